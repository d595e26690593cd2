// Device side of the contextual-biasing beam-search decoder (gfx950).
//
// One workgroup owns one channel for a whole cbd_advance call and walks its
// frames in order; channels never interact (paper Sec. 3.2: streams are decoded
// in parallel, each with its own boosting; the graph is shared and read-only).
// Per frame the workgroup runs, separated by workgroup barriers only:
//   emit     wave-level prefix scan over the surviving tokens' emitting
//            out-degrees, one lane per arc (the "load balancing expand" of
//            Sec. 3.2), bias lookup per arc (Sec. 4.2), candidate cost, cutoff
//            against the running minimum, recombination by a 64-bit atomic min
//            on (orderable cost << 32 | arc) in an open-addressing state table;
//   closure  rounds over the change log: states whose value changed and that
//            have epsilon-input arcs are expanded again until nothing changes;
//   compact  the change log names each state's winning update exactly once;
//            the winner writes the token, its back-pointer record and the
//            pruning histogram, and clears its table slot.
// The state table, the token list and the log-likelihood row live in LDS when
// they fit (kLds), otherwise the tables are per-channel arrays in device memory.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cbd {

constexpr uint32_t kEmptyKey = 0xFFFFFFFFu;   // state table: free slot
constexpr uint64_t kEmptyVal = ~0ull;
constexpr uint32_t kArcNone = 0xFFFFFFFFu;    // start token's arc; sorts after every real arc
constexpr uint32_t kSrcEps = 0x80000000u;     // change-log src: index into the current frame's tokens
constexpr uint32_t kSrcHasEps = 0x40000000u;  // change-log src: the updated state has epsilon-input arcs
constexpr uint32_t kSrcMask = 0x3FFFFFFFu;
constexpr uint32_t kSrcNone = 0x3FFFFFFFu;    // start token: no predecessor
constexpr uint32_t kMetaDstHasEps = 0x80000000u;

constexpr int kStatusOk = 0;
constexpr int kStatusCapacity = -2;
constexpr int kStatusEpsDiverged = -3;
constexpr int kStatusNoTokens = -4;
constexpr int kStatusBuffer = -5;

// One arc in the library's own order (per state: emitting arcs, then epsilon-input arcs).
struct __attribute__((aligned(16))) ArcRec {
  int32_t dst;
  float weight;
  uint32_t meta;   // bits 0..30 ilabel (0 = epsilon input, else pdf + 1); bit 31: dst has epsilon-input arcs
  int32_t olabel;
};

// One table update: slot h took the value `key` through an arc leaving token `src`.
struct __attribute__((aligned(16))) LogEntry {
  uint64_t key;
  uint32_t h;
  uint32_t src;
};

// Per-channel state that survives between calls.
struct __attribute__((aligned(128))) ChanState {
  int32_t n_tok;        // entries of the current token list (dead ones included)
  int32_t frame_base;   // back-pointer record of token 0 of the current frame
  int32_t n_rec;        // back-pointer records in use
  int32_t status;       // sticky
  float best;           // minimum cost of the current table
  int32_t cut_bin;      // histogram cut for the next prune; 255 = none
  int32_t ctx_n;
  float ctx_offset;
  long long frames, active_tokens, emit_arcs, eps_arcs, candidates, improvements, tokens, eps_rounds;
  int32_t max_tokens;
  int32_t pad[7];
};

struct AdvanceParams {
  const int2 *off2;        // [S+1]: x = first arc of the state, y = first epsilon-input arc of the state
  const ArcRec *arcs;      // [A]
  int32_t start_state;
  int32_t num_pdfs;
  ChanState *chan;         // [C]
  const int32_t *chan_ids; // [grid] channel of each workgroup
  const float *loglikes;
  long long channel_stride;
  int32_t n_frames;
  int32_t do_reset;
  float beam;
  int32_t max_active;
  int32_t max_eps_iters;
  int32_t lookup_mode;
  int32_t log_h;           // table slots = 1 << log_h
  int32_t tok_cap;
  int32_t log_cap;
  int32_t bp_cap;
  int32_t max_ctx;         // row length of ctx
  int32_t ctx_lds_cap;     // context entries that fit the LDS copy
  int32_t *tok_state;      // [C][tok_cap]
  float *tok_cost;         // [C][tok_cap]
  int2 *bp;                // [C][bp_cap] (arc, predecessor record or -1)
  LogEntry *log;           // [C][log_cap]
  const int32_t *ctx;      // [C][max_ctx] sorted, library arc order
  uint32_t *g_hkey;        // [C][H]  tables in device memory (unused with kLds)
  uint64_t *g_hval;        // [C][H]
  uint32_t *g_haux;        // [C][H]
};

// Workgroup-shared scalars.
struct Shared {
  uint32_t m_ord;      // running minimum of emitting candidates (orderable bits)
  uint32_t best_ord;   // minimum over all accepted candidates of the frame
  int32_t n_claim;     // states in the table = tokens of the frame
  int32_t log_n;
  int32_t n_front;     // log entries of the last phase whose state has epsilon-input arcs
  int32_t n_surv;      // tokens within the beam of best
  int32_t n_live;      // tokens that passed the frame cutoff
  int32_t fault;       // capacity overflow seen
  int32_t n_tok, frame_base, n_rec, status, cut_bin, fr_begin, fr_end, rounds;
  float best;
  uint32_t c_active, c_emit, c_eps, c_cand;
};

struct LdsLayout {
  uint32_t sh, hist, bitmap, ctx, L, hval, hkey, haux, tst, tco, total;
};

__host__ __device__ inline uint32_t align_up(uint32_t x, uint32_t a) { return (x + a - 1) / a * a; }

__host__ __device__ inline LdsLayout make_layout(int num_pdfs, int ctx_lds_cap, int log_h, int tok_cap, bool lds_tables) {
  LdsLayout l;
  uint32_t o = 0;
  l.sh = o; o += align_up((uint32_t)sizeof(Shared), 16);
  l.hist = o; o += 256 * 4;
  l.bitmap = o; o += 256 * 4;
  l.ctx = o; o += align_up((uint32_t)ctx_lds_cap * 4, 16);
  l.L = o; o += align_up((uint32_t)num_pdfs * 4, 16);
  l.hval = l.hkey = l.haux = l.tst = l.tco = 0;
  if (lds_tables) {
    uint32_t H = 1u << log_h;
    l.hval = o; o += H * 8;
    l.hkey = o; o += H * 4;
    l.haux = o; o += H * 4;
    l.tst = o; o += align_up((uint32_t)tok_cap * 4, 16);
    l.tco = o; o += align_up((uint32_t)tok_cap * 4, 16);
  }
  l.total = o;
  return l;
}

// ---- small helpers -------------------------------------------------------

// Monotone map of fp32 to uint32 (exact: no quantisation).  -0 is folded into +0 first.
__device__ __forceinline__ uint32_t f2ord(float f) {
  uint32_t b = __float_as_uint(f + 0.0f);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t o) {
  uint32_t b = o ^ ((o >> 31) ? 0x80000000u : 0xFFFFFFFFu);
  return __uint_as_float(b);
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    uint32_t t = (uint32_t)__shfl_xor((int)v, d, 64);
    v = t < v ? t : v;
  }
  return v;
}

// Accessors for values that other waves change with atomics.
template <bool kLds> __device__ __forceinline__ uint32_t ld32(const uint32_t *p) {
  if (kLds) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool kLds> __device__ __forceinline__ uint64_t ld64(const uint64_t *p) {
  if (kLds) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool kLds> __device__ __forceinline__ void st32(uint32_t *p, uint32_t v) {
  if (kLds) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool kLds> __device__ __forceinline__ void st64(uint64_t *p, uint64_t v) {
  if (kLds) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sec. 4.2: the listed arc indices are kept sorted and searched per expanded arc.
__device__ __forceinline__ bool sorted_contains(const int32_t *list, int n, int32_t a) {
  int lo = 0, hi = n;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (list[mid] < a) lo = mid + 1; else hi = mid;
  }
  return lo < n && list[lo] == a;
}

__device__ __forceinline__ uint32_t bitmap_bit(int32_t a) { return ((uint32_t)a * 2654435761u) >> 19; }  // 13 bits

struct Ctx {
  const int32_t *lds_list;
  const int32_t *g_list;
  const uint32_t *bitmap;
  int n;
  bool in_lds;
  bool use_bitmap;
  float offset;
};

__device__ __forceinline__ bool ctx_contains(const Ctx &cx, int32_t a) {
  if (cx.n == 0) return false;
  if (cx.use_bitmap) {
    uint32_t b = bitmap_bit(a);
    if (!((cx.bitmap[b >> 5] >> (b & 31)) & 1u)) return false;
  }
  if (cx.in_lds) return sorted_contains(cx.lds_list, cx.n, a);
  return sorted_contains(cx.g_list, cx.n, a);
}

template <bool kLds> struct Tables {
  uint64_t *hval;
  uint32_t *hkey;
  uint32_t *haux;
  int32_t *tok_state;
  float *tok_cost;
  uint32_t mask;
  int shift;
};

// Recombination: E[state] = min key.  Returns true if this call lowered the
// state's value (old > key); h receives the slot.
template <bool kLds>
__device__ __forceinline__ bool table_min(const Tables<kLds> &T, Shared *sh, int tok_cap, uint32_t state, uint64_t key,
                                          uint32_t &h_out) {
  uint32_t h = (state * 2654435761u) >> T.shift;
  for (uint32_t probe = 0; probe <= T.mask; ++probe) {
    uint32_t k = ld32<kLds>(&T.hkey[h]);
    if (k == kEmptyKey) {
      k = atomicCAS(&T.hkey[h], kEmptyKey, state);
      if (k == kEmptyKey) {
        int idx = atomicAdd(&sh->n_claim, 1);
        if (idx >= tok_cap) sh->fault = 1;
        st32<kLds>(&T.haux[h], (uint32_t)idx);
        k = state;
      }
    }
    if (k == state) {
      uint64_t old = atomicMin((unsigned long long *)&T.hval[h], (unsigned long long)key);
      h_out = h;
      return old > key;
    }
    h = (h + 1) & T.mask;
  }
  sh->fault = 1;
  h_out = 0;
  return false;
}

// Append the updates of this wave's lanes to the channel's change log.
__device__ __forceinline__ void log_append(LogEntry *log, int log_cap, Shared *sh, bool improved, uint64_t key,
                                           uint32_t h, uint32_t src, int lane) {
  unsigned long long mask = __ballot(improved);
  if (mask == 0) return;
  int leader = __ffsll((long long)mask) - 1;
  int n = __popcll(mask);
  int nf = __popcll(__ballot(improved && (src & kSrcHasEps)));
  int base = 0;
  if (lane == leader) {
    base = atomicAdd(&sh->log_n, n);
    if (nf) atomicAdd(&sh->n_front, nf);
  }
  base = __shfl(base, leader, 64);
  if (improved) {
    int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
    if (pos < log_cap) {
      LogEntry e; e.key = key; e.h = h; e.src = src;
      log[pos] = e;
    } else {
      sh->fault = 1;
    }
  }
}

// Expand `deg` arcs starting at `first` for each lane's item (deg = 0: none),
// one lane per arc.  kEmit: cand = (cost + w') - L[pdf]; else cand = cost + w'.
template <bool kLds, bool kEmit>
__device__ __forceinline__ void expand_rows(const AdvanceParams &p, const Tables<kLds> &T, Shared *sh, const Ctx &cx,
                                            const float *Lrow, LogEntry *log, int first, int deg, float cost,
                                            uint32_t src_tag, float m_fixed, int lane) {
  int incl = wave_incl_scan(deg, lane);
  int pos = incl - deg;
  int total = __shfl(incl, 63, 64);
  if (total == 0) return;
  if (lane == 0) {
    if (kEmit) atomicAdd(&sh->c_emit, (uint32_t)total); else atomicAdd(&sh->c_eps, (uint32_t)total);
  }
  int rel = first - pos;  // arc index = rel + position in the wave's arc list
  for (int j0 = 0; j0 < total; j0 += 64) {
    int jj = j0 + lane;
    bool act = jj < total;
    // owner = last lane whose first position is <= jj
    int owner = 0;
#pragma unroll
    for (int step = 32; step >= 1; step >>= 1) {
      int cand = owner + step;
      int pc = __shfl(pos, cand & 63, 64);
      if (cand < 64 && pc <= jj) owner = cand;
    }
    int a = __shfl(rel, owner, 64) + jj;
    float c_own = __shfl(cost, owner, 64);
    uint32_t s_own = (uint32_t)__shfl((int)src_tag, owner, 64);
    bool pass = false;
    float cand = 0.0f;
    ArcRec rec; rec.dst = 0; rec.weight = 0.0f; rec.meta = 0; rec.olabel = 0;
    if (act) {
      rec = p.arcs[a];
      float w = rec.weight;
      if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
      if (kEmit) {
        cand = (c_own + w) - Lrow[(rec.meta & 0x7FFFFFFFu) - 1u];
        float mrun = ord2f(__hip_atomic_load(&sh->m_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
        pass = !(cand - mrun > p.beam);
      } else {
        cand = c_own + w;
        pass = !(cand - m_fixed > p.beam);
      }
    }
    uint32_t co = pass ? f2ord(cand) : 0xFFFFFFFFu;
    uint32_t wmin = wave_min_u32(co);
    unsigned long long pmask = __ballot(pass);
    if (pmask == 0) continue;
    if (lane == 0) {
      if (kEmit) atomicMin(&sh->m_ord, wmin); else atomicMin(&sh->best_ord, wmin);
      atomicAdd(&sh->c_cand, (uint32_t)__popcll(pmask));
    }
    bool improved = false;
    uint32_t h = 0;
    uint64_t key = ((uint64_t)co << 32) | (uint32_t)a;
    if (pass && !sh->fault) improved = table_min<kLds>(T, sh, p.tok_cap, (uint32_t)rec.dst, key, h);
    uint32_t src = s_own | ((rec.meta & kMetaDstHasEps) ? kSrcHasEps : 0u);
    log_append(log, p.log_cap, sh, improved, key, h, src, lane);
  }
}

template <bool kLds, int kBlock>
__global__ __launch_bounds__(kBlock) void advance_kernel(AdvanceParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NW = kBlock / 64;
  constexpr int kPre = 8;  // log-likelihood values each thread holds while the next row is in flight
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = p.chan_ids[blockIdx.x];
  ChanState *cs = p.chan + c;
  const LdsLayout lay = make_layout(p.num_pdfs, p.ctx_lds_cap, p.log_h, p.tok_cap, kLds);
  Shared *sh = (Shared *)(smem + lay.sh);
  uint32_t *hist = (uint32_t *)(smem + lay.hist);
  uint32_t *bitmap = (uint32_t *)(smem + lay.bitmap);
  int32_t *ctx_lds = (int32_t *)(smem + lay.ctx);
  float *Lrow = (float *)(smem + lay.L);
  const uint32_t H = 1u << p.log_h;

  Tables<kLds> T;
  T.mask = H - 1; T.shift = 32 - p.log_h;
  if (kLds) {
    T.hval = (uint64_t *)(smem + lay.hval);
    T.hkey = (uint32_t *)(smem + lay.hkey);
    T.haux = (uint32_t *)(smem + lay.haux);
    T.tok_state = (int32_t *)(smem + lay.tst);
    T.tok_cost = (float *)(smem + lay.tco);
  } else {
    T.hval = p.g_hval + (size_t)c * H;
    T.hkey = p.g_hkey + (size_t)c * H;
    T.haux = p.g_haux + (size_t)c * H;
    T.tok_state = p.tok_state + (size_t)c * p.tok_cap;
    T.tok_cost = p.tok_cost + (size_t)c * p.tok_cap;
  }
  int32_t *g_tok_state = p.tok_state + (size_t)c * p.tok_cap;
  float *g_tok_cost = p.tok_cost + (size_t)c * p.tok_cap;
  int2 *bp = p.bp + (size_t)c * p.bp_cap;
  LogEntry *log = p.log + (size_t)c * p.log_cap;
  const float *Lbase = p.loglikes + (long long)blockIdx.x * p.channel_stride;

  if (tid == 0) {
    sh->status = p.do_reset ? kStatusOk : cs->status;
    sh->n_tok = p.do_reset ? 0 : cs->n_tok;
    sh->frame_base = p.do_reset ? 0 : cs->frame_base;
    sh->n_rec = p.do_reset ? 0 : cs->n_rec;
    sh->best = p.do_reset ? 0.0f : cs->best;
    sh->cut_bin = p.do_reset ? 255 : cs->cut_bin;
    sh->fault = 0;
    sh->n_claim = 1;  // only a decoded frame that produced nothing parks the channel
    sh->c_active = sh->c_emit = sh->c_eps = sh->c_cand = 0;
  }
  __syncthreads();
  if (sh->status != kStatusOk) return;  // uniform: the channel is parked until reset

  // context of this call (Sec. 4.3: whichever list is current is the one used)
  Ctx cx;
  cx.n = cs->ctx_n; cx.offset = cs->ctx_offset;
  cx.g_list = p.ctx + (size_t)c * p.max_ctx;
  cx.lds_list = ctx_lds; cx.bitmap = bitmap;
  cx.in_lds = cx.n <= p.ctx_lds_cap;
  cx.use_bitmap = p.lookup_mode == 1;
  if (cx.in_lds) for (int i = tid; i < cx.n; i += kBlock) ctx_lds[i] = cx.g_list[i];
  if (cx.use_bitmap) {
    for (int i = tid; i < 256; i += kBlock) bitmap[i] = 0;
    __syncthreads();
    for (int i = tid; i < cx.n; i += kBlock) {
      uint32_t b = bitmap_bit(cx.g_list[i]);
      atomicOr(&bitmap[b >> 5], 1u << (b & 31));
    }
  }
  if (kLds) {
    for (uint32_t i = tid; i < H; i += kBlock) { T.hval[i] = kEmptyVal; T.hkey[i] = kEmptyKey; }
    for (int i = tid; i < sh->n_tok; i += kBlock) { T.tok_state[i] = g_tok_state[i]; T.tok_cost[i] = g_tok_cost[i]; }
  }
  if (p.n_frames > 0) for (int i = tid; i < p.num_pdfs; i += kBlock) Lrow[i] = Lbase[i];

  long long st_frames = 0, st_active = 0, st_emit = 0, st_eps = 0, st_cand = 0, st_impr = 0, st_tok = 0, st_rounds = 0;
  int st_maxtok = 0;
  const bool hist_on = p.max_active > 0 && p.beam > 0.0f && p.beam < __builtin_inff();
  const float inv = 256.0f / p.beam;

  for (int f = p.do_reset ? -1 : 0; f < p.n_frames; ++f) {
    if (tid == 0) {
      sh->m_ord = f < 0 ? f2ord(0.0f) : 0xFFFFFFFFu;
      sh->n_claim = 0; sh->log_n = 0; sh->n_front = 0; sh->n_surv = 0; sh->n_live = 0; sh->rounds = 0;
    }
    for (int i = tid; i < 256; i += kBlock) hist[i] = 0;
    __syncthreads();

    // next frame's row starts its way from HBM now and is parked in registers
    float pre[kPre];
    const bool have_next = f + 1 < p.n_frames && f >= 0;
    const float *Lnext = Lbase + (long long)(f + 1) * p.num_pdfs;
#pragma unroll
    for (int k = 0; k < kPre; ++k) {
      int i = tid + k * kBlock;
      pre[k] = (have_next && i < p.num_pdfs) ? Lnext[i] : 0.0f;
    }

    if (f < 0) {
      // reset: one start token at cost 0
      if (wave == 0) {
        bool me = lane == 0;
        uint32_t h = 0;
        uint64_t key = ((uint64_t)f2ord(0.0f) << 32) | kArcNone;
        bool improved = false;
        if (me) improved = table_min<kLds>(T, sh, p.tok_cap, (uint32_t)p.start_state, key, h);
        int2 o = p.off2[p.start_state], o2 = p.off2[p.start_state + 1];
        uint32_t src = kSrcNone | ((o2.x > o.y) ? kSrcHasEps : 0u);
        log_append(log, p.log_cap, sh, improved, key, h, src, lane);
      }
    } else {
      // ---- emit: prune (step 1) and expand emitting arcs (step 2)
      const int n_tok = sh->n_tok;
      const float best = sh->best;
      const int cut = sh->cut_bin;
      for (int tile = wave; tile * 64 < n_tok; tile += NW) {
        int i = tile * 64 + lane;
        bool alive = false;
        float cost = 0.0f;
        int s = -1;
        if (i < n_tok) {
          s = T.tok_state[i];
          cost = T.tok_cost[i];
          if (s >= 0) {
            float r = cost - best;
            alive = !(r > p.beam);
            if (alive && cut < 255) {
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              alive = bin <= cut;
            }
          }
        }
        int first = 0, deg = 0;
        if (alive) {
          int2 o = p.off2[s];
          first = o.x; deg = o.y - o.x;
        }
        unsigned long long am = __ballot(alive);
        if (lane == 0 && am) atomicAdd(&sh->c_active, (uint32_t)__popcll(am));
        expand_rows<kLds, true>(p, T, sh, cx, Lrow, log, first, deg, cost, (uint32_t)i, 0.0f, lane);
      }
    }
    __syncthreads();

    // ---- step 3: the emission minimum fixes the frame's cutoff
    const float m = ord2f(sh->m_ord);
    if (tid == 0) { sh->best_ord = sh->m_ord; sh->fr_begin = 0; sh->fr_end = sh->log_n; }
    __syncthreads();
    if (sh->n_claim == 0 || sh->fault) break;

    // ---- step 4: epsilon closure, one round per barrier
    while (sh->n_front > 0) {
      const int fb = sh->fr_begin, fe = sh->fr_end;
      __syncthreads();
      if (tid == 0) sh->n_front = 0;
      __syncthreads();
      for (int tile = wave; fb + tile * 64 < fe; tile += NW) {
        int j = fb + tile * 64 + lane;
        bool act = false;
        float cost = 0.0f;
        int first = 0, deg = 0;
        uint32_t src_tag = 0;
        if (j < fe) {
          LogEntry e = log[j];
          if (e.src & kSrcHasEps) {
            uint64_t cur = ld64<kLds>(&T.hval[e.h]);
            cost = ord2f((uint32_t)(e.key >> 32));
            act = cur == e.key && !(cost - m > p.beam);
            if (act) {
              uint32_t s = ld32<kLds>(&T.hkey[e.h]);
              int2 o = p.off2[s], o2 = p.off2[s + 1];
              first = o.y; deg = o2.x - o.y;
              src_tag = ld32<kLds>(&T.haux[e.h]) | kSrcEps;
            }
          }
        }
        expand_rows<kLds, false>(p, T, sh, cx, Lrow, log, first, deg, cost, src_tag, m, lane);
      }
      __syncthreads();
      if (tid == 0) {
        sh->fr_begin = fe; sh->fr_end = sh->log_n; sh->rounds++;
        if (sh->n_front > 0 && sh->rounds >= p.max_eps_iters) sh->status = kStatusEpsDiverged;
      }
      __syncthreads();
      if (sh->status != kStatusOk || sh->fault) break;
    }
    if (sh->status != kStatusOk || sh->fault) break;
    if (sh->n_rec + sh->n_claim > p.bp_cap || sh->n_claim > p.tok_cap) {
      __syncthreads();
      if (tid == 0) sh->fault = 1;
      __syncthreads();
      break;
    }

    // ---- step 5 and bookkeeping: every state's winning update writes the token
    {
      const float best = ord2f(sh->best_ord);
      const int base_cur = sh->n_rec, base_prev = sh->frame_base, log_n = sh->log_n;
      int my_surv = 0, my_live = 0;
      for (int j = tid; j < log_n; j += kBlock) {
        LogEntry e = log[j];
        uint64_t cur = ld64<kLds>(&T.hval[e.h]);
        if (cur != e.key) continue;
        int idx = (int)ld32<kLds>(&T.haux[e.h]);
        int s = (int)ld32<kLds>(&T.hkey[e.h]);
        float cost = ord2f((uint32_t)(e.key >> 32));
        bool dead = cost - m > p.beam;
        uint32_t sf = e.src & kSrcMask;
        int prev = sf == kSrcNone ? -1 : ((e.src & kSrcEps) ? base_cur + (int)sf : base_prev + (int)sf);
        T.tok_state[idx] = dead ? -1 : s;
        T.tok_cost[idx] = cost;
        bp[base_cur + idx] = make_int2((int)(uint32_t)e.key, prev);
        if (!dead) {
          my_live++;
          float r = cost - best;
          if (!(r > p.beam)) {
            my_surv++;
            if (hist_on) {
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              atomicAdd(&hist[bin], 1u);
            }
          }
        }
        st32<kLds>(&T.hkey[e.h], kEmptyKey);
        st64<kLds>(&T.hval[e.h], kEmptyVal);
      }
      if (my_surv) atomicAdd(&sh->n_surv, my_surv);
      if (my_live) atomicAdd(&sh->n_live, my_live);
    }
    __syncthreads();

    // ---- close the frame
    if (wave == 0) {
      int cut = 255;
      if (hist_on && sh->n_surv > p.max_active) {
        // largest bin B whose cumulative count fits max_active (0 if bin 0 alone does not)
        int loc[4], sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { loc[k] = (int)hist[lane * 4 + k]; sum += loc[k]; }
        int incl = wave_incl_scan(sum, lane);
        int run = incl - sum;
        int myB = -1;
#pragma unroll
        for (int k = 0; k < 4; ++k) { run += loc[k]; if (run <= p.max_active) myB = lane * 4 + k; }
        // cumulative counts are monotone, so the bins that fit form a prefix: take the maximum
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { int t = __shfl_xor(myB, d, 64); myB = t > myB ? t : myB; }
        cut = myB < 0 ? 0 : myB;
      }
      if (lane == 0) {
        sh->cut_bin = cut;
        sh->n_tok = sh->n_claim;
        sh->frame_base = sh->n_rec;
        sh->n_rec += sh->n_claim;
        sh->best = ord2f(sh->best_ord);
        if (f >= 0) {  // the table made at reset is not a decoded frame
          st_frames++;
          st_tok += sh->n_live;
          if (sh->n_live > st_maxtok) st_maxtok = sh->n_live;
        }
        st_active += sh->c_active; st_emit += sh->c_emit; st_eps += sh->c_eps; st_cand += sh->c_cand;
        st_impr += sh->log_n; st_rounds += sh->rounds;
        sh->c_active = sh->c_emit = sh->c_eps = sh->c_cand = 0;
      }
    }
    // park the prefetched row in LDS for the next frame
    if (have_next) {
#pragma unroll
      for (int k = 0; k < kPre; ++k) {
        int i = tid + k * kBlock;
        if (i < p.num_pdfs) Lrow[i] = pre[k];
      }
      for (int i = tid + kPre * kBlock; i < p.num_pdfs; i += kBlock) Lrow[i] = Lnext[i];
    }
    __syncthreads();
  }

  // ---- leave: a frame that produced nothing or overflowed parks the channel
  __syncthreads();
  if (tid == 0) {
    int status = sh->status;
    if (status == kStatusOk && sh->fault) status = kStatusCapacity;
    if (status == kStatusOk && sh->n_claim == 0) { status = kStatusNoTokens; sh->n_tok = 0; sh->frame_base = sh->n_rec; }
    sh->status = status;
    cs->status = status;
    cs->n_tok = status == kStatusOk ? sh->n_tok : 0;
    cs->frame_base = sh->frame_base;
    cs->n_rec = sh->n_rec;
    cs->best = sh->best;
    cs->cut_bin = sh->cut_bin;
    if (p.do_reset) {
      cs->frames = 0; cs->active_tokens = 0; cs->emit_arcs = 0; cs->eps_arcs = 0; cs->candidates = 0;
      cs->improvements = 0; cs->tokens = 0; cs->eps_rounds = 0; cs->max_tokens = 0;
    }
    cs->frames += st_frames; cs->active_tokens += st_active; cs->emit_arcs += st_emit; cs->eps_arcs += st_eps;
    cs->candidates += st_cand; cs->improvements += st_impr; cs->tokens += st_tok; cs->eps_rounds += st_rounds;
    if (st_maxtok > cs->max_tokens) cs->max_tokens = st_maxtok;
  }
  __syncthreads();
  if (kLds && sh->status == kStatusOk) {
    for (int i = tid; i < sh->n_tok; i += kBlock) { g_tok_state[i] = T.tok_state[i]; g_tok_cost[i] = T.tok_cost[i]; }
  }
  if (!kLds && sh->status != kStatusOk) {
    // leave the device-memory table empty for the next utterance
    for (uint32_t i = tid; i < H; i += kBlock) { st32<false>(&T.hkey[i], kEmptyKey); st64<false>(&T.hval[i], kEmptyVal); }
  }
}

// ---- contexts ---------------------------------------------------------------

// One workgroup per listed channel copies its sorted list into the channel's row.
__global__ void scatter_contexts_kernel(const int32_t *chan_ids, const int32_t *list_off, const float *offsets,
                                        const int32_t *lists, int32_t *ctx, int max_ctx, ChanState *chan) {
  int i = blockIdx.x;
  int c = chan_ids[i];
  int b = list_off[i], n = list_off[i + 1] - b;
  for (int k = threadIdx.x; k < n; k += blockDim.x) ctx[(size_t)c * max_ctx + k] = lists[b + k];
  if (threadIdx.x == 0) { chan[c].ctx_n = n; chan[c].ctx_offset = offsets[i]; }
}

__global__ void init_tables_kernel(uint32_t *hkey, uint64_t *hval, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { hkey[i] = kEmptyKey; hval[i] = kEmptyVal; }
}

__global__ void init_chan_kernel(ChanState *chan, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    ChanState z;
    unsigned char *b = (unsigned char *)&z;
    for (size_t k = 0; k < sizeof(ChanState); ++k) b[k] = 0;
    z.status = kStatusNoTokens;  // until reset
    z.cut_bin = 255;
    chan[i] = z;
  }
}

// ---- best path ----------------------------------------------------------------

struct BestParams {
  const ChanState *chan;
  const int32_t *chan_ids;
  const int32_t *tok_state;
  const float *tok_cost;
  const int2 *bp;
  const ArcRec *arcs;
  const int32_t *int2pub;   // library arc order -> caller's numbering
  const float *final_cost;  // or null
  int32_t tok_cap, bp_cap, use_final, capacity;
  int32_t *out_arcs;        // [n][capacity]
  int32_t *out_words;       // [n][capacity]
  int32_t *out_meta;        // [n][4]: status, n_arcs, n_words, cost bits
};

// One wave per channel: best token (Sec. 1: the current best token sequence is
// read directly, no lattice), then the back-pointer walk, then olabels in time order.
__global__ __launch_bounds__(64) void best_path_kernel(BestParams p) {
  const int lane = threadIdx.x;
  const int i = blockIdx.x;
  const int c = p.chan_ids[i];
  const ChanState *cs = p.chan + c;
  int32_t *meta = p.out_meta + (size_t)i * 4;
  int32_t *oarcs = p.out_arcs + (size_t)i * p.capacity;
  int32_t *owords = p.out_words + (size_t)i * p.capacity;
  if (cs->status != kStatusOk) {
    if (lane == 0) { meta[0] = cs->status; meta[1] = 0; meta[2] = 0; meta[3] = (int)__float_as_uint(__builtin_inff()); }
    return;
  }
  const int n = cs->n_tok, base = cs->frame_base;
  const int32_t *ts = p.tok_state + (size_t)c * p.tok_cap;
  const float *tc = p.tok_cost + (size_t)c * p.tok_cap;
  const int2 *bp = p.bp + (size_t)c * p.bp_cap;
  uint64_t bestk = kEmptyVal;
  int besti = -1;
  for (int t = lane; t < n; t += 64) {
    int s = ts[t];
    if (s < 0) continue;
    float cost = tc[t];
    if (p.use_final && p.final_cost) cost = cost + p.final_cost[s];
    if (!(cost < __builtin_inff())) continue;
    uint64_t k = ((uint64_t)f2ord(cost) << 32) | (uint32_t)bp[base + t].x;
    if (k < bestk) { bestk = k; besti = t; }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    uint64_t ok = (uint64_t)__shfl_xor((long long)bestk, d, 64);
    int oi = __shfl_xor(besti, d, 64);
    if (ok < bestk) { bestk = ok; besti = oi; }
  }
  if (besti < 0) {
    if (lane == 0) { meta[0] = kStatusNoTokens; meta[1] = 0; meta[2] = 0; meta[3] = (int)__float_as_uint(__builtin_inff()); }
    return;
  }
  // walk back: lane 0 writes the arcs newest-first into the output row
  // (a path can never be longer than the records in use; the bound also ends
  // the walk on a predecessor cycle, which zero-weight epsilon cycles can form)
  const int max_steps = cs->n_rec;
  int na = 0;
  if (lane == 0) {
    int r = base + besti;
    while (r >= 0 && na <= max_steps) {
      int2 rec = bp[r];
      if ((uint32_t)rec.x == kArcNone) break;
      if (na < p.capacity) oarcs[na] = rec.x;
      na++;
      r = rec.y;
    }
  }
  na = __shfl(na, 0, 64);
  __threadfence_block();
  if (na > max_steps) {
    if (lane == 0) { meta[0] = kStatusEpsDiverged; meta[1] = 0; meta[2] = 0; meta[3] = (int)__float_as_uint(__builtin_inff()); }
    return;
  }
  if (na > p.capacity) {
    // count the words too so the caller learns both sizes
    int nw = 0;
    if (lane == 0) {
      int r = base + besti;
      for (int step = 0; r >= 0 && step < na; ++step) {
        int2 rec = bp[r];
        if ((uint32_t)rec.x == kArcNone) break;
        if (p.arcs[rec.x].olabel != 0) nw++;
        r = rec.y;
      }
      meta[0] = kStatusBuffer; meta[1] = na; meta[2] = nw; meta[3] = (int)__float_as_uint(ord2f((uint32_t)(bestk >> 32)));
    }
    return;
  }
  // reverse into time order, pick up word labels, translate to the caller's numbering
  int nw_total = 0;
  for (int j0 = 0; j0 < (na + 1) / 2; j0 += 64) {
    int j = j0 + lane;
    if (j < (na + 1) / 2) {
      int k = na - 1 - j;
      int a = oarcs[j], b = oarcs[k];
      oarcs[j] = b; oarcs[k] = a;
    }
  }
  __threadfence_block();
  for (int j0 = 0; j0 < na; j0 += 64) {
    int j = j0 + lane;
    int w = 0, a = 0;
    if (j < na) { a = oarcs[j]; w = p.arcs[a].olabel; }
    unsigned long long wm = __ballot(w != 0);
    if (w != 0) owords[nw_total + __popcll(wm & ((1ull << lane) - 1ull))] = w;
    nw_total += __popcll(wm);
    if (j < na) oarcs[j] = p.int2pub[a];
  }
  if (lane == 0) {
    meta[0] = kStatusOk; meta[1] = na; meta[2] = nw_total;
    meta[3] = (int)__float_as_uint(ord2f((uint32_t)(bestk >> 32)));
  }
}

}  // namespace cbd
