// Device side of the contextual-biasing beam-search decoder (gfx950).
//
// One workgroup owns one channel for a whole cbd_advance call and walks its
// frames in order; channels never interact (paper Sec. 3.2: streams are decoded
// in parallel, each with its own boosting; the graph is shared and read-only).
// Per frame the workgroup runs, separated by workgroup barriers only:
//   emit     wave-level prefix scan over the surviving tokens' emitting
//            out-degrees, one lane per arc (the "load balancing expand" of
//            Sec. 3.2), bias lookup per arc (Sec. 4.2), candidate cost.  A
//            batch's candidates wait in registers until the batch minimum is
//            known, then pass the cutoff and are recombined by a 64-bit atomic
//            min on (orderable cost << 32 | arc) in an open-addressing table;
//   closure  states whose value changed and that have epsilon-input arcs are
//            expanded again until nothing changes: every wave follows the chains
//            it starts without barriers (the children of a pass stay in its
//            registers); only oversized passes go back through the change log;
//   compact  the change log names each state's winning update exactly once;
//            the winner writes the token, its back-pointer record and the
//            pruning histogram, and frees its table slot.
// Every arc record carries the row of its destination state, so expanding a
// token needs no offset lookup: the only dependent HBM access of a phase is the
// arc read itself.  Table, tokens, change log and the log-likelihood row live in
// LDS (kLds); a frame that outgrows them is redone with per-channel tables in
// device memory, and decoding returns to LDS once the token list fits again.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cbd {

constexpr uint32_t kEmptyKey = 0xFFFFFFFFu;   // state table: free slot
constexpr uint64_t kEmptyVal = ~0ull;
constexpr uint32_t kArcNone = 0xFFFFFFFFu;    // start token's arc; sorts after every real arc

constexpr int kStatusOk = 0;
constexpr int kStatusCapacity = -2;
constexpr int kStatusEpsDiverged = -3;
constexpr int kStatusNoTokens = -4;
constexpr int kStatusBuffer = -5;

// frame outcomes inside the kernel
constexpr int kFrameOk = 0, kFrameOverflow = 1, kFrameNoTokens = 2, kFrameDiverged = 3, kFrameRecordsFull = 4,
              kFrameRedo = 5;   // (lean frames only) nothing lasting was written: decode the frame with the general code

// One record of the arc array.  Per state the array holds: its emitting arcs, its epsilon-input arcs, and then
// its closure list: every state reachable from it through epsilon-input arcs alone, one record per path, in
// depth-first preorder (a copy of the arc that ends the path, with the path's depth).  With the closure list a
// whole epsilon closure is one contiguous read.  Arcs keep their identity: a record of a closure list names the
// arc it copies (its position among the state rows) in the parallel array `canon`.
struct __attribute__((aligned(16))) ArcRec {
  int32_t dst;
  float weight;
  int32_t row;     // first arc of dst
  uint32_t meta;   // bits 0..15: ilabel (0 = epsilon input, else pdf + 1); in a closure list: bits 0..3 the path's
                   //   depth (1..), bits 4..9 the position in the list of the record one arc shorter, plus 1 (0: none)
                   // bits 16..21 number of emitting arcs of dst, 22..25 number of epsilon-input arcs of dst
                   //   (all ones in either field: look the row up in the offsets array)
                   // bits 26..31 records in dst's closure list (all ones: the list is not stored, too deep or long)
};
constexpr uint32_t kEdEscape = 63, kXdEscape = 15, kClEscape = 63;
constexpr int kClosureMaxDepth = 15;   // deeper closures are not flattened (the general closure code takes them);
                                       // the depth field of a closure record holds 4 bits
__host__ __device__ inline uint32_t meta_ed(uint32_t m) { return (m >> 16) & 63u; }
__host__ __device__ inline uint32_t meta_xd(uint32_t m) { return (m >> 22) & 15u; }
__host__ __device__ inline uint32_t meta_cl(uint32_t m) { return m >> 26; }
__host__ __device__ inline uint32_t make_meta(uint32_t low16, uint32_t ed, uint32_t xd, uint32_t cl) {
  return (low16 & 0xFFFFu) | ((ed < kEdEscape ? ed : kEdEscape) << 16) | ((xd < kXdEscape ? xd : kXdEscape) << 22) |
         ((cl < kClEscape ? cl : kClEscape) << 26);
}

// Change-log entry: slot h took a value through arc `arc`.  `src` names where the arc
// started: a token index of the previous frame (emitting arc), or, with kSrcEps, the
// table slot of the source state in this frame (epsilon-input arc).  kSrcHasEps marks an
// entry whose state has epsilon-input arcs that nobody has expanded for this value yet.
// LDS form: 8 bytes; device-memory form: wide indices.
template <bool kLds> struct LogT;
template <> struct LogT<true> {
  uint32_t arc; uint16_t h; uint16_t src;
  static constexpr uint32_t kSrcEps = 0x8000u, kSrcHasEps = 0x4000u, kSrcMask = 0x3FFFu, kSrcNone = 0x3FFFu;
};
template <> struct __attribute__((aligned(16))) LogT<false> {
  uint32_t arc; uint32_t h; uint32_t src; uint32_t pad;
  static constexpr uint32_t kSrcEps = 0x80000000u, kSrcHasEps = 0x40000000u, kSrcMask = 0x3FFFFFFFu,
                            kSrcNone = 0x3FFFFFFFu;
};
constexpr int kLdsTokLimit = 0x3FFE;  // token indices must fit the 14-bit src field

template <bool kLds> struct IdxT { typedef uint32_t type; };
template <> struct IdxT<true> { typedef uint16_t type; };

// Per-channel state that survives between calls.
struct __attribute__((aligned(128))) ChanState {
  int32_t n_tok;        // entries of the current token list (dead ones included)
  int32_t frame_base;   // back-pointer record of token 0 of the current frame
  int32_t n_rec;        // back-pointer records in use
  int32_t status;       // sticky
  float best;           // minimum cost of the current table
  int32_t cut_bin;      // histogram cut for the next prune; 255 = none
  int32_t ctx_slot;     // which stored context the channel decodes with
  int32_t row_buf;      // which of the two row buffers (tok_row) belongs to the current token list
  long long frames, active_tokens, emit_arcs, eps_arcs, candidates, improvements, tokens, eps_rounds;
  int32_t max_tokens;
  int32_t slow_frames;  // frames decoded with the device-memory tables
  int32_t gc_base;      // records below this one survived the last compaction and are never examined again
  int32_t gc_runs;      // compactions since reset
  long long gc_dropped; // records they removed
  int32_t n_fixed_arcs;  // arcs / words of the paths' shared beginning written out so far (in time order, to the
  int32_t n_fixed_words; // channel's fixed_arcs / fixed_words rows)
  long long lean_frames; // frames decoded by the lean code
  long long spare[15];
#ifdef CBD_PROFILE
  long long timeline[16];  // diagnostic build: the workgroup of the channel's last call with frames (start, end, ids)
#endif
};
#ifndef CBD_PROFILE
static_assert(sizeof(ChanState) == 256, "one channel's state fills two 128-byte lines");
#endif

struct AdvanceParams {
  const int4 *off2;        // [S]: x = first arc of the state, y = its first epsilon-input arc, z = end of those
                           //      (start of its closure list), w = end of the closure list
  const ArcRec *arcs;      // [A]
  const int32_t *canon;    // [A] the arc a record stands for (itself, except in closure lists)
  int32_t start_state;
  int32_t num_pdfs;
  ChanState *chan;         // [C]
  const int32_t *chan_ids; // [grid] the call's channel list
  const float *loglikes;
  long long channel_stride;
  int32_t n_frames;
  int32_t do_reset;
  float beam;
  int32_t max_active;
  int32_t max_eps_iters;
  int32_t lookup_mode;
  int32_t lds_tok_cap;     // token capacity of the LDS tables (0: LDS tables unused)
  int32_t lds_slots;       // state-table slots in LDS
  int32_t lds_log_cap;
  int32_t g_tok_cap;       // the same for the device-memory tables
  int32_t g_slots;
  int32_t g_log_cap;
  int32_t bp_cap;
  int32_t max_ctx;         // row length of ctx
  int32_t ctx_lds_cap;     // context entries that fit the LDS copy
  int32_t stage_rows;      // 1: the frame's log-likelihood row is copied to LDS; 0: read from device memory
  int32_t lean_frames;     // 1: frames that qualify are decoded by the lean code (run_frame_lean)
  int32_t lean_log_per_wave;  // entries of a wave's commit log in lean frames
  // per channel, device memory
  int32_t *tok_state;      // [C][g_tok_cap] states of the current tokens (written on the last frame of a call)
  float *tok_cost;         // [C][g_tok_cap]
  int4 *tok_row;           // [C][2][g_tok_cap] per token: first emitting arc, first epsilon arc, end of row (two buffers)
  int2 *bp;                // [C][bp_cap] (arc, predecessor record or -1)
  LogT<false> *g_log;      // [C][g_log_cap]
  const int32_t *ctx;      // [C + pool][max_ctx] stored contexts: sorted, library arc order
  const int32_t *ctx_n;    // [C + pool] entries of each stored context
  const float *ctx_off;    // [C + pool] its offset
  uint32_t *g_hkey;        // [C][g_slots]
  uint64_t *g_hval;
  uint32_t *g_hidx;
  int32_t *auto_snap;      // [grid][kSnapInts] or null: where each workgroup leaves its channel's best token when done
  int2 *new_records;       // [C] or null (pinned host memory): x = the channel's records above gc_base after this
  int32_t call_seq;        //     call, y = call_seq: lets the host see when no compaction is due without waiting
  unsigned long long *due_max;  // or null: (call_seq << 32 | largest such count among the call's channels)
};

constexpr int kSnapInts = 8;   // a best-token snapshot: status, best record, cost bits, records in use, channel,
                               // gc_base, fixed arcs, fixed words
constexpr int kMetaInts = 8;   // a result's header: status, arcs, words, cost bits, fixed arcs, fixed words

constexpr int kBigRows = 32;      // slots for such rows per frame
constexpr int kBigRowArcs = 512;  // a row with more arcs than this is shared out over all waves

// Workgroup-shared scalars.
struct Shared {
  uint32_t m_ord;      // running minimum of emitting candidates (orderable bits)
  uint32_t best_ord;   // minimum over all accepted candidates of the frame
  unsigned long long log_claim;  // low 32 bits: change-log entries; high 32 bits: states in the table (= tokens)
  int32_t n_front[2];  // log entries of the last / the running phase whose state has epsilon-input arcs
  int32_t n_surv;      // tokens within the beam of best
  int32_t n_live;      // tokens that passed the frame cutoff
  int32_t fault;       // capacity overflow seen
  int32_t n_tok, frame_base, n_rec, status, cut_bin, fr_begin, fr_end, rounds;
  float best;
  int32_t diverged;
  int32_t halt;               // fault or diverged, latched by one thread between two barriers
  int32_t n_big;              // rows too long for one wave, expanded by the whole workgroup (emit)
  int32_t big_first[kBigRows], big_deg[kBigRows];
  float big_cost[kBigRows];
  uint32_t big_src[kBigRows];
  int32_t n_done;             // lean frame: waves through with the look-up phase
  int32_t redo, redo_b;       // lean frame: something this frame needs the general code (the frame is redone there);
                              // set before the first / between the first and the second barrier of the frame
  int32_t wcount[16];         // lean frame: states each wave created; wbase: the same as exclusive prefix sums
  int32_t wbase[16];
  int32_t a_maxtok, a_slow;   // counters of this call
  int32_t a_lean;             // frames decoded by the lean code
  unsigned long long a_lean_pack[2];   // its counters, two to a word: active tokens | emitting arcs << 32,
                                       // epsilon-input arcs | candidates << 32
#ifdef CBD_PROFILE
  long long prof[12];
  long long prof_last;
  int32_t prof_redo;
  int32_t prof_why[8];   // why lean frames went back to the general code (see CBD_WHY)
  long long prof_general;   // time in those frames' second run
#endif
  unsigned long long a_frames, a_active, a_emit, a_eps, a_cand, a_impr, a_tokens, a_rounds;
};

__device__ __forceinline__ int sh_log_n(const Shared *sh) { return (int)(uint32_t)sh->log_claim; }
__device__ __forceinline__ int sh_n_claim(const Shared *sh) { return (int)(uint32_t)(sh->log_claim >> 32); }

// Bloom filter in front of the context list's binary search: an arc sets two bits of one 32-bit word, so a test is
// one LDS read.  64 Kbit: with a 1,000-arc list 3 % of the bits are set and one lane in a thousand passes by chance;
// the search loop runs for a whole wave whenever one of its lanes passes (with 16 Kbit that was 6 in 10 wave
// instructions on 1,000-arc lists, and cost 3 % of the launch; 32 and 128 Kbit measured no better: the filter's
// 8 KB come out of the LDS tables).
#ifndef CBD_BLOOM_LOG2_WORDS
#define CBD_BLOOM_LOG2_WORDS 11
#endif
constexpr int kBloomLog2Words = CBD_BLOOM_LOG2_WORDS;
constexpr int kBloomWords = 1 << kBloomLog2Words;

struct LdsLayout {
  uint32_t sh, hist, bitmap, owner, cmap, ctx, L, hval, hkey, hidx, tcost, log, total;
};

__host__ __device__ inline uint32_t align_up(uint32_t x, uint32_t a) { return (x + a - 1) / a * a; }

// What the lean frame code keeps where the general code has its change log: the tokens' rows (4 + 2 bytes per
// token), the rows of the states in the table (4 + 1 bytes per slot) and the waves' commit logs (8-byte entries).
__host__ __device__ inline uint32_t lean_region_bytes(int tok_cap, int slots, int log_entries) {
  return align_up((uint32_t)tok_cap * 6, 16) + align_up((uint32_t)slots * 5, 16) + (uint32_t)log_entries * 8;
}

// lean_log_entries: room for the lean frame code's commit logs (all waves together); its region is shared with
// the change log and sized for whichever needs more.
__host__ __device__ inline LdsLayout make_layout(int num_pdfs, int ctx_lds_cap, int tok_cap, int slots, int log_cap,
                                                 int lean_log_entries = 0) {
  LdsLayout l;
  uint32_t o = 0;
  l.sh = o; o += align_up((uint32_t)sizeof(Shared), 16);
  l.hist = o; o += 256 * 4;
  l.bitmap = o; o += kBloomWords * 4;
  l.owner = o; o += 16 * 256;   // per-wave owner map of the first 256 arcs of a tile
  l.cmap = o; o += 16 * 64;     // per-wave owner map of a closure stage's records
  l.ctx = o; o += align_up((uint32_t)ctx_lds_cap * 4, 16);
  l.L = o; o += align_up((uint32_t)num_pdfs * 4, 16);
  l.hval = o; o += (uint32_t)slots * 8;
  l.hkey = o; o += (uint32_t)slots * 4;
  l.hidx = o; o += align_up((uint32_t)slots * 2, 16);
  l.tcost = o; o += align_up((uint32_t)tok_cap * 4, 16);
  l.log = o;
  {
    const uint32_t general = align_up((uint32_t)log_cap * 8, 16);
    const uint32_t lean = lean_log_entries > 0 ? lean_region_bytes(tok_cap, slots, lean_log_entries) : 0;
    o += general > lean ? general : lean;
  }
  l.total = o;
  return l;
}

// LDS per token of capacity: 1.5 slots x 14 B + 4 B of cost + 1.5 log entries x 8 B = 37 B.  (The tokens' arc
// rows, written once and read once a frame later, live in device memory: they stream, they are not looked up.)
__host__ __device__ inline int lds_slots_for(int tok_cap) { return tok_cap + tok_cap / 2; }
__host__ __device__ inline int lds_log_for(int tok_cap) { return tok_cap + tok_cap / 2; }

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

// Cross-lane steps on the DPP path (no LDS round trip).  Lanes that a step does not reach
// (row/bank masked off, or whose source lies outside the 16-lane row) receive `identity`.
template <int kCtrl, int kRowMask, int kBankMask>
__device__ __forceinline__ int dpp_step(int identity, int v) {
  return __builtin_amdgcn_update_dpp(identity, v, kCtrl, kRowMask, kBankMask, false);
}
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr3 = 0x113, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;

// Inclusive prefix sum over the 64 lanes: three shifts inside groups of four, two
// shifts inside the 16-lane row, then the row totals are carried across rows.
__device__ __forceinline__ int wave_incl_scan(int v) {
  int s = v;
  s += dpp_step<kRowShr1, 0xf, 0xf>(0, v);
  s += dpp_step<kRowShr2, 0xf, 0xf>(0, v);
  s += dpp_step<kRowShr3, 0xf, 0xf>(0, v);
  s += dpp_step<kRowShr4, 0xf, 0xe>(0, s);
  s += dpp_step<kRowShr8, 0xf, 0xc>(0, s);
  s += dpp_step<kRowBcast15, 0xa, 0xf>(0, s);
  s += dpp_step<kRowBcast31, 0xc, 0xf>(0, s);
  return s;
}

// Inclusive running maximum over the 64 lanes (values >= 0), same ladder.  The arithmetic is unsigned: 0 is then
// the maximum's identity, and a lane a step does not reach keeps its value in one instruction.
__device__ __forceinline__ int wave_incl_scan_max(int v) {
  uint32_t s = (uint32_t)v;
  s = max(s, (uint32_t)dpp_step<kRowShr1, 0xf, 0xf>(0, v));
  s = max(s, (uint32_t)dpp_step<kRowShr2, 0xf, 0xf>(0, v));
  s = max(s, (uint32_t)dpp_step<kRowShr3, 0xf, 0xf>(0, v));
  s = max(s, (uint32_t)dpp_step<kRowShr4, 0xf, 0xe>(0, (int)s));
  s = max(s, (uint32_t)dpp_step<kRowShr8, 0xf, 0xc>(0, (int)s));
  s = max(s, (uint32_t)dpp_step<kRowBcast15, 0xa, 0xf>(0, (int)s));
  s = max(s, (uint32_t)dpp_step<kRowBcast31, 0xc, 0xf>(0, (int)s));
  return (int)s;
}

__device__ __forceinline__ uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }

// Minimum over the 64 lanes (same ladder with min instead of add), returned in every lane.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  const int id = -1;  // 0xFFFFFFFF
  uint32_t s = v;
  s = umin32(s, (uint32_t)dpp_step<kRowShr1, 0xf, 0xf>(id, (int)v));
  s = umin32(s, (uint32_t)dpp_step<kRowShr2, 0xf, 0xf>(id, (int)v));
  s = umin32(s, (uint32_t)dpp_step<kRowShr3, 0xf, 0xf>(id, (int)v));
  s = umin32(s, (uint32_t)dpp_step<kRowShr4, 0xf, 0xe>(id, (int)s));
  s = umin32(s, (uint32_t)dpp_step<kRowShr8, 0xf, 0xc>(id, (int)s));
  s = umin32(s, (uint32_t)dpp_step<kRowBcast15, 0xa, 0xf>(id, (int)s));
  s = umin32(s, (uint32_t)dpp_step<kRowBcast31, 0xc, 0xf>(id, (int)s));
  return (uint32_t)__builtin_amdgcn_readlane((int)s, 63);
}

// Workgroup barrier.  A frame whose working set is in LDS only has to order LDS traffic;
// outstanding HBM loads and stores (the next log-likelihood row, back-pointer records) keep flying.
template <bool kLds> __device__ __forceinline__ void wg_barrier() {
  if (kLds) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else __syncthreads();
}

// Accessors for values that other waves change with atomics.
template <bool kLds, typename T> __device__ __forceinline__ T ldv(const T *p) {
  if (kLds) return __hip_atomic_load(const_cast<T *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return __hip_atomic_load(const_cast<T *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool kLds, typename T> __device__ __forceinline__ void stv(T *p, T v) {
  if (kLds) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Sec. 4.2: the listed arc indices are kept sorted and searched per expanded arc.
template <typename ListPtr>
__device__ __forceinline__ bool sorted_contains(ListPtr list, int n, int32_t a) {
  int lo = 0, hi = n;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (list[mid] < a) lo = mid + 1; else hi = mid;
  }
  return lo < n && list[lo] == a;
}

__device__ __forceinline__ uint32_t bloom_hash(int32_t a) { return (uint32_t)a * 2654435761u; }
__device__ __forceinline__ uint32_t bloom_word(uint32_t h) { return h >> (32 - kBloomLog2Words); }
__device__ __forceinline__ uint32_t bloom_mask(uint32_t h) {
  return (1u << ((h >> (27 - kBloomLog2Words)) & 31u)) | (1u << ((h >> (22 - kBloomLog2Words)) & 31u));
}

// LDS-typed pointers: reads through them are plain LDS reads, not generic loads
typedef const __attribute__((address_space(3))) float *lds_cfloat_ptr;
typedef const __attribute__((address_space(3))) int32_t *lds_cint_ptr;

struct Ctx {
  lds_cint_ptr lds_list;
  const int32_t *g_list;
  const uint32_t *bitmap;
  int n;
  bool in_lds;
  bool use_bitmap;
  float offset;
};

// The current frame's log-likelihood row: the LDS copy, or (when LDS is kept for more resident
// workgroups instead) the row in device memory, which stays in L2 while the frame lasts.
struct Rows {
  lds_cfloat_ptr lds;   // typed as LDS so that the staged case is a plain LDS read, not a generic load
  const float *glob;
  bool staged;
  __device__ __forceinline__ float at(uint32_t i) const {
    if (staged) return lds[i];
    return glob[i];
  }
};

__device__ __forceinline__ bool ctx_contains(const Ctx &cx, int32_t a) {
  if (cx.n == 0) return false;
  if (cx.use_bitmap) {
    const uint32_t h = bloom_hash(a), mask = bloom_mask(h);
    if ((cx.bitmap[bloom_word(h)] & mask) != mask) return false;
  }
  if (cx.in_lds) return sorted_contains(cx.lds_list, cx.n, a);
  return sorted_contains(cx.g_list, cx.n, a);
}

// A token's arc row as another wave of the workgroup stored it to device memory: read past the L1.
__device__ __forceinline__ int2 load_row_fe(const int4 *row) {
  unsigned long long v = __hip_atomic_load((const unsigned long long *)row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_int2((int)(uint32_t)v, (int)(uint32_t)(v >> 32));
}
__device__ __forceinline__ int2 load_row_end(const int4 *row) {
  unsigned long long v = __hip_atomic_load((const unsigned long long *)row + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_int2((int)(uint32_t)v, (int)(uint32_t)(v >> 32));
}

// Where a frame's working set lives.
template <bool kLds> struct Mem {
  typedef typename IdxT<kLds>::type idx_t;
  uint64_t *hval;
  uint32_t *hkey;
  idx_t *hidx;
  int4 *t_row;   // device memory, two buffers: buffer b starts at b * row_cap
  float *t_cost;
  LogT<kLds> *log;
  uint32_t slots;
  int tok_cap, log_cap, row_cap;
};

struct RowInfo { int first, eps, end; };

__device__ __forceinline__ RowInfo row_of(const AdvanceParams &p, const ArcRec &rec) {
  RowInfo r;
  uint32_t ed = meta_ed(rec.meta), xd = meta_xd(rec.meta);
  r.first = rec.row;
  if (ed == kEdEscape || xd == kXdEscape) {
    // a long row (rare): its bounds come from the offsets.  The wait is taken here, inside the rare branch, so
    // that code after it never has to wait for "a load that may have happened" (which would also make it wait
    // for the arc records requested ahead of need).
    int4 o = p.off2[rec.dst];
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    r.eps = o.y; r.end = o.z;
  } else {
    r.eps = r.first + (int)ed; r.end = r.eps + (int)xd;
  }
  return r;
}

// The overflow flag as some wave last wrote it (a hint: the decision is taken after a barrier).
__device__ __forceinline__ int load_fault(const Shared *sh) {
  return __hip_atomic_load(&sh->fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Recombination: E[state] = min key.  Returns true if this call lowered the
// state's value (old > key); h receives the slot, claimed tells whether this
// lane created the state's entry.
template <bool kLds>
__device__ __forceinline__ bool table_min(const Mem<kLds> &M, Shared *sh, uint32_t state, uint64_t key, uint32_t &h_out,
                                          bool &claimed) {
  uint32_t h = __umulhi(state * 2654435761u, M.slots);
  // most candidates open a new state or find theirs at the home slot: try to take it straight away,
  // and walk on only after a collision
  uint32_t k = atomicCAS(&M.hkey[h], kEmptyKey, state);
  if (__builtin_expect(k != kEmptyKey && k != state, 0)) {
    uint32_t probe = 1;
    do {
      h = h + 1 == M.slots ? 0 : h + 1;
      k = atomicCAS(&M.hkey[h], kEmptyKey, state);
      // (a long walk means a nearly full table: stop as soon as anybody has declared the overflow)
    } while (k != kEmptyKey && k != state && ++probe < M.slots && !((probe & 63u) == 0 && load_fault(sh)));
    if (k != kEmptyKey && k != state) {   // every slot holds another state, or the frame is being given up
      sh->fault = 1;
      claimed = false;
      h_out = 0;
      return false;
    }
  }
  uint64_t old = atomicMin((unsigned long long *)&M.hval[h], (unsigned long long)key);
  claimed = k == kEmptyKey;
  h_out = h;
  return old > key;
}

// Book the updates of this wave's lanes: one atomic on the packed counter yields the
// change-log positions and, for lanes that created a state, the token indices; those
// lanes file the state's row under their index (no = offset of the row buffer being built).
template <bool kLds>
__device__ __forceinline__ void record(const Mem<kLds> &M, Shared *sh, int32_t *front, int no, bool improved,
                                       bool claimed, uint32_t arc, uint32_t h, uint32_t src, const RowInfo &row,
                                       int lane) {
  unsigned long long imask = __ballot(improved);
  unsigned long long cmask = __ballot(claimed);
  // (a lane can create a state's entry and still lose the minimum to a lane of another wave
  // that reached the value first: it must get its token index all the same)
  if ((imask | cmask) == 0) return;
  int leader = __ffsll((long long)(imask | cmask)) - 1;
  int nf = __popcll(__ballot(improved && (src & LogT<kLds>::kSrcHasEps)));
  unsigned long long base = 0;
  if (lane == leader) {
    base = atomicAdd(&sh->log_claim, (unsigned long long)__popcll(imask) | ((unsigned long long)__popcll(cmask) << 32));
    if (nf) atomicAdd(front, nf);
  }
  int base_log = __builtin_amdgcn_readlane((int)(uint32_t)base, leader);
  int base_tok = __builtin_amdgcn_readlane((int)(uint32_t)(base >> 32), leader);
  unsigned long long below = (1ull << lane) - 1ull;
  if (claimed) {
    int idx = base_tok + __popcll(cmask & below);
    if (idx < M.tok_cap) {
      M.t_row[no + idx] = make_int4(row.first, row.eps, row.end, 0);
      stv<kLds>(&M.hidx[h], (typename Mem<kLds>::idx_t)idx);
    } else {
      sh->fault = 1;
    }
  }
  if (improved) {
    int pos = base_log + __popcll(imask & below);
    if (pos < M.log_cap) {
      LogT<kLds> e;
      e.arc = arc; e.h = (decltype(e.h))h; e.src = (decltype(e.src))src;
      M.log[pos] = e;
    } else {
      sh->fault = 1;
    }
  }
}

// The wave's arc list: lane i contributes `deg` arcs starting at `first`.
struct ArcList { int pos, rel, total; uint8_t *owner; };
constexpr int kOwnerMap = 256;   // list positions covered by the per-wave owner map

__device__ __forceinline__ ArcList make_arc_list(int first, int deg, int lane, uint8_t *owner_map) {
  ArcList L;
  int incl = wave_incl_scan(deg);
  L.pos = incl - deg;
  L.rel = first - L.pos;   // arc index = rel(owner) + position in the list
  L.total = __builtin_amdgcn_readlane(incl, 63);
  L.owner = owner_map;
  // every contributing lane signs the positions it owns (rows are short: a few stores)
  for (int k = 0; k < deg && L.pos + k < kOwnerMap; ++k) owner_map[L.pos + k] = (uint8_t)lane;
  return L;
}

// owner of list position jj: from the map, or (long lists) the last lane whose first position is <= jj
__device__ __forceinline__ int arc_owner(const ArcList &L, int jj, int j0) {
  if (j0 + 64 <= kOwnerMap) return L.owner[jj < kOwnerMap ? jj : 0];   // j0 is uniform
  int owner = 0;
#pragma unroll
  for (int step = 32; step >= 1; step >>= 1) {
    int cand = owner + step;
    int pc = __shfl(L.pos, cand & 63, 64);
    if (cand < 64 && pc <= jj) owner = cand;
  }
  return owner;
}

// Cutoff test, recombination and logging of one candidate per lane (called by whole waves).
// n_cand counts the candidates that passed the cutoff (same value in every lane).
template <bool kLds, bool kEmit>
__device__ __forceinline__ void commit(const AdvanceParams &p, const Mem<kLds> &M, Shared *sh, int32_t *front, int no,
                                       bool act, float cand, int a, const ArcRec &rec, uint32_t src_tag, float m_fixed,
                                       uint32_t &n_cand, int lane, bool flag_children, int fault, bool &improved,
                                       uint32_t &h, RowInfo &row, bool have_row = false) {
  // fault: a recent reading of the overflow flag (see load_fault); once set, the tables are left alone.
  // have_row: row already holds the destination's row (else it is worked out here for candidates that pass).
  improved = false; h = 0;
  if (!have_row) row.first = row.eps = row.end = 0;
  bool pass = false;
  if (act) {
    float mref = kEmit ? ord2f(__hip_atomic_load(&sh->m_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) : m_fixed;
    pass = !(cand - mref > p.beam);
  }
  unsigned long long pmask = __ballot(pass);
  if (pmask == 0) return;
  n_cand += (uint32_t)__popcll(pmask);
  uint32_t co = pass ? f2ord(cand) : 0xFFFFFFFFu;
  if (!kEmit && __ballot(co < f2ord(m_fixed)) != 0) {
    // the frame's minimum is min(m, closure candidates): only a candidate below m can move it
    uint32_t wmin = wave_min_u32(co);
    if (lane == 0) atomicMin(&sh->best_ord, wmin);
  }
  bool claimed = false;
  uint32_t src = src_tag;
  if (pass && !fault) {
    if (!have_row) row = row_of(p, rec);
    if (flag_children && row.end > row.eps) src |= LogT<kLds>::kSrcHasEps;   // flag_children may differ per lane
    uint64_t key = ((uint64_t)co << 32) | (uint32_t)a;
    improved = table_min<kLds>(M, sh, (uint32_t)rec.dst, key, h, claimed);
  }
  record<kLds>(M, sh, front, no, improved, claimed, (uint32_t)a, h, src, row, lane);
}

// Expand positions [j_begin, total) of the wave's arc list of epsilon-input arcs, one lane per arc, committing
// each candidate at once and leaving the children flagged in the change log (closure levels of more than 64 arcs).
template <bool kLds>
__device__ __forceinline__ void expand_direct(const AdvanceParams &p, const Mem<kLds> &M, Shared *sh, int32_t *front,
                                              const Ctx &cx, int no, const ArcList &AL, int j_begin, float cost,
                                              uint32_t src_tag, float m_fixed, uint32_t &n_cand, int lane) {
  for (int j0 = j_begin; j0 < AL.total; j0 += 64) {
    int jj = j0 + lane;
    bool act = jj < AL.total;
    const int fault = load_fault(sh);
    int owner = arc_owner(AL, jj, j0);
    int a = __shfl(AL.rel, owner, 64) + jj;
    float c_own = __shfl(cost, owner, 64);
    uint32_t s_own = (uint32_t)__shfl((int)src_tag, owner, 64);
    float cand = 0.0f;
    ArcRec rec; rec.dst = 0; rec.weight = 0.0f; rec.row = 0; rec.meta = 0;
    if (act) {
      rec = p.arcs[a];
      float w = rec.weight;
      if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
      cand = c_own + w;
    }
    bool imp; uint32_t hh; RowInfo rr;
    commit<kLds, false>(p, M, sh, front, no, act, cand, a, rec, s_own, m_fixed, n_cand, lane, true, fault, imp, hh, rr);
  }
}

// A state whose value a lane has just lowered and whose epsilon-input arcs it will expand itself:
// the row [first, first+deg), the value, the state's table slot, and the row's first arc record,
// fetched ahead of need.
struct Pending {
  int first, deg;
  float cost;
  uint32_t slot;
  ArcRec nxt;
  bool have_nxt;
  // a second state waiting behind the first (taken up when the lane's current chain ends)
  int first2, deg2;
  float cost2;
  uint32_t slot2;
};

__device__ __forceinline__ void pending_clear(Pending &pd) {
  pd.first = 0; pd.deg = 0; pd.cost = 0.0f; pd.slot = 0; pd.have_nxt = false;
  pd.nxt.dst = 0; pd.nxt.weight = 0.0f; pd.nxt.row = 0; pd.nxt.meta = 0;
  pd.first2 = 0; pd.deg2 = 0; pd.cost2 = 0.0f; pd.slot2 = 0;
}

constexpr int kEmitSlots = 2;  // candidates a lane holds while the batch minimum settles (more cost registers:
                               // at 2 the kernel fits 120 VGPRs, which leaves room on every SIMD for a wave of another kernel)

// Recombination of the emit phase's candidates: kPair (1 or 2) slots of each lane, holding list positions
// jb + lane and jb + 64 + lane (a slot is in use if its first position lies below total).  Same steps as commit(), but taken for both slots together, so that a lane with two candidates
// waits once per step, not once per candidate: cutoff against the running minimum; home-slot claims; (rarely)
// walks after collisions; minima; one counter update for the wave; rows, table indices and log entries.  A lane
// keeps the first two states it lowered that have epsilon-input arcs as its own pending work for the closure
// (asking for the first one's arc record right away); any further ones are flagged in the change log.
template <bool kLds, int kPair>
__device__ __forceinline__ void commit_emit_n(const AdvanceParams &p, const Mem<kLds> &M, Shared *sh, int no,
                                                 int total, int jb, const float *cand, const int *arc,
                                                 const ArcRec *rec, const uint32_t *srct, uint32_t &n_cand, int lane,
                                                 Pending &pd, uint32_t &pd_arc, uint32_t &pd_arc2) {
  typedef LogT<kLds> LogE;
  const int fault = load_fault(sh);
  const float mref = ord2f(__hip_atomic_load(&sh->m_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
  bool ok[kPair], claimed[kPair], improved[kPair];
  uint32_t h[kPair], k[kPair], src[kPair];
  unsigned long long any = 0;
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    const int j0 = jb + q * 64;
    ok[q] = j0 + lane < total && !(cand[q] - mref > p.beam) && !fault;   // for now: "passes and will be tried"
    claimed[q] = false; improved[q] = false; h[q] = 0; k[q] = 0; src[q] = srct[q];
    if (j0 < total) {
      unsigned long long pm = __ballot(j0 + lane < total && !(cand[q] - mref > p.beam));
      n_cand += (uint32_t)__popcll(pm);
      any |= pm;
    }
  }
  if (any == 0) return;
  // home slots
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    if (jb + q * 64 < total && ok[q]) {
      h[q] = __umulhi((uint32_t)rec[q].dst * 2654435761u, M.slots);
      k[q] = atomicCAS(&M.hkey[h[q]], kEmptyKey, (uint32_t)rec[q].dst);
    }
  }
  // collisions: walk on (rare)
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    if (jb + q * 64 < total) {
      const uint32_t state = (uint32_t)rec[q].dst;
      const bool collided = ok[q] && k[q] != kEmptyKey && k[q] != state;
      if (__ballot(collided) != 0) {
        if (collided) {
          uint32_t hh = h[q], kk = k[q], probe = 1;
          do {
            hh = hh + 1 == M.slots ? 0 : hh + 1;
            kk = atomicCAS(&M.hkey[hh], kEmptyKey, state);
          } while (kk != kEmptyKey && kk != state && ++probe < M.slots && !((probe & 63u) == 0 && load_fault(sh)));
          if (kk == kEmptyKey || kk == state) { h[q] = hh; k[q] = kk; }
          else { ok[q] = false; sh->fault = 1; }   // every slot holds another state, or the frame is being given up
        }
      }
    }
  }
  // minima
  uint64_t old[kPair];
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    old[q] = 0;
    if (jb + q * 64 < total && ok[q]) {
      const uint64_t key = ((uint64_t)f2ord(cand[q]) << 32) | (uint32_t)arc[q];
      old[q] = atomicMin((unsigned long long *)&M.hval[h[q]], (unsigned long long)key);
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // both minima are on their way before anything below is looked at
  // who lowered what; which states the lane keeps for the closure
  unsigned long long imask[kPair], cmask[kPair];
  RowInfo row[kPair];
  int n_imp = 0, n_claim = 0, n_flag = 0;
  bool took_first = false;
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    imask[q] = cmask[q] = 0;
    row[q].first = row[q].eps = row[q].end = 0;
    if (jb + q * 64 < total) {
      const uint64_t key = ((uint64_t)f2ord(cand[q]) << 32) | (uint32_t)arc[q];
      improved[q] = ok[q] && old[q] > key;
      claimed[q] = ok[q] && k[q] == kEmptyKey;
      if (improved[q] || claimed[q]) row[q] = row_of(p, rec[q]);
      if (improved[q] && row[q].end > row[q].eps) {
        if (pd.deg == 0) {
          pd.first = row[q].eps; pd.deg = row[q].end - row[q].eps; pd.cost = cand[q]; pd.slot = h[q];
          pd_arc = (uint32_t)arc[q];
          took_first = true;
        } else if (pd.deg2 == 0) {
          pd.first2 = row[q].eps; pd.deg2 = row[q].end - row[q].eps; pd.cost2 = cand[q]; pd.slot2 = h[q];
          pd_arc2 = (uint32_t)arc[q];
        } else {
          src[q] |= LogE::kSrcHasEps;
        }
      }
      imask[q] = __ballot(improved[q]);
      cmask[q] = __ballot(claimed[q]);
      n_imp += __popcll(imask[q]); n_claim += __popcll(cmask[q]);
      n_flag += __popcll(__ballot(improved[q] && (src[q] & LogE::kSrcHasEps)));
    }
  }
  // The first arc record of the lane's first pending row is asked for now.  Every lane issues the load (lanes
  // that took nothing new ask again for what they hold, or for record 0): with no branch around it, nothing
  // below has to wait for it, and it has arrived by the time the closure starts.
  if (__ballot(took_first) != 0) {
    pd.nxt = p.arcs[(took_first || pd.have_nxt) ? pd.first : 0];
    pd.have_nxt = pd.have_nxt || took_first;
  }
  // (a lane can create a state's entry and still lose the minimum to a lane of another wave
  // that reached the value first: it must get its token index all the same)
  if ((n_imp | n_claim) == 0) return;
  unsigned long long base = 0;
  if (lane == 0) {
    base = atomicAdd(&sh->log_claim, (unsigned long long)n_imp | ((unsigned long long)n_claim << 32));
    if (n_flag) atomicAdd(&sh->n_front[0], n_flag);
  }
  int base_log = __builtin_amdgcn_readfirstlane((int)(uint32_t)base);
  int base_tok = __builtin_amdgcn_readfirstlane((int)(uint32_t)(base >> 32));
  const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
  for (int q = 0; q < kPair; ++q) {
    if (jb + q * 64 < total) {
      if (claimed[q]) {
        int idx = base_tok + __popcll(cmask[q] & below);
        if (idx < M.tok_cap) {
          M.t_row[no + idx] = make_int4(row[q].first, row[q].eps, row[q].end, 0);
          stv<kLds>(&M.hidx[h[q]], (typename Mem<kLds>::idx_t)idx);
        } else {
          sh->fault = 1;
        }
      }
      if (improved[q]) {
        int pos = base_log + __popcll(imask[q] & below);
        if (pos < M.log_cap) {
          LogE e;
          e.arc = (uint32_t)arc[q]; e.h = (decltype(e.h))h[q]; e.src = (decltype(e.src))src[q];
          M.log[pos] = e;
        } else {
          sh->fault = 1;
        }
      }
      base_tok += __popcll(cmask[q]);
      base_log += __popcll(imask[q]);
    }
  }
}

// Epsilon closure from this wave's pending states.  While every pending row has one arc (the
// usual case) each lane expands its own arc: no scan, no cross-lane traffic, and the record
// of the next level's arc is requested before the table update that decides whether it is
// needed.  Rows with several arcs go through the wave's arc list, one lane per arc; a level of
// more than 64 arcs is expanded in bulk and its children are left flagged in the change log
// for the next round.  No barrier anywhere: a wave follows the chains it starts.
template <bool kLds>
__device__ __forceinline__ void chase(const AdvanceParams &p, const Mem<kLds> &M, Shared *sh, int32_t *front,
                                      const Ctx &cx, int no, uint8_t *owner_map, Pending &pd, float m,
                                      uint32_t &n_eps, uint32_t &n_cand, int &levels, int lane) {
  typedef LogT<kLds> LogE;
  int depth = 0;   // levels of this call: bounds the length of the chains it follows (a lane's second chain included)
  while (true) {
    if (pd.deg == 0 && pd.deg2 > 0) {
      pd.first = pd.first2; pd.deg = pd.deg2; pd.cost = pd.cost2; pd.slot = pd.slot2; pd.have_nxt = false;
      pd.deg2 = 0;
    }
    unsigned long long pend = __ballot(pd.deg > 0);
    if (pend == 0) return;
    const int fault = load_fault(sh);   // asked for here, back by the time the arcs have arrived
    levels = max(levels, ++depth);
    if (depth > p.max_eps_iters) {
      if (lane == 0) sh->diverged = 1;
      pd.deg = 0;
      return;
    }
    if (__ballot(pd.deg > 1) == 0) {
      // every pending row is a single arc: each lane takes its own
      n_eps += (uint32_t)__popcll(pend);
      const bool act = pd.deg > 0;
      const int a = pd.first;
      if (act && !pd.have_nxt) pd.nxt = p.arcs[a];
      const ArcRec rec = pd.nxt;
      float w = rec.weight;
      if (act && ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1
      const float cand = pd.cost + w;
      // the record of the next level's arc is asked for now, by every lane (lanes without one ask for record 0:
      // no branch around the load, so nothing downstream has to wait for it before it is needed)
      const RowInfo ahead = row_of(p, rec);
      const bool more = act && !(cand - m > p.beam) && ahead.end > ahead.eps;
      Pending nx;
      nx.nxt = p.arcs[more ? ahead.eps : 0];
      nx.have_nxt = more;
      bool improved; uint32_t h; RowInfo row = ahead;
      commit<kLds, false>(p, M, sh, front, no, act, cand, a, rec, pd.slot | LogE::kSrcEps, m, n_cand, lane, false,
                          fault, improved, h, row, true);
      const bool go = improved && row.end > row.eps;
      nx.first = go ? row.eps : 0; nx.deg = go ? row.end - row.eps : 0; nx.cost = cand; nx.slot = h;
      nx.have_nxt = nx.have_nxt && go;
      nx.first2 = pd.first2; nx.deg2 = pd.deg2; nx.cost2 = pd.cost2; nx.slot2 = pd.slot2;
      pd = nx;
      continue;
    }
    ArcList AL = make_arc_list(pd.first, pd.deg, lane, owner_map);
    n_eps += (uint32_t)AL.total;
    const uint32_t tag = pd.slot | LogE::kSrcEps;
    if (AL.total > 64) {
      expand_direct<kLds>(p, M, sh, front, cx, no, AL, 0, pd.cost, tag, m, n_cand, lane);
      pd.deg = 0;
      continue;   // lanes with a second state still have it to do
    }
    bool act = lane < AL.total;
    int owner = arc_owner(AL, lane, 0);
    int a = __shfl(AL.rel, owner, 64) + lane;
    float c_own = __shfl(pd.cost, owner, 64);
    uint32_t s_own = (uint32_t)__shfl((int)tag, owner, 64);
    float cand = 0.0f;
    ArcRec rec; rec.dst = 0; rec.weight = 0.0f; rec.row = 0; rec.meta = 0;
    if (act) {
      rec = p.arcs[a];
      float w = rec.weight;
      if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1
      cand = c_own + w;
    }
    bool improved; uint32_t h; RowInfo row;
    commit<kLds, false>(p, M, sh, front, no, act, cand, a, rec, s_own, m, n_cand, lane, false, fault, improved, h, row);
    bool go = improved && row.end > row.eps;
    pd.first = go ? row.eps : 0;
    pd.deg = go ? row.end - row.eps : 0;
    pd.cost = cand;
    pd.slot = h;
    pd.have_nxt = false;   // (asking for the child's first record here was measured: it costs more than it saves)
  }
}

// Per-frame scalars and the pruning histogram, set by one wave; a barrier must follow before use.
// start: the frame is the start of an utterance (its cutoff reference is the start token's cost 0).
__device__ __forceinline__ void frame_init(Shared *sh, uint32_t *hist, bool start, int lane, bool zero_hist = true) {
  if (zero_hist) {   // (uniform) a frame that did not fill the histogram leaves it empty
#pragma unroll
    for (int k = 0; k < 4; ++k) hist[lane * 4 + k] = 0;
  }
  if (lane == 0) {
    sh->m_ord = start ? f2ord(0.0f) : 0xFFFFFFFFu;
    sh->best_ord = 0xFFFFFFFFu;   // minimum over closure candidates; the table's minimum is min(m, this)
    sh->log_claim = 0; sh->n_front[0] = 0; sh->n_front[1] = 0; sh->n_surv = 0; sh->n_live = 0; sh->rounds = 0;
    sh->fault = 0; sh->diverged = 0; sh->halt = 0; sh->n_big = 0; sh->redo = 0; sh->redo_b = 0; sh->n_done = 0;
  }
}

// One frame (f >= 0) or the start of an utterance (f < 0).  Uniform control flow; returns a kFrame* code.
// Nothing that outlives the frame is written before the capacity checks have passed.
template <bool kLds, int kBlock>
__device__ __forceinline__ int run_frame(const AdvanceParams &p, const Mem<kLds> &M, Shared *sh, const Ctx &cx,
                                         float *Lstage, const Rows &Lrow, const float *Lnext, uint32_t *hist,
                                         uint8_t *owner_maps, int f,
                                         int cur, int2 *bp, int32_t *g_tok_state, bool last_frame) {
  // Lnext: the next frame's log-likelihood row in HBM (null: none).  It starts its way now, waits in
  // registers during the emit phase and is parked in the LDS row Lstage once the emit phase is over.
  constexpr int NW = kBlock / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int co = cur * M.row_cap, no = (cur ^ 1) * M.row_cap;   // row buffer read / built
  // The arc row of this lane's token in the first batch comes from device memory: ask for it before
  // anything else (loads return in order), so that it is there when the token's cost has been looked at.
  int2 fe0 = make_int2(0, 0);
  if (f >= 0) {
    const int nb0 = min(kBlock, sh->n_tok);
    const int tpw0 = (nb0 + NW - 1) / NW;
    const int i0 = wave * tpw0 + lane;
    if (lane < tpw0 && i0 < nb0) fe0 = load_row_fe(&M.t_row[co + i0]);
  }
  constexpr int kPre = kBlock >= 1024 ? 6 : (kBlock >= 960 ? 7 : 8);
  float pre[kPre];
#pragma unroll
  for (int k = 0; k < kPre; ++k) {
    int i = threadIdx.x + k * kBlock;
    pre[k] = (Lnext && i < p.num_pdfs) ? Lnext[i] : 0.0f;
  }
  const bool hist_on = p.max_active > 0 && p.beam > 0.0f && p.beam < __builtin_inff();
  const float inv = 256.0f / p.beam;
  typedef LogT<kLds> LogE;
  uint8_t *owner_map = owner_maps + wave * kOwnerMap;

  uint32_t n_active = 0, n_emit = 0, n_eps = 0, n_cand = 0;   // this wave's share of the frame's counters
  Pending pd; pending_clear(pd);   // the state this lane will start the closure from
  uint32_t pd_arc = 0, pd_arc2 = 0;   // the arcs that produced them: a state's value names its arc
  if (f < 0) {
    // reset: one start token at cost 0
    if (wave == 0) {
      uint32_t h = 0;
      uint64_t key = ((uint64_t)f2ord(0.0f) << 32) | kArcNone;
      bool improved = false, claimed = false;
      int4 o = p.off2[p.start_state];
      RowInfo row; row.first = o.x; row.eps = o.y; row.end = o.z;
      if (lane == 0) improved = table_min<kLds>(M, sh, (uint32_t)p.start_state, key, h, claimed);
      uint32_t src = LogE::kSrcNone | ((row.end > row.eps) ? LogE::kSrcHasEps : 0u);
      record<kLds>(M, sh, &sh->n_front[0], no, improved, claimed, kArcNone, h, src, row, lane);
    }
  } else {
    // ---- emit: prune (step 1), expand emitting arcs (step 2), in batches of one tile per wave
    const int n_tok = sh->n_tok;
    const float best = sh->best;
    const int cut = sh->cut_bin;
    const int n_batches = (n_tok + kBlock - 1) / kBlock;
    int big_arcs = 0;
    for (int b = 0; b < n_batches; ++b) {
      // a batch holds up to kBlock tokens, shared evenly by the waves: with few tokens every
      // wave still gets some, and each lane ends up with about one arc
      const int nb = min(kBlock, n_tok - b * kBlock);
      const int tpw = (nb + NW - 1) / NW;
      const int tile0 = b * kBlock + wave * tpw;
      int i = tile0 + lane;
      bool alive = false;
      float cost = 0.0f;
      int first = 0, deg = 0;
      if (lane < tpw && i < b * kBlock + nb) {
        cost = M.t_cost[i];
        float r = cost - best;
        alive = !(r > p.beam) && cost < __builtin_inff();
        if (alive && cut < 255) {
          int bin = (int)floorf(r * inv);
          bin = bin > 255 ? 255 : bin;
          alive = bin <= cut;
        }
        if (alive) { int2 fe = b == 0 ? fe0 : load_row_fe(&M.t_row[co + i]); first = fe.x; deg = fe.y - first; }
      }
      if (deg > kBigRowArcs) {
        // a hub-like row: one wave would walk it alone, so park it for the whole workgroup
        int slot = atomicAdd(&sh->n_big, 1);
        if (slot < kBigRows) {
          sh->big_first[slot] = first; sh->big_deg[slot] = deg; sh->big_cost[slot] = cost; sh->big_src[slot] = (uint32_t)i;
          big_arcs += deg;
          deg = 0;
        }
      }
      unsigned long long am = __ballot(alive);
      ArcList AL = make_arc_list(first, deg, lane, owner_map);
      n_active += (uint32_t)__popcll(am); n_emit += (uint32_t)AL.total;
      if (__ballot(big_arcs > 0) != 0) {
        int wb = wave_incl_scan(big_arcs);
        n_emit += (uint32_t)__builtin_amdgcn_readlane(wb, 63);
        big_arcs = 0;
      }
      // The wave's arcs are taken kEmitSlots * 64 at a time (one round is the rule).  Phase A fetches the
      // records and keeps the candidates in registers; phase B cuts and recombines them.  Before the first
      // round's phase B every wave waits for the others' minima (few doomed candidates reach the table);
      // later rounds cut against the running minimum, which never lies below the final one.
      for (int jb = 0; jb == 0 || jb < AL.total; jb += kEmitSlots * 64) {
        float cand[kEmitSlots];
        int arc[kEmitSlots];
        ArcRec rec[kEmitSlots];
        uint32_t srct[kEmitSlots];
        uint32_t lmin = 0xFFFFFFFFu;
#pragma unroll
        for (int r = 0; r < kEmitSlots; ++r) {
          const int j0 = jb + r * 64, jj = j0 + lane;
          bool act = jj < AL.total;
          cand[r] = 0.0f; arc[r] = 0; srct[r] = 0;
          rec[r].dst = 0; rec[r].weight = 0.0f; rec[r].row = 0; rec[r].meta = 0;
          if (j0 < AL.total) {   // uniform
            int owner = arc_owner(AL, jj, j0);
            arc[r] = __shfl(AL.rel, owner, 64) + jj;
            float c_own = __shfl(cost, owner, 64);
            srct[r] = (uint32_t)(tile0 + owner);
            if (act) {
              rec[r] = p.arcs[arc[r]];
              float w = rec[r].weight;
              if (ctx_contains(cx, arc[r])) w = w + cx.offset;   // Sec. 4.1
              cand[r] = (c_own + w) - Lrow.at((rec[r].meta & 0xFFFFu) - 1u);
              uint32_t o = f2ord(cand[r]);
              lmin = o < lmin ? o : lmin;
            }
          }
        }
        uint32_t wmin = wave_min_u32(lmin);
        if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->m_ord, wmin);
        if (jb == 0) wg_barrier<kLds>();   // (every wave passes here exactly once per batch)
        commit_emit_n<kLds, 2>(p, M, sh, no, AL.total, jb, cand, arc, rec, srct, n_cand, lane, pd, pd_arc, pd_arc2);
        if constexpr (kEmitSlots > 2) {
          if (jb + 128 < AL.total)
            commit_emit_n<kLds, kEmitSlots - 2>(p, M, sh, no, AL.total, jb + 128, &cand[2], &arc[2], &rec[2], &srct[2], n_cand,
                                                lane, pd, pd_arc, pd_arc2);
        }
      }
    }
  }
  wg_barrier<kLds>();
  if (sh->n_big > 0) {
    // the parked long rows: every wave takes every NW-th group of 64 arcs
    const int nbig = min(sh->n_big, kBigRows);
    for (int r = 0; r < nbig; ++r) {
      const int first = sh->big_first[r], deg = sh->big_deg[r];
      const float c_own = sh->big_cost[r];
      const uint32_t src = sh->big_src[r];
      for (int j0 = wave * 64; j0 < deg; j0 += NW * 64) {
        int jj = j0 + lane;
        bool act = jj < deg;
        int a = first + jj;
        float cand = 0.0f;
        ArcRec rec; rec.dst = 0; rec.weight = 0.0f; rec.row = 0; rec.meta = 0;
        if (act) {
          rec = p.arcs[a];
          float w = rec.weight;
          if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1
          cand = (c_own + w) - Lrow.at((rec.meta & 0xFFFFu) - 1u);
        }
        uint32_t wmin = wave_min_u32(act ? f2ord(cand) : 0xFFFFFFFFu);
        if (lane == 0) atomicMin(&sh->m_ord, wmin);
        bool imp; uint32_t hh; RowInfo rr;
        commit<kLds, true>(p, M, sh, &sh->n_front[0], no, act, cand, a, rec, src, 0.0f, n_cand, lane, true, load_fault(sh), imp, hh, rr);
      }
    }
    wg_barrier<kLds>();
  }

  // ---- step 3: the emission minimum fixes the frame's cutoff
  const float m = ord2f(sh->m_ord);
  // (no test of sh->fault here: waves already in the closure may set it while others have not read it yet;
  // after an overflow the updates below do nothing, and the flag is read once every writer has passed a barrier)
  if (sh_n_claim(sh) == 0) return kFrameNoTokens;   // stable: nothing can be added to an empty table

  // ---- step 4: epsilon closure.  First every lane follows the state it kept from the emit phase,
  // provided that is still the state's value and survived the cutoff ...
  int levels = 0;   // deepest run of closure levels this wave has made in one go
  if (pd.deg > 0) {
    uint64_t curv = ldv<kLds>(&M.hval[pd.slot]);
    if ((uint32_t)curv != pd_arc || pd.cost - m > p.beam) pd.deg = 0;
  }
  if (pd.deg2 > 0) {
    uint64_t curv = ldv<kLds>(&M.hval[pd.slot2]);
    if ((uint32_t)curv != pd_arc2 || pd.cost2 - m > p.beam) pd.deg2 = 0;
  }
  chase<kLds>(p, M, sh, &sh->n_front[0], cx, no, owner_map, pd, m, n_eps, n_cand, levels, lane);
  // This wave has stored the last token row it will store in this frame (the rare rounds below have full
  // barriers of their own): once the stores have landed, the barrier makes them the next frame's to read.
  // The frame's log-likelihood row is no longer needed either (only the emit phase reads it), so the next
  // one is parked now, by waves that would otherwise just wait for the deepest chain.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  if (Lnext) {
#pragma unroll
    for (int k = 0; k < kPre; ++k) {
      int i = tid + k * kBlock;
      if (i < p.num_pdfs) Lstage[i] = pre[k];
    }
    for (int i = tid + kPre * kBlock; i < p.num_pdfs; i += kBlock) Lstage[i] = Lnext[i];
  }
  wg_barrier<kLds>();
  // ... then, rarely, rounds over the change log for what was left flagged there: round r reads the
  // entries logged before it and counts the entries it flags for round r+1 in the other counter
  if (sh->n_front[0] > 0 && !sh->diverged && !sh->fault) {
    if (tid == 0) { sh->fr_begin = 0; sh->fr_end = sh_log_n(sh); }
    __syncthreads();   // (full: the rounds read token rows that other waves stored to device memory)
    for (int r = 0; sh->n_front[r & 1] > 0; ++r) {
      const int fb = sh->fr_begin, fe = sh->fr_end;
      int32_t *front = &sh->n_front[(r + 1) & 1];
      for (int base = fb; base < fe; base += kBlock) {
        // the round's entries are shared evenly by the waves
        const int nb = min(kBlock, fe - base);
        const int tpw = (nb + NW - 1) / NW;
        int j = lane < tpw ? base + wave * tpw + lane : fe;
        if (j >= base + nb) j = fe;
        pending_clear(pd);
        if (j < fe) {
          LogE e = M.log[j];
          if (e.src & LogE::kSrcHasEps) {
            uint64_t curv = ldv<kLds>(&M.hval[e.h]);
            float cost = ord2f((uint32_t)(curv >> 32));
            // still this state's value, and not dropped by the emission cutoff
            if ((uint32_t)curv == e.arc && curv != kEmptyVal && !(cost - m > p.beam)) {
              uint32_t idx = ldv<kLds>(&M.hidx[e.h]);
              const int eps0 = load_row_fe(&M.t_row[no + idx]).y, end0 = load_row_end(&M.t_row[no + idx]).x;
              pd.first = eps0;
              pd.deg = end0 - eps0;
              pd.cost = cost;
              pd.slot = e.h;
            }
          }
        }
        chase<kLds>(p, M, sh, front, cx, no, owner_map, pd, m, n_eps, n_cand, levels, lane);
      }
      wg_barrier<kLds>();
      if (tid == 0) {
        sh->fr_begin = fe; sh->fr_end = sh_log_n(sh);
        sh->n_front[r & 1] = 0;
        if (*front > 0 && r + 1 >= p.max_eps_iters) sh->diverged = 1;
        sh->halt = sh->diverged | sh->fault;   // latched between barriers, so every wave takes the same branch
      }
      __syncthreads();
      if (sh->halt) break;
    }
  }
  if (sh->fault) return kFrameOverflow;
  if (sh->diverged) return kFrameDiverged;
  if (sh->n_rec + sh_n_claim(sh) > p.bp_cap) return kFrameRecordsFull;

  // ---- step 5 and bookkeeping: every state's winning update writes the token
  // (the histogram only matters when more tokens than max_active can survive; the table holds at least as many)
  const bool hist_need = hist_on && sh_n_claim(sh) > p.max_active;
  {
    const float best = ord2f(umin32(sh->m_ord, sh->best_ord));
    const int base_cur = sh->n_rec, base_prev = sh->frame_base, log_n = sh_log_n(sh);
    int w_surv = 0, w_live = 0;   // per wave, counted with ballots (same-address LDS atomics from many lanes crawl)
    for (int j0 = wave * 64; j0 < log_n; j0 += kBlock) {
      const int j = j0 + lane;
      bool live = false, surv = false;
      if (j < log_n) {
      LogE e = M.log[j];
      uint64_t curv = ldv<kLds>(&M.hval[e.h]);
      // an arc can appear twice for a slot (its source improved in a later round): one of them takes the slot
      if ((uint32_t)curv == e.arc && curv != kEmptyVal &&
          atomicCAS((unsigned long long *)&M.hval[e.h], (unsigned long long)curv, (unsigned long long)kEmptyVal) == curv) {
        int idx = (int)ldv<kLds>(&M.hidx[e.h]);
        float cost = ord2f((uint32_t)(curv >> 32));
        bool dead = cost - m > p.beam;
        uint32_t sf = e.src & LogE::kSrcMask;
        int prev = -1;
        if (e.src & LogE::kSrcEps) prev = base_cur + (int)ldv<kLds>(&M.hidx[sf]);   // source state's token, via its slot
        else if (sf != LogE::kSrcNone) prev = base_prev + (int)sf;
        M.t_cost[idx] = dead ? __builtin_inff() : cost;
        bp[base_cur + idx] = make_int2((int)e.arc, prev);
        if (last_frame) g_tok_state[idx] = (int)ldv<kLds>(&M.hkey[e.h]);
        if (!dead) {
          live = true;
          float r = cost - best;
          if (!(r > p.beam)) {
            surv = true;
            if (hist_need) {
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              atomicAdd(&hist[bin], 1u);
            }
          }
        }
        stv<kLds>(&M.hkey[e.h], kEmptyKey);
      }
      }
      w_live += __popcll(__ballot(live));
      w_surv += __popcll(__ballot(surv));
    }
    if (lane == 0) {
      if (w_surv) atomicAdd(&sh->n_surv, w_surv);
      if (w_live) atomicAdd(&sh->n_live, w_live);
      // (no failure return lies behind this point, so a frame is counted once)
      if (n_active) atomicAdd(&sh->a_active, (unsigned long long)n_active);
      if (n_emit) atomicAdd(&sh->a_emit, (unsigned long long)n_emit);
      if (n_eps) atomicAdd(&sh->a_eps, (unsigned long long)n_eps);
      if (n_cand) atomicAdd(&sh->a_cand, (unsigned long long)n_cand);
      if (levels) atomicMax(&sh->rounds, levels);
    }
  }
  wg_barrier<kLds>();

  // ---- close the frame
  if (wave == 0) {
    int cut = 255;
    if (hist_need && sh->n_surv > p.max_active) {
      // largest bin B whose cumulative count fits max_active (0 if bin 0 alone does not)
      int loc[4], sum = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) { loc[k] = (int)hist[lane * 4 + k]; sum += loc[k]; }
      int incl = wave_incl_scan(sum);
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
      sh->n_tok = sh_n_claim(sh);
      sh->frame_base = sh->n_rec;
      sh->n_rec += sh_n_claim(sh);
      sh->best = ord2f(umin32(sh->m_ord, sh->best_ord));
      if (f >= 0) {  // the table made at reset is not a decoded frame
        atomicAdd(&sh->a_frames, 1ull);
        atomicAdd(&sh->a_tokens, (unsigned long long)sh->n_live);
        atomicMax(&sh->a_maxtok, sh->n_live);
        if (!kLds) atomicAdd(&sh->a_slow, 1);
      }
      atomicAdd(&sh->a_impr, (unsigned long long)sh_log_n(sh));
      atomicAdd(&sh->a_rounds, (unsigned long long)sh->rounds);
    }
    frame_init(sh, hist, false, lane, hist_need);   // for the next frame
  }
  wg_barrier<kLds>();   // (back-pointer stores need not have landed: nothing in the next frame reads them)
  return kFrameOk;
}

}  // namespace cbd
#include "cbd_lean.hpp"
namespace cbd {

// Where the current tokens' arc rows are kept changes with the code that decodes the next frame: the lean code
// wants them in LDS, the general code in the channel's row buffer in device memory.
template <int kBlock>
__device__ __forceinline__ void rows_to_lds(const Mem<true> &M, const LeanMem &R, int n_tok, int row_buf) {
  const int4 *rows = M.t_row + (size_t)row_buf * M.row_cap;
  for (int i = threadIdx.x; i < n_tok; i += kBlock) {
    const int2 fe = load_row_fe(&rows[i]);
    const int deg = fe.y - fe.x;
    R.t_first[i] = fe.x;
    R.t_deg[i] = deg < (int)kEdEscape ? (uint16_t)deg : kLeanDegEscape;
  }
  __syncthreads();
}
template <int kBlock>
__device__ __forceinline__ void rows_to_device(const Mem<true> &M, const LeanMem &R, int n_tok, int row_buf) {
  int4 *rows = M.t_row + (size_t)row_buf * M.row_cap;
  for (int i = threadIdx.x; i < n_tok; i += kBlock) {
    const int first = R.t_first[i];
    const uint16_t deg = R.t_deg[i];
    // (a row too long for the count field was written to the row buffer when its token was made)
    if (deg != kLeanDegEscape) rows[i] = make_int4(first, first + (int)deg, 0, 0);
  }
  __syncthreads();   // (waits for the stores: other waves read the rows past their L1)
}

// One call's work on one channel: `pos` is the channel's place in the call's list.
template <int kBlock>
__device__ __forceinline__ void advance_channel(const AdvanceParams &p, const int pos, unsigned char *smem) {
  const int tid = threadIdx.x;
  const int c = p.chan_ids[pos];
  ChanState *cs = p.chan + c;
  const LdsLayout lay = make_layout(p.stage_rows ? p.num_pdfs : 0, p.ctx_lds_cap, p.lds_tok_cap, p.lds_slots,
                                    p.lds_log_cap, p.lean_log_per_wave * (kBlock / 64));
  Shared *sh = (Shared *)(smem + lay.sh);
  uint32_t *hist = (uint32_t *)(smem + lay.hist);
  uint32_t *bitmap = (uint32_t *)(smem + lay.bitmap);
  uint8_t *owner_maps = (uint8_t *)(smem + lay.owner);
  uint8_t *closure_maps = (uint8_t *)(smem + lay.cmap);
  int32_t *ctx_lds = (int32_t *)(smem + lay.ctx);
  float *Lrow = (float *)(smem + lay.L);

  Mem<true> ML;
  ML.hval = (uint64_t *)(smem + lay.hval);
  ML.hkey = (uint32_t *)(smem + lay.hkey);
  ML.hidx = (uint16_t *)(smem + lay.hidx);
  ML.t_cost = (float *)(smem + lay.tcost);
  ML.log = (LogT<true> *)(smem + lay.log);
  ML.t_row = p.tok_row + (size_t)c * 2 * p.g_tok_cap;
  ML.slots = (uint32_t)p.lds_slots; ML.tok_cap = p.lds_tok_cap; ML.log_cap = p.lds_log_cap; ML.row_cap = p.g_tok_cap;

  // (the tables in device memory are described where they are used: few frames need them, and every pointer that
  // lives through the frame loop costs the lean frames registers)
  auto make_MG = [&]() {
    Mem<false> G;
    G.hval = p.g_hval + (size_t)c * p.g_slots;
    G.hkey = p.g_hkey + (size_t)c * p.g_slots;
    G.hidx = p.g_hidx + (size_t)c * p.g_slots;
    G.t_row = p.tok_row + (size_t)c * 2 * p.g_tok_cap;
    G.t_cost = p.tok_cost + (size_t)c * p.g_tok_cap;
    G.log = p.g_log + (size_t)c * p.g_log_cap;
    G.slots = (uint32_t)p.g_slots; G.tok_cap = p.g_tok_cap; G.log_cap = p.g_log_cap; G.row_cap = p.g_tok_cap;
    return G;
  };
  auto g_cost = [&]() { return p.tok_cost + (size_t)c * p.g_tok_cap; };
  int32_t *g_tok_state = p.tok_state + (size_t)c * p.g_tok_cap;
  int2 *bp = p.bp + (size_t)c * p.bp_cap;
  const float *Lbase = p.loglikes + (long long)pos * p.channel_stride;

  if (tid == 0) {
    sh->status = p.do_reset ? kStatusOk : cs->status;
    sh->n_tok = p.do_reset ? 0 : cs->n_tok;
    sh->frame_base = p.do_reset ? 0 : cs->frame_base;
    sh->n_rec = p.do_reset ? 0 : cs->n_rec;
    sh->best = p.do_reset ? 0.0f : cs->best;
    sh->cut_bin = p.do_reset ? 255 : cs->cut_bin;
    sh->a_maxtok = 0; sh->a_slow = 0;
    sh->a_frames = sh->a_active = sh->a_emit = sh->a_eps = sh->a_cand = sh->a_impr = sh->a_tokens = sh->a_rounds = 0;
  }
  __syncthreads();
  if (sh->status != kStatusOk) {  // uniform: the channel is parked until reset
    if (p.new_records && tid == 0) p.new_records[c] = make_int2(0, p.call_seq);
    if (p.auto_snap && tid == 0) {
      int32_t *snap = p.auto_snap + (size_t)pos * kSnapInts;
      snap[0] = sh->status; snap[1] = -1; snap[2] = (int)0xFFFFFFFFu; snap[3] = cs->n_rec; snap[4] = c;
      snap[5] = 0; snap[6] = 0; snap[7] = 0;
    }
    return;
  }

  // context of this call (Sec. 4.3: whichever list is current is the one used)
  Ctx cx;
  const int cslot = cs->ctx_slot;
  cx.n = p.ctx_n[cslot]; cx.offset = p.ctx_off[cslot];
  cx.g_list = p.ctx + (size_t)cslot * p.max_ctx;
  cx.lds_list = (lds_cint_ptr)ctx_lds; cx.bitmap = bitmap;
  cx.in_lds = cx.n <= p.ctx_lds_cap;
  cx.use_bitmap = p.lookup_mode == 1;
  if (cx.in_lds) for (int i = tid; i < cx.n; i += kBlock) ctx_lds[i] = cx.g_list[i];
  if (cx.use_bitmap) {
    for (int i = tid; i < kBloomWords; i += kBlock) bitmap[i] = 0;
    __syncthreads();
    for (int i = tid; i < cx.n; i += kBlock) {
      const uint32_t h = bloom_hash(cx.g_list[i]);
      atomicOr(&bitmap[bloom_word(h)], bloom_mask(h));
    }
  }
  // the tokens' costs enter through device memory; LDS takes them over when they fit
  bool fast = p.lds_tok_cap > 0 && sh->n_tok <= p.lds_tok_cap;
  int cur = p.do_reset ? 0 : (cs->row_buf & 1);
  for (int i = tid; i < p.lds_slots; i += kBlock) { ML.hval[i] = kEmptyVal; ML.hkey[i] = kEmptyKey; }
  if (fast) {
    { float *gc = g_cost(); for (int i = tid; i < sh->n_tok; i += kBlock) ML.t_cost[i] = gc[i]; }
  }
  if (p.n_frames > 0 && p.stage_rows) for (int i = tid; i < p.num_pdfs; i += kBlock) Lrow[i] = Lbase[i];
  __syncthreads();

  int outcome = kFrameOk;
  if (tid < 64) frame_init(sh, hist, p.do_reset != 0, tid);
  if (tid == 0) { sh->a_lean = 0; sh->a_lean_pack[0] = 0; sh->a_lean_pack[1] = 0; }
#ifdef CBD_PROFILE
  if (tid == 0) {
    for (int k = 0; k < 12; ++k) sh->prof[k] = 0;
    for (int k = 0; k < 8; ++k) sh->prof_why[k] = 0;
    sh->prof_redo = 0; sh->prof_general = 0;
  }
  const long long prof_k0 = wall_clock64();
#endif
  __syncthreads();
  const LeanMem LM = make_lean_mem(ML.log, p.lds_tok_cap, p.lds_slots, p.lean_log_per_wave);
  bool rows_in_lds = false;   // the current tokens' rows: in LDS (lean frames) or in the row buffer `cur`
  for (int f = p.do_reset ? -1 : 0; f < p.n_frames; ++f) {
    // the next frame's row (staged rows: copied to LDS during this frame; others: only the lean code uses it)
    const float *Lnext = (f >= 0 && f + 1 < p.n_frames) ? Lbase + (long long)(f + 1) * p.num_pdfs : nullptr;
    Rows rows;
    rows.lds = (lds_cfloat_ptr)Lrow; rows.glob = Lbase + (long long)(f < 0 ? 0 : f) * p.num_pdfs; rows.staged = p.stage_rows != 0;
    const bool last = f == p.n_frames - 1;
    bool slow = !fast;
    if (fast) {
      // frames go to the lean code; whatever that cannot take comes back
      const bool lean = p.lean_frames && f >= 0;
      if (lean) {
        if (!rows_in_lds) { rows_to_lds<kBlock>(ML, LM, sh->n_tok, cur); rows_in_lds = true; }
        outcome = run_frame_lean<kBlock>(p, ML, LM, sh, cx, Lrow, rows, Lnext, hist, owner_maps, closure_maps, cur, bp,
                                         g_tok_state, last);
        if (outcome == kFrameRedo) {
#ifdef CBD_PROFILE
          if (tid == 0) { sh->prof_redo += 1; sh->prof_general -= wall_clock64(); }
#endif
          // wipe the table, bring this frame's log-likelihood row back, hand the rows to the general code
          __syncthreads();
          for (int i = tid; i < p.lds_slots; i += kBlock) { ML.hval[i] = kEmptyVal; ML.hkey[i] = kEmptyKey; }
          if (p.stage_rows) for (int i = tid; i < p.num_pdfs; i += kBlock) Lrow[i] = rows.glob[i];
          rows_to_device<kBlock>(ML, LM, sh->n_tok, cur);
          rows_in_lds = false;
          if (tid < 64) frame_init(sh, hist, false, tid);
          __syncthreads();
        }
      }
      if (!lean || outcome == kFrameRedo) {
        if (rows_in_lds) { rows_to_device<kBlock>(ML, LM, sh->n_tok, cur); rows_in_lds = false; }
        outcome = run_frame<true, kBlock>(p, ML, sh, cx, Lrow, rows, p.stage_rows ? Lnext : nullptr, hist, owner_maps, f, cur, bp, g_tok_state, last);
        if (outcome == kFrameOk) cur ^= 1;
#ifdef CBD_PROFILE
        if (lean && tid == 0) sh->prof_general += wall_clock64();
#endif
      }
      if (outcome == kFrameOverflow) {
        // redo the frame with the tables in device memory: wipe the LDS table, hand the costs over
        for (int i = tid; i < p.lds_slots; i += kBlock) { ML.hval[i] = kEmptyVal; ML.hkey[i] = kEmptyKey; }
        { float *gc = g_cost(); for (int i = tid; i < sh->n_tok; i += kBlock) gc[i] = ML.t_cost[i]; }
        // (the abandoned attempt has already parked the next frame's log-likelihood row: bring this frame's back)
        if (p.stage_rows && f >= 0) for (int i = tid; i < p.num_pdfs; i += kBlock) Lrow[i] = rows.glob[i];
        __syncthreads();
        if (tid < 64) frame_init(sh, hist, f < 0, tid);
        __syncthreads();
        fast = false; slow = true;
      }
    }
    if (slow) {
      const Mem<false> MG = make_MG();
      outcome = run_frame<false, kBlock>(p, MG, sh, cx, Lrow, rows, p.stage_rows ? Lnext : nullptr, hist, owner_maps, f, cur, bp, g_tok_state, last);
      if (outcome == kFrameOk) cur ^= 1;
    }
    if (outcome != kFrameOk) break;
    if (!fast && p.lds_tok_cap > 0 && sh->n_tok <= p.lds_tok_cap) {
      // the token list fits LDS again
      { float *gc = g_cost(); for (int i = tid; i < sh->n_tok; i += kBlock) ML.t_cost[i] = gc[i]; }
      fast = true;
      __syncthreads();
    }
  }

  // ---- leave: a frame that produced nothing, overflowed or diverged parks the channel
  __syncthreads();
  if (rows_in_lds && outcome == kFrameOk) rows_to_device<kBlock>(ML, LM, sh->n_tok, cur);   // the next call finds them there
  int status = kStatusOk;
  if (outcome == kFrameOverflow || outcome == kFrameRecordsFull) status = kStatusCapacity;
  else if (outcome == kFrameNoTokens) status = kStatusNoTokens;
  else if (outcome == kFrameDiverged) status = kStatusEpsDiverged;
  if (status == kStatusOk) {
    // the tokens' costs leave through device memory
    const int n = sh->n_tok;
    if (fast) {
      { float *gc = g_cost(); for (int i = tid; i < n; i += kBlock) gc[i] = ML.t_cost[i]; }
    }
  } else if (outcome != kFrameNoTokens) {
    // leave the device-memory table empty for the next utterance
    { const Mem<false> MG = make_MG(); for (int i = tid; i < p.g_slots; i += kBlock) { stv<false>(&MG.hkey[i], kEmptyKey); stv<false>(&MG.hval[i], kEmptyVal); } }
  }
  if (tid == 0) {
    cs->status = status;
    cs->n_tok = status == kStatusOk ? sh->n_tok : 0;
    cs->frame_base = status == kStatusOk ? sh->frame_base : sh->n_rec;
    cs->n_rec = sh->n_rec;
    cs->best = sh->best;
    cs->cut_bin = sh->cut_bin;
    cs->row_buf = status == kStatusOk ? cur : 0;
    if (p.do_reset) {
      cs->frames = 0; cs->active_tokens = 0; cs->emit_arcs = 0; cs->eps_arcs = 0; cs->candidates = 0;
      cs->improvements = 0; cs->tokens = 0; cs->eps_rounds = 0; cs->max_tokens = 0; cs->slow_frames = 0;
      cs->gc_base = 0; cs->gc_runs = 0; cs->gc_dropped = 0; cs->n_fixed_arcs = 0; cs->n_fixed_words = 0;
      cs->lean_frames = 0;
    }
    cs->lean_frames += sh->a_lean;
#ifdef CBD_PROFILE
    if (p.do_reset) for (int k = 0; k < 15; ++k) cs->spare[k] = 0;
    for (int k = 0; k < 7; ++k) cs->spare[k] += sh->prof[k];
    cs->spare[12] += sh->prof[7]; cs->spare[13] += sh->prof[8];
    cs->spare[8] += sh->prof_redo;
    cs->spare[7] += sh->prof_general;
    {
      long long packed = 0;   // eight 8-bit counts (saturating) would be too small: four 16-bit counts per word
      for (int k = 0; k < 4; ++k) packed |= (long long)(sh->prof_why[k] & 0x7FFF) << (16 * k);
      cs->spare[14] += packed;
    }
    cs->spare[9] += wall_clock64() - prof_k0;   // the workgroup's whole run
    if (p.n_frames > 0) {
      // when and where the workgroup ran: the 100 MHz counter is the same on all compute units; hardware register
      // 4 (HW_ID) holds the compute unit, shader array and engine, register 20 (XCC_ID) the die
      cs->timeline[0] = prof_k0; cs->timeline[1] = wall_clock64();
      cs->timeline[2] = ((long long)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 20) << 32) |
                        (unsigned)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4);
      cs->timeline[3] = pos;
    }
    cs->spare[10] += sh->a_lean;
    cs->spare[11] += (long long)sh->a_frames;
#endif
    cs->frames += sh->a_frames;
    cs->active_tokens += sh->a_active + (sh->a_lean_pack[0] & 0xFFFFFFFFull);
    cs->emit_arcs += sh->a_emit + (sh->a_lean_pack[0] >> 32);
    cs->eps_arcs += sh->a_eps + (sh->a_lean_pack[1] & 0xFFFFFFFFull);
    cs->candidates += sh->a_cand + (sh->a_lean_pack[1] >> 32);
    cs->improvements += sh->a_impr;
    cs->tokens += sh->a_tokens; cs->eps_rounds += sh->a_rounds;
    if (sh->a_maxtok > cs->max_tokens) cs->max_tokens = sh->a_maxtok;
    cs->slow_frames += sh->a_slow;
    const int n_new = sh->n_rec - (p.do_reset ? 0 : cs->gc_base);
    if (p.new_records) p.new_records[c] = make_int2(n_new, p.call_seq);
    if (p.due_max) atomicMax(p.due_max, ((unsigned long long)(uint32_t)p.call_seq << 32) | (uint32_t)n_new);
  }
  // Sec. 1 / 3.2: the partial result is the best current token's sequence.  The workgroup leaves that token
  // here (arg-min of (cost, arc) over its final table, as the stand-alone snapshot kernel would find it), so a
  // request for partial results right after this call only has to walk.
  if (p.auto_snap) {
    __syncthreads();   // this call's last costs and records are in device memory
    if (tid < 64) {
      const int lane = tid;
      uint64_t bestk = kEmptyVal;
      int besti = -1;
      if (status == kStatusOk) {
        const int n = sh->n_tok, base = sh->frame_base;
        for (int t = lane; t < n; t += 64) {
          const float cost = __hip_atomic_load(&g_cost()[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (!(cost < __builtin_inff())) continue;   // dropped by the frame cutoff
          const unsigned long long rec = __hip_atomic_load((const unsigned long long *)&bp[base + t], __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
          const uint64_t k = ((uint64_t)f2ord(cost) << 32) | (uint32_t)rec;   // low word of a record: its arc
          if (k < bestk) { bestk = k; besti = t; }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
          uint64_t ok = (uint64_t)__shfl_xor((long long)bestk, d, 64);
          int oi = __shfl_xor(besti, d, 64);
          if (ok < bestk) { bestk = ok; besti = oi; }
        }
      }
      if (lane == 0) {
        int32_t *snap = p.auto_snap + (size_t)pos * kSnapInts;
        snap[0] = status != kStatusOk ? status : (besti < 0 ? kStatusNoTokens : kStatusOk);
        snap[1] = besti < 0 ? -1 : sh->frame_base + besti;
        snap[2] = (int)(uint32_t)(bestk >> 32);
        snap[3] = sh->n_rec; snap[4] = c;
        snap[5] = cs->gc_base; snap[6] = cs->n_fixed_arcs; snap[7] = cs->n_fixed_words;
      }
    }
  }
}

// The decode kernel: workgroup b takes place b of the call's channel list.
template <int kBlock>
__global__ __launch_bounds__(kBlock, 4) void advance_kernel(AdvanceParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  advance_channel<kBlock>(p, (int)blockIdx.x, smem);
}

// The same with 120 instead of 128 vector registers per wave, for launches that start while result walks of
// earlier calls are still on the side stream.  Sixteen waves of 128 registers take a compute unit's whole register
// file: no wave of another kernel fits beside them, so a walk (two waves of 16 registers, half a KB of LDS) that
// gets onto a compute unit first keeps the decoding workgroup off it until it is through, and the launch ends that
// much later (Large, a partial result per chunk: 0.69 ms per launch against 0.59 without the walks).  With 8
// registers per wave left over, and 2 KB of LDS left free by the decoder's layout, walk and decoding share the
// unit: 0.63 ms.  The 8 registers cost 2-4 % where nothing runs beside the launch, hence two kernels.  (The
// attribute counts registers of one kind; for this device's unified file the compiler doubles it: 60 -> 120.)
template <int kBlock>
__global__ __launch_bounds__(kBlock, 4) __attribute__((amdgpu_num_vgpr(60))) void advance_beside_kernel(AdvanceParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  advance_channel<kBlock>(p, (int)blockIdx.x, smem);
}

// ---- self-test of the cross-lane primitives ------------------------------------

// One wave: prefix sums of in[0..63] and the minimum of in[64..127] (as unsigned).
__global__ __launch_bounds__(64) void selftest_kernel(const int32_t *in, int32_t *out_scan, uint32_t *out_min) {
  int lane = threadIdx.x;
  out_scan[lane] = wave_incl_scan(in[lane]);
  out_min[lane] = wave_min_u32((uint32_t)in[64 + lane]);
}

// ---- contexts ---------------------------------------------------------------

// One workgroup per uploaded list copies it into its slot of the context store; with `bind`,
// channel bind[i] is switched to that slot as well.
__global__ void scatter_contexts_kernel(const int32_t *slots, const int32_t *bind, const int32_t *list_off,
                                        const float *offsets, const int32_t *lists, int32_t *ctx, int max_ctx,
                                        int32_t *ctx_n, float *ctx_off, ChanState *chan) {
  int i = blockIdx.x;
  int slot = slots[i];
  int b = list_off[i], n = list_off[i + 1] - b;
  for (int k = threadIdx.x; k < n; k += blockDim.x) ctx[(size_t)slot * max_ctx + k] = lists[b + k];
  if (threadIdx.x == 0) {
    ctx_n[slot] = n; ctx_off[slot] = offsets[i];
    if (bind) chan[bind[i]].ctx_slot = slot;
  }
}

// Sec. 4.2 asks for the listed arc indices sorted; the list is a set.  One workgroup per uploaded list does
// all of it on the device: caller's arc numbering -> library numbering, bitonic sort in LDS, removal of
// repeats, and the store into the list's slot (with `bind`, channel bind[i] is switched to that slot too).
// Lists longer than kPrepMaxList are prepared on the host instead.
constexpr int kPrepMaxList = 8192;
constexpr int kPrepThreads = 256;

__global__ __launch_bounds__(kPrepThreads) void prepare_contexts_kernel(
    const int32_t *slots, const int32_t *bind, const int32_t *list_off, const float *offsets, const int32_t *lists,
    const int32_t *pub2int, int32_t *ctx, int max_ctx, int32_t *ctx_n, float *ctx_off, ChanState *chan) {
  extern __shared__ __align__(16) int32_t prep_v[];   // the next power of two >= the longest list of the launch
  __shared__ int32_t prep_cnt[kPrepThreads];
  const int tid = threadIdx.x;
  const int i = blockIdx.x;
  const int slot = slots[i];
  const int b = list_off[i], n = list_off[i + 1] - b;
  int N = 1;
  while (N < n) N <<= 1;
  const int32_t kPad = 0x7FFFFFFF;   // no arc has this number; pads sort to the end
  for (int k = tid; k < N; k += kPrepThreads) prep_v[k] = k < n ? pub2int[lists[b + k]] : kPad;
  __syncthreads();
  for (int k = 2; k <= N; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (N >> 1); t += kPrepThreads) {
        const int lo = 2 * j * (t / j) + (t % j), hi = lo + j;
        const bool ascending = (lo & k) == 0;
        const int32_t x = prep_v[lo], y = prep_v[hi];
        if ((x > y) == ascending) { prep_v[lo] = y; prep_v[hi] = x; }
      }
      __syncthreads();
    }
  }
  // each thread owns a run of consecutive positions: count the first occurrences in it, ...
  const int per = (N + kPrepThreads - 1) / kPrepThreads;
  const int e0 = min(tid * per, N), e1 = min(e0 + per, N);
  int cnt = 0;
  for (int e = e0; e < e1; ++e) cnt += prep_v[e] != kPad && (e == 0 || prep_v[e] != prep_v[e - 1]);
  prep_cnt[tid] = cnt;
  __syncthreads();
  // ... turn the counts into positions (inclusive scan over the threads), ...
  for (int d = 1; d < kPrepThreads; d <<= 1) {
    const int add = tid >= d ? prep_cnt[tid - d] : 0;
    __syncthreads();
    prep_cnt[tid] += add;
    __syncthreads();
  }
  // ... and store them in order
  int pos = prep_cnt[tid] - cnt;
  int32_t *out = ctx + (size_t)slot * max_ctx;
  for (int e = e0; e < e1; ++e)
    if (prep_v[e] != kPad && (e == 0 || prep_v[e] != prep_v[e - 1])) out[pos++] = prep_v[e];   // pos < n <= max_ctx
  if (tid == 0) {
    ctx_n[slot] = prep_cnt[kPrepThreads - 1]; ctx_off[slot] = offsets[i];
    if (bind) chan[bind[i]].ctx_slot = slot;
  }
}

// Sec. 4.3: switching a channel to a context that is already on the device is one store.
__global__ void bind_contexts_kernel(const int32_t *chan_ids, const int32_t *slots, int n, ChanState *chan) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) chan[chan_ids[i]].ctx_slot = slots[i];
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
    z.ctx_slot = i;              // the channel's own (empty) context
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
  const int32_t *olabel;    // library arc order
  const int32_t *int2pub;   // library arc order -> caller's numbering
  const float *final_cost;  // or null
  int32_t tok_cap, bp_cap, use_final, capacity;
  int32_t row_pitch;        // entries between consecutive output rows (>= capacity)
  int32_t *out_arcs;        // [n][row_pitch]
  int32_t *out_words;       // [n][row_pitch]
  int32_t *out_meta;        // [n][kMetaInts]: status, n_arcs, n_words, cost bits, fixed arcs, fixed words
  int32_t tail_only;        // 1: the path is followed down to the paths' shared beginning only (see the compaction)
  // that shared beginning in time order, or null if no compaction has run ([C][fixed_cap] each): whole-path
  // requests copy it instead of walking it
  const int32_t *fixed_arcs, *fixed_words;
  int32_t fixed_cap;
  int32_t *snap;            // [n][kSnapInts] snapshot taken on the decode stream (two-stage form only)
};

// Best token of a channel's current table (Sec. 1: the current best token sequence is read
// directly, no lattice).  All kThreads threads of the workgroup call it (a team's token list has tens of thousands
// of places: one wave alone needed 200 us); s_key / s_idx: one LDS entry per wave.  Every thread returns the
// record index or -1; key receives (cost, arc).  Keys are unique (an arc leads to one state, a state has one token).
template <int kThreads>
__device__ __forceinline__ int find_best(const BestParams &p, int c, const ChanState *cs, uint64_t &key, int tid,
                                         unsigned long long *s_key, int *s_idx) {
  const int n = cs->n_tok, base = cs->frame_base;
  const int32_t *ts = p.tok_state + (size_t)c * p.tok_cap;
  const float *tc = p.tok_cost + (size_t)c * p.tok_cap;
  const int2 *bp = p.bp + (size_t)c * p.bp_cap;
  uint64_t bestk = kEmptyVal;
  int besti = -1;
  for (int t = tid; t < n; t += kThreads) {
    float cost = tc[t];
    if (!(cost < __builtin_inff())) continue;   // dropped by the frame cutoff
    if (p.use_final && p.final_cost) cost = cost + p.final_cost[ts[t]];
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
  if (kThreads > 64) {
    if ((tid & 63) == 0) { s_key[tid >> 6] = bestk; s_idx[tid >> 6] = besti; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
      const uint64_t ok = s_key[w];
      if (ok < bestk) { bestk = ok; besti = s_idx[w]; }
    }
  }
  key = bestk;
  return besti < 0 ? -1 : base + besti;
}

// The walk below is one lane's chain of dependent reads, a round trip to device memory each.  Records lie in the
// order of the frames that wrote them, and a step of the walk leads about one frame's records back.  A second wave
// therefore reads ahead of it: it looks where the walk is (walk_pos, in LDS) and asks for the lines a few frames
// further down (64 bytes = 8 records each), so that the walk finds its records in the L2 cache.  It reads only and
// ends when the walk says so.
constexpr int kWalkDone = -2;
constexpr int kWalkChunk = 128;   // arcs the walk notes in LDS before the wave writes them out

// One pass of the wave that reads ahead of a walk at record r: asks for the 64-byte lines below `low` (the lowest
// record asked for so far) that the walk will reach next, never below `floor`.  Returns false when it is far
// enough ahead.  prev_r: where the walk was at the last pass.
__device__ __forceinline__ bool read_ahead_pass(const int2 *bp, int r, int floor, int lane, int &prev_r, int &low) {
  if (low < 0 || r < low) low = r;   // (first pass, or the walk has overtaken the reads)
  // how far the walk came since the last look tells how far it will be when these reads are back:
  // stay three such stretches and one span of the wave ahead of it, at most four spans per pass
  int moved = prev_r < 0 ? 64 : prev_r - r;
  moved = moved < 64 ? 64 : moved;
  prev_r = r;
  int target = r - 3 * moved - 512;
  target = target < floor ? floor : target;
  int spans = (low - target + 511) >> 9;
  spans = spans > 4 ? 4 : spans;
  if (spans <= 0) return false;
  // (always four reads, all under way together; spans not wanted yet repeat the first one's addresses)
  int v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int q = low - 8 - lane * 8 - (k < spans ? k : 0) * 512;
    v[k] = bp[q < floor ? floor : q].x;
  }
  asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]));   // (the values are not used: this keeps the reads)
  low -= spans * 512;
  if (low < floor) low = floor;
  return true;
}

__device__ __forceinline__ void walk_read_ahead(const BestParams &p, int c, int lane, const int *walk_pos) {
  const int2 *bp = p.bp + (size_t)c * p.bp_cap;
  int prev_r = -1, low = -1;
  for (;;) {
    const int r = __hip_atomic_load(walk_pos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (r == kWalkDone) break;
    if (!read_ahead_pass(bp, r, 0, lane, prev_r, low)) __builtin_amdgcn_s_sleep(8);   // look again shortly
  }
}

// Back-pointer walk from record `rec` and labels in time order.  One wave.  Only records below
// n_rec are touched (they never change once written), so this may run beside later decoding.
__device__ __forceinline__ void walk_path(const BestParams &p, int i, int c, int rec, int n_rec, uint32_t cost_ord,
                                          int lane, int *walk_pos, int *walk_arcs, int stop_below, int front_arcs,
                                          int front_words) {
  // stop_below: records below this one are not followed (0: the whole path).  front_arcs / front_words: that many
  // arcs / words of the channel's fixed part are put in front of what the walk finds (a plain copy: the fixed
  // part is kept in time order and in the caller's numbering).
  const int Fa = front_arcs, Fw = front_words;
  int32_t *meta = p.out_meta + (size_t)i * kMetaInts;
  int32_t *oarcs = p.out_arcs + (size_t)i * p.row_pitch;
  int32_t *owords = p.out_words + (size_t)i * p.row_pitch;
  const int2 *bp = p.bp + (size_t)c * p.bp_cap;
  const int inf_bits = (int)__float_as_uint(__builtin_inff());
  // lane 0 writes the arcs newest-first into the output row.  A path can never be longer than the
  // records in use; the bound also ends the walk on a predecessor cycle, which zero-weight epsilon
  // cycles can form.
  const int max_steps = n_rec;
  int na = 0;
  {
    // Lane 0 follows the predecessors and notes the arcs in LDS; every kWalkChunk steps the wave writes them out
    // together.  (A store to device memory per step would sit in the chain: the wait for the next record also
    // waits for the store before it.)
    int r = rec;
    while (r >= stop_below && na <= max_steps) {   // uniform
      int n_chunk = 0;
      if (lane == 0) {
        while (r >= stop_below && na + n_chunk <= max_steps && n_chunk < kWalkChunk) {
          int2 e = bp[r];
          // where the walk is, for the wave that reads ahead of it (an atomic store: a plain one is dropped)
          __hip_atomic_store(walk_pos, r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if ((uint32_t)e.x == kArcNone) { r = -1; break; }
          walk_arcs[n_chunk++] = e.x;
          r = e.y;
        }
      }
      n_chunk = __shfl(n_chunk, 0, 64);
      r = __shfl(r, 0, 64);
      __threadfence_block();
      for (int j = lane; j < n_chunk; j += 64)
        if (Fa + na + j < p.capacity) oarcs[Fa + na + j] = walk_arcs[j];
      __threadfence_block();
      na += n_chunk;
    }
    if (lane == 0) __hip_atomic_store(walk_pos, kWalkDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __threadfence_block();
  if (na > max_steps) {
    if (lane == 0) { meta[0] = kStatusEpsDiverged; meta[1] = 0; meta[2] = 0; meta[3] = inf_bits; }
    return;
  }
  if (Fa + na > p.capacity) {
    // count the words too so the caller learns both sizes
    int nw = 0;
    if (lane == 0) {
      int r = rec;
      for (int step = 0; r >= 0 && step < na; ++step) {
        int2 e = bp[r];
        if ((uint32_t)e.x == kArcNone) break;
        if (p.olabel[e.x] != 0) nw++;
        r = e.y;
      }
      meta[0] = kStatusBuffer; meta[1] = Fa + na; meta[2] = Fw + nw; meta[3] = (int)__float_as_uint(ord2f(cost_ord));
    }
    return;
  }
  // reverse into time order, pick up word labels, translate to the caller's numbering
  int nw_total = 0;
  int32_t *tail = oarcs + Fa;
  for (int j0 = 0; j0 < (na + 1) / 2; j0 += 64) {
    int j = j0 + lane;
    if (j < (na + 1) / 2) {
      int k = na - 1 - j;
      int a = tail[j], b = tail[k];
      tail[j] = b; tail[k] = a;
    }
  }
  __threadfence_block();
  for (int j0 = 0; j0 < na; j0 += 64) {
    int j = j0 + lane;
    int w = 0, a = 0;
    if (j < na) { a = tail[j]; w = p.olabel[a]; }
    unsigned long long wm = __ballot(w != 0);
    if (w != 0) owords[Fw + nw_total + __popcll(wm & ((1ull << lane) - 1ull))] = w;
    nw_total += __popcll(wm);
    if (j < na) tail[j] = p.int2pub[a];
  }
  if (Fa > 0) {
    const int32_t *fa = p.fixed_arcs + (size_t)c * p.fixed_cap, *fw = p.fixed_words + (size_t)c * p.fixed_cap;
    for (int j = lane; j < Fa; j += 64) oarcs[j] = fa[j];
    for (int j = lane; j < Fw; j += 64) owords[j] = fw[j];
  }
  if (lane == 0) {
    meta[0] = kStatusOk; meta[1] = Fa + na; meta[2] = Fw + nw_total;
    meta[3] = (int)__float_as_uint(ord2f(cost_ord));
  }
}

constexpr int kWalkThreads = 128;   // per channel: the wave that walks and the wave that reads ahead of it

// One workgroup per channel: best token, then its path.
__global__ __launch_bounds__(kWalkThreads) void best_path_kernel(BestParams p) {
  __shared__ int s_walk_pos;
  __shared__ int s_walk_arcs[kWalkChunk];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = blockIdx.x;
  const int c = p.chan_ids[i];
  const ChanState *cs = p.chan + c;
  int32_t *meta = p.out_meta + (size_t)i * kMetaInts;
  const int inf_bits = (int)__float_as_uint(__builtin_inff());
  if (threadIdx.x == 0) {
    meta[4] = p.tail_only ? cs->n_fixed_arcs : 0;
    meta[5] = p.tail_only ? cs->n_fixed_words : 0;
  }
  if (cs->status != kStatusOk) {   // (uniform)
    if (threadIdx.x == 0) { meta[0] = cs->status; meta[1] = 0; meta[2] = 0; meta[3] = inf_bits; }
    return;
  }
  __shared__ unsigned long long s_key[kWalkThreads / 64];
  __shared__ int s_idx[kWalkThreads / 64];
  uint64_t key = kEmptyVal;
  const int rec = find_best<kWalkThreads>(p, c, cs, key, (int)threadIdx.x, s_key, s_idx);
  if (threadIdx.x == 0) s_walk_pos = rec < 0 ? kWalkDone : rec;
  __syncthreads();
  if (wave == 1) {
    walk_read_ahead(p, c, lane, &s_walk_pos);
    return;
  }
  if (rec < 0) {
    if (lane == 0) { meta[0] = kStatusNoTokens; meta[1] = 0; meta[2] = 0; meta[3] = inf_bits; }
    return;
  }
  // (whole paths: what lies below gc_base is not walked but copied from the fixed part, where there is one)
  const bool have_fixed = p.fixed_arcs != nullptr;
  walk_path(p, i, c, rec, cs->n_rec, (uint32_t)(key >> 32), lane, &s_walk_pos, s_walk_arcs,
            (p.tail_only || have_fixed) ? cs->gc_base : 0, (!p.tail_only && have_fixed) ? cs->n_fixed_arcs : 0,
            (!p.tail_only && have_fixed) ? cs->n_fixed_words : 0);
}

// Two-stage form for results delivered beside later decoding.  Stage 1 (decode stream): pick the
// best token and note everything the walk needs, before the next call changes the channel.
constexpr int kSnapThreads = 512;
__global__ __launch_bounds__(kSnapThreads) void best_snapshot_kernel(BestParams p) {
  __shared__ unsigned long long s_key[kSnapThreads / 64];
  __shared__ int s_idx[kSnapThreads / 64];
  const int i = blockIdx.x;
  const int c = p.chan_ids[i];
  const ChanState *cs = p.chan + c;
  int32_t *snap = p.snap + (size_t)i * kSnapInts;
  int status = cs->status, rec = -1;
  uint64_t key = kEmptyVal;
  if (status == kStatusOk) {   // (uniform)
    rec = find_best<kSnapThreads>(p, c, cs, key, (int)threadIdx.x, s_key, s_idx);
    if (rec < 0) status = kStatusNoTokens;
  }
  if (threadIdx.x == 0) {
    snap[0] = status; snap[1] = rec; snap[2] = (int)(uint32_t)(key >> 32); snap[3] = cs->n_rec; snap[4] = c;
    snap[5] = cs->gc_base; snap[6] = cs->n_fixed_arcs; snap[7] = cs->n_fixed_words;
  }
}

// Stage 2 (side stream): the walk, from the snapshot only.
__global__ __launch_bounds__(kWalkThreads) void best_walk_kernel(BestParams p) {
  __shared__ int s_walk_pos;
  __shared__ int s_walk_arcs[kWalkChunk];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = blockIdx.x;
  const int32_t *snap = p.snap + (size_t)i * kSnapInts;
  int32_t *meta = p.out_meta + (size_t)i * kMetaInts;
  if (threadIdx.x == 0) {
    meta[4] = p.tail_only ? snap[6] : 0;
    meta[5] = p.tail_only ? snap[7] : 0;
  }
  if (snap[0] != kStatusOk) {   // (uniform)
    if (threadIdx.x == 0) { meta[0] = snap[0]; meta[1] = 0; meta[2] = 0; meta[3] = (int)__float_as_uint(__builtin_inff()); }
    return;
  }
  if (threadIdx.x == 0) s_walk_pos = snap[1];
  __syncthreads();
  if (wave == 1) {
    walk_read_ahead(p, snap[4], lane, &s_walk_pos);
    return;
  }
  const bool have_fixed = p.fixed_arcs != nullptr;
  walk_path(p, i, snap[4], snap[1], snap[3], (uint32_t)snap[2], lane, &s_walk_pos, s_walk_arcs,
            (p.tail_only || have_fixed) ? snap[5] : 0, (!p.tail_only && have_fixed) ? snap[6] : 0,
            (!p.tail_only && have_fixed) ? snap[7] : 0);
}

// ---- compaction of the back-pointer records ------------------------------------------

// Partial results are read off the best current token (Sec. 1, 3.2), so the only records ever read again are
// those on a path from a token of the current frame.  This kernel drops the others and renumbers the rest,
// which lets an utterance run on (the 3-minute recordings of Sec. 5.3 and beyond) in a buffer sized for the
// stretch between two compactions.  Results are unaffected: every kept record keeps its arc, and its
// predecessor is the same record under its new number.
//
// The paths of all current tokens share their beginning.  Records below gc_base are that shared beginning as
// an earlier compaction found it: one chain, part of every path from now on, never examined again (the marking
// walks stop there).  Above it lie the records examined each time: the tree the last compaction kept and
// whatever has been written since.  After marking, the kernel looks for the highest place in this stretch that
// exactly one marked link crosses: every path runs through that link, so the marked records below it are one
// chain, and gc_base moves up to there.  The cost of a call therefore follows the frames since the last one
// (plus the depth at which the paths merge), not the length of the utterance, and so does the memory in use.
// The records of the current frame (one per token, dead ones included) are all kept.
struct CompactParams {
  ChanState *chan;
  const int32_t *chan_ids;  // [grid]
  int2 *bp;                 // [C][bp_cap]
  const float *tok_cost;    // [C][tok_cap]
  uint32_t *mark;           // [C][mark_words] one bit per examined record
  uint32_t *prefix;         // [C][mark_words] marked records before each bitmap word
  int32_t *cross;           // [C][mark_words + 2] marked links crossing the place before each bitmap word
  int32_t bp_cap, tok_cap, mark_words;
  int32_t min_new;          // channels with at most this many records above gc_base are left alone ...
  const unsigned long long *due_max;  // ... or with at most half as many, if this (see AdvanceParams; null: not used)
  int32_t due_seq;                    //     comes from call due_seq and shows a channel above min_new
  // the shared beginning of the paths, written out in time order as it is found (append-only per utterance)
  int32_t *fixed_arcs;      // [C][fixed_cap] arcs, caller's numbering
  int32_t *fixed_words;     // [C][fixed_cap] their word labels
  int32_t fixed_cap;
  const int32_t *olabel;    // library arc order
  const int32_t *int2pub;   // library arc order -> caller's numbering
};

constexpr int kCompactBlock = 1024;
constexpr int kCompactPerThread = 4;
constexpr int kCompactStage = 4096;   // records the workgroup stages in LDS
constexpr int kCompactLdsWords = 16384;   // bitmap words (32 records each) the marking keeps in LDS

__device__ __forceinline__ uint32_t ld_agent_u32(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// New number of record q: g0 = gc_base, fb = first record of the current frame, new_fb = where that one moves.
__device__ __forceinline__ int compact_remap(int q, int g0, int fb, int new_fb, const uint32_t *mark,
                                             const uint32_t *prefix) {
  if (q < g0) return q;   // the shared beginning, or -1 (no predecessor)
  if (q >= fb) return q - fb + new_fb;
  const uint32_t r = (uint32_t)(q - g0), bit = 1u << (r & 31);
  const uint32_t wv = ld_agent_u32(&mark[r >> 5]);
  if (!(wv & bit)) return -1;   // only a dead token's record can point at a dropped one
  return g0 + (int)ld_agent_u32(&prefix[r >> 5]) + __popc(wv & (bit - 1u));
}

// A marked link between examined positions lo < hi (relative to gc_base; -1 = below it) crosses the places
// before bitmap words lo/32 + 1 .. hi/32: noted as +1 / -1 steps, summed up afterwards.
__device__ __forceinline__ void compact_note_link(int32_t *cross, int a, int b) {
  const int lo = a < b ? a : b, hi = a < b ? b : a;
  const int b_lo = (lo >> 5) + 1, b_hi = hi >> 5;   // (arithmetic shift: -1 >> 5 = -1)
  if (b_lo <= b_hi) {
    atomicAdd(&cross[b_lo], 1);
    atomicAdd(&cross[b_hi + 1], -1);
  }
}

// Workgroup-wide exclusive prefix sums of one value per thread (s_tot: one int per wave); returns the total.
__device__ __forceinline__ int compact_block_scan(int v, int &excl, int *s_tot, int lane, int wave) {
  const int incl = wave_incl_scan(v);
  if (lane == 63) s_tot[wave] = incl;
  __syncthreads();
  int before = 0, total = 0;
#pragma unroll
  for (int k = 0; k < kCompactBlock / 64; ++k) {
    const int t = s_tot[k];
    before += k < wave ? t : 0;
    total += t;
  }
  excl = before + incl - v;
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(kCompactBlock) void compact_records_kernel(CompactParams p) {
  __shared__ int s_tot[kCompactBlock / 64];
  __shared__ int s_cut, s_top, s_pos, s_done;
  __shared__ int2 s_stage[kCompactStage];
  __shared__ uint32_t s_mark[kCompactLdsWords];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = p.chan_ids[blockIdx.x];
  ChanState *cs = p.chan + c;
  if (cs->status != kStatusOk) return;   // (uniform) a parked channel has nothing worth keeping
  const int n_tok = cs->n_tok, fb = cs->frame_base, n_rec = cs->n_rec, g0 = cs->gc_base;
  const int young = fb - g0;      // records examined
  const int n_cur = n_rec - fb;   // records of the current frame
  // A compaction holds up its call for as long as one lane needs to walk the frames since the last one, however
  // many channels take part: so when one channel of the call is due, those half-way there join in.
  int min_new = p.min_new;
  if (p.due_max) {
    const unsigned long long dm = *p.due_max;
    if ((int32_t)(dm >> 32) == p.due_seq && (int32_t)(uint32_t)dm > p.min_new) min_new = p.min_new / 2;
  }
  if (young <= 0 || n_rec - g0 <= min_new) return;
  int2 *bp = p.bp + (size_t)c * p.bp_cap;
  const float *tc = p.tok_cost + (size_t)c * p.tok_cap;
  uint32_t *mark = p.mark + (size_t)c * p.mark_words;
  uint32_t *prefix = p.prefix + (size_t)c * p.mark_words;
  int32_t *cross = p.cross + (size_t)c * (p.mark_words + 2);
  const int W = (young + 31) >> 5;   // bitmap words in use (<= mark_words: the host sizes them for bp_cap records)
  const int B = young >> 5;          // places 0..B: place b lies before examined record 32 b

  // While the walks run, the bitmap is in LDS if it fits (a walk's step then waits for a record from L2 and an LDS
  // atomic, not for an atomic's trip to device memory); it is copied out afterwards for the passes that follow.
  const bool lds_marks = W <= kCompactLdsWords;
  if (lds_marks) {
    for (int i = tid; i < W; i += kCompactBlock) s_mark[i] = 0;
  } else {
    for (int i = tid; i < W; i += kCompactBlock) mark[i] = 0;
  }
  for (int i = tid; i < B + 2; i += kCompactBlock) cross[i] = 0;
  if (tid == 0) { s_cut = -1; s_top = -1; s_pos = fb; s_done = 0; }
  __syncthreads();
  // mark: from every live token's record, back to the first record that is already marked or lies below gc_base.
  // Links inside the current frame (epsilon-input arcs) are not followed: their targets are tokens with walks of
  // their own.  A walk that runs into a loop of predecessors stops at its first marked record like any other.
  // The walks soon merge into one lane's chain of dependent reads, a trip to device memory each; as for the
  // result walks, the last wave reads ahead of the lowest position any walk has reached (s_pos).
  constexpr int kWalkWaves = kCompactBlock / 64 - 1;
  if (wave == kWalkWaves) {
    int prev_r = -1, low = -1;
    while (__hip_atomic_load(&s_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < kWalkWaves) {
      const int r = __hip_atomic_load(&s_pos, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      if (!read_ahead_pass(bp, r, g0, lane, prev_r, low)) __builtin_amdgcn_s_sleep(8);
    }
  } else {
    if (lds_marks) {
      for (int i = tid; i < n_tok && i < n_cur; i += kWalkWaves * 64) {
        if (!(tc[i] < __builtin_inff())) continue;   // dropped by the frame cutoff
        int q = bp[fb + i].y;
        if (q < fb) compact_note_link(cross, q < g0 ? -1 : q - g0, young);
        while (q >= g0 && q < fb) {
          const uint32_t r = (uint32_t)(q - g0), bit = 1u << (r & 31);
          const int nxt = bp[q].y;   // asked for before the mark's answer is in
          atomicMin(&s_pos, q);
          if (atomicOr(&s_mark[r >> 5], bit) & bit) break;
          q = nxt;
        }
      }
    } else {
      for (int i = tid; i < n_tok && i < n_cur; i += kWalkWaves * 64) {
        if (!(tc[i] < __builtin_inff())) continue;
        int q = bp[fb + i].y;
        if (q < fb) compact_note_link(cross, q < g0 ? -1 : q - g0, young);
        while (q >= g0 && q < fb) {
          const uint32_t r = (uint32_t)(q - g0), bit = 1u << (r & 31);
          const int nxt = bp[q].y;   // asked for before the mark's answer is in: one round trip per step, not two
          atomicMin(&s_pos, q);
          if (atomicOr(&mark[r >> 5], bit) & bit) break;
          q = nxt;
        }
      }
    }
    if (lane == 0) atomicAdd(&s_done, 1);   // (the wave is through with its tokens)
  }
  __syncthreads();
  if (lds_marks) {
    for (int i = tid; i < W; i += kCompactBlock) mark[i] = s_mark[i];
    __syncthreads();
  }
  // the links of the marked records (noted here, by all threads, rather than by the walks: the long walk is one
  // lane's chain of dependent loads and should wait for nothing else).  One bitmap word per thread: few bits
  // are set, and a word's records are asked for four at a time.
  for (int w = tid; w < W; w += kCompactBlock) {
    uint32_t m = ld_agent_u32(&mark[w]);
    while (m) {
      int r[4], u[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        r[k] = -1;
        if (m) { r[k] = (w << 5) + __builtin_ctz(m); m &= m - 1u; }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) u[k] = bp[g0 + (r[k] < 0 ? 0 : r[k])].y;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (r[k] >= 0) compact_note_link(cross, u[k] < g0 ? -1 : u[k] - g0, r[k]);
    }
  }
  __syncthreads();
  // how many marked records precede each bitmap word; how many marked links cross each place
  int carry = 0, run = 0;
  for (int base = 0; base < W || base < B + 1; base += kCompactBlock) {
    const int w = base + tid;
    int excl;
    const int cnt = w < W ? __popc(ld_agent_u32(&mark[w])) : 0;
    const int total = compact_block_scan(cnt, excl, s_tot, lane, wave);
    if (w < W) prefix[w] = (uint32_t)(carry + excl);
    carry += total;
    const int step = w <= B ? __hip_atomic_load(&cross[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    const int total2 = compact_block_scan(step, excl, s_tot, lane, wave);
    if (w <= B && run + excl + step == 1) atomicMax(&s_cut, w);   // exactly one link crosses place w
    run += total2;
  }
  __syncthreads();
  const int n_keep = carry;
  const int new_fb = g0 + n_keep;
  // marked records below the highest place that a single link crosses: the new part of the shared beginning
  const int cut = s_cut;
  int n_fixed = cut < 0 ? 0 : (cut < W ? (int)ld_agent_u32(&prefix[cut]) : n_keep);
  // The new part of the shared beginning will be written out in time order: that takes its uppermost record, the
  // lower end of the one link that crosses the cut.  (Record 0, the start token's, carries no arc.)
  const int n_new_arcs = n_fixed - (g0 == 0 && n_fixed > 0 ? 1 : 0);
  const int nf_arcs = cs->n_fixed_arcs, nf_words = cs->n_fixed_words;
  if (nf_arcs + n_new_arcs > p.fixed_cap) n_fixed = 0;   // (uniform) no room to write it out: leave it for later
  if (n_fixed > 0) {
    const int edge = cut << 5;   // examined records below this one are the new part
    for (int w = cut + tid; w < W; w += kCompactBlock) {
      uint32_t m = ld_agent_u32(&mark[w]);
      while (m) {
        const int r = (w << 5) + __builtin_ctz(m);
        m &= m - 1u;
        const int u = bp[g0 + r].y;
        if (u >= g0 && u - g0 < edge) s_top = u - g0;
      }
    }
    for (int i = tid; i < n_tok && i < n_cur; i += kCompactBlock) {
      if (!(tc[i] < __builtin_inff())) continue;
      const int u = bp[fb + i].y;
      if (u >= g0 && u < fb && u - g0 < edge) s_top = u - g0;
    }
    __syncthreads();
    if (s_top < 0) n_fixed = 0;   // (uniform; cannot happen while the marked records below the cut are one chain)
  }
  if (n_keep < young) {   // (uniform) something to drop
    // Move the kept records down.  Few records are kept, so the bitmap is taken a word per thread, 1024 words at
    // a time; each thread brings its word's records (with their predecessors renumbered) to LDS, in the order
    // they will have, and the workgroup writes them out together.  A record never moves up: what is written lies
    // below every record that is still to be read.  (More than kCompactStage kept records in one stretch of 1024
    // words take several passes over it.)
    for (int w0 = 0; w0 < W; w0 += kCompactBlock) {
      const int w = w0 + tid;
      const uint32_t m0 = w < W ? ld_agent_u32(&mark[w]) : 0u;
      const int first = w < W ? (int)ld_agent_u32(&prefix[w]) : 0;   // the new place (above g0) of the word's first record
      const int t_lo = (int)ld_agent_u32(&prefix[w0]);
      const int t_hi = w0 + kCompactBlock < W ? (int)ld_agent_u32(&prefix[w0 + kCompactBlock]) : n_keep;
      for (int lo = t_lo; lo < t_hi; lo += kCompactStage) {   // (uniform)
        uint32_t m = m0;
        int k = first;
        while (m) {
          const int r = (w << 5) + __builtin_ctz(m);
          m &= m - 1u;
          if (k >= lo && k < lo + kCompactStage) {
            int2 rec = bp[g0 + r];
            rec.y = compact_remap(rec.y, g0, fb, new_fb, mark, prefix);
            s_stage[k - lo] = rec;
          }
          ++k;
        }
        __syncthreads();
        const int n_out = t_hi - lo < kCompactStage ? t_hi - lo : kCompactStage;
        for (int j = tid; j < n_out; j += kCompactBlock) bp[g0 + lo + j] = s_stage[j];
        __syncthreads();
      }
    }
    constexpr int kTile = kCompactBlock * kCompactPerThread;
    __syncthreads();
    // ... then the current frame's records, in the same way
    for (int base = 0; base < n_cur; base += kTile) {
      int2 rec[kCompactPerThread];
#pragma unroll
      for (int k = 0; k < kCompactPerThread; ++k) {
        const int i = base + k * kCompactBlock + tid;
        rec[k] = make_int2(0, 0);
        if (i < n_cur) {
          rec[k] = bp[fb + i];
          rec[k].y = compact_remap(rec[k].y, g0, fb, new_fb, mark, prefix);
        }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < kCompactPerThread; ++k) {
        const int i = base + k * kCompactBlock + tid;
        if (i < n_cur) bp[new_fb + i] = rec[k];
      }
    }
  }
  __syncthreads();   // every wave is done with the channel's old numbers
  int nw_new = 0;
  bool wrote = true;
  // The new part of the shared beginning now lies in records [g0, g0 + n_fixed).  Lane 0 follows it down from its
  // uppermost record and writes the arcs where they belong in time order; the wave then adds the word labels and
  // turns the arcs into the caller's numbers.  The walk runs in LDS where the stretch fits there.
  const bool staged = n_fixed > 0 && n_fixed <= kCompactStage;
  if (staged && n_new_arcs > 0) {
    for (int j = tid; j < n_fixed; j += kCompactBlock) {
      const unsigned long long e = __hip_atomic_load((const unsigned long long *)&bp[g0 + j], __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
      s_stage[j] = make_int2((int)(uint32_t)e, (int)(uint32_t)(e >> 32));
    }
    __syncthreads();
  }
  if (n_fixed > 0 && n_new_arcs > 0 && tid < 64) {
    int32_t *fa = p.fixed_arcs + (size_t)c * p.fixed_cap + nf_arcs;
    int32_t *fw = p.fixed_words + (size_t)c * p.fixed_cap + nf_words;
    if (lane == 0) {
      int r = compact_remap(g0 + s_top, g0, fb, new_fb, mark, prefix);
      int k = 0;
      if (staged) {   // (two loops: the one in LDS should not inherit the other's waits for device memory)
        while (r >= g0 && r < g0 + n_fixed && k < n_new_arcs) {
          const int2 e = s_stage[r - g0];
          if ((uint32_t)e.x != kArcNone) fa[n_new_arcs - 1 - k++] = e.x;
          r = e.y;
        }
      } else {
        while (r >= g0 && r < g0 + n_fixed && k < n_new_arcs) {
          const unsigned long long v = __hip_atomic_load((const unsigned long long *)&bp[r], __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
          if ((uint32_t)v != kArcNone) fa[n_new_arcs - 1 - k++] = (int)(uint32_t)v;
          r = (int)(uint32_t)(v >> 32);
        }
      }
      wrote = k == n_new_arcs;   // else the records were not the chain they should be: nothing is declared fixed
    }
    wrote = __shfl((int)wrote, 0, 64) != 0;
    __threadfence_block();
    for (int j0 = 0; j0 < n_new_arcs; j0 += 64) {
      const int j = j0 + lane;
      int w = 0, a = 0;
      if (j < n_new_arcs && wrote) {
        a = fa[j];
        w = p.olabel[a];
      }
      const unsigned long long wm = __ballot(w != 0);
      if (w != 0) fw[nw_new + __popcll(wm & ((1ull << lane) - 1ull))] = w;
      nw_new += __popcll(wm);
      if (j < n_new_arcs && wrote) fa[j] = p.int2pub[a];
    }
  }
  if (tid == 0) {
    cs->frame_base = new_fb;
    cs->n_rec = new_fb + n_cur;
    cs->gc_runs += 1;
    cs->gc_dropped += young - n_keep;
    if (n_fixed > 0 && wrote) {
      cs->gc_base = g0 + n_fixed;
      cs->n_fixed_arcs = nf_arcs + n_new_arcs;
      cs->n_fixed_words = nf_words + nw_new;
    }
  }
}

}  // namespace cbd
#include "cbd_team.hpp"
