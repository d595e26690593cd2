// The lean frame: the same frame as run_frame() computes (same table, same records, same counters), for frames
// whose tables fit LDS, over rows of ordinary length and closure lists stored with the graph.  What it leaves
// out is dependent waiting and per-wave bookkeeping:
//   - the emit phase reads the tokens' rows from LDS and one arc record per lane from device memory; every
//     wave posts its minimum, one barrier, and the frame's cutoff m is final before anything reaches the table
//     (so nothing is ever marked dead afterwards).  A wave holds 128 candidates in registers; what a heavy frame
//     has beyond that counts for the minimum before the barrier and is computed again after it;
//   - the epsilon closure of a state is one contiguous list stored with the graph (depth-first, parents first,
//     each record naming its parent's position).  The lists behind a wave's committed candidates are spread
//     over its lanes, one record per lane: one read for all of them, costs handed down the lists' trees level
//     by level, one table update for all.  A list is walked for every candidate that passes the cutoff, whether
//     or not it lowered its state: a walk from a value that is not the state's final one only produces
//     candidates that the walk from the final value dominates (fp32 addition is monotone), so the fixed point
//     is the one of paper Sec. 3.2's expansion;
//   - no change log shared by the workgroup and no counter atomics: every wave logs its own commits (8 bytes
//     each) and, after the second barrier, looks up which of them is its state's value ("the winner writes" the
//     token and its back-pointer record); token indices are wave-local ordinals, made dense by a prefix sum
//     over the waves' counts.
// Whatever does not fit (a tile with more than 256 arcs, a hub row, a closure without stored list, a full table
// or log) sets Shared::redo (before the first barrier) or Shared::redo_b (between the barriers); each is read by
// all waves after the barrier that follows, and the frame is then decoded again by run_frame(), which handles
// everything.
#pragma once

namespace cbd {

// Diagnostic build only (-DCBD_PROFILE): thread 0 stamps the phases of every lean frame with the 100 MHz counter
// and the sums go out through ChanState::spare.
#ifdef CBD_PROFILE
#define CBD_STAMP(k)                                                                                     \
  do {                                                                                                   \
    if (threadIdx.x == 0) { const long long t_ = wall_clock64(); sh->prof[k] += t_ - sh->prof_last; sh->prof_last = t_; } \
  } while (0)
// why a lean frame is given back: 0 closure stage over 64 records, 1 commit log full, 2 too many tokens, 3 other
#define CBD_WHY(k) atomicAdd(&sh->prof_why[k], 1)
#else
#define CBD_STAMP(k) do {} while (0)
#define CBD_WHY(k) do {} while (0)
#endif

constexpr uint16_t kLeanDegEscape = 0xFFFF;   // t_deg: the row is too long for the lean code
constexpr int kLeanLidBits = 10;              // a wave-local token id: wave << 10 | ordinal within the wave
constexpr int kLeanLidMask = (1 << kLeanLidBits) - 1;

// One commit as its wave logged it: slot h took (some cost, arc).  from: where the arc started, a token of the
// previous frame (kLeanFromToken set: an emitting arc) or a table slot of this frame (an epsilon-input arc).
struct __attribute__((aligned(8))) LeanLog {
  uint32_t arc;
  uint16_t h;
  uint16_t from;
};
constexpr uint16_t kLeanFromToken = 0x8000;

// The tokens' rows and the commit logs live where the general code keeps its change log.
struct LeanMem {
  int32_t *t_first;    // [tok_cap] first emitting arc of each current token's state
  uint16_t *t_deg;     // [tok_cap] number of emitting arcs
  int32_t *hrow;       // [slots] the same for the states in the table, written by whoever creates the entry
  uint8_t *hed;        // [slots]  (kLeanEdEscape: the row is too long for the lean code)
  LeanLog *clog;       // [waves][clog_per_wave]
  int clog_per_wave;
};
constexpr uint8_t kLeanEdEscape = 0xFF;

constexpr int kLeanLogPerWave = 256;   // commits a wave can log per frame (more: the frame goes to the general code)
constexpr int kLeanLogEntryBytes = 8;

__device__ __forceinline__ LeanMem make_lean_mem(void *log_region, int tok_cap, int slots, int log_per_wave) {
  LeanMem R;
  unsigned char *b = (unsigned char *)log_region;
  R.t_first = (int32_t *)b;
  R.t_deg = (uint16_t *)(b + (size_t)tok_cap * 4);
  b += align_up((uint32_t)tok_cap * 6u, 16u);
  R.hrow = (int32_t *)b;
  R.hed = (uint8_t *)(b + (size_t)slots * 4);
  b += align_up((uint32_t)slots * 5u, 16u);
  R.clog = (LeanLog *)b;
  R.clog_per_wave = log_per_wave;
  return R;
}

// table slot of a state: home slot first, then linear probing (same function as table_min)
__device__ __forceinline__ uint32_t lean_home(uint32_t state, uint32_t slots) {
  return __umulhi(state * 2654435761u, slots);
}

// Finds or creates the slot of `state` after a collision at its home slot.  Returns false if the table is full.
__device__ __forceinline__ bool lean_probe(const Mem<true> &M, uint32_t state, uint32_t &h, uint32_t &k) {
  uint32_t probe = 1;
  do {
    h = h + 1 == M.slots ? 0 : h + 1;
    k = atomicCAS(&M.hkey[h], kEmptyKey, state);
  } while (k != kEmptyKey && k != state && ++probe < M.slots);
  return k == kEmptyKey || k == state;
}

// A tile: up to 64 tokens of the previous frame, one per lane, and the list of their emitting arcs.
struct LeanTile {
  float cost;     // this lane's token
  int rel;        // first arc of its row minus the row's position in the arc list
  int base;       // index of lane 0's token
  int total;      // arcs in the list (uniform)
};

// Loads tile `st` of this wave (tokens tile0 + st * 64 + lane, below tile_end), prunes (step 1), and writes the
// heads of its arc list into omap: the owner of a list position is the last head at or before it.
__device__ __forceinline__ LeanTile lean_load_tile(const AdvanceParams &p, const Mem<true> &M, const LeanMem &R,
                                                   Shared *sh, uint8_t *omap, int tile0, int tile_end, int st, int lane,
                                                   float best, int cut, float inv, uint32_t &n_active) {
  LeanTile T;
  T.base = tile0 + st * 64;
  const int i = T.base + lane;
  bool alive = false;
  T.cost = 0.0f;
  int first = 0, deg = 0;
  if (i < tile_end) {
    T.cost = M.t_cost[i];
    const float r = T.cost - best;
    alive = !(r > p.beam) && T.cost < __builtin_inff();
    if (alive && cut < 255) {
      int bin = (int)floorf(r * inv);
      bin = bin > 255 ? 255 : bin;
      alive = bin <= cut;
    }
    if (alive) { first = R.t_first[i]; deg = (int)R.t_deg[i]; }
  }
  if (deg == (int)kLeanDegEscape) { sh->redo = 1; deg = 0; CBD_WHY(3); }
  const int incl = wave_incl_scan(deg);
  const int pos = incl - deg;
  T.total = __builtin_amdgcn_readlane(incl, 63);
  if (T.total > kOwnerMap) { if (lane == 0) { sh->redo = 1; CBD_WHY(3); } T.total = 0; }
  ((uint32_t *)omap)[lane] = 0;
  if (deg > 0 && pos < kOwnerMap) omap[pos] = (uint8_t)(lane + 1);
  T.rel = first - pos;
  n_active += (uint32_t)__popcll(__ballot(alive));
  return T;
}

// One emitting candidate per lane and slot: two slots, list positions jb + lane and jb + 64 + lane.
struct LeanEmit {
  float cand[2];
  int arc[2];
  ArcRec rec[2];
  int src[2];      // token (index in the previous frame's list) the arc leaves from
  bool act[2];
};

// Candidates of list positions [jb, jb + 128) of tile T (jb a multiple of 128).  Returns the minimum (orderable
// bits) over the candidates computed.
template <bool kRowFromLds>
__device__ __forceinline__ uint32_t lean_candidates(const AdvanceParams &p, const Ctx &cx, const Rows &Lrow,
                                                    const uint8_t *omap, int jb, int lane, const LeanTile &T,
                                                    LeanEmit &E) {
  uint32_t lmin = 0xFFFFFFFFu;
  // owner + 1 of the last position before jb
  int carry = 0;
  for (int b = 0; b < jb; b += 64) {   // (uniform; only beyond the first 128 arcs of a tile)
    const int t = __builtin_amdgcn_readlane(wave_incl_scan_max((int)omap[b + lane]), 63);
    carry = t > carry ? t : carry;
  }
  // both slots' arc records are asked for before either is used (one wait for both)
  float c_own[2] = {0.0f, 0.0f};
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int j0 = jb + q * 64, j = j0 + lane;
    E.act[q] = j < T.total;
    E.cand[q] = 0.0f; E.arc[q] = 0; E.src[q] = 0;
    E.rec[q].dst = 0; E.rec[q].weight = 0.0f; E.rec[q].row = 0; E.rec[q].meta = 0;
    if (j0 < T.total) {   // uniform
      // the lane that owns position j: the last head at or before j (heads carry lane + 1)
      int own1 = wave_incl_scan_max((int)omap[j]);
      own1 = own1 > carry ? own1 : carry;
      carry = __builtin_amdgcn_readlane(own1, 63);
      const int owner = own1 - 1;
      E.arc[q] = __shfl(T.rel, owner, 64) + j;
      c_own[q] = __shfl(T.cost, owner, 64);
      E.src[q] = T.base + owner;
      if (E.act[q]) E.rec[q] = p.arcs[E.arc[q]];
    }
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (jb + q * 64 < T.total && E.act[q]) {
      float w = E.rec[q].weight;
      if (ctx_contains(cx, E.arc[q])) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
      const uint32_t pdf = (E.rec[q].meta & 0xFFFFu) - 1u;
      const float ll = kRowFromLds ? Lrow.at(pdf) : Lrow.glob[pdf];
      E.cand[q] = (c_own[q] + w) - ll;
      const uint32_t o = f2ord(E.cand[q]);
      lmin = o < lmin ? o : lmin;
    }
  }
  return lmin;
}

// Per-wave running state of the commit phase.
struct LeanWave {
  int n_claimed;     // states this wave created so far (uniform)
  int n_clog;        // commits it logged (uniform)
  uint32_t n_cand, n_eps;
  int max_depth;
};

// Copies a log-likelihood row from device memory into LDS without passing through registers: every wave asks for
// 1 KB pieces (16 bytes per lane) that the memory pipeline writes straight into LDS.  The caller waits for its own
// requests (vmcnt) and passes a barrier before anyone reads the row.  Rows whose size or address is not a
// multiple of 16 bytes go 4 bytes per lane.
template <int kBlock>
__device__ __forceinline__ void stage_row_async(float *lds_row, const float *row, int num_pdfs, int wave, int lane) {
  constexpr int NW = kBlock / 64;
  typedef const __attribute__((address_space(1))) void *gptr;
  typedef __attribute__((address_space(3))) void *lptr;
  if ((num_pdfs & 3) == 0 && (((unsigned long long)row) & 15ull) == 0) {
    for (int base = wave * 256; base < num_pdfs; base += NW * 256) {   // uniform
      const int i = base + lane * 4;
      if (i < num_pdfs)
        __builtin_amdgcn_global_load_lds((gptr)(row + i), (lptr)(lds_row + base), 16, 0, 0);
    }
  } else {
    for (int base = wave * 64; base < num_pdfs; base += NW * 64) {
      const int i = base + lane;
      if (i < num_pdfs)
        __builtin_amdgcn_global_load_lds((gptr)(row + i), (lptr)(lds_row + base), 4, 0, 0);
    }
  }
}

// Asks for the table slot of `state` for lanes with ok set: h, and k = what the slot held before (kEmptyKey: this
// lane created the entry).
__device__ __forceinline__ void lean_slot(const Mem<true> &M, bool ok, uint32_t state, uint32_t &h, uint32_t &k) {
  k = 0; h = 0;
  if (ok) {
    h = lean_home(state, M.slots);
    k = atomicCAS(&M.hkey[h], kEmptyKey, state);
  }
}
// After a collision at the home slot: walks on.  Clears ok and sets sh->redo_b if the table is full.
__device__ __forceinline__ void lean_slot_collisions(const Mem<true> &M, Shared *sh, bool &ok, uint32_t state,
                                                     uint32_t &h, uint32_t &k) {
  const bool collided = ok && k != kEmptyKey && k != state;
  if (__ballot(collided) != 0) {   // rare
    if (collided && !lean_probe(M, state, h, k)) { sh->redo_b = 1; ok = false; CBD_WHY(3); }
  }
}

// E[state] = min key for lanes with ok set (slot h, previous holder k from lean_slot), the token's wave-local id
// and the state's row if the lane created the entry, and the log entry for the look-up after the barrier.
// Returns whether this lane created the entry.
__device__ __forceinline__ bool lean_min_and_log(const Mem<true> &M, const LeanMem &R, Shared *sh, bool ok, uint32_t h,
                                                 uint32_t k, uint64_t key, const ArcRec &rec, uint32_t from, int wave,
                                                 int lane, LeanWave &W) {
  if (ok) atomicMin((unsigned long long *)&M.hval[h], (unsigned long long)key);
  const bool claimed = ok && k == kEmptyKey;
  const unsigned long long om = __ballot(ok);
  const unsigned long long cm = __ballot(claimed);
  const unsigned long long below = (1ull << lane) - 1ull;
  if (claimed) {
    // this lane created the state's entry: it names the token (wave-local id, made dense after the barrier) and
    // files the state's row, which the next frame expands
    const int ord = W.n_claimed + __popcll(cm & below);
    if (ord <= kLeanLidMask) M.hidx[h] = (uint16_t)((wave << kLeanLidBits) | ord);
    else { sh->redo_b = 1; CBD_WHY(3); }
    const uint32_t ed = meta_ed(rec.meta);
    R.hrow[h] = rec.row;
    R.hed[h] = ed == kEdEscape ? kLeanEdEscape : (uint8_t)ed;
  }
  if (ok) {
    const int e = W.n_clog + __popcll(om & below);
    if (e < R.clog_per_wave) {
      LeanLog le;
      le.arc = (uint32_t)key; le.h = (uint16_t)h; le.from = (uint16_t)from;
      (R.clog + (size_t)wave * R.clog_per_wave)[e] = le;
    } else {
      sh->redo_b = 1;
      CBD_WHY(1);
    }
  }
  W.n_claimed += __popcll(cm);
  W.n_clog += __popcll(om);
  return claimed;
}

// The closure stage, first half.  A lane may bring up to two lists: the stored closure lists of the states it is
// committing candidates to (len[q] records from pos[q]; root[q]: the candidate's cost).  The records of all the
// wave's lists are spread over the lanes, one record per lane, and asked for with one read.
struct LeanClosure {
  int total;        // records (uniform); 0: nothing to do
  bool act, second; // this lane holds a record; it is of its owner's second list
  int owner;        // the lane whose list it belongs to
  int plane;        // the lane before the list's first record (the parent's position is added to it)
  float o_root;     // cost of the candidate the list hangs from
  ArcRec rec;
  int can;
};

__device__ __forceinline__ LeanClosure lean_closure_begin(const AdvanceParams &p, Shared *sh, int lane, uint8_t *cmap,
                                                          const int *pos, const int *len, const float *root) {
  LeanClosure C;
  C.act = false; C.second = false; C.owner = 0; C.plane = 0; C.o_root = 0.0f; C.can = 0;
  C.rec.dst = 0; C.rec.weight = 0.0f; C.rec.row = 0; C.rec.meta = 0;
  const int mine = len[0] + len[1];
  const int incl = wave_incl_scan(mine);
  C.total = __builtin_amdgcn_readlane(incl, 63);
  if (C.total == 0) return C;   // uniform
  if (C.total > 64) {           // (rare: the general code takes the frame)
    if (lane == 0) { sh->redo_b = 1; CBD_WHY(0); }
    C.total = 0;
    return C;
  }
  const int start = incl - mine;
  // which lane's lists a record belongs to: the last head at or before its position
  if (lane < 16) ((uint32_t *)cmap)[lane] = 0;
  if (mine > 0) cmap[start] = (uint8_t)(lane + 1);
  C.owner = wave_incl_scan_max((int)cmap[lane]) - 1;   // (position 0 is a head)
  C.act = lane < C.total;
  const int o_start = __shfl(start, C.owner, 64);
  const int o_len0 = __shfl(len[0], C.owner, 64);
  const int kk = lane - o_start;                 // position among the owner's records
  C.second = kk >= o_len0;
  const int o_pos0 = __shfl(pos[0], C.owner, 64);
  const int o_pos1 = __shfl(pos[1] - len[0], C.owner, 64);
  const int rpos = (C.second ? o_pos1 : o_pos0) + kk;
  if (C.act) { C.rec = p.arcs[rpos]; C.can = p.canon[rpos]; }
  const float o_root0 = __shfl(root[0], C.owner, 64), o_root1 = __shfl(root[1], C.owner, 64);
  C.o_root = C.second ? o_root1 : o_root0;
  C.plane = o_start + (C.second ? o_len0 : 0) - 1;
  return C;
}

// Second half: costs follow the lists' trees level by level (a record names its parent's position), a dropped
// record drops its subtree, and everything that passes is committed in one go.  root_h: the slots of the states
// this lane's lists hang from.
__device__ __forceinline__ void lean_closure_end(const AdvanceParams &p, const Mem<true> &M, const LeanMem &R,
                                                 Shared *sh, const Ctx &cx, float m, int wave, int lane, LeanWave &W,
                                                 const LeanClosure &C, const uint32_t *root_h) {
  if (C.total == 0) return;   // uniform
  const uint32_t o_hh = (uint32_t)__shfl((int)(root_h[0] | (root_h[1] << 16)), C.owner, 64);
  const uint32_t o_h = C.second ? o_hh >> 16 : o_hh & 0xFFFFu;
  W.n_eps += (uint32_t)C.total;
  const ArcRec &rec = C.rec;
  const int depth = C.act ? (int)(rec.meta & 0xFu) : 0;   // 1..kClosureMaxDepth
  const int plane = (C.plane + (int)((rec.meta >> 4) & 0x3Fu)) & 63;   // the lane that holds the parent record
  float w = rec.weight;
  if (C.act && ctx_contains(cx, C.can)) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
  const float beam = p.beam;
  float c = __builtin_inff();
  bool ok = false;
  if (depth == 1) {
    const float cc = C.o_root + w;
    ok = cc < __builtin_inff() && !(cc - m > beam);
    if (ok) c = cc;
  }
  const int maxd = __builtin_amdgcn_readlane(wave_incl_scan_max(depth), 63);
  for (int d = 2; d <= maxd; ++d) {   // uniform
    const float pc = __shfl(c, plane, 64);
    if (depth == d) {
      const float cc = pc + w;
      ok = cc < __builtin_inff() && !(cc - m > beam);
      if (ok) c = cc;
    }
  }
  W.max_depth = max(W.max_depth, maxd);
  const unsigned long long om = __ballot(ok);
  if (om == 0) return;
  W.n_cand += (uint32_t)__popcll(om);
  const uint32_t co = ok ? f2ord(c) : 0xFFFFFFFFu;
  if (__ballot(ok && co < f2ord(m)) != 0) {
    // the frame's minimum is min(m, closure candidates): only a candidate below m can move it
    const uint32_t wmin = wave_min_u32(co);
    if (lane == 0) atomicMin(&sh->best_ord, wmin);
  }
  uint32_t h, k;
  lean_slot(M, ok, (uint32_t)rec.dst, h, k);
  lean_slot_collisions(M, sh, ok, (uint32_t)rec.dst, h, k);
  // the source state's slot: the list's state, or the parent record's (found a moment ago by its lane)
  const uint32_t ph = (uint32_t)__shfl((int)h, plane, 64);
  lean_min_and_log(M, R, sh, ok, h, k, ((uint64_t)co << 32) | (uint32_t)C.can, rec, depth == 1 ? o_h : ph, wave, lane,
                   W);
}

// Commits the emitting candidates in E (the cutoff m is final) and walks the closure lists behind them.  The
// steps are ordered so that waits overlap: the table slots are asked for, then the closure records, and only
// then are the slots looked at.
__device__ __forceinline__ void lean_commit(const AdvanceParams &p, const Mem<true> &M, const LeanMem &R, Shared *sh,
                                            const Ctx &cx, float m, int wave, int lane, LeanWave &W, uint8_t *cmap,
                                            const LeanEmit &E) {
  bool pass[2];
  uint32_t h[2], k[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) pass[q] = E.act[q] && !(E.cand[q] - m > p.beam);
  if (__ballot(pass[0] || pass[1]) == 0) return;   // uniform
#pragma unroll
  for (int q = 0; q < 2; ++q) lean_slot(M, pass[q], (uint32_t)E.rec[q].dst, h[q], k[q]);
  // the closure lists of the destinations
  int pos[2] = {0, 0}, len[2] = {0, 0};
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const uint32_t cl = meta_cl(E.rec[q].meta);
    if (pass[q] && cl > 0) {
      if (cl == kClEscape) {
        sh->redo_b = 1;   // no stored list: the general code follows this closure
        CBD_WHY(3);
      } else {
        pos[q] = E.rec[q].row + (int)meta_ed(E.rec[q].meta) + (int)meta_xd(E.rec[q].meta);
        len[q] = (int)cl;
      }
    }
  }
  const LeanClosure C = lean_closure_begin(p, sh, lane, cmap, pos, len, E.cand);
  CBD_STAMP(6);   // (diagnostic: cutoff, slot requests, closure records requested)
  // now the emitting candidates' slots
#pragma unroll
  for (int q = 0; q < 2; ++q) lean_slot_collisions(M, sh, pass[q], (uint32_t)E.rec[q].dst, h[q], k[q]);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (__ballot(pass[q]) == 0) continue;   // uniform
    W.n_cand += (uint32_t)__popcll(__ballot(pass[q]));
    const uint64_t key = ((uint64_t)f2ord(E.cand[q]) << 32) | (uint32_t)E.arc[q];
    lean_min_and_log(M, R, sh, pass[q], h[q], k[q], key, E.rec[q], (uint32_t)E.src[q] | kLeanFromToken, wave, lane, W);
  }
  CBD_STAMP(7);   // (diagnostic: emitting candidates committed)
  lean_closure_end(p, M, R, sh, cx, m, wave, lane, W, C, h);
  CBD_STAMP(8);   // (diagnostic: closure records committed)
}

// One frame by the lean code.  Returns kFrameOk, kFrameNoTokens, kFrameRecordsFull, or kFrameRedo (then nothing
// that outlives the frame has been written, but the state table holds entries and the staged log-likelihood
// row may already be the next frame's: the caller cleans up and runs the general code).
template <int kBlock>
__device__ __forceinline__ int run_frame_lean(const AdvanceParams &p, const Mem<true> &M, const LeanMem &R, Shared *sh,
                                              const Ctx &cx, float *Lstage, const Rows &Lrow, const float *Lnext,
                                              uint32_t *hist, uint8_t *owner_maps, uint8_t *closure_maps, int row_buf,
                                              int2 *bp, int32_t *g_tok_state, bool last_frame) {
  constexpr int NW = kBlock / 64;
  static_assert(NW <= 16, "Shared::wcount holds 16 waves");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#ifdef CBD_PROFILE
  if (tid == 0) sh->prof_last = wall_clock64();
#endif
  const bool hist_on = p.max_active > 0 && p.beam > 0.0f && p.beam < __builtin_inff();
  const float inv = 256.0f / p.beam;
  uint8_t *omap = owner_maps + wave * kOwnerMap;
  uint8_t *cmap = closure_maps + wave * 64;

  // ---- emit: prune (step 1), expand (step 2).  The wave's share of the tokens is taken in tiles of 64, a tile's
  // arcs 128 at a time; tile 0's first 128 come last and stay in registers.
  const int n_tok = sh->n_tok;
  const float best = sh->best;
  const int cut = sh->cut_bin;
  const int tpw = (n_tok + NW - 1) / NW;
  const int tile0 = wave * tpw;
  const int tile_end = min(tile0 + tpw, n_tok);
  const int n_tiles = (tpw + 63) >> 6;   // (uniform over the workgroup)
  uint32_t n_active = 0, n_emit = 0;
  uint32_t lmin = 0xFFFFFFFFu;
  LeanEmit E;
  LeanTile T;
  for (int st = n_tiles - 1; st >= 0; --st) {
    T = lean_load_tile(p, M, R, sh, omap, tile0, tile_end, st, lane, best, cut, inv, n_active);
    n_emit += (uint32_t)T.total;
    for (int jb = T.total > 0 ? ((T.total - 1) >> 7) << 7 : 0; jb >= 0; jb -= 128) {
      const uint32_t l = lean_candidates<true>(p, cx, Lrow, omap, jb, lane, T, E);
      lmin = l < lmin ? l : lmin;
    }
  }
  const uint32_t n_active_frame = n_active;
  const uint32_t wmin = wave_min_u32(lmin);
  if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->m_ord, wmin);
  CBD_STAMP(0);   // emit phase of wave 0
  wg_barrier<true>();
  CBD_STAMP(1);   // its wait at the first barrier

  // ---- step 3: the emission minimum fixes the frame's cutoff
  const uint32_t m_ord = sh->m_ord;
  if (sh->redo) return kFrameRedo;              // (uniform: set before the barrier, or never)
  if (m_ord == 0xFFFFFFFFu) return kFrameNoTokens;
  const float m = ord2f(m_ord);

  // ---- recombination (step 2, second half) and epsilon closure (step 4): the candidates in registers first,
  // then whatever the tiles hold beyond them, computed again (the staged row may be on its way out by then: these
  // read the row in device memory)
  LeanWave W;
  W.n_claimed = 0; W.n_clog = 0; W.n_cand = 0; W.n_eps = 0; W.max_depth = 0;
  {
    bool have = true;   // E holds tile 0's first 128 candidates
    for (int st = 0; st < n_tiles; ++st) {
      if (st > 0) T = lean_load_tile(p, M, R, sh, omap, tile0, tile_end, st, lane, best, cut, inv, n_active);
      for (int jb = 0; jb == 0 || jb < T.total; jb += 128) {
        if (!have) lean_candidates<false>(p, cx, Lrow, omap, jb, lane, T, E);
        have = false;
        lean_commit(p, M, R, sh, cx, m, wave, lane, W, cmap, E);
      }
    }
  }
  // The emit phase is long over: the next frame's row starts its way.  (Not earlier: loads return in order, and
  // the closure stages' reads would queue behind the row.)
  // A row that is not staged is touched instead, one lane per 64 bytes: the next frame's emit phase then finds it
  // in L2 (the value is asked for again at the end of the frame, so that the read is kept and nothing waits for it).
  float touched = 0.0f;
  if (Lnext) {
    if (Lrow.staged) stage_row_async<kBlock>(Lstage, Lnext, p.num_pdfs, wave, lane);
    else if (tid * 16 < p.num_pdfs) touched = Lnext[tid * 16];
  }
  if (lane == 0) sh->wcount[wave] = W.n_claimed;
  CBD_STAMP(2);   // commit phase of wave 0
  wg_barrier<true>();
  CBD_STAMP(3);   // its wait at the second barrier

  // ---- step 5 and bookkeeping: the winner of each state writes the token
  if (sh->redo_b) return kFrameRedo;   // (uniform: set between the two barriers, or never)
  // dense token indices: prefix sums over the waves' counts (every wave computes the same numbers)
  int n_claim;
  {
    const int c = lane < NW ? sh->wcount[lane] : 0;
    const int inc = wave_incl_scan(c);
    n_claim = __builtin_amdgcn_readlane(inc, 63);
    if (lane < NW) sh->wbase[lane] = inc - c;
  }
  if (n_claim > M.tok_cap) {   // (the general code decides what an overflow means)
    if (tid == 0) CBD_WHY(2);
    return kFrameRedo;
  }
  if (sh->n_rec + n_claim > p.bp_cap) return kFrameRecordsFull;
  const bool hist_need = hist_on && n_claim > p.max_active;
  const float fbest = ord2f(umin32(m_ord, sh->best_ord));
  const int base_cur = sh->n_rec, base_prev = sh->frame_base;
  int4 *hbm_rows = M.t_row + (size_t)row_buf * M.row_cap;
  int w_surv = 0;
  // Every commit of this wave is in its log.  A state's value names its arc, so the entry whose arc is the
  // state's value is the winner and writes the token: cost, row, back-pointer record, state (last frame),
  // histogram.  An emitting arc is expanded once per frame, so its entry is unique; a closure record can have
  // been committed twice with the same (cost, arc) (two walks of one list from values that round to the same
  // sum): the compare-and-swap lets one of the two write.
  {
    const LeanLog *clog = R.clog + (size_t)wave * R.clog_per_wave;
    for (int j0 = 0; j0 < W.n_clog; j0 += 64) {
      const int j = j0 + lane;
      bool surv = false;
      if (j < W.n_clog) {
        const LeanLog e = clog[j];
        // everything the winner will need is asked for together: the state's value, row and token id, the source
        // state's token id, and the waves' bases
        const uint64_t v = M.hval[e.h];
        const int row = R.hrow[e.h];
        const uint32_t ed = R.hed[e.h];
        const int lid = (int)M.hidx[e.h];
        const bool from_token = (e.from & kLeanFromToken) != 0;
        const int from = (int)(e.from & (kLeanFromToken - 1));
        const int plid = (int)M.hidx[from_token ? 0 : from];
        const int idx = sh->wbase[(lid >> kLeanLidBits) & 15] + (lid & kLeanLidMask);
        const int pidx = sh->wbase[(plid >> kLeanLidBits) & 15] + (plid & kLeanLidMask);
        bool win = (uint32_t)v == e.arc && v != kEmptyVal;
        if (win && !from_token)
          win = atomicCAS((unsigned long long *)&M.hval[e.h], (unsigned long long)v, (unsigned long long)kEmptyVal) == v;
        if (win) {
          const float c = ord2f((uint32_t)(v >> 32));
          M.t_cost[idx] = c;
          R.t_first[idx] = row;
          R.t_deg[idx] = ed == kLeanEdEscape ? kLeanDegEscape : (uint16_t)ed;
          bp[base_cur + idx] = make_int2((int)e.arc, from_token ? base_prev + from : base_cur + pidx);
          uint32_t state = 0;
          if (last_frame || ed == kLeanEdEscape) state = M.hkey[e.h];
          if (last_frame) g_tok_state[idx] = (int)state;
          if (ed == kLeanEdEscape) {
            // a row too long for the count field (rare): its bounds go to the row buffer in device memory, where
            // the general code, which will take the next frame, looks for them
            const int4 o = p.off2[state];
            hbm_rows[idx] = make_int4(o.x, o.y, o.z, 0);
          }
          M.hkey[e.h] = kEmptyKey;
          if (from_token) M.hval[e.h] = kEmptyVal;
          if (hist_need) {
            const float r = c - fbest;
            if (!(r > p.beam)) {
              surv = true;
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              atomicAdd(&hist[bin], 1u);
            }
          }
        }
      }
      if (hist_need) w_surv += __popcll(__ballot(surv));
    }
  }
  // ---- close the frame: the wave that gets here last does it (every wave's LDS traffic of this phase lies
  // before its count, and LDS keeps a wave's operations in order)
  int done = 0;
  if (lane == 0) {
    if (w_surv) atomicAdd(&sh->n_surv, w_surv);
    // (two counters to an atomic; they are taken apart when the call ends)
    atomicAdd(&sh->a_lean_pack[0], (unsigned long long)n_active_frame | ((unsigned long long)n_emit << 32));
    atomicAdd(&sh->a_lean_pack[1], (unsigned long long)W.n_eps | ((unsigned long long)W.n_cand << 32));
    if (W.max_depth) atomicMax(&sh->rounds, W.max_depth);
    done = atomicAdd(&sh->n_done, 1);
  }
  CBD_STAMP(4);   // look-up phase of wave 0
  if (__builtin_amdgcn_readfirstlane(done) == NW - 1) {
    int cutb = 255;
    if (hist_need && sh->n_surv > p.max_active) {
      int loc[4], sum = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) { loc[k] = (int)hist[lane * 4 + k]; sum += loc[k]; }
      const int inc = wave_incl_scan(sum);
      int run = inc - sum;
      int myB = -1;
#pragma unroll
      for (int k = 0; k < 4; ++k) { run += loc[k]; if (run <= p.max_active) myB = lane * 4 + k; }
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) { const int t = __shfl_xor(myB, d, 64); myB = t > myB ? t : myB; }
      cutb = myB < 0 ? 0 : myB;
    }
    if (lane == 0) {
      sh->cut_bin = cutb;
      sh->n_tok = n_claim;
      sh->frame_base = sh->n_rec;
      sh->n_rec += n_claim;
      sh->best = fbest;
      atomicAdd(&sh->a_frames, 1ull);
      atomicAdd(&sh->a_tokens, (unsigned long long)n_claim);
      atomicMax(&sh->a_maxtok, n_claim);
      atomicAdd(&sh->a_impr, (unsigned long long)n_claim);
      atomicAdd(&sh->a_rounds, (unsigned long long)sh->rounds);
      sh->a_lean += 1;
    }
    frame_init(sh, hist, false, lane, hist_need);   // for the next frame
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's pieces of the next row have arrived in LDS
  wg_barrier<true>();
  CBD_STAMP(5);   // its wait at the last barrier (with the closing of the frame by the last wave)
  asm volatile("" ::"v"(touched));
  return kFrameOk;
}

}  // namespace cbd
