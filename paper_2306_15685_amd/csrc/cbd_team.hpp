// Dense frames: several workgroups decode one channel together.
//
// Where a frame holds far more tokens than one compute unit's LDS can take (thousands of word starts behind a hub
// state, Sec. 6: graphs of end-to-end units), one workgroup per channel has to keep its state table in device
// memory, and the tables of all channels together do not stay in L2.  Here a TEAM of k workgroups shares the channel:
// the states are split over the team by a hash, each member keeps the table of its share in LDS, and candidates
// travel from the member that expands an arc to the member that owns the arc's destination through queues in
// device memory.  A frame has four phases, separated by barriers across the team:
//
//   1  every member prunes and expands its own tokens (steps 1 and 2 of the frame) and appends each candidate to
//      the queue (owner of the destination, sender); rows with hundreds of arcs are shared out over the team;
//      the team's emission minimum m is taken with one atomic per wave                            -- barrier 1
//   2  owners drop what m cuts off, recombine the rest in their LDS table (E[state] = min key) and walk the stored
//      epsilon closure list of every candidate that passed; closure candidates go to a second set of queues
//                                                                                                  -- barrier 2
//   3  owners recombine the closure candidates, then go through what they received once more: the entry whose arc
//      is the state's value is the winner and writes the token (cost, row, state) and, for an emitting arc, the
//      back-pointer record; tokens of member q live at [q * cap, q * cap + n_q) of the channel's token arrays, so
//      their record numbers are known at once.  Each member publishes (state -> token) of its share  -- barrier 3
//   4  back-pointer records of closure winners (their predecessor is a token of this frame, found in its owner's
//      published table); histogram cut and scalars of the next frame, computed by every member alike.
//
// Results are those of the one-workgroup code bit for bit (the same keys compete for every state); only the numbering
// of tokens and records differs (token arrays and record blocks have unused places between the members' shares).
//
// The barrier is a counter in device memory that every member's thread 0 increments and then polls (agent-scope
// atomics, release / acquire fences around them, a bounded number of polls: a member that waits too long marks the
// channel failed and leaves, and so then do the others).  All members of all teams have to be resident at once:
// the kernel is launched cooperatively and the host refuses more teams than the device has compute units.
#pragma once

namespace cbd {

constexpr int kTeamMax = 8;       // members of a team
constexpr int kTeamBig = 32;      // long rows a frame can share out
constexpr int kTeamSpinLimit = 4 << 20;   // polls of a barrier before a member gives up (seconds)
constexpr int kStatusTeam = -6;   // a member waited too long at a team barrier (reported as a HIP-level failure)

// A candidate on its way to the owner of its destination state.
struct __attribute__((aligned(8))) TeamEntry {
  uint32_t dst;
  float cost;
  uint32_t arc;     // library arc index (closure records: the arc they stand for)
  int32_t from;     // emitting arc: the source token's place in the previous frame; closure: the source STATE
  int32_t row;      // first arc of dst
  uint32_t meta;    // degrees and closure length of dst (ArcRec::meta with the low 16 bits cleared)
};
static_assert(sizeof(TeamEntry) == 24, "queue entries are 24 bytes");

struct TeamClosureWin { int32_t idx; uint32_t arc; uint32_t parent_state; };

// One frame's team-wide scalars (two copies, used by even and odd frames in turn).
struct TeamFrame {
  uint32_t m_ord, best_ord;
  int32_t n_big, pad0;
  int32_t count[kTeamMax];              // tokens each member made
  int32_t qn[kTeamMax][kTeamMax];       // entries of queue [owner][sender], emitting candidates
  int32_t q2n[kTeamMax][kTeamMax];      // the same, closure candidates
  uint32_t hist[256];
  // long rows among this frame's tokens: expanded by the whole team in the next frame
  int32_t big_first[kTeamBig], big_deg[kTeamBig], big_src[kTeamBig];
  float big_cost[kTeamBig];
};

struct __attribute__((aligned(256))) TeamChan {
  uint32_t barrier;        // arrivals at team barriers since the decoder was made
  int32_t status;          // why the channel is parked (sticky until reset)
  int32_t flag[4];         // a failure met before team barrier n is noted in flag[n & 3] and looked for there after
                           // that barrier: a member that is already past it cannot change what a slower one reads
  int32_t partitioned;     // 0: the token list is the dense one a reset leaves; 1: members' shares
  int32_t ntok[kTeamMax];  // tokens of each member's share
  int32_t carry_n;         // long rows found in the last frame of the previous call
  int32_t carry_first[kTeamBig], carry_deg[kTeamBig], carry_src[kTeamBig];
  float carry_cost[kTeamBig];
  TeamFrame fr[2];
};

struct TeamParams {
  AdvanceParams a;
  TeamChan *team;          // [C]
  TeamEntry *q1, *q2;      // [C][k][k][q_cap]
  TeamClosureWin *cwin;    // [C][k][part_cap]
  uint32_t *pub_key;       // [C][k][slots] each member's table keys as of the end of phase 3
  uint16_t *pub_lid;       // [C][k][slots] and the tokens they name
  int32_t k;               // members per team
  int32_t q_cap;
  int32_t part_cap;        // tokens per member and frame
  int32_t slots;           // table slots per member (LDS)
  int32_t stage_rows;      // the frame's log-likelihood row is copied to LDS
  int32_t ctx_lds_cap;
};

struct TeamLayout { uint32_t sh, hist, bitmap, ctx, L, hval, hkey, hidx, total; };
struct TeamShared {
  int32_t abort_flag, fault, failed;
  int32_t n_mine;            // tokens this member has made in the current frame
  int32_t n_cwin;            // closure winners noted for phase 4
  int32_t cnt1[kTeamMax], cnt2[kTeamMax];   // entries pushed to each owner's queues
  uint32_t m_ord, best_ord;  // this member's minima before they go to the team
  int32_t n_big;             // long rows met unannounced in this member's own tokens
  int32_t big_first[kBigRows], big_deg[kBigRows], big_src[kBigRows];
  float big_cost[kBigRows];
  int32_t cut_bin, n_surv;
  unsigned long long a_active, a_emit, a_eps, a_cand;
};

__host__ __device__ inline TeamLayout team_layout(int num_pdfs_staged, int ctx_lds_cap, int slots) {
  TeamLayout l;
  uint32_t o = 0;
  l.sh = o; o += align_up((uint32_t)sizeof(TeamShared), 16);
  l.hist = o; o += 256 * 4;
  l.bitmap = o; o += kBloomWords * 4;
  l.ctx = o; o += align_up((uint32_t)ctx_lds_cap * 4, 16);
  l.L = o; o += align_up((uint32_t)num_pdfs_staged * 4, 16);
  l.hval = o; o += (uint32_t)slots * 8;
  l.hkey = o; o += (uint32_t)slots * 4;
  l.hidx = o; o += align_up((uint32_t)slots * 2, 16);
  l.total = o;
  return l;
}

__device__ __forceinline__ uint32_t team_hash(uint32_t state) { return state * 2654435761u; }
// which member owns a state, and the state's home slot in that member's table (different bits of the hash)
__device__ __forceinline__ int team_owner(uint32_t state, int k) { return (int)__umulhi(team_hash(state), (uint32_t)k); }
__device__ __forceinline__ uint32_t team_home(uint32_t state, uint32_t slots) {
  return __umulhi(team_hash(state) * 0x9E3779B1u, slots);
}

// Barrier across the k members of a team; `seq` counts the team barriers of this call.  A member that met a
// failure on its way here says so first.  Returns false if the team has to give up waiting (then abort_flag is
// set); `failed` receives the failure, if any, that some member met before this barrier.
__device__ __forceinline__ bool team_barrier(TeamChan *tc, TeamShared *sh, int k, int &seq, int &failed) {
  __syncthreads();
  if (threadIdx.x == 0) {
    if (sh->fault) atomicCAS(&tc->flag[seq & 3], 0, kStatusCapacity);
    __threadfence();   // what this member wrote is visible to the device before its arrival is
    const uint32_t old = atomicAdd(&tc->barrier, 1u);
    const uint32_t target = (old / (uint32_t)k + 1u) * (uint32_t)k;
    int polls = 0;
    while ((int32_t)(__hip_atomic_load(&tc->barrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
      __builtin_amdgcn_s_sleep(8);
      if (++polls > kTeamSpinLimit) { sh->abort_flag = 1; break; }
    }
    __threadfence();   // and what the others wrote before theirs is visible here
    sh->failed = __hip_atomic_load(&tc->flag[seq & 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  failed = sh->failed;
  seq += 1;
  return sh->abort_flag == 0;
}

// Appends one entry per lane with `act` set to the queues of the entries' owners: one LDS atomic per wave and
// owner hands out the places.
__device__ __forceinline__ void team_push(TeamEntry *q_base, int32_t *cnt, TeamShared *sh, int k, int q_cap, int me,
                                          bool act, int owner, const TeamEntry &e, int lane) {
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int o = 0; o < k; ++o) {   // uniform
    const unsigned long long m = __ballot(act && owner == o);
    if (m == 0) continue;
    int base = 0;
    if (lane == (int)__builtin_ctzll(m)) base = atomicAdd(&cnt[o], (int)__popcll(m));
    base = __shfl(base, (int)__builtin_ctzll(m), 64);
    if (act && owner == o) {
      const int pos = base + (int)__popcll(m & below);
      if (pos < q_cap) q_base[((size_t)o * k + me) * q_cap + pos] = e;
      else sh->fault = 1;
    }
  }
}

// Finds or makes the slot of `state` in this member's table.  Returns false if the table is full.
__device__ __forceinline__ bool team_slot(uint32_t *hkey, uint32_t slots, uint32_t state, uint32_t &h) {
  h = team_home(state, slots);
  uint32_t k = atomicCAS(&hkey[h], kEmptyKey, state);
  uint32_t probe = 1;
  while (k != kEmptyKey && k != state && probe < slots) {
    h = h + 1 == slots ? 0 : h + 1;
    k = atomicCAS(&hkey[h], kEmptyKey, state);
    ++probe;
  }
  return k == kEmptyKey || k == state;
}
// The slot of a state that is known to be in the table.
__device__ __forceinline__ uint32_t team_find(const uint32_t *hkey, uint32_t slots, uint32_t state) {
  uint32_t h = team_home(state, slots);
  uint32_t probe = 0;
  while (hkey[h] != state && probe < slots) { h = h + 1 == slots ? 0 : h + 1; ++probe; }
  return h;
}

// E[state] = min key for the lanes with `act` set.  Candidates of one wave often share their destination (every
// word end leads to the hub): if they all do, the wave's minimum is taken first and one lane commits it.
__device__ __forceinline__ void team_min(uint64_t *hval, uint32_t *hkey, uint32_t slots, TeamShared *sh, bool act,
                                         uint32_t state, uint64_t key, int lane) {
  const unsigned long long am = __ballot(act);
  if (am == 0) return;
  const int first = (int)__builtin_ctzll(am);
  const uint32_t s0 = (uint32_t)__shfl((int)state, first, 64);
  if (__popcll(am) > 1 && __ballot(act && state == s0) == am) {
    const uint32_t hi = act ? (uint32_t)(key >> 32) : 0xFFFFFFFFu;
    const uint32_t mhi = wave_min_u32(hi);
    const uint32_t lo = (act && hi == mhi) ? (uint32_t)key : 0xFFFFFFFFu;
    const uint32_t mlo = wave_min_u32(lo);
    if (lane == first) {
      uint32_t h;
      if (team_slot(hkey, slots, s0, h)) atomicMin((unsigned long long *)&hval[h], ((unsigned long long)mhi << 32) | mlo);
      else sh->fault = 1;
    }
    return;
  }
  if (act) {
    uint32_t h;
    if (team_slot(hkey, slots, state, h)) atomicMin((unsigned long long *)&hval[h], (unsigned long long)key);
    else sh->fault = 1;
  }
}

// Expansion of one emitting arc per lane: candidate cost (step 2: cost + biased weight - log-likelihood), the
// member's running minimum, and the entry on its way to the destination's owner.
__device__ __forceinline__ void team_emit(const TeamParams &tp, const Ctx &cx, const Rows &Lrow, TeamShared *sh,
                                          TeamEntry *q1c, int me, bool act, int a, float c_own, int src_tok, int lane,
                                          uint32_t &lmin) {
  TeamEntry e; e.dst = 0; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0;
  int owner = 0;
  if (act) {
    const ArcRec rec = tp.a.arcs[a];
    float w = rec.weight;
    if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
    const float cand = (c_own + w) - Lrow.at((rec.meta & 0xFFFFu) - 1u);
    const uint32_t o = f2ord(cand);
    lmin = o < lmin ? o : lmin;
    e.dst = (uint32_t)rec.dst; e.cost = cand; e.arc = (uint32_t)a; e.from = src_tok; e.row = rec.row;
    e.meta = rec.meta & 0xFFFF0000u;
    owner = team_owner(e.dst, tp.k);
  }
  team_push(q1c, sh->cnt1, sh, tp.k, tp.q_cap, me, act, owner, e, lane);
}

// A reset leaves the dense token list of the one-workgroup code behind and clears what the team kept.
__global__ void team_reset_kernel(TeamChan *team, const int32_t *chan_ids, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  TeamChan *tc = team + chan_ids[i];
  tc->status = 0; tc->partitioned = 0; tc->carry_n = 0;
  tc->barrier = 0;   // (a team that gave up waiting leaves its count between two multiples of k)
  for (int q = 0; q < 4; ++q) tc->flag[q] = 0;
  for (int q = 0; q < kTeamMax; ++q) tc->ntok[q] = 0;
}

__global__ __launch_bounds__(1024) void advance_team_kernel(TeamParams tp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const AdvanceParams &p = tp.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = 16;
  const int k = tp.k;
  const int ci = blockIdx.x / k, me = blockIdx.x % k;   // (members of a team are neighbours in the grid)
  const int c = p.chan_ids[ci];
  ChanState *cs = p.chan + c;
  TeamChan *tc = tp.team + c;

  const TeamLayout lay = team_layout(tp.stage_rows ? p.num_pdfs : 0, tp.ctx_lds_cap, tp.slots);
  TeamShared *sh = (TeamShared *)(smem + lay.sh);
  uint32_t *hist = (uint32_t *)(smem + lay.hist);
  uint32_t *bitmap = (uint32_t *)(smem + lay.bitmap);
  int32_t *ctx_lds = (int32_t *)(smem + lay.ctx);
  float *Lstage = (float *)(smem + lay.L);
  uint64_t *hval = (uint64_t *)(smem + lay.hval);
  uint32_t *hkey = (uint32_t *)(smem + lay.hkey);
  uint16_t *hidx = (uint16_t *)(smem + lay.hidx);
  const uint32_t slots = (uint32_t)tp.slots;

  float *t_cost = p.tok_cost + (size_t)c * p.g_tok_cap;
  int4 *t_row = p.tok_row + (size_t)c * 2 * p.g_tok_cap;
  int32_t *t_state = p.tok_state + (size_t)c * p.g_tok_cap;
  int2 *bp = p.bp + (size_t)c * p.bp_cap;
  const float *Lbase = p.loglikes + (long long)ci * p.channel_stride;
  TeamEntry *q1c = tp.q1 + (size_t)c * k * k * tp.q_cap;
  TeamEntry *q2c = tp.q2 + (size_t)c * k * k * tp.q_cap;
  TeamClosureWin *cwin = tp.cwin + ((size_t)c * k + me) * tp.part_cap;
  uint32_t *pub_key = tp.pub_key + (size_t)c * k * slots;
  uint16_t *pub_lid = tp.pub_lid + (size_t)c * k * slots;

  // a parked channel stays parked until it is reset (every member reads the same status: it only changes when a
  // call ends); nothing below runs for it, in particular no team barrier
  if (cs->status != kStatusOk || tc->status != 0) return;

  // ---- enter: context, empty table, the team's scalars
  if (tid == 0) {
    sh->abort_flag = 0; sh->fault = 0;
    sh->a_active = sh->a_emit = sh->a_eps = sh->a_cand = 0;
  }
  Ctx cx;
  const int cslot = cs->ctx_slot;
  cx.n = p.ctx_n[cslot]; cx.offset = p.ctx_off[cslot];
  cx.g_list = p.ctx + (size_t)cslot * p.max_ctx;
  cx.lds_list = (lds_cint_ptr)ctx_lds; cx.bitmap = bitmap;
  cx.in_lds = cx.n <= tp.ctx_lds_cap;
  cx.use_bitmap = p.lookup_mode == 1;
  if (cx.in_lds) for (int i = tid; i < cx.n; i += 1024) ctx_lds[i] = cx.g_list[i];
  for (int i = tid; i < kBloomWords; i += 1024) bitmap[i] = 0;
  for (uint32_t i = tid; i < slots; i += 1024) { hval[i] = kEmptyVal; hkey[i] = kEmptyKey; }
  __syncthreads();
  if (cx.use_bitmap) {
    for (int i = tid; i < cx.n; i += 1024) {
      const uint32_t h = bloom_hash(cx.g_list[i]);
      atomicOr(&bitmap[bloom_word(h)], bloom_mask(h));
    }
  }
  // (what the previous call left is read before anyone changes it: the first barrier lies between)
  int status = cs->status;
  if (status == kStatusOk && tc->status != 0) status = tc->status;
  const bool dense = tc->partitioned == 0;
  int n_dense = cs->n_tok;
  int n_mine_prev = dense ? 0 : tc->ntok[me];
  int frame_base = cs->frame_base, n_rec = cs->n_rec;
  float best = cs->best;
  int cut_bin = cs->cut_bin;
  int cur = cs->row_buf & 1;
  const int carry_n = tc->carry_n;
  if (me == 0 && tid < 64) {
    // both copies of the frame scalars start clean; the long rows left by the previous call go where frame 0
    // looks for them (the copy of the frame before it)
    for (int b = 0; b < 2; ++b) {
      TeamFrame *fr = &tc->fr[b];
      for (int i = tid; i < 256; i += 64) fr->hist[i] = 0;
      if (tid < kTeamMax) fr->count[tid] = 0;
      for (int i = tid; i < kTeamMax * kTeamMax; i += 64) { (&fr->qn[0][0])[i] = 0; (&fr->q2n[0][0])[i] = 0; }
      if (tid == 0) { fr->m_ord = 0xFFFFFFFFu; fr->best_ord = 0xFFFFFFFFu; fr->n_big = 0; }
    }
    TeamFrame *f1 = &tc->fr[1];
    if (tid < carry_n && tid < kTeamBig) {
      f1->big_first[tid] = tc->carry_first[tid]; f1->big_deg[tid] = tc->carry_deg[tid];
      f1->big_src[tid] = tc->carry_src[tid]; f1->big_cost[tid] = tc->carry_cost[tid];
    }
    if (tid == 0) f1->n_big = carry_n < kTeamBig ? carry_n : kTeamBig;
  }
  int bar_seq = 0, failed = 0;
  bool alive_team = team_barrier(tc, sh, k, bar_seq, failed);
  if (failed != 0 && status == kStatusOk) status = failed;
  const bool hist_on = p.max_active > 0 && p.beam > 0.0f && p.beam < __builtin_inff();
  const float inv = 256.0f / p.beam;
  const int part_cap = tp.part_cap;
  int frames_done = 0, max_tok = 0;
  long long tokens_made = 0;

  for (int f = 0; f < p.n_frames && alive_team && status == kStatusOk; ++f) {
    TeamFrame *fr = &tc->fr[f & 1];
    TeamFrame *fprev = &tc->fr[(f + 1) & 1];
    const bool last = f == p.n_frames - 1;
    const int co = cur * p.g_tok_cap, no = (cur ^ 1) * p.g_tok_cap;
    Rows Lrow;
    Lrow.lds = (lds_cfloat_ptr)Lstage; Lrow.glob = Lbase + (long long)f * p.num_pdfs; Lrow.staged = tp.stage_rows != 0;
    if (tp.stage_rows) for (int i = tid; i < p.num_pdfs; i += 1024) Lstage[i] = Lrow.glob[i];
    if (tid == 0) {
      sh->n_mine = 0; sh->n_cwin = 0; sh->m_ord = 0xFFFFFFFFu; sh->best_ord = 0xFFFFFFFFu; sh->n_big = 0; sh->n_surv = 0;
    }
    if (tid < kTeamMax) { sh->cnt1[tid] = 0; sh->cnt2[tid] = 0; }
    for (int i = tid; i < 256; i += 1024) hist[i] = 0;
    __syncthreads();

    // ================= phase 1: prune and expand this member's tokens
    uint32_t n_active = 0, n_emit = 0;
    uint32_t lmin = 0xFFFFFFFFu;
    {
      // this member's tokens: its share, or (first frame after a reset) its part of the dense list
      const int t0 = dense && f == 0 ? (int)((long long)n_dense * me / k) : me * part_cap;
      const int t1 = dense && f == 0 ? (int)((long long)n_dense * (me + 1) / k) : t0 + n_mine_prev;
      for (int i0 = t0 + wave * 64; i0 < t1; i0 += NW * 64) {
        const int i = i0 + lane;
        bool alive = false;
        float cost = 0.0f;
        int first = 0, deg = 0;
        if (i < t1) {
          cost = t_cost[i];
          const float r = cost - best;
          alive = !(r > p.beam) && cost < __builtin_inff();
          if (alive && cut_bin < 255) {
            int bin = (int)floorf(r * inv);
            bin = bin > 255 ? 255 : bin;
            alive = bin <= cut_bin;
          }
          if (alive) { const int4 row = t_row[co + i]; first = row.x; deg = row.y - row.x; }
        }
        n_active += (uint32_t)__popcll(__ballot(alive));
        if (deg > kBigRowArcs) {
          // a long row that was not announced (the start token's): this member's waves share it out below
          const int slot = atomicAdd(&sh->n_big, 1);
          if (slot < kBigRows) {
            sh->big_first[slot] = first; sh->big_deg[slot] = deg; sh->big_cost[slot] = cost; sh->big_src[slot] = i;
            deg = 0;
          }
        }
        // one lane per token, its arcs one after the other (rows are short: the long ones are shared out)
        int maxdeg = deg;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { const int t = __shfl_xor(maxdeg, d, 64); maxdeg = t > maxdeg ? t : maxdeg; }
        for (int j = 0; j < maxdeg; ++j) {   // uniform
          const bool act = j < deg;
          n_emit += (uint32_t)__popcll(__ballot(act));
          team_emit(tp, cx, Lrow, sh, q1c, me, act, first + j, cost, i, lane, lmin);
        }
      }
      // long rows announced by the previous frame: every wave of every member takes every (k * NW)-th group of 64
      const int nbig = fprev->n_big < kTeamBig ? fprev->n_big : kTeamBig;
      for (int r = 0; r < nbig; ++r) {
        const float cost = fprev->big_cost[r];
        const float rr = cost - best;
        bool alive = !(rr > p.beam) && cost < __builtin_inff();
        if (alive && cut_bin < 255) {
          int bin = (int)floorf(rr * inv);
          bin = bin > 255 ? 255 : bin;
          alive = bin <= cut_bin;
        }
        if (!alive) continue;   // uniform (the token itself is counted where it lives, with an empty row)
        const int first = fprev->big_first[r], deg = fprev->big_deg[r], src = fprev->big_src[r];
        for (int j0 = (me * NW + wave) * 64; j0 < deg; j0 += k * NW * 64) {
          const bool act = j0 + lane < deg;
          n_emit += (uint32_t)__popcll(__ballot(act));
          team_emit(tp, cx, Lrow, sh, q1c, me, act, first + j0 + lane, cost, src, lane, lmin);
        }
      }
      __syncthreads();
      const int nloc = sh->n_big < kBigRows ? sh->n_big : kBigRows;
      for (int r = 0; r < nloc; ++r) {
        const int first = sh->big_first[r], deg = sh->big_deg[r], src = sh->big_src[r];
        const float cost = sh->big_cost[r];
        for (int j0 = wave * 64; j0 < deg; j0 += NW * 64) {
          const bool act = j0 + lane < deg;
          n_emit += (uint32_t)__popcll(__ballot(act));
          team_emit(tp, cx, Lrow, sh, q1c, me, act, first + j0 + lane, cost, src, lane, lmin);
        }
      }
      const uint32_t wmin = wave_min_u32(lmin);
      if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->m_ord, wmin);
      __syncthreads();
      if (tid < k) fr->qn[tid][me] = sh->cnt1[tid] < tp.q_cap ? sh->cnt1[tid] : tp.q_cap;
      if (tid == 0 && sh->m_ord != 0xFFFFFFFFu) atomicMin(&fr->m_ord, sh->m_ord);
    }
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    if (me == 0 && tid < 64) {
      // the other copy of the frame scalars is free now (its long rows have been expanded): clean it for frame f + 1
      for (int i = tid; i < 256; i += 64) fprev->hist[i] = 0;
      if (tid < kTeamMax) fprev->count[tid] = 0;
      for (int i = tid; i < kTeamMax * kTeamMax; i += 64) { (&fprev->qn[0][0])[i] = 0; (&fprev->q2n[0][0])[i] = 0; }
      if (tid == 0) { fprev->m_ord = 0xFFFFFFFFu; fprev->best_ord = 0xFFFFFFFFu; fprev->n_big = 0; }
    }
    if (failed != 0) { status = failed; break; }
    const uint32_t m_ord = __hip_atomic_load(&fr->m_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (m_ord == 0xFFFFFFFFu) { status = kStatusNoTokens; break; }   // (every member sees the same)
    const float m = ord2f(m_ord);

    // ================= phase 2: what this member owns of the emitting candidates; closure lists of what passes
    uint32_t n_cand = 0, n_eps = 0;
    uint32_t cmin = 0xFFFFFFFFu;
    {
      int qn[kTeamMax], total = 0;
      for (int s = 0; s < k; ++s) { qn[s] = __hip_atomic_load(&fr->qn[me][s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); total += qn[s]; }
      const int rounds = (total + 1023) / 1024;
      for (int rd = 0; rd < rounds; ++rd) {   // uniform
        int t = rd * 1024 + tid;
        bool act = t < total;
        int s = 0;
        if (act) { while (t >= qn[s]) { t -= qn[s]; ++s; } }
        TeamEntry e; e.dst = 0; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0;
        if (act) e = q1c[((size_t)me * k + s) * tp.q_cap + t];
        const bool pass = act && !(e.cost - m > p.beam);
        n_cand += (uint32_t)__popcll(__ballot(pass));
        team_min(hval, hkey, slots, sh, pass, e.dst, ((uint64_t)f2ord(e.cost) << 32) | e.arc, lane);
        // the closure list of the state reached (stored with the graph: depth-first preorder, a record's source
        // is the latest record one level up)
        int pos = 0, len = 0;
        if (pass) {
          const uint32_t cl = meta_cl(e.meta);
          if (cl == kClEscape || meta_ed(e.meta) == kEdEscape || meta_xd(e.meta) == kXdEscape) {
            const int4 o = p.off2[e.dst];
            pos = o.z; len = o.w - o.z;
            if (len == 0 && o.z > o.y) sh->fault = 1;   // epsilon arcs without a stored list: not for this code
          } else {
            pos = e.row + (int)meta_ed(e.meta) + (int)meta_xd(e.meta); len = (int)cl;
          }
        }
        int maxlen = len;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) { const int tt = __shfl_xor(maxlen, d, 64); maxlen = tt > maxlen ? tt : maxlen; }
        float cstack[kClosureMaxDepth + 1];
        uint32_t sstack[kClosureMaxDepth + 1];
#pragma unroll
        for (int d = 0; d <= kClosureMaxDepth; ++d) { cstack[d] = __builtin_inff(); sstack[d] = 0; }
        cstack[0] = e.cost; sstack[0] = e.dst;
        for (int j = 0; j < maxlen; ++j) {   // uniform
          const bool has = j < len;
          bool ok = false;
          TeamEntry ce; ce.dst = 0; ce.cost = 0.0f; ce.arc = 0; ce.from = 0; ce.row = 0; ce.meta = 0;
          int owner = 0;
          if (has) {
            const ArcRec rec = p.arcs[pos + j];
            const int can = p.canon[pos + j];
            const int depth = (int)(rec.meta & 0xFu);
            float w = rec.weight;
            if (ctx_contains(cx, can)) w = w + cx.offset;   // Sec. 4.1
            float pc = __builtin_inff();
            uint32_t ps = 0;
#pragma unroll
            for (int d = 1; d <= kClosureMaxDepth; ++d) if (d == depth) { pc = cstack[d - 1]; ps = sstack[d - 1]; }
            const float cc = pc + w;
            ok = cc < __builtin_inff() && !(cc - m > p.beam);
#pragma unroll
            for (int d = 1; d <= kClosureMaxDepth; ++d) if (d == depth) { cstack[d] = ok ? cc : __builtin_inff(); sstack[d] = (uint32_t)rec.dst; }
            if (ok) {
              ce.dst = (uint32_t)rec.dst; ce.cost = cc; ce.arc = (uint32_t)can; ce.from = (int32_t)ps; ce.row = rec.row;
              ce.meta = rec.meta & 0xFFFF0000u;
              owner = team_owner(ce.dst, k);
              const uint32_t o = f2ord(cc);
              cmin = o < cmin ? o : cmin;
            }
          }
          n_eps += (uint32_t)__popcll(__ballot(has));
          n_cand += (uint32_t)__popcll(__ballot(ok));
          // candidates of one wave for one state (every word end leads to the hub): only the least key travels
          const unsigned long long om = __ballot(ok);
          if (om != 0) {
            const int fl = (int)__builtin_ctzll(om);
            const uint32_t d0 = (uint32_t)__shfl((int)ce.dst, fl, 64);
            if (__popcll(om) > 1 && __ballot(ok && ce.dst == d0) == om) {
              const uint32_t hi = ok ? f2ord(ce.cost) : 0xFFFFFFFFu;
              const uint32_t mhi = wave_min_u32(hi);
              const uint32_t lo = (ok && hi == mhi) ? ce.arc : 0xFFFFFFFFu;
              const uint32_t mlo = wave_min_u32(lo);
              ok = ok && hi == mhi && ce.arc == mlo;
              // (two lanes can hold the same least key: one of them goes)
              const unsigned long long wm = __ballot(ok);
              ok = ok && lane == (int)__builtin_ctzll(wm);
            }
          }
          team_push(q2c, sh->cnt2, sh, k, tp.q_cap, me, ok, owner, ce, lane);
        }
      }
      const uint32_t wmin = wave_min_u32(cmin);
      if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->best_ord, wmin);
      __syncthreads();
      if (tid < k) fr->q2n[tid][me] = sh->cnt2[tid] < tp.q_cap ? sh->cnt2[tid] : tp.q_cap;
      if (tid == 0 && sh->best_ord != 0xFFFFFFFFu) atomicMin(&fr->best_ord, sh->best_ord);
    }
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    if (failed != 0) { status = failed; break; }
    if (n_rec + k * part_cap > p.bp_cap) { status = kStatusCapacity; break; }   // (the same for all)

    // ================= phase 3: closure candidates in; winners write their tokens
    const uint32_t best_ord = umin32(m_ord, __hip_atomic_load(&fr->best_ord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const float fbest = ord2f(best_ord);
    int qn1[kTeamMax], qn2[kTeamMax], tot1 = 0, tot2 = 0;
    for (int s = 0; s < k; ++s) {
      qn1[s] = __hip_atomic_load(&fr->qn[me][s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); tot1 += qn1[s];
      qn2[s] = __hip_atomic_load(&fr->q2n[me][s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); tot2 += qn2[s];
    }
    for (int rd = 0; rd * 1024 < tot2; ++rd) {   // uniform
      int t = rd * 1024 + tid;
      const bool act = t < tot2;
      int s = 0;
      if (act) { while (t >= qn2[s]) { t -= qn2[s]; ++s; } }
      TeamEntry e; e.dst = 0; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0;
      if (act) e = q2c[((size_t)me * k + s) * tp.q_cap + t];
      team_min(hval, hkey, slots, sh, act, e.dst, ((uint64_t)f2ord(e.cost) << 32) | e.arc, lane);
    }
    __syncthreads();
    const int tok0 = me * part_cap;
    for (int rd = 0; rd * 1024 < tot1 + tot2; ++rd) {   // uniform
      int t = rd * 1024 + tid;
      const bool act = t < tot1 + tot2;
      const bool closure = act && t >= tot1;
      TeamEntry e; e.dst = 0; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0;
      if (act) {
        int s = 0;
        if (!closure) { while (t >= qn1[s]) { t -= qn1[s]; ++s; } e = q1c[((size_t)me * k + s) * tp.q_cap + t]; }
        else { t -= tot1; while (t >= qn2[s]) { t -= qn2[s]; ++s; } e = q2c[((size_t)me * k + s) * tp.q_cap + t]; }
      }
      bool win = false;
      uint32_t h = 0;
      uint64_t v = 0;
      if (act && !(e.cost - m > p.beam)) {
        h = team_find(hkey, slots, e.dst);
        v = hval[h];
        // the entry whose key is the state's value wins; equal keys (a closure record reached twice, or a copy
        // of an entry) are told apart by the exchange
        win = v != kEmptyVal && (uint32_t)v == e.arc && (uint32_t)(v >> 32) == f2ord(e.cost) &&
              atomicCAS((unsigned long long *)&hval[h], (unsigned long long)v, (unsigned long long)kEmptyVal) == v;
      }
      const unsigned long long wm = __ballot(win);
      if (wm == 0) continue;   // uniform
      int base = 0;
      if (lane == (int)__builtin_ctzll(wm)) base = atomicAdd(&sh->n_mine, (int)__popcll(wm));
      base = __shfl(base, (int)__builtin_ctzll(wm), 64);
      bool surv = false;
      if (win) {
        const int lid = base + (int)__popcll(wm & ((1ull << lane) - 1ull));
        if (lid >= part_cap) { sh->fault = 1; }
        else {
          hidx[h] = (uint16_t)lid;
          const int idx = tok0 + lid;
          // the state's row: from the arc record's fields, or (long rows) from the offsets
          int first = e.row, eps, end;
          const uint32_t ed = meta_ed(e.meta), xd = meta_xd(e.meta);
          if (ed == kEdEscape || xd == kXdEscape) { const int4 o = p.off2[e.dst]; eps = o.y; end = o.z; }
          else { eps = first + (int)ed; end = eps + (int)xd; }
          if (eps - first > kBigRowArcs) {
            const int slot = atomicAdd(&fr->n_big, 1);
            if (slot < kTeamBig) {
              fr->big_first[slot] = first; fr->big_deg[slot] = eps - first; fr->big_src[slot] = idx; fr->big_cost[slot] = e.cost;
              first = eps;   // (the token's own row has no emitting arcs left: the team expands them)
            }
          }
          t_cost[idx] = e.cost;
          t_row[no + idx] = make_int4(first, eps, end, 0);
          if (last) t_state[idx] = (int32_t)e.dst;
          if (!closure) {
            bp[n_rec + idx] = make_int2((int)e.arc, frame_base + e.from);
          } else {
            const int w = atomicAdd(&sh->n_cwin, 1);
            TeamClosureWin cw; cw.idx = idx; cw.arc = e.arc; cw.parent_state = (uint32_t)e.from;
            cwin[w] = cw;   // (w < part_cap: one per token)
          }
          if (hist_on) {
            const float r = e.cost - fbest;
            if (!(r > p.beam)) {
              surv = true;
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              atomicAdd(&hist[bin], 1u);
            }
          }
        }
      }
      const unsigned long long sm = __ballot(surv);
      if (sm != 0 && lane == 0) atomicAdd(&sh->n_surv, (int)__popcll(sm));
    }
    __syncthreads();
    // publish (state -> token) of this share, then empty the table for the next frame
    const int n_mine = sh->n_mine < part_cap ? sh->n_mine : part_cap;
    for (uint32_t i = tid; i < slots; i += 1024) {
      const uint32_t key = hkey[i];
      pub_key[(size_t)me * slots + i] = key;
      if (key != kEmptyKey) pub_lid[(size_t)me * slots + i] = hidx[i];
      hkey[i] = kEmptyKey; hval[i] = kEmptyVal;
    }
    if (last) for (int i = tid + n_mine; i < part_cap; i += 1024) t_cost[tok0 + i] = __builtin_inff();   // unused places
    if (hist_on) for (int i = tid; i < 256; i += 1024) if (hist[i]) atomicAdd(&fr->hist[i], hist[i]);
    if (tid == 0) fr->count[me] = n_mine;
    if (lane == 0) {   // (per-wave counters of the frame)
      atomicAdd(&sh->a_active, (unsigned long long)n_active); atomicAdd(&sh->a_emit, (unsigned long long)n_emit);
      atomicAdd(&sh->a_eps, (unsigned long long)n_eps); atomicAdd(&sh->a_cand, (unsigned long long)n_cand);
    }
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    if (failed != 0) { status = failed; break; }

    // ================= phase 4: records of the closure winners; the next frame's scalars
    {
      const int ncw = sh->n_cwin;
      for (int i = tid; i < ncw; i += 1024) {
        const TeamClosureWin cw = cwin[i];
        const int o = team_owner(cw.parent_state, k);
        const uint32_t *pk = pub_key + (size_t)o * slots;
        uint32_t h = team_home(cw.parent_state, slots);
        uint32_t probe = 0;
        while (__hip_atomic_load(&pk[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != cw.parent_state && probe < slots) {
          h = h + 1 == slots ? 0 : h + 1; ++probe;
        }
        const int plid = (int)__hip_atomic_load(&pub_lid[(size_t)o * slots + h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bp[n_rec + cw.idx] = make_int2((int)cw.arc, n_rec + o * part_cap + plid);
      }
      int n_total = 0, n_surv = 0;
      for (int s = 0; s < k; ++s) n_total += __hip_atomic_load(&fr->count[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      int cutb = 255;
      if (hist_on && n_total > p.max_active) {
        // (every member computes the same cut from the team's histogram; only wave 0's result is kept)
        if (wave == 0) {
          int loc[4], sum = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) { loc[q] = (int)__hip_atomic_load(&fr->hist[lane * 4 + q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); sum += loc[q]; }
          const int inc = wave_incl_scan(sum);
          n_surv = __builtin_amdgcn_readlane(inc, 63);
          if (n_surv > p.max_active) {
            int run = inc - sum, myB = -1;
#pragma unroll
            for (int q = 0; q < 4; ++q) { run += loc[q]; if (run <= p.max_active) myB = lane * 4 + q; }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) { const int t = __shfl_xor(myB, d, 64); myB = t > myB ? t : myB; }
            cutb = myB < 0 ? 0 : myB;
          }
          if (lane == 0) sh->cut_bin = cutb;
        }
        __syncthreads();
        cutb = sh->cut_bin;
      }
      cut_bin = cutb;
      best = fbest;
      frame_base = n_rec;
      n_rec += k * part_cap;
      n_mine_prev = n_mine;
      cur ^= 1;
      frames_done += 1;
      tokens_made += n_total;
      max_tok = n_total > max_tok ? n_total : max_tok;
      __syncthreads();   // (cut_bin in LDS is free again)
    }
  }

  // ---- leave
  __syncthreads();
  if (!alive_team) status = kStatusTeam;
  if (tid == 0) {
    tc->ntok[me] = status == kStatusOk ? n_mine_prev : 0;
    // every member adds its counters; member 0 writes what all members hold alike
    atomicAdd((unsigned long long *)&cs->active_tokens, sh->a_active);
    atomicAdd((unsigned long long *)&cs->emit_arcs, sh->a_emit);
    atomicAdd((unsigned long long *)&cs->eps_arcs, sh->a_eps);
    atomicAdd((unsigned long long *)&cs->candidates, sh->a_cand);
    if (me == 0) {
      if (status != kStatusOk) tc->status = status;
      cs->status = status;
      cs->n_tok = status == kStatusOk ? k * part_cap : 0;
      cs->frame_base = status == kStatusOk ? frame_base : n_rec;
      cs->n_rec = n_rec;
      cs->best = best;
      cs->cut_bin = cut_bin;
      cs->row_buf = status == kStatusOk ? cur : 0;
      cs->frames += frames_done;
      cs->tokens += tokens_made;
      cs->improvements += tokens_made;
      if (max_tok > cs->max_tokens) cs->max_tokens = max_tok;
      tc->partitioned = 1;
      // long rows among the last frame's tokens wait for the next call
      const TeamFrame *lf = &tc->fr[(p.n_frames - 1) & 1];
      const int nb = frames_done == p.n_frames && p.n_frames > 0 ? (lf->n_big < kTeamBig ? lf->n_big : kTeamBig) : 0;
      tc->carry_n = nb;
      for (int i = 0; i < nb; ++i) {
        tc->carry_first[i] = lf->big_first[i]; tc->carry_deg[i] = lf->big_deg[i];
        tc->carry_src[i] = lf->big_src[i]; tc->carry_cost[i] = lf->big_cost[i];
      }
      const int n_new = n_rec - cs->gc_base;
      if (p.new_records) p.new_records[c] = make_int2(n_new, p.call_seq);
      if (p.due_max) atomicMax(p.due_max, ((unsigned long long)(uint32_t)p.call_seq << 32) | (uint32_t)n_new);
    }
  }
}

}  // namespace cbd
