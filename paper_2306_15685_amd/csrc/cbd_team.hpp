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
// the host refuses more members than the device has compute units, and a member fills its unit's LDS.
#pragma once

namespace cbd {

constexpr int kTeamMax = 8;       // members of a team
constexpr int kTeamBig = 32;      // long rows a frame can share out
constexpr int kTeamSpinLimit = 8 << 20;   // polls of a barrier before a member gives up (seconds)
constexpr int kStatusTeam = -6;   // a member waited too long at a team barrier (reported as a HIP-level failure)

// A candidate on its way to the owner of its destination state.
struct __attribute__((aligned(16))) TeamEntry {
  uint32_t dst;
  float cost;
  uint32_t arc;     // library arc index (closure records: the arc they stand for)
  int32_t from;     // emitting arc: the source token's place in the previous frame; closure: the source STATE
  int32_t row;      // first arc of dst
  uint32_t meta;    // degrees and closure length of dst (ArcRec::meta with the low 16 bits cleared)
  uint32_t pad[2];  // (an entry is one aligned 32-byte sector: written whole, so nothing has to be read to merge it)
};
static_assert(sizeof(TeamEntry) == 32, "queue entries are 32 bytes");

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
  int32_t big_id[kTeamBig];   // the row's place in TeamParams::big_rows, or -1
};

struct __attribute__((aligned(256))) TeamChan {
  uint32_t barrier;        // arrivals at team barriers since the last reset (low 30 bits), failure marks (bits 30, 31)
  int32_t status;          // why the channel is parked (sticky until reset)
  int32_t partitioned;     // 0: the token list is the dense one a reset leaves; 1: members' shares
  int32_t ntok[kTeamMax];  // tokens of each member's share
  int32_t carry_n;         // long rows found in the last frame of the previous call
  int32_t carry_first[kTeamBig], carry_deg[kTeamBig], carry_src[kTeamBig], carry_id[kTeamBig];
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
  int32_t n_teams;         // channels of this launch (the grid may hold more teams: padding, they return at once)
  // Rows with more than kBigRowArcs emitting arcs, known when the graph was loaded: for each, its arcs sorted by the
  // member that owns their destination (a member then expands the arcs it owns itself: nothing travels)
  const int4 *big_rows;    // [n_big_rows] x = state (ascending), y = first emitting arc, z = emitting arcs, w = start in big_perm
  const int32_t *big_group;  // [n_big_rows][k + 1] where each member's arcs begin in the row's stretch of big_perm
  const int32_t *big_perm;   // library arc indices
  int32_t n_big_rows;
  int32_t k;               // members per team
  int32_t q_cap;
  int32_t part_cap;        // tokens per member and frame
  int32_t slots;           // table slots per member (LDS)
  int32_t stage_rows;      // the frame's log-likelihood row is copied to LDS
  int32_t ctx_lds_cap;
};

struct TeamLayout { uint32_t sh, hist, bitmap, stage, ctx, L, hval, hkey, hidx, total; };
struct TeamLive { float cost; int32_t first; int32_t deg; int32_t idx; };   // a token that survived pruning, on its way to a lane
struct TeamShared {
  int32_t abort_flag, fault, failed;
  int32_t n_mine;            // tokens this member has made in the current frame
  int32_t n_cwin;            // closure winners noted for phase 4
  unsigned long long cnt1[2], cnt2[2];       // entries pushed to each owner's queues (16 bits per owner)
  uint32_t m_ord, best_ord;  // this member's minima before they go to the team
  int32_t n_big;             // long rows met unannounced in this member's own tokens
  int32_t big_first[kBigRows], big_deg[kBigRows], big_src[kBigRows];
  float big_cost[kBigRows];
  int32_t cut_bin;
  unsigned long long a_active, a_emit, a_eps, a_cand;
};

__host__ __device__ inline TeamLayout team_layout(int num_pdfs_staged, int ctx_lds_cap, int slots, int n_waves) {
  TeamLayout l;
  uint32_t o = 0;
  l.sh = o; o += align_up((uint32_t)sizeof(TeamShared), 16);
  l.hist = o; o += 256 * 4;
  l.bitmap = o; o += kBloomWords * 4;
  l.stage = o; o += (uint32_t)n_waves * 64 * (uint32_t)sizeof(TeamLive);   // per wave: up to 64 live tokens waiting for a full group
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

// Barrier across the k members of a team.  The word counts arrivals in its low 30 bits (the counter runs on from
// barrier to barrier: a barrier is complete when the count reaches the next multiple of k; a reset starts it again)
// and carries two failure marks, one for even and one for odd barriers of the call: a member that met a failure
// on its way to barrier n sets the mark of n's parity before it arrives, and whoever leaves barrier n looks at that
// mark only (a member that is already on its way to barrier n + 1 sets the other one).  Returns false if the team
// has to give up waiting (then abort_flag is set); `failed` receives the failure, if any, met before this barrier.
constexpr uint32_t kTeamCountMask = 0x3FFFFFFFu;
__device__ __forceinline__ bool team_barrier(TeamChan *tc, TeamShared *sh, int k, int &seq, int &failed) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t mark = 0x40000000u << (seq & 1);
    if (sh->fault) atomicOr(&tc->barrier, mark);
    __threadfence();   // what this member wrote is visible to the device before its arrival is
    uint32_t v = atomicAdd(&tc->barrier, 1u) + 1u;
    const uint32_t target = (((v & kTeamCountMask) - 1u) / (uint32_t)k + 1u) * (uint32_t)k;
    int polls = 0;
    while ((v & kTeamCountMask) < target) {   // (the last to arrive does not wait)
      __builtin_amdgcn_s_sleep(2);
      v = __hip_atomic_load(&tc->barrier, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (++polls > kTeamSpinLimit) { sh->abort_flag = 1; break; }
    }
    __threadfence();   // and what the others wrote before theirs is visible here
    sh->failed = (v & mark) ? kStatusCapacity : 0;
  }
  __syncthreads();
  failed = sh->failed;
  seq += 1;
  return sh->abort_flag == 0;
}

// Appends up to U entries per lane (those with act[u] set) to the queues of the entries' owners.  The members'
// counters are 16-bit fields of 64-bit LDS words (owners 0-3 and 4-7), so ONE atomic per wave hands out the places
// of all owners and all U groups at once (the waves of a member all add to the same word, and such atomics queue).
// (A queue holds fewer than 32,768 entries; once one is full nothing is added any more, so no field overflows.)
template <int U>
__device__ __forceinline__ void team_push(TeamEntry *q_base, unsigned long long *cnt, TeamShared *sh, int k, int q_cap,
                                          int me, const bool (&act)[U], const int (&owner)[U], const TeamEntry (&e)[U],
                                          int lane) {
  bool any = false;
#pragma unroll
  for (int u = 0; u < U; ++u) any = any || act[u];
  if (__ballot(any) == 0) return;   // uniform
  if (__hip_atomic_load(&sh->fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0) return;
  const unsigned long long below = (1ull << lane) - 1ull;
  unsigned long long add[2] = {0, 0};
  int rank[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    rank[u] = 0;
    for (int o = 0; o < k; ++o) {   // uniform
      const unsigned long long m = __ballot(act[u] && owner[u] == o);
      if (owner[u] == o) rank[u] = (int)__popcll(m & below) + (int)((add[o >> 2] >> (16 * (o & 3))) & 0xFFFFull);
      add[o >> 2] += (unsigned long long)__popcll(m) << (16 * (o & 3));
    }
  }
  unsigned long long base[2] = {0, 0};
  if (lane == 0) {
    if (add[0]) base[0] = atomicAdd(&cnt[0], add[0]);
    if (add[1]) base[1] = atomicAdd(&cnt[1], add[1]);
  }
  base[0] = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(base[0] >> 32), 0) << 32) |
            (uint32_t)__builtin_amdgcn_readlane((int)base[0], 0);
  if (k > 4) base[1] = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(base[1] >> 32), 0) << 32) |
                       (uint32_t)__builtin_amdgcn_readlane((int)base[1], 0);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (act[u]) {
      const int pos = (int)((base[owner[u] >> 2] >> (16 * (owner[u] & 3))) & 0xFFFFull) + rank[u];
      if (pos < q_cap) q_base[((size_t)owner[u] * k + me) * q_cap + pos] = e[u];
      else sh->fault = 1;
    }
  }
}
__device__ __forceinline__ int team_count(const unsigned long long *cnt, int o) {
  return (int)((cnt[o >> 2] >> (16 * (o & 3))) & 0xFFFFull);
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
  const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)state, first);
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

// Expansion of one emitting arc per lane, in two halves so that several records can be on their way at once:
// the record is asked for, and later the candidate cost (step 2: cost + biased weight - log-likelihood) joins the
// member's running minimum and the entry goes on its way to the destination's owner.
__device__ __forceinline__ ArcRec team_arc(const TeamParams &tp, bool act, int a) {
  ArcRec rec; rec.dst = 0; rec.weight = 0.0f; rec.row = 0; rec.meta = 0;
  if (act) rec = tp.a.arcs[a];
  return rec;
}
template <int U>
__device__ __forceinline__ void team_emit(const TeamParams &tp, const Ctx &cx, const Rows &Lrow, TeamShared *sh,
                                          TeamEntry *q1c, int me, const bool (&act)[U], const int (&a)[U],
                                          const ArcRec (&rec)[U], float c_own, int src_tok, int lane, uint32_t &lmin) {
  TeamEntry e[U];
  int owner[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    e[u].dst = 0; e[u].cost = 0.0f; e[u].arc = 0; e[u].from = 0; e[u].row = 0; e[u].meta = 0; e[u].pad[0] = 0; e[u].pad[1] = 0;
    owner[u] = 0;
    if (act[u]) {
      float w = rec[u].weight;
      if (ctx_contains(cx, a[u])) w = w + cx.offset;   // Sec. 4.1: boosted weight = weight + discount
      const float cand = (c_own + w) - Lrow.at((rec[u].meta & 0xFFFFu) - 1u);
      const uint32_t o = f2ord(cand);
      lmin = o < lmin ? o : lmin;
      e[u].dst = (uint32_t)rec[u].dst; e[u].cost = cand; e[u].arc = (uint32_t)a[u]; e[u].from = src_tok; e[u].row = rec[u].row;
      e[u].meta = rec[u].meta & 0xFFFF0000u;
      owner[u] = team_owner(e[u].dst, tp.k);
    }
  }
  team_push<U>(q1c, sh->cnt1, sh, tp.k, tp.q_cap, me, act, owner, e, lane);
}
// A long row shared out: this wave takes the groups of 64 arcs at j_begin, j_begin + j_step, ..., four at a time:
// all four records are asked for before the first entry is stored (loads and stores complete in order, so a
// load issued behind stores also waits for them).
__device__ __forceinline__ void team_long_row(const TeamParams &tp, const Ctx &cx, const Rows &Lrow, TeamShared *sh,
                                              TeamEntry *q1c, int me, int first, int deg, float cost, int src,
                                              int j_begin, int j_step, int lane, uint32_t &lmin, uint32_t &n_emit) {
  for (int j0 = j_begin; j0 < deg; j0 += 4 * j_step) {   // uniform
    ArcRec r[4];
    bool act[4];
    int a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * j_step + lane;
      act[u] = j < deg;
      a[u] = first + j;
      r[u] = team_arc(tp, act[u], a[u]);
      n_emit += (uint32_t)__popcll(__ballot(act[u]));
    }
    team_emit<4>(tp, cx, Lrow, sh, q1c, me, act, a, r, cost, src, lane, lmin);
  }
}

// One workgroup per long row: sorts the row's arcs by the member that owns their destination (counting sort; the
// order inside a member's group does not matter).
__global__ __launch_bounds__(256) void team_prepare_rows_kernel(const ArcRec *arcs, const int4 *big_rows, int32_t *big_group,
                                                                int32_t *big_perm, int k) {
  __shared__ int32_t count[kTeamMax + 1], fill[kTeamMax];
  const int4 row = big_rows[blockIdx.x];
  if (threadIdx.x <= kTeamMax) count[threadIdx.x] = 0;
  __syncthreads();
  for (int j = threadIdx.x; j < row.z; j += blockDim.x) atomicAdd(&count[team_owner((uint32_t)arcs[row.y + j].dst, k)], 1);
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int o = 0; o < k; ++o) { const int c = count[o]; big_group[blockIdx.x * (k + 1) + o] = run; fill[o] = run; run += c; }
    big_group[blockIdx.x * (k + 1) + k] = run;
  }
  __syncthreads();
  for (int j = threadIdx.x; j < row.z; j += blockDim.x) {
    const int o = team_owner((uint32_t)arcs[row.y + j].dst, k);
    big_perm[row.w + atomicAdd(&fill[o], 1)] = row.y + j;
  }
}
// The place of `state` among the long rows, or -1.
__device__ __forceinline__ int team_long_row_id(const TeamParams &tp, uint32_t state) {
  int lo = 0, hi = tp.n_big_rows;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((uint32_t)tp.big_rows[mid].x < state) lo = mid + 1; else hi = mid;
  }
  return (lo < tp.n_big_rows && (uint32_t)tp.big_rows[lo].x == state) ? lo : -1;
}

// A reset leaves the dense token list of the one-workgroup code behind and clears what the team kept.
__global__ void team_reset_kernel(TeamChan *team, const int32_t *chan_ids, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  TeamChan *tc = team + chan_ids[i];
  tc->status = 0; tc->partitioned = 0; tc->carry_n = 0;
  tc->barrier = 0;   // (a team that gave up waiting leaves its count between two multiples of k)
  for (int q = 0; q < kTeamMax; ++q) tc->ntok[q] = 0;
}

#ifdef CBD_PROFILE
#define TEAM_STAMP(k_) do { if (tid == 0) { const long long t_ = wall_clock64(); tprof[k_] += t_ - tlast; tlast = t_; } } while (0)
#else
#define TEAM_STAMP(k_) do {} while (0)
#endif

template <int kBlock>
__global__ __launch_bounds__(kBlock) void advance_team_kernel(TeamParams tp) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const AdvanceParams &p = tp.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NW = kBlock / 64;
  const int k = tp.k;
  // Workgroups are handed to the chip's eight dies in turn.  With the teams' members a whole number of rounds apart
  // in the grid (the host pads the number of teams to a multiple of 8), a team sits on one die and its queues stay in
  // that die's L2.  (Only speed depends on it: the fences and atomics are device-wide.)
  const int n_teams = (int)gridDim.x / k;
  const int ci = blockIdx.x % n_teams, me = blockIdx.x / n_teams;
  if (ci >= tp.n_teams) return;
  const int c = p.chan_ids[ci];
  ChanState *cs = p.chan + c;
  TeamChan *tc = tp.team + c;

  const TeamLayout lay = team_layout(tp.stage_rows ? p.num_pdfs : 0, tp.ctx_lds_cap, tp.slots, NW);
  TeamShared *sh = (TeamShared *)(smem + lay.sh);
  uint32_t *hist = (uint32_t *)(smem + lay.hist);
  uint32_t *bitmap = (uint32_t *)(smem + lay.bitmap);
  TeamLive *stage = (TeamLive *)(smem + lay.stage) + wave * 64;
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
  if (cx.in_lds) for (int i = tid; i < cx.n; i += kBlock) ctx_lds[i] = cx.g_list[i];
  for (int i = tid; i < kBloomWords; i += kBlock) bitmap[i] = 0;
  for (uint32_t i = tid; i < slots; i += kBlock) { hval[i] = kEmptyVal; hkey[i] = kEmptyKey; }
  __syncthreads();
  if (cx.use_bitmap) {
    for (int i = tid; i < cx.n; i += kBlock) {
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
      f1->big_src[tid] = tc->carry_src[tid]; f1->big_cost[tid] = tc->carry_cost[tid]; f1->big_id[tid] = tc->carry_id[tid];
    }
    if (tid == 0) f1->n_big = carry_n < kTeamBig ? carry_n : kTeamBig;
  }
#ifdef CBD_PROFILE
  long long tprof[14] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  long long tlast = wall_clock64();
#endif
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
    if (tp.stage_rows) for (int i = tid; i < p.num_pdfs; i += kBlock) Lstage[i] = Lrow.glob[i];
    if (tid == 0) {
      sh->n_mine = 0; sh->n_cwin = 0; sh->m_ord = 0xFFFFFFFFu; sh->best_ord = 0xFFFFFFFFu; sh->n_big = 0;
    }
    if (tid < 2) { sh->cnt1[tid] = 0; sh->cnt2[tid] = 0; }
    for (int i = tid; i < 256; i += kBlock) hist[i] = 0;
    __syncthreads();

    // a token's fate at the start of this frame (step 1), and one arc of a long row as the candidate it makes
    auto row_alive = [&](float cost) {
      const float rr = cost - best;
      bool alive = !(rr > p.beam) && cost < __builtin_inff();
      if (alive && cut_bin < 255) {
        int bin = (int)floorf(rr * inv);
        bin = bin > 255 ? 255 : bin;
        alive = bin <= cut_bin;
      }
      return alive;
    };
    // (asked for a round ahead: the arc's place in the sorted list, then its record; made into an entry afterwards)
    auto long_load = [&](int perm0, int t, int t_end, int &a, ArcRec &rec) {
      a = -1; rec.dst = 0; rec.weight = 0.0f; rec.row = 0; rec.meta = 0;
      if (t < t_end) { a = tp.big_perm[perm0 + t]; rec = p.arcs[a]; }
    };
    auto long_entry = [&](int a, const ArcRec &rec, float cost, int src) {
      TeamEntry e; e.dst = kEmptyKey; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0; e.pad[0] = 0; e.pad[1] = 0;
      if (a >= 0) {
        float w = rec.weight;
        if (ctx_contains(cx, a)) w = w + cx.offset;   // Sec. 4.1
        e.dst = (uint32_t)rec.dst; e.cost = (cost + w) - Lrow.at((rec.meta & 0xFFFFu) - 1u); e.arc = (uint32_t)a; e.from = src;
        e.row = rec.row; e.meta = rec.meta & 0xFFFF0000u;
      }
      return e;
    };
    const int nbig_prev = fprev->n_big < kTeamBig ? fprev->n_big : kTeamBig;
    // every candidate this member owns of the announced long rows with sorted arcs, one per thread and round
    auto for_owned_long_arcs = [&](auto &&fn) {
      for (int r = 0; r < nbig_prev; ++r) {
        const int id = fprev->big_id[r];
        const float cost = fprev->big_cost[r];
        if (id < 0 || !row_alive(cost)) continue;   // uniform
        const int src = fprev->big_src[r];
        const int4 row = tp.big_rows[id];
        const int g0 = tp.big_group[id * (k + 1) + me], g1 = tp.big_group[id * (k + 1) + me + 1];
        int a0, a1;
        ArcRec r0, r1;
        long_load(row.w, g0 + tid, g1, a0, r0);
        for (int t0 = g0; t0 < g1; t0 += kBlock) {   // uniform
          long_load(row.w, t0 + kBlock + tid, g1, a1, r1);
          fn(long_entry(a0, r0, cost, src));
          a0 = a1; r0 = r1;
        }
      }
    };

    // ================= phase 1: prune and expand this member's tokens
    uint32_t n_active = 0, n_emit = 0;
    uint32_t lmin = 0xFFFFFFFFu;
    {
      // this member's tokens: its share, or (first frame after a reset) its part of the dense list
      const int t0 = dense && f == 0 ? (int)((long long)n_dense * me / k) : me * part_cap;
      const int t1 = dense && f == 0 ? (int)((long long)n_dense * (me + 1) / k) : t0 + n_mine_prev;
      // Most tokens of a dense frame fall to the histogram cut.  So only the costs are read for all of them (four
      // tiles of a wave at a time); the live ones are gathered in the wave's staging list and expanded a full
      // group at a time: their rows are read then, one lane per token (rows are short, the long ones are shared
      // out), two arcs of a token together.
      auto expand_staged = [&](int n) {
        TeamLive tk; tk.cost = 0.0f; tk.first = 0; tk.deg = 0; tk.idx = 0;
        if (lane < n) {
          tk = stage[lane];
          // (the team keeps 8 bytes of a token's row: first emitting arc, first epsilon arc; the list a reset leaves
          // has the one-workgroup code's 16-byte rows)
          if (dense && f == 0) { const int4 row = t_row[co + tk.idx]; tk.first = row.x; tk.deg = row.y - row.x; }
          else { const int2 row = ((const int2 *)(t_row + co))[tk.idx]; tk.first = row.x; tk.deg = row.y - row.x; }
          if (tk.deg > kBigRowArcs) {
            // a long row that was not announced (the start token's): this member's waves share it out below
            const int slot = atomicAdd(&sh->n_big, 1);
            if (slot < kBigRows) {
              sh->big_first[slot] = tk.first; sh->big_deg[slot] = tk.deg; sh->big_cost[slot] = tk.cost; sh->big_src[slot] = tk.idx;
              tk.deg = 0;
            }
          }
        }
        for (int j = 0; __ballot(j < tk.deg) != 0; j += 2) {   // uniform
          bool act[2] = {j < tk.deg, j + 1 < tk.deg};
          int a[2] = {tk.first + j, tk.first + j + 1};
          ArcRec r[2];
          r[0] = team_arc(tp, act[0], a[0]);
          r[1] = team_arc(tp, act[1], a[1]);
          n_emit += (uint32_t)__popcll(__ballot(act[0])) + (uint32_t)__popcll(__ballot(act[1]));
          team_emit<2>(tp, cx, Lrow, sh, q1c, me, act, a, r, tk.cost, tk.idx, lane, lmin);
        }
      };
      int n_staged = 0;
      for (int base = t0 + wave * 64; base < t1; base += 4 * NW * 64) {   // uniform
        float c4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int i = base + u * NW * 64 + lane;
          c4[u] = i < t1 ? t_cost[i] : __builtin_inff();
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (base + u * NW * 64 >= t1) break;   // uniform
          const int i = base + u * NW * 64 + lane;
          const bool alive = i < t1 && row_alive(c4[u]);
          const unsigned long long lm = __ballot(alive);
          const int n_new = (int)__popcll(lm);
          n_active += (uint32_t)n_new;
          if (n_new == 0) continue;   // uniform
          if (n_staged + n_new > 64) { expand_staged(n_staged); n_staged = 0; }
          if (alive) {
            TeamLive tk; tk.cost = c4[u]; tk.first = 0; tk.deg = 0; tk.idx = i;
            stage[n_staged + (int)__popcll(lm & ((1ull << lane) - 1ull))] = tk;
          }
          n_staged += n_new;
        }
      }
      if (n_staged > 0) expand_staged(n_staged);
      TEAM_STAMP(7);   // (diagnostic: own tokens expanded)
      // long rows announced by the previous frame: every wave of every member takes every (k * NW)-th group of 64
      for (int r = 0; r < nbig_prev; ++r) {
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
        if (fprev->big_id[r] < 0) {
          team_long_row(tp, cx, Lrow, sh, q1c, me, first, deg, cost, src, (me * NW + wave) * 64, k * NW * 64, lane, lmin, n_emit);
          continue;
        }
        // its arcs are sorted by owner: every member will expand the ones it owns after the barrier.  Here the team
        // only needs their minimum (each wave looks at its share of the row)
        for (int j0 = (me * NW + wave) * 64; j0 < deg; j0 += k * NW * 64) {   // uniform
          const int j = j0 + lane;
          if (j < deg) {
            const ArcRec rec = p.arcs[first + j];
            float w = rec.weight;
            if (ctx_contains(cx, first + j)) w = w + cx.offset;   // Sec. 4.1
            const uint32_t o = f2ord((cost + w) - Lrow.at((rec.meta & 0xFFFFu) - 1u));
            lmin = o < lmin ? o : lmin;
          }
          n_emit += (uint32_t)__popcll(__ballot(j < deg));
        }
      }
      TEAM_STAMP(8);   // (diagnostic: announced long rows expanded)
      __syncthreads();
      TEAM_STAMP(9);   // (diagnostic: wait for the member's other waves)
      const int nloc = sh->n_big < kBigRows ? sh->n_big : kBigRows;
      for (int r = 0; r < nloc; ++r) {
        const int first = sh->big_first[r], deg = sh->big_deg[r], src = sh->big_src[r];
        team_long_row(tp, cx, Lrow, sh, q1c, me, first, deg, sh->big_cost[r], src, wave * 64, NW * 64, lane, lmin, n_emit);
      }
      const uint32_t wmin = wave_min_u32(lmin);
      if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->m_ord, wmin);
      __syncthreads();
      if (tid < k) fr->qn[tid][me] = team_count(sh->cnt1, tid) < tp.q_cap ? team_count(sh->cnt1, tid) : tp.q_cap;
      if (tid == 0 && sh->m_ord != 0xFFFFFFFFu) atomicMin(&fr->m_ord, sh->m_ord);
    }
    TEAM_STAMP(0);
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    TEAM_STAMP(1);
    if (me == 0 && tid < 64) {
      // the other copy of the frame scalars is free now (its long rows have been expanded): clean it for frame f + 1
      for (int i = tid; i < 256; i += 64) fprev->hist[i] = 0;
      if (tid < kTeamMax) fprev->count[tid] = 0;
      for (int i = tid; i < kTeamMax * kTeamMax; i += 64) { (&fprev->qn[0][0])[i] = 0; (&fprev->q2n[0][0])[i] = 0; }
      if (tid == 0) { fprev->m_ord = 0xFFFFFFFFu; fprev->best_ord = 0xFFFFFFFFu; fprev->n_big = 0; }
    }
    if (failed != 0) { status = failed; break; }
    const uint32_t m_ord = fr->m_ord;
    if (m_ord == 0xFFFFFFFFu) { status = kStatusNoTokens; break; }   // (every member sees the same)
    const float m = ord2f(m_ord);

    // ================= phase 2: what this member owns of the emitting candidates; closure lists of what passes
    uint32_t n_cand = 0, n_eps = 0;
    uint32_t cmin = 0xFFFFFFFFu;
    {
      int qn[kTeamMax], total = 0;
      for (int s = 0; s < k; ++s) { qn[s] = fr->qn[me][s]; total += qn[s]; }   // (plain reads: the barrier's fence made them current)
      const int rounds = (total + kBlock - 1) / kBlock;
      auto fetch = [&](int rd) {   // this thread's entry of round rd (dst = kEmptyKey: none)
        TeamEntry e; e.dst = kEmptyKey; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0; e.pad[0] = 0; e.pad[1] = 0;
        int t = rd * kBlock + tid;
        if (t < total) {
          int s = 0;
          while (t >= qn[s]) { t -= qn[s]; ++s; }
          e = q1c[((size_t)me * k + s) * tp.q_cap + t];
        }
        return e;
      };
      // what happens to one received candidate (dst = kEmptyKey: this lane has none)
      auto recombine = [&](const TeamEntry &e) {
        const bool act = e.dst != kEmptyKey;
        const bool pass = act && !(e.cost - m > p.beam);
        n_cand += (uint32_t)__popcll(__ballot(pass));
        // the closure list of the state reached (stored with the graph: depth-first preorder, a record's source
        // is the latest record one level up); its first record is asked for before the table is touched
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
        ArcRec rec0; rec0.dst = 0; rec0.weight = 0.0f; rec0.row = 0; rec0.meta = 0;
        int can0 = 0;
        if (len > 0) { rec0 = p.arcs[pos]; can0 = p.canon[pos]; }
        team_min(hval, hkey, slots, sh, pass, e.dst, ((uint64_t)f2ord(e.cost) << 32) | e.arc, lane);
        float cstack[kClosureMaxDepth + 1];
        uint32_t sstack[kClosureMaxDepth + 1];
        const bool flat = __ballot(len > 1) == 0;   // (uniform) no list of this wave is longer than one arc: no levels to keep
        if (!flat) {
#pragma unroll
          for (int d = 0; d <= kClosureMaxDepth; ++d) { cstack[d] = __builtin_inff(); sstack[d] = 0; }
          cstack[0] = e.cost; sstack[0] = e.dst;
        }
        for (int j = 0; __ballot(j < len) != 0; ++j) {   // uniform
          const bool has = j < len;
          bool ok = false;
          TeamEntry ce; ce.dst = 0; ce.cost = 0.0f; ce.arc = 0; ce.from = 0; ce.row = 0; ce.meta = 0; ce.pad[0] = 0; ce.pad[1] = 0;
          int owner = 0;
          if (has) {
            const ArcRec rec = j == 0 ? rec0 : p.arcs[pos + j];
            const int can = j == 0 ? can0 : p.canon[pos + j];
            const int depth = (int)(rec.meta & 0xFu);
            float w = rec.weight;
            if (ctx_contains(cx, can)) w = w + cx.offset;   // Sec. 4.1
            float pc = e.cost;
            uint32_t ps = e.dst;
            if (!flat) {
#pragma unroll
              for (int d = 1; d <= kClosureMaxDepth; ++d) if (d == depth) { pc = cstack[d - 1]; ps = sstack[d - 1]; }
            }
            const float cc = pc + w;
            ok = cc < __builtin_inff() && !(cc - m > p.beam);
            if (!flat) {
#pragma unroll
              for (int d = 1; d <= kClosureMaxDepth; ++d) if (d == depth) { cstack[d] = ok ? cc : __builtin_inff(); sstack[d] = (uint32_t)rec.dst; }
            }
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
            const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)ce.dst, fl);
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
          {
            const bool act1[1] = {ok};
            const int owner1[1] = {owner};
            const TeamEntry e1[1] = {ce};
            team_push<1>(q2c, sh->cnt2, sh, k, tp.q_cap, me, act1, owner1, e1, lane);
          }
        }
      };
      TeamEntry e_next = fetch(0);
      for (int rd = 0; rd < rounds; ++rd) {   // uniform
        const TeamEntry e = e_next;
        if (rd + 1 < rounds) e_next = fetch(rd + 1);
        recombine(e);
      }
      // long rows whose arcs are sorted by owner: this member expands the arcs it owns, here, with the cutoff known
      TEAM_STAMP(12);   // (diagnostic: candidates from the queues recombined)
      for_owned_long_arcs([&](const TeamEntry &e) { recombine(e); });
      const uint32_t wmin = wave_min_u32(cmin);
      if (lane == 0 && wmin != 0xFFFFFFFFu) atomicMin(&sh->best_ord, wmin);
      __syncthreads();
      if (tid < k) fr->q2n[tid][me] = team_count(sh->cnt2, tid) < tp.q_cap ? team_count(sh->cnt2, tid) : tp.q_cap;
      if (tid == 0 && sh->best_ord != 0xFFFFFFFFu) atomicMin(&fr->best_ord, sh->best_ord);
    }
    TEAM_STAMP(2);
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    TEAM_STAMP(3);
    if (failed != 0) { status = failed; break; }
    if (n_rec + k * part_cap > p.bp_cap) { status = kStatusCapacity; break; }   // (the same for all)

    // ================= phase 3: closure candidates in; winners write their tokens
    const uint32_t best_ord = umin32(m_ord, fr->best_ord);
    const float fbest = ord2f(best_ord);
    int qn1[kTeamMax], qn2[kTeamMax], tot1 = 0, tot2 = 0;
    for (int s = 0; s < k; ++s) {
      qn1[s] = fr->qn[me][s]; tot1 += qn1[s];
      qn2[s] = fr->q2n[me][s]; tot2 += qn2[s];
    }
    for (int rd = 0; rd * kBlock < tot2; ++rd) {   // uniform
      int t = rd * kBlock + tid;
      const bool act = t < tot2;
      int s = 0;
      if (act) { while (t >= qn2[s]) { t -= qn2[s]; ++s; } }
      TeamEntry e; e.dst = 0; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0; e.pad[0] = 0; e.pad[1] = 0;
      if (act) e = q2c[((size_t)me * k + s) * tp.q_cap + t];
      team_min(hval, hkey, slots, sh, act, e.dst, ((uint64_t)f2ord(e.cost) << 32) | e.arc, lane);
    }
    __syncthreads();
    TEAM_STAMP(10);   // (diagnostic: closure candidates recombined)
    const int tok0 = me * part_cap;
    auto fetch_any = [&](int rd, bool &closure) {   // this thread's entry of round rd over both sets of queues
      TeamEntry e; e.dst = kEmptyKey; e.cost = 0.0f; e.arc = 0; e.from = 0; e.row = 0; e.meta = 0; e.pad[0] = 0; e.pad[1] = 0;
      int t = rd * kBlock + tid;
      closure = t >= tot1;
      if (t < tot1 + tot2) {
        int s = 0;
        if (!closure) { while (t >= qn1[s]) { t -= qn1[s]; ++s; } e = q1c[((size_t)me * k + s) * tp.q_cap + t]; }
        else { t -= tot1; while (t >= qn2[s]) { t -= qn2[s]; ++s; } e = q2c[((size_t)me * k + s) * tp.q_cap + t]; }
      }
      return e;
    };
    // the entry whose key is its state's value writes the token
    auto winner = [&](const TeamEntry &e, bool closure) {
      const bool act = e.dst != kEmptyKey;
      bool win = false;
      uint32_t h = 0;
      uint64_t v = 0;
      if (act && !(e.cost - m > p.beam)) {
        h = team_find(hkey, slots, e.dst);
        v = hval[h];
        // the entry whose key is the state's value wins.  An emitting arc is expanded once per frame, so its entry
        // is the only one with its key; a closure record can have been reached twice with the same key: there an
        // exchange lets one of the two through
        win = v != kEmptyVal && (uint32_t)v == e.arc && (uint32_t)(v >> 32) == f2ord(e.cost);
        if (win && closure)
          win = atomicCAS((unsigned long long *)&hval[h], (unsigned long long)v, (unsigned long long)kEmptyVal) == v;
      }
      const unsigned long long wm = __ballot(win);
      if (wm == 0) return;   // uniform
      int base = 0;
      if (lane == (int)__builtin_ctzll(wm)) base = atomicAdd(&sh->n_mine, (int)__popcll(wm));
      base = __builtin_amdgcn_readlane(base, (int)__builtin_ctzll(wm));
      if (win) {
        const int lid = base + (int)__popcll(wm & ((1ull << lane) - 1ull));
        if (lid >= part_cap) { sh->fault = 1; }
        else {
          hidx[h] = (uint16_t)lid;
          const int idx = tok0 + lid;
          // the state's row: from the arc record's fields, or (long rows) from the offsets
          int first = e.row, eps;
          const uint32_t ed = meta_ed(e.meta);
          if (ed == kEdEscape) eps = p.off2[e.dst].y;
          else eps = first + (int)ed;
          if (eps - first > kBigRowArcs) {
            const int slot = atomicAdd(&fr->n_big, 1);
            if (slot < kTeamBig) {
              fr->big_first[slot] = first; fr->big_deg[slot] = eps - first; fr->big_src[slot] = idx; fr->big_cost[slot] = e.cost;
              fr->big_id[slot] = team_long_row_id(tp, e.dst);
              first = eps;   // (the token's own row has no emitting arcs left: the team expands them)
            }
          }
          t_cost[idx] = e.cost;
          ((int2 *)(t_row + no))[idx] = make_int2(first, eps);
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
              int bin = (int)floorf(r * inv);
              bin = bin > 255 ? 255 : bin;
              atomicAdd(&hist[bin], 1u);
            }
          }
        }
      }
    };
    bool closure_next = false;
    TeamEntry w_next = fetch_any(0, closure_next);
    for (int rd = 0; rd * kBlock < tot1 + tot2; ++rd) {   // uniform
      const TeamEntry e = w_next;
      const bool closure = closure_next;
      if ((rd + 1) * kBlock < tot1 + tot2) w_next = fetch_any(rd + 1, closure_next);
      winner(e, closure);
    }
    TEAM_STAMP(13);   // (diagnostic: winners among the queues' candidates)
    for_owned_long_arcs([&](const TeamEntry &e) { winner(e, false); });   // (made once more: the same bits)
    __syncthreads();
    TEAM_STAMP(11);   // (diagnostic: winners done)
    // publish (state -> token) of this share, then empty the table for the next frame
    const int n_mine = sh->n_mine < part_cap ? sh->n_mine : part_cap;
    for (uint32_t i = tid; i < slots; i += kBlock) {
      const uint32_t key = hkey[i];
      pub_key[(size_t)me * slots + i] = key;
      if (key != kEmptyKey) pub_lid[(size_t)me * slots + i] = hidx[i];
      hkey[i] = kEmptyKey; hval[i] = kEmptyVal;
    }
    if (last) for (int i = tid + n_mine; i < part_cap; i += kBlock) t_cost[tok0 + i] = __builtin_inff();   // unused places
    if (hist_on) for (int i = tid; i < 256; i += kBlock) if (hist[i]) atomicAdd(&fr->hist[i], hist[i]);
    if (tid == 0) fr->count[me] = n_mine;
    if (lane == 0) {   // (per-wave counters of the frame)
      atomicAdd(&sh->a_active, (unsigned long long)n_active); atomicAdd(&sh->a_emit, (unsigned long long)n_emit);
      atomicAdd(&sh->a_eps, (unsigned long long)n_eps); atomicAdd(&sh->a_cand, (unsigned long long)n_cand);
    }
    TEAM_STAMP(4);
    if (!(alive_team = team_barrier(tc, sh, k, bar_seq, failed))) break;
    TEAM_STAMP(5);
    if (failed != 0) { status = failed; break; }

    // ================= phase 4: records of the closure winners; the next frame's scalars
    {
      const int ncw = sh->n_cwin;
      for (int i = tid; i < ncw; i += kBlock) {
        const TeamClosureWin cw = cwin[i];
        const int o = team_owner(cw.parent_state, k);
        const uint32_t *pk = pub_key + (size_t)o * slots;
        uint32_t h = team_home(cw.parent_state, slots);
        uint32_t probe = 0;
        while (pk[h] != cw.parent_state && probe < slots) {   // (plain reads: the barrier's fence made them current)
          h = h + 1 == slots ? 0 : h + 1; ++probe;
        }
        const int plid = (int)pub_lid[(size_t)o * slots + h];
        bp[n_rec + cw.idx] = make_int2((int)cw.arc, n_rec + o * part_cap + plid);
      }
      int n_total = 0, n_surv = 0;
      for (int s = 0; s < k; ++s) n_total += fr->count[s];
      int cutb = 255;
      if (hist_on && n_total > p.max_active) {
        // (every member computes the same cut from the team's histogram; only wave 0's result is kept)
        if (wave == 0) {
          int loc[4], sum = 0;
#pragma unroll
          for (int q = 0; q < 4; ++q) { loc[q] = (int)fr->hist[lane * 4 + q]; sum += loc[q]; }
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
    TEAM_STAMP(6);
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
        tc->carry_src[i] = lf->big_src[i]; tc->carry_cost[i] = lf->big_cost[i]; tc->carry_id[i] = lf->big_id[i];
      }
#ifdef CBD_PROFILE
      for (int q = 0; q < 7; ++q) cs->spare[q] += tprof[q];
      cs->spare[12] += tprof[7]; cs->spare[13] += tprof[8]; cs->spare[14] += tprof[9];
      cs->spare[7] += tprof[10]; cs->spare[8] += tprof[11]; cs->spare[9] += tprof[12]; cs->spare[10] += tprof[13];
      cs->spare[11] += frames_done;
#endif
      const int n_new = n_rec - cs->gc_base;
      if (p.new_records) p.new_records[c] = make_int2(n_new, p.call_seq);
      if (p.due_max) atomicMax(p.due_max, ((unsigned long long)(uint32_t)p.call_seq << 32) | (uint32_t)n_new);
    }
  }
}

}  // namespace cbd
