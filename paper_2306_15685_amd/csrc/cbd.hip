// Host runtime and C ABI of the decoder: buffer ownership, validation, context
// upload, kernel sequencing.  See include/cbd.h for the contract of each call.
#include "../../include/cbd.h"

#include <algorithm>
#include <atomic>
#include <thread>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <stdexcept>
#include <string>
#include <vector>

#include "cbd_device.hpp"

// Device-side result rows of cbd_best_paths_static (headers, words, arcs): a fixed array in the code object instead
// of buffers from hipMalloc, for callers that must not allocate.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels and copies get
// the device address it returns (static_scratch()).
constexpr size_t kStaticScratchInts = (size_t)2 << 20;   // 8 MiB
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

namespace {

thread_local std::string g_last_error;

constexpr int kMaxDevices = 64;
int32_t *g_scratch_ptr[kMaxDevices] = {};   // per device: where `scratch` lives there

// The address of `scratch` on `device` (made current by the caller), looked up once per device.
hipError_t static_scratch(int device, int32_t **out) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[device]) {
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = (int32_t *)p;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

int32_t fail(int32_t code, const std::string &msg) {
  g_last_error = msg;
  return code;
}

#define HIPCHK(expr)                                                                              \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return fail(CBD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));                  \
  } while (0)

template <typename T> hipError_t dmalloc(T **p, size_t n, size_t *total) {
  size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
  hipError_t e = hipMalloc((void **)p, bytes);
  if (e == hipSuccess && total) *total += bytes;
  return e;
}

// A small ring of pinned host buffers with matching device buffers, so that
// argument lists can be uploaded asynchronously without racing their reuse.
struct StageRing {
  static constexpr int kSlots = 8;
  void *host[kSlots] = {};
  void *dev[kSlots] = {};
  hipEvent_t ev[kSlots] = {};
  bool busy[kSlots] = {};
  size_t cap = 0;
  int next = 0;

  hipError_t init(size_t bytes) {
    cap = bytes;
    for (int i = 0; i < kSlots; ++i) {
      hipError_t e = hipHostMalloc(&host[i], bytes, hipHostMallocDefault);
      if (e != hipSuccess) return e;
      e = hipMalloc(&dev[i], bytes);
      if (e != hipSuccess) return e;
      e = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  void destroy() {
    for (int i = 0; i < kSlots; ++i) {
      if (host[i]) (void)hipHostFree(host[i]);
      if (dev[i]) (void)hipFree(dev[i]);
      if (ev[i]) (void)hipEventDestroy(ev[i]);
    }
  }
  // Returns a slot whose previous upload has been consumed.
  hipError_t acquire(int *slot) {
    int s = next;
    next = (next + 1) % kSlots;
    if (busy[s]) {
      hipError_t e = hipEventSynchronize(ev[s]);
      if (e != hipSuccess) return e;
      busy[s] = false;
    }
    *slot = s;
    return hipSuccess;
  }
  // Upload `bytes` of the slot's host buffer; call release() after the consumer is enqueued.
  hipError_t upload(int s, size_t bytes, hipStream_t st) {
    return hipMemcpyAsync(dev[s], host[s], bytes, hipMemcpyHostToDevice, st);
  }
  hipError_t release(int s, hipStream_t st) {
    if (s < 0) return hipSuccess;   // (nothing was uploaded: the list was already on the device)
    busy[s] = true;
    return hipEventRecord(ev[s], st);
  }
};

}  // namespace

struct cbd_graph {
  int device = 0;
  int32_t S = 0, A = 0, P = 0, start = 0;
  int32_t A_lib = 0;              // records of the library's arc array (arcs + closure lists)
  int4 *d_off2 = nullptr;
  cbd::ArcRec *d_arcs = nullptr;
  int32_t *d_canon = nullptr;
  int32_t *d_int2pub = nullptr;
  int32_t *d_pub2int = nullptr;   // caller's arc numbering -> library numbering (context lists are translated on the device)
  int32_t *d_olabel = nullptr;
  float *d_final = nullptr;
  std::vector<int32_t> pub2int, int2pub;
  // host copy in the caller's numbering, for building contexts from word sequences
  std::vector<int32_t> h_row, h_dst, h_olabel;
  std::vector<int32_t> word_arcs;   // arcs that carry a word, ordered by (word, arc); built on first use
  std::vector<int32_t> word_first;  // [num_words + 2] start of each word's run in word_arcs
  std::vector<int32_t> visit;       // [S] search stamps
  int32_t visit_stamp = 0;
  int32_t max_word = 0;
  int32_t unstored_closures = 0;    // states whose epsilon closure is not stored as a list (too deep or too long)
  std::vector<int4> long_rows;      // states with more than kBigRowArcs emitting arcs: (state, first arc, arcs, 0), by state
  size_t bytes = 0;
};

struct cbd_decoder {
  const cbd_graph *g = nullptr;
  cbd_config cfg{};
  hipStream_t stream = nullptr;
  int32_t C = 0, bp_cap = 0, max_ctx = 0, ctx_lds_cap = 0;
  int32_t lds_tok_cap = 0, lds_slots = 0, lds_log_cap = 0;  // LDS tables (0: unused)
  int32_t g_tok_cap = 0, g_slots = 0, g_log_cap = 0;        // device-memory tables
  int block = 1024;
  int stage_rows = 1;
  int lean_log_per_wave = 0;
  uint32_t lds_bytes = 0;
  cbd::ChanState *d_chan = nullptr;
  int32_t *d_tok_state = nullptr;
  float *d_tok_cost = nullptr;
  int4 *d_tok_row = nullptr;
  int2 *d_bp = nullptr;
  cbd::LogT<false> *d_log = nullptr;
  int32_t *d_ctx = nullptr;      // [C + pool][max_ctx]
  int32_t *d_ctx_n = nullptr;    // [C + pool]
  float *d_ctx_off = nullptr;
  int32_t pool = 0;              // pre-loaded contexts the store has room for
  std::vector<uint8_t> pool_used;
  uint32_t *d_hkey = nullptr;
  uint64_t *d_hval = nullptr;
  uint32_t *d_hidx = nullptr;
  // record compaction: one bit per back-pointer record, and two counts per bitmap word (allocated on first use)
  uint32_t *d_gc_mark = nullptr, *d_gc_prefix = nullptr;
  int32_t *d_gc_cross = nullptr;
  // automatic compaction: each decoding launch leaves (records above gc_base, call number) per channel here (pinned
  // host memory the kernel writes to), so cbd_advance can tell when a compaction is due without synchronising
  int2 *h_new = nullptr, *dv_new = nullptr;
  unsigned long long *d_due_max = nullptr;   // the same for the device: (call number, largest count of that call)
  int64_t last_compact_call = -1;
  // the shared beginning of each channel's paths in time order, as the compactions find it ([C][bp_cap] each)
  int32_t *d_fixed_arcs = nullptr, *d_fixed_words = nullptr;
  int32_t gc_words = 0;
  // best-path results: slot 0 serves the synchronous calls, the others asynchronous requests
  static constexpr int kOutSlots = 5;
  struct OutSlot {
    int32_t *d_arcs = nullptr, *d_snap = nullptr;
    int32_t *h_arcs = nullptr, *h_words = nullptr, *h_meta = nullptr;   // pinned
    // words and the per-channel header are written by the kernels straight into the pinned host buffers (through
    // these device-side addresses): no copy, and no copy kernel competing with the decoding for compute units
    int32_t *dv_words = nullptr, *dv_meta = nullptr;
    int32_t rows = 0, capacity = 0;
    int32_t n = 0, req_capacity = 0;
    bool want_arcs = false, pending = false, tail_only = false;
    int snap_slot = -1;   // ring slot of d_auto_snap the request reads (-1: its own snapshot)
    hipEvent_t done = nullptr;
  } out[kOutSlots];
  hipStream_t side = nullptr;      // walks and copies of asynchronous requests
  bool walk_room = false;          // the LDS layout leaves room for walks beside a decoding workgroup
  int walk_room_min_grid = 0;      // calls with at least this many channels use it
  // Best-token snapshots left by the decoding kernel itself, one ring slot per advance / reset call
  static constexpr int kSnapRing = 8;
  int32_t *d_auto_snap = nullptr;  // [kSnapRing][C][kSnapInts]
  int64_t adv_calls = 0;           // advance / reset calls so far
  std::vector<int32_t> last_list;  // channel list of the latest one (empty: none)
  hipEvent_t snap_ev = nullptr;
  StageRing ids;   // channel lists
  // A server passes the same channel list call after call: the second time in a row a list is seen it is kept
  // on the device, and calls with that list upload nothing (one small copy kernel and its gap less per call).
  int32_t *d_ids_kept = nullptr;
  std::vector<int32_t> kept_ids, last_ids;
  StageRing ctxs;  // context uploads
  // teams (workgroups_per_channel > 1)
  int team_k = 0, team_block = 1024, team_slots = 0, team_part_cap = 0, team_q_cap = 0, team_stage_rows = 0;
  uint32_t team_lds = 0;
  cbd::TeamChan *d_team = nullptr;
  cbd::TeamEntry *d_team_q1 = nullptr, *d_team_q2 = nullptr;
  cbd::TeamClosureWin *d_team_cwin = nullptr;
  uint32_t *d_team_pub_key = nullptr;
  uint16_t *d_team_pub_lid = nullptr;
  int4 *d_team_big_rows = nullptr;
  int32_t *d_team_big_group = nullptr, *d_team_big_perm = nullptr;
  int32_t team_n_big_rows = 0;
  std::vector<int32_t> h_tmp;
  std::vector<int32_t> h_static_meta;   // result headers of cbd_best_paths_static on their way to the caller
  size_t bytes = 0;
};

namespace {

using cbd::AdvanceParams;

template <int kBlock> hipError_t launch_advance_t(const AdvanceParams &p, int grid, uint32_t lds, hipStream_t st) {
  hipLaunchKernelGGL((cbd::advance_kernel<kBlock>), dim3(grid), dim3(kBlock), lds, st, p);
  return hipGetLastError();
}

template <int kBlock> hipError_t set_attr_t(uint32_t lds) {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&cbd::advance_kernel<kBlock>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

hipError_t set_attr(int block, uint32_t lds) {
  if (block == 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&cbd::advance_beside_kernel<1024>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (block == 256) return set_attr_t<256>(lds);
  if (block == 512) return set_attr_t<512>(lds);
  if (block == 960) return set_attr_t<960>(lds);
  return set_attr_t<1024>(lds);
}

// Workgroups of the decode kernel that one compute unit holds at once (registers, waves and LDS together).
hipError_t resident_per_cu(int block, uint32_t lds, int *n) {
  if (block == 256) return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, cbd::advance_kernel<256>, 256, lds);
  if (block == 512) return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, cbd::advance_kernel<512>, 512, lds);
  if (block == 960) return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, cbd::advance_kernel<960>, 960, lds);
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(n, cbd::advance_kernel<1024>, 1024, lds);
}

// A team launch.  The members of a team wait for one another inside the kernel, so all of a launch's workgroups
// have to become resident without waiting for one another: the grid never exceeds the device's compute units
// (checked when the decoder is made), a workgroup fills a compute unit's LDS, launches of one decoder follow one
// another on its stream, and whatever else runs on the device (result walks on the side stream) is finite.  The
// members' polls are bounded all the same.
hipError_t launch_team(const cbd_decoder *d, const AdvanceParams &p, int n_channels) {
  cbd::TeamParams tp{};
  tp.a = p;
  tp.team = d->d_team; tp.q1 = d->d_team_q1; tp.q2 = d->d_team_q2; tp.cwin = d->d_team_cwin;
  tp.pub_key = d->d_team_pub_key; tp.pub_lid = d->d_team_pub_lid;
  tp.big_rows = d->d_team_big_rows; tp.big_group = d->d_team_big_group; tp.big_perm = d->d_team_big_perm;
  tp.n_big_rows = d->team_n_big_rows;
  // (teams padded to a multiple of 8 where the device has room: see the kernel's note on dies)
  int n_cu = 0;
  (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, d->g->device);
  int padded = (n_channels + 7) / 8 * 8;
  if ((int64_t)padded * d->team_k > n_cu) padded = n_channels;
  tp.n_teams = n_channels;
  tp.k = d->team_k; tp.q_cap = d->team_q_cap; tp.part_cap = d->team_part_cap; tp.slots = d->team_slots;
  tp.stage_rows = d->team_stage_rows; tp.ctx_lds_cap = d->ctx_lds_cap;
  hipLaunchKernelGGL(cbd::advance_team_kernel<1024>, dim3((unsigned)(padded * d->team_k)), dim3(1024), d->team_lds, d->stream, tp);
  return hipGetLastError();
}

// Has the caller begun a request for results that it has not finished yet?  Its walk may then still be on the side
// stream when the launch starts.  (Asked of the host's own bookkeeping, not of the event: what a call does should
// not depend on how far the device has come.)
bool walks_in_flight(const cbd_decoder *d) {
  for (int k = 1; k < cbd_decoder::kOutSlots; ++k)
    if (d->out[k].pending) return true;
  return false;
}

hipError_t launch_advance(const cbd_decoder *d, const AdvanceParams &p, int grid) {
  if (d->walk_room && d->block == 1024 && grid >= d->walk_room_min_grid && walks_in_flight(d)) {
    // leave the walks room on the compute units (see advance_beside_kernel)
    hipLaunchKernelGGL((cbd::advance_beside_kernel<1024>), dim3(grid), dim3(1024), d->lds_bytes, d->stream, p);
    return hipGetLastError();
  }
  if (d->block == 256) return launch_advance_t<256>(p, grid, d->lds_bytes, d->stream);
  if (d->block == 512) return launch_advance_t<512>(p, grid, d->lds_bytes, d->stream);
  if (d->block == 960) return launch_advance_t<960>(p, grid, d->lds_bytes, d->stream);
  return launch_advance_t<1024>(p, grid, d->lds_bytes, d->stream);
}

AdvanceParams base_params(const cbd_decoder *d) {
  AdvanceParams p{};
  p.off2 = d->g->d_off2; p.arcs = d->g->d_arcs; p.canon = d->g->d_canon; p.start_state = d->g->start; p.num_pdfs = d->g->P;
  p.chan = d->d_chan;
  p.beam = d->cfg.beam; p.max_active = d->cfg.max_active; p.max_eps_iters = d->cfg.max_eps_iters;
  p.lookup_mode = d->cfg.lookup_mode;
  p.lds_tok_cap = d->lds_tok_cap; p.lds_slots = d->lds_slots; p.lds_log_cap = d->lds_log_cap;
  p.g_tok_cap = d->g_tok_cap; p.g_slots = d->g_slots; p.g_log_cap = d->g_log_cap;
  p.bp_cap = d->bp_cap; p.max_ctx = d->max_ctx; p.ctx_lds_cap = d->ctx_lds_cap; p.stage_rows = d->stage_rows;
  p.lean_frames = d->cfg.frame_code == 0 && d->lean_log_per_wave > 0 ? 1 : 0;
  p.lean_log_per_wave = d->lean_log_per_wave;
  p.tok_state = d->d_tok_state; p.tok_cost = d->d_tok_cost;
  p.tok_row = d->d_tok_row;
  p.bp = d->d_bp; p.g_log = d->d_log; p.ctx = d->d_ctx; p.ctx_n = d->d_ctx_n; p.ctx_off = d->d_ctx_off;
  p.g_hkey = d->d_hkey; p.g_hval = d->d_hval; p.g_hidx = d->d_hidx;
  return p;
}

void free_out_slot(cbd_decoder::OutSlot &o) {
  if (o.d_arcs) (void)hipFree(o.d_arcs);
  if (o.d_snap) (void)hipFree(o.d_snap);
  if (o.h_arcs) (void)hipHostFree(o.h_arcs);
  if (o.h_words) (void)hipHostFree(o.h_words);
  if (o.h_meta) (void)hipHostFree(o.h_meta);
  o.d_arcs = o.d_snap = o.h_arcs = o.h_words = o.h_meta = o.dv_words = o.dv_meta = nullptr;
  o.rows = o.capacity = 0;
}

// Makes the slot's buffers hold at least n rows of `capacity` entries (the slot must be idle).
int32_t size_out_slot(cbd_decoder *d, cbd_decoder::OutSlot &o, int32_t n, int32_t capacity) {
  if (o.capacity >= capacity && o.rows >= n) return CBD_OK;
  const int32_t rows = std::max(n, o.rows), cap = std::max(capacity, o.capacity);
  HIPCHK(hipStreamSynchronize(d->stream));
  free_out_slot(o);
  HIPCHK(dmalloc(&o.d_arcs, (size_t)rows * cap, nullptr));
  HIPCHK(dmalloc(&o.d_snap, (size_t)rows * cbd::kSnapInts, nullptr));
  HIPCHK(hipHostMalloc((void **)&o.h_arcs, sizeof(int32_t) * (size_t)rows * cap, hipHostMallocDefault));
  HIPCHK(hipHostMalloc((void **)&o.h_words, sizeof(int32_t) * (size_t)rows * cap, hipHostMallocDefault));
  HIPCHK(hipHostMalloc((void **)&o.h_meta, sizeof(int32_t) * (size_t)rows * cbd::kMetaInts, hipHostMallocDefault));
  HIPCHK(hipHostGetDevicePointer((void **)&o.dv_words, o.h_words, 0));
  HIPCHK(hipHostGetDevicePointer((void **)&o.dv_meta, o.h_meta, 0));
  o.rows = rows; o.capacity = cap;
  return CBD_OK;
}

cbd::BestParams best_params(const cbd_decoder *d, const cbd_decoder::OutSlot &o, const int32_t *chan_ids,
                            int32_t use_final, int32_t capacity, bool tail_only) {
  cbd::BestParams bp{};
  bp.chan = d->d_chan; bp.chan_ids = chan_ids; bp.tok_state = d->d_tok_state; bp.tok_cost = d->d_tok_cost;
  bp.bp = d->d_bp; bp.olabel = d->g->d_olabel; bp.int2pub = d->g->d_int2pub; bp.final_cost = d->g->d_final;
  bp.tok_cap = d->g_tok_cap; bp.bp_cap = d->bp_cap; bp.use_final = use_final; bp.capacity = capacity;
  bp.row_pitch = o.capacity;
  bp.tail_only = tail_only ? 1 : 0;
  bp.fixed_arcs = d->d_fixed_arcs; bp.fixed_words = d->d_fixed_words; bp.fixed_cap = d->bp_cap;
  bp.out_arcs = o.d_arcs; bp.out_words = o.dv_words; bp.out_meta = o.dv_meta; bp.snap = o.d_snap;
  return bp;
}

// Waits for the kernels on stream `st` (headers and words are then in the slot's pinned host buffers), copies as
// many columns of the arc rows as the longest path needs if arcs are wanted, and hands the rows to the caller.
int32_t fetch_results(cbd_decoder *d, cbd_decoder::OutSlot &o, hipStream_t st, int32_t n, int32_t capacity,
                      int32_t *words, int32_t *arcs, int32_t *n_words, int32_t *n_arcs, float *cost,
                      int32_t *status, int32_t *n_fixed_words = nullptr, int32_t *n_fixed_arcs = nullptr) {
  constexpr size_t M = cbd::kMetaInts;
  int32_t *meta = o.h_meta;
  HIPCHK(hipStreamSynchronize(st));   // the kernel has written headers and words into host memory
  if (arcs) {
    int32_t max_na = 0;
    for (int32_t i = 0; i < n; ++i)
      if (meta[(size_t)i * M] == CBD_OK) max_na = std::max(max_na, meta[(size_t)i * M + 1]);
    const size_t pitch = sizeof(int32_t) * (size_t)o.capacity;
    if (max_na > 0) {
      HIPCHK(hipMemcpy2DAsync(o.h_arcs, pitch, o.d_arcs, pitch, sizeof(int32_t) * (size_t)max_na, (size_t)n,
                              hipMemcpyDeviceToHost, st));
      HIPCHK(hipStreamSynchronize(st));
    }
  }
  for (int32_t i = 0; i < n; ++i) {
    status[i] = meta[(size_t)i * M + 0];
    n_arcs[i] = meta[(size_t)i * M + 1];
    n_words[i] = meta[(size_t)i * M + 2];
    if (n_fixed_arcs) n_fixed_arcs[i] = meta[(size_t)i * M + 4];
    if (n_fixed_words) n_fixed_words[i] = meta[(size_t)i * M + 5];
    uint32_t bits = (uint32_t)meta[(size_t)i * M + 3];
    memcpy(&cost[i], &bits, 4);
    if (status[i] != CBD_OK) continue;
    memcpy(words + (size_t)i * capacity, o.h_words + (size_t)i * o.capacity, sizeof(int32_t) * (size_t)n_words[i]);
    if (arcs)
      memcpy(arcs + (size_t)i * capacity, o.h_arcs + (size_t)i * o.capacity, sizeof(int32_t) * (size_t)n_arcs[i]);
  }
  return CBD_OK;
}

// Gives the coming advance / reset call the next slot of the snapshot ring (the stream first waits for any
// unfinished request that still reads that slot) and remembers the call's channel list.
int32_t claim_snapshot_slot(cbd_decoder *d, const int32_t *channels, int32_t n, AdvanceParams *p) {
  const int s = (int)(d->adv_calls % cbd_decoder::kSnapRing);
  for (int k = 1; k < cbd_decoder::kOutSlots; ++k)
    if (d->out[k].pending && d->out[k].snap_slot == s) HIPCHK(hipStreamWaitEvent(d->stream, d->out[k].done, 0));
  p->auto_snap = d->d_auto_snap + (size_t)s * d->C * cbd::kSnapInts;
  d->last_list.assign(channels, channels + n);
  d->adv_calls++;
  return CBD_OK;
}

// Validates a channel list and uploads it; *dev receives the device copy.
int32_t stage_channels(cbd_decoder *d, const int32_t *channels, int32_t n, const int32_t **dev, int *slot) {
  if (!channels || n <= 0 || n > d->C) return fail(CBD_E_INVALID, "channel list: bad length");
  if ((size_t)n == d->kept_ids.size() && memcmp(channels, d->kept_ids.data(), sizeof(int32_t) * (size_t)n) == 0) {
    *dev = d->d_ids_kept;   // checked and uploaded before
    *slot = -1;
    return CBD_OK;
  }
  d->h_tmp.assign((size_t)d->C, 0);
  for (int32_t i = 0; i < n; ++i) {
    int32_t c = channels[i];
    if (c < 0 || c >= d->C) return fail(CBD_E_INVALID, "channel list: index out of range");
    if (d->h_tmp[c]) return fail(CBD_E_INVALID, "channel list: duplicate channel");
    d->h_tmp[c] = 1;
  }
  HIPCHK(d->ids.acquire(slot));
  memcpy(d->ids.host[*slot], channels, sizeof(int32_t) * (size_t)n);
  HIPCHK(d->ids.upload(*slot, sizeof(int32_t) * (size_t)n, d->stream));
  *dev = (const int32_t *)d->ids.dev[*slot];
  if ((size_t)n == d->last_ids.size() && memcmp(channels, d->last_ids.data(), sizeof(int32_t) * (size_t)n) == 0) {
    // (stream-ordered like every use of the kept copy, so kernels already enqueued with it are not disturbed)
    HIPCHK(hipMemcpyAsync(d->d_ids_kept, d->ids.dev[*slot], sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice,
                          d->stream));
    d->kept_ids = d->last_ids;
  } else {
    d->last_ids.assign(channels, channels + n);
  }
  return CBD_OK;
}

// Enqueues the record compaction for the channels in `dev` (a staged list of n).  It renumbers records, so the
// stream first waits for every unfinished asynchronous walk, and snapshots left by earlier calls are retired.
// due_seq >= 0: channels half-way to min_new join in if call due_seq left a count above min_new (automatic mode).
int32_t enqueue_compaction(cbd_decoder *d, const int32_t *dev, int32_t n, int32_t min_new, int64_t due_seq = -1) {
  d->gc_words = (d->bp_cap + 31) / 32;
  if (!d->d_gc_mark) HIPCHK(dmalloc(&d->d_gc_mark, (size_t)d->C * d->gc_words, &d->bytes));
  if (!d->d_gc_prefix) HIPCHK(dmalloc(&d->d_gc_prefix, (size_t)d->C * d->gc_words, &d->bytes));
  if (!d->d_gc_cross) HIPCHK(dmalloc(&d->d_gc_cross, (size_t)d->C * (d->gc_words + 2), &d->bytes));
  if (!d->d_fixed_arcs) HIPCHK(dmalloc(&d->d_fixed_arcs, (size_t)d->C * d->bp_cap, &d->bytes));
  if (!d->d_fixed_words) HIPCHK(dmalloc(&d->d_fixed_words, (size_t)d->C * d->bp_cap, &d->bytes));
  for (int k = 1; k < cbd_decoder::kOutSlots; ++k)
    if (d->out[k].pending) HIPCHK(hipStreamWaitEvent(d->stream, d->out[k].done, 0));
  d->last_list.clear();
  cbd::CompactParams cp{};
  cp.chan = d->d_chan; cp.chan_ids = dev; cp.bp = d->d_bp; cp.tok_cost = d->d_tok_cost;
  cp.mark = d->d_gc_mark; cp.prefix = d->d_gc_prefix; cp.cross = d->d_gc_cross;
  cp.bp_cap = d->bp_cap; cp.tok_cap = d->g_tok_cap; cp.mark_words = d->gc_words; cp.min_new = min_new;
  cp.fixed_arcs = d->d_fixed_arcs; cp.fixed_words = d->d_fixed_words; cp.fixed_cap = d->bp_cap;
  cp.olabel = d->g->d_olabel; cp.int2pub = d->g->d_int2pub;
  if (due_seq >= 0) { cp.due_max = d->d_due_max; cp.due_seq = (int32_t)due_seq; }
  hipLaunchKernelGGL(cbd::compact_records_kernel, dim3((unsigned)n), dim3(cbd::kCompactBlock), 0, d->stream, cp);
  HIPCHK(hipGetLastError());
  return CBD_OK;
}

}  // namespace

extern "C" {

const char *cbd_strerror(int32_t status) {
  switch (status) {
    case CBD_OK: return "ok";
    case CBD_E_INVALID: return "invalid argument";
    case CBD_E_CAPACITY: return "channel capacity exceeded (token table, change log or back-pointers)";
    case CBD_E_EPS_DIVERGED: return "epsilon closure did not converge";
    case CBD_E_NO_TOKENS: return "no tokens (dead end or channel not reset)";
    case CBD_E_BUFFER: return "output buffer too small";
    case CBD_E_HIP: return "HIP runtime error";
    case CBD_E_NOMEM: return "out of memory";
    default: return "unknown status";
  }
}

const char *cbd_last_error(void) { return g_last_error.c_str(); }

int32_t cbd_graph_load(const cbd_graph_desc *desc, cbd_graph **out) try {
  if (!desc || !out) return fail(CBD_E_INVALID, "graph: null argument");
  const int32_t S = desc->num_states, A = desc->num_arcs, P = desc->num_pdfs;
  if (S <= 0 || A < 0 || P <= 0 || desc->start_state < 0 || desc->start_state >= S)
    return fail(CBD_E_INVALID, "graph: bad sizes");
  if (P > 65535) return fail(CBD_E_INVALID, "graph: more than 65535 pdfs (the arc record keeps ilabel in 16 bits)");
  if (!desc->row_offsets || (A > 0 && (!desc->dst || !desc->ilabel || !desc->olabel || !desc->weight)))
    return fail(CBD_E_INVALID, "graph: null array");
  const int32_t *row = desc->row_offsets;
  if (row[0] != 0 || row[S] != A) return fail(CBD_E_INVALID, "graph: row_offsets must span [0, num_arcs]");
  for (int32_t s = 0; s < S; ++s)
    if (row[s + 1] < row[s]) return fail(CBD_E_INVALID, "graph: row_offsets not monotone");
  for (int32_t a = 0; a < A; ++a) {
    if (desc->dst[a] < 0 || desc->dst[a] >= S) return fail(CBD_E_INVALID, "graph: dst out of range");
    if (desc->ilabel[a] < 0 || desc->ilabel[a] > P) return fail(CBD_E_INVALID, "graph: ilabel out of range");
    if (desc->olabel[a] < 0) return fail(CBD_E_INVALID, "graph: negative olabel");
    if (!std::isfinite(desc->weight[a])) return fail(CBD_E_INVALID, "graph: non-finite weight");
  }
  if (desc->final_cost)
    for (int32_t s = 0; s < S; ++s)   // +inf marks a state that is not final
      if (std::isnan(desc->final_cost[s]) || desc->final_cost[s] == -INFINITY)
        return fail(CBD_E_INVALID, "graph: final_cost must be finite or +inf");
  cbd_graph *g = new (std::nothrow) cbd_graph();
  if (!g) return fail(CBD_E_NOMEM, "graph: host allocation");
  struct Guard {   // frees the half-built graph if anything below throws
    cbd_graph *g;
    ~Guard() { if (g) cbd_graph_free(g); }
  } guard{g};
  g->S = S; g->A = A; g->P = P; g->start = desc->start_state;
  g->h_row.assign(row, row + S + 1);
  g->h_dst.assign(desc->dst, desc->dst + A);
  g->h_olabel.assign(desc->olabel, desc->olabel + A);
  if (hipGetDevice(&g->device) != hipSuccess) return fail(CBD_E_HIP, "hipGetDevice failed");
  // Library order: per state, its emitting arcs, then its epsilon-input arcs (each in the caller's order), then
  // its closure list: one record per path of epsilon-input arcs that starts at the state, depth-first, parents
  // before children.  A state whose closure is deeper than kClosureMaxDepth or longer than the count field holds
  // gets no list (the decoding kernel then takes the general closure code for it).
  std::vector<int32_t> n_emit((size_t)S, 0), n_eps((size_t)S, 0), n_clo((size_t)S, 0);
  for (int32_t s = 0; s < S; ++s)
    for (int32_t a = row[s]; a < row[s + 1]; ++a) (desc->ilabel[a] != 0 ? n_emit : n_eps)[(size_t)s]++;
  struct Frame { int32_t next, end, depth, parent1; };
  std::vector<Frame> stack;
  // walks the closure of s depth-first; visit(arc, depth, parent1) per record, parent1 = position of the record
  // of the arc's source state in the list + 1 (0: s itself); false if the closure is too deep or too long
  auto walk_closure = [&](int32_t s, auto &&visit) -> bool {
    stack.clear();
    stack.push_back({row[s], row[s + 1], 1, 0});
    int32_t count = 0;
    while (!stack.empty()) {
      Frame &f = stack.back();
      while (f.next < f.end && desc->ilabel[f.next] != 0) ++f.next;
      if (f.next >= f.end) { stack.pop_back(); continue; }
      const int32_t a = f.next++;
      const int32_t depth = f.depth, parent1 = f.parent1;
      if (depth > cbd::kClosureMaxDepth || ++count >= (int32_t)cbd::kClEscape) return false;
      visit(a, depth, parent1);
      const int32_t t = desc->dst[a];
      if (n_eps[(size_t)t] > 0) stack.push_back({row[t], row[t + 1], depth + 1, count});   // (f is dead after this)
    }
    return true;
  };
  constexpr int32_t kNoList = -1;
  for (int32_t s = 0; s < S; ++s) {
    if (n_eps[(size_t)s] == 0) continue;
    int32_t cnt = 0;
    const bool ok = n_emit[(size_t)s] < (int32_t)cbd::kEdEscape && n_eps[(size_t)s] < (int32_t)cbd::kXdEscape &&
                    walk_closure(s, [&](int32_t, int32_t, int32_t) { ++cnt; });
    n_clo[(size_t)s] = ok ? cnt : kNoList;
    if (!ok) g->unstored_closures += 1;
  }
  std::vector<int4> off2((size_t)S);
  int64_t total = 0;
  for (int32_t s = 0; s < S; ++s) {
    const int64_t first = total, eps = first + n_emit[(size_t)s], end_x = eps + n_eps[(size_t)s];
    total = end_x + std::max(n_clo[(size_t)s], 0);
    if (total > 0x7FFFFFF0) return fail(CBD_E_INVALID, "graph: too many arc records");
    off2[(size_t)s] = make_int4((int)first, (int)eps, (int)end_x, (int)total);
    if (n_emit[(size_t)s] > cbd::kBigRowArcs) g->long_rows.push_back(make_int4(s, (int)first, n_emit[(size_t)s], 0));
  }
  const int32_t AL = (int32_t)total;   // records in the library's arc array
  g->A_lib = AL;
  std::vector<cbd::ArcRec> arcs((size_t)std::max(AL, 1));
  std::vector<int32_t> canon((size_t)std::max(AL, 1)), olab((size_t)std::max(AL, 1));
  g->pub2int.resize((size_t)std::max(A, 1));
  g->int2pub.resize((size_t)std::max(AL, 1));
  for (int32_t s = 0; s < S; ++s) {
    int32_t ke = off2[(size_t)s].x, kx = off2[(size_t)s].y;
    for (int32_t a = row[s]; a < row[s + 1]; ++a) {
      int32_t &k = desc->ilabel[a] != 0 ? ke : kx;
      g->pub2int[(size_t)a] = k;
      ++k;
    }
  }
  auto record_of = [&](int32_t a, uint32_t low16) {
    const int32_t dst = desc->dst[a];
    cbd::ArcRec r;
    r.dst = dst;
    r.weight = desc->weight[a];
    r.row = off2[(size_t)dst].x;
    const int32_t cl = n_clo[(size_t)dst];
    r.meta = cbd::make_meta(low16, (uint32_t)n_emit[(size_t)dst], (uint32_t)n_eps[(size_t)dst],
                            cl == kNoList ? cbd::kClEscape : (uint32_t)cl);
    return r;
  };
  for (int32_t a = 0; a < A; ++a) {
    const int32_t i = g->pub2int[(size_t)a];
    arcs[(size_t)i] = record_of(a, (uint32_t)desc->ilabel[a]);
    canon[(size_t)i] = i;
    g->int2pub[(size_t)i] = a;
    olab[(size_t)i] = desc->olabel[a];
  }
  for (int32_t s = 0; s < S; ++s) {
    if (n_clo[(size_t)s] <= 0) continue;
    int32_t k = off2[(size_t)s].z;
    walk_closure(s, [&](int32_t a, int32_t depth, int32_t parent1) {
      arcs[(size_t)k] = record_of(a, (uint32_t)depth | ((uint32_t)parent1 << 4));
      canon[(size_t)k] = g->pub2int[(size_t)a];
      g->int2pub[(size_t)k] = a;
      olab[(size_t)k] = desc->olabel[a];
      ++k;
    });
  }
#define GCHK(expr)                                                                     \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) {                                                            \
      return fail(CBD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));       \
    }                                                                                  \
  } while (0)
  GCHK(dmalloc(&g->d_off2, (size_t)S, &g->bytes));
  GCHK(dmalloc(&g->d_arcs, (size_t)AL, &g->bytes));
  GCHK(dmalloc(&g->d_canon, (size_t)AL, &g->bytes));
  GCHK(dmalloc(&g->d_int2pub, (size_t)AL, &g->bytes));
  GCHK(dmalloc(&g->d_pub2int, (size_t)A, &g->bytes));
  GCHK(dmalloc(&g->d_olabel, (size_t)AL, &g->bytes));
  GCHK(hipMemcpy(g->d_off2, off2.data(), sizeof(int4) * (size_t)S, hipMemcpyHostToDevice));
  if (A > 0) {
    GCHK(hipMemcpy(g->d_arcs, arcs.data(), sizeof(cbd::ArcRec) * (size_t)AL, hipMemcpyHostToDevice));
    GCHK(hipMemcpy(g->d_canon, canon.data(), sizeof(int32_t) * (size_t)AL, hipMemcpyHostToDevice));
    GCHK(hipMemcpy(g->d_int2pub, g->int2pub.data(), sizeof(int32_t) * (size_t)AL, hipMemcpyHostToDevice));
    GCHK(hipMemcpy(g->d_pub2int, g->pub2int.data(), sizeof(int32_t) * (size_t)A, hipMemcpyHostToDevice));
    GCHK(hipMemcpy(g->d_olabel, olab.data(), sizeof(int32_t) * (size_t)AL, hipMemcpyHostToDevice));
  }
  if (desc->final_cost) {
    GCHK(dmalloc(&g->d_final, (size_t)S, &g->bytes));
    GCHK(hipMemcpy(g->d_final, desc->final_cost, sizeof(float) * (size_t)S, hipMemcpyHostToDevice));
  }
#undef GCHK
  guard.g = nullptr;
  *out = g;
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "graph_load: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("graph_load: ") + e.what());
}

namespace {

// source state of an arc in the caller's numbering
int32_t arc_source(const cbd_graph *g, int32_t a) {
  return (int32_t)(std::upper_bound(g->h_row.begin(), g->h_row.end(), a) - g->h_row.begin()) - 1;
}

void build_word_index(cbd_graph *g) {
  if (!g->word_first.empty()) return;
  int32_t mw = 0;
  for (int32_t w : g->h_olabel) mw = std::max(mw, w);
  g->max_word = mw;
  g->word_first.assign((size_t)mw + 2, 0);
  for (int32_t w : g->h_olabel)
    if (w > 0) g->word_first[(size_t)w + 1]++;
  for (size_t w = 1; w < g->word_first.size(); ++w) g->word_first[w] += g->word_first[w - 1];
  g->word_arcs.resize((size_t)g->word_first.back());
  std::vector<int32_t> fill(g->word_first.begin(), g->word_first.end() - 1);
  for (int32_t a = 0; a < g->A; ++a) {
    int32_t w = g->h_olabel[(size_t)a];
    if (w > 0) g->word_arcs[(size_t)fill[(size_t)w]++] = a;
  }
  g->visit.assign((size_t)g->S, 0);
}

bool state_outputs(const cbd_graph *g, int32_t s, int32_t w) {
  for (int32_t a = g->h_row[(size_t)s]; a < g->h_row[(size_t)s + 1]; ++a)
    if (g->h_olabel[(size_t)a] == w) return true;
  return false;
}

// Algorithm 1 for one word sequence; arcs are appended to `out` (duplicates possible).
void arcs_for_sequence(cbd_graph *g, const int32_t *words, int32_t k, std::vector<int32_t> &out) {
  if (k <= 0) return;
  auto run = [&](int32_t w, const int32_t **b, const int32_t **e) {
    if (w <= 0 || w > g->max_word) { *b = *e = nullptr; return; }
    *b = g->word_arcs.data() + g->word_first[(size_t)w];
    *e = g->word_arcs.data() + g->word_first[(size_t)w + 1];
  };
  // states that output w_1: the sequence may start anywhere (Sec. 4.1)
  std::vector<int32_t> reached, next, stack;
  const int32_t *b, *e;
  run(words[0], &b, &e);
  for (const int32_t *p = b; p != e; ++p) reached.push_back(arc_source(g, *p));
  std::sort(reached.begin(), reached.end());
  reached.erase(std::unique(reached.begin(), reached.end()), reached.end());
  for (int32_t t = 1; t < k; ++t) {
    const int32_t w_prev = words[t - 1], w_next = words[t];
    next.clear();
    if (++g->visit_stamp == 0x7FFFFFFF) { std::fill(g->visit.begin(), g->visit.end(), 0); g->visit_stamp = 1; }
    const int32_t stamp = g->visit_stamp;
    for (int32_t s_p : reached) {
      // leave s_p through an arc that outputs the previous word, then follow arcs without output
      // label; states on the way that can output the next word are where the sequence continues
      for (int32_t a = g->h_row[(size_t)s_p]; a < g->h_row[(size_t)s_p + 1]; ++a) {
        if (g->h_olabel[(size_t)a] != w_prev) continue;
        out.push_back(a);
        stack.push_back(g->h_dst[(size_t)a]);
      }
      while (!stack.empty()) {
        int32_t q = stack.back();
        stack.pop_back();
        if (g->visit[(size_t)q] == stamp) continue;   // shared by all s_p of this step: the result is a union
        g->visit[(size_t)q] = stamp;
        if (state_outputs(g, q, w_next)) next.push_back(q);
        for (int32_t a = g->h_row[(size_t)q]; a < g->h_row[(size_t)q + 1]; ++a)
          if (g->h_olabel[(size_t)a] == 0) stack.push_back(g->h_dst[(size_t)a]);
      }
    }
    std::sort(next.begin(), next.end());
    next.erase(std::unique(next.begin(), next.end()), next.end());
    reached.swap(next);
  }
  const int32_t w_last = words[k - 1];
  for (int32_t s : reached)
    for (int32_t a = g->h_row[(size_t)s]; a < g->h_row[(size_t)s + 1]; ++a)
      if (g->h_olabel[(size_t)a] == w_last) out.push_back(a);
}

}  // namespace

int32_t cbd_context_from_words(cbd_graph *g, const int32_t *words, const int32_t *seq_offsets, int32_t n_seq,
                               int32_t *arcs, int32_t capacity, int32_t *n_arcs) try {
  if (!g || !seq_offsets || !n_arcs) return fail(CBD_E_INVALID, "context_from_words: null argument");
  if (n_seq < 0 || seq_offsets[0] != 0) return fail(CBD_E_INVALID, "context_from_words: bad sequence offsets");
  for (int32_t i = 0; i < n_seq; ++i)
    if (seq_offsets[i + 1] < seq_offsets[i]) return fail(CBD_E_INVALID, "context_from_words: offsets not monotone");
  if (n_seq > 0 && seq_offsets[n_seq] > 0 && !words) return fail(CBD_E_INVALID, "context_from_words: null words");
  build_word_index(g);
  std::vector<int32_t> out;
  for (int32_t i = 0; i < n_seq; ++i)
    arcs_for_sequence(g, words + seq_offsets[i], seq_offsets[i + 1] - seq_offsets[i], out);
  std::sort(out.begin(), out.end());
  out.erase(std::unique(out.begin(), out.end()), out.end());
  *n_arcs = (int32_t)out.size();
  if ((int32_t)out.size() > capacity) return CBD_E_BUFFER;
  if (!out.empty()) {
    if (!arcs) return fail(CBD_E_INVALID, "context_from_words: null output");
    memcpy(arcs, out.data(), sizeof(int32_t) * out.size());
  }
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "context_from_words: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("context_from_words: ") + e.what());
}

int32_t cbd_graph_free(cbd_graph *g) {
  if (!g) return CBD_OK;
  if (g->d_off2) (void)hipFree(g->d_off2);
  if (g->d_arcs) (void)hipFree(g->d_arcs);
  if (g->d_canon) (void)hipFree(g->d_canon);
  if (g->d_int2pub) (void)hipFree(g->d_int2pub);
  if (g->d_pub2int) (void)hipFree(g->d_pub2int);
  if (g->d_olabel) (void)hipFree(g->d_olabel);
  if (g->d_final) (void)hipFree(g->d_final);
  delete g;
  return CBD_OK;
}

int32_t cbd_decoder_create(const cbd_graph *g, const cbd_config *cfg, void *hip_stream, cbd_decoder **out) try {
  if (!g || !cfg || !out) return fail(CBD_E_INVALID, "decoder: null argument");
  if (cfg->num_channels < 1) return fail(CBD_E_INVALID, "decoder: num_channels < 1");
  if (!(cfg->beam >= 0.0f)) return fail(CBD_E_INVALID, "decoder: beam must be >= 0");
  if (cfg->max_active < 0 || cfg->max_frames < 1 || cfg->max_context_arcs < 0)
    return fail(CBD_E_INVALID, "decoder: negative size");
  if (cfg->lookup_mode < 0 || cfg->lookup_mode > 1) return fail(CBD_E_INVALID, "decoder: lookup_mode");
  if (cfg->hash_capacity_log2 < 6 || cfg->hash_capacity_log2 > 24)
    return fail(CBD_E_INVALID, "decoder: hash_capacity_log2 must be in [6, 24]");
  if (cfg->table_location < 0 || cfg->table_location > 2) return fail(CBD_E_INVALID, "decoder: table_location");
  if (cfg->lds_token_cap < 0) return fail(CBD_E_INVALID, "decoder: lds_token_cap");
  if (cfg->max_pool_contexts < 0) return fail(CBD_E_INVALID, "decoder: max_pool_contexts");
  if (cfg->workgroups_per_cu < 0 || cfg->workgroups_per_cu > 4) return fail(CBD_E_INVALID, "decoder: workgroups_per_cu");
  if (cfg->compact_records_above < 0) return fail(CBD_E_INVALID, "decoder: compact_records_above");
  if (cfg->frame_code < 0 || cfg->frame_code > 1) return fail(CBD_E_INVALID, "decoder: frame_code");
  {
    const int k = cfg->workgroups_per_channel;
    if (k != 0 && k != 1 && k != 2 && k != 4 && k != 8)
      return fail(CBD_E_INVALID, "decoder: workgroups_per_channel must be 0, 1, 2, 4 or 8");
    if (k > 1 && cfg->compact_records_above > 0)
      return fail(CBD_E_INVALID, "decoder: record compaction is not available with workgroups_per_channel > 1");
    if (k > 1 && g->unstored_closures > 0)
      return fail(CBD_E_INVALID, "decoder: workgroups_per_channel > 1 needs every epsilon closure of the graph stored as a list");
  }
  if (cfg->block_threads != 0 && cfg->block_threads != 256 && cfg->block_threads != 512 && cfg->block_threads != 960 &&
      cfg->block_threads != 1024)
    return fail(CBD_E_INVALID, "decoder: block_threads must be 0, 256, 512, 960 or 1024");
  cbd_decoder *d = new (std::nothrow) cbd_decoder();
  if (!d) return fail(CBD_E_NOMEM, "decoder: host allocation");
  struct Guard {   // frees the half-built decoder on every early return and if anything below throws
    cbd_decoder *d;
    ~Guard() { if (d) cbd_decoder_free(d); }
  } guard{d};
  d->g = g; d->cfg = *cfg; d->stream = (hipStream_t)hip_stream;
  if (d->cfg.max_eps_iters <= 0) d->cfg.max_eps_iters = 64;
  d->C = cfg->num_channels;
  d->g_slots = (int32_t)1 << cfg->hash_capacity_log2;
  d->g_tok_cap = d->g_slots / 2;
  d->g_log_cap = d->g_slots;
  int64_t rpf = cfg->records_per_frame > 0 ? cfg->records_per_frame : d->g_tok_cap;
  int64_t bp = rpf * ((int64_t)cfg->max_frames + 1) + d->g_tok_cap;
  if (bp > 0x7FFFFFF0) return fail(CBD_E_INVALID, "decoder: back-pointer buffer too large per channel");
  d->bp_cap = (int32_t)bp;
  d->max_ctx = std::max(cfg->max_context_arcs, 1);
  d->ctx_lds_cap = std::min((d->max_ctx + 15) / 16 * 16, 2048);

#define DCHK(expr)                                                                     \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) {                                                            \
      return fail(CBD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));       \
    }                                                                                  \
  } while (0)
  DCHK(hipSetDevice(g->device));
  {
    int32_t *sp = nullptr;   // cbd_best_paths_static's array on this device: resolved here, once
    DCHK(static_scratch(g->device, &sp));
  }
  int lds_limit = 0;
  DCHK(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, g->device));
  {
    // How many workgroups (channels) share a compute unit's LDS.  One 1024-thread workgroup per compute unit is
    // the default at every channel count: the frame code keeps the vector units busy about half the time, two
    // 512-thread workgroups side by side each run their frames 1.6 times slower (two rounds per wave, and the
    // halved table capacity sends their larger frames to the tables in device memory) and gain nothing back from
    // sharing the unit (measured with 512 channels: 2.8 instead of 2.0 ms per launch; with 2048: 8.8 instead of
    // 5.6 ms).  A caller can still ask for 2 or 4 (the kernel is held to 128 vector registers for that).
    int wgs = cfg->workgroups_per_cu;
    if (wgs == 0) wgs = 1;
    // Result walks run beside the decoding (side stream).  Where a call's workgroups fill the device in one round
    // (more than half of the compute units, not more than all), a walk that holds a compute unit delays that
    // unit's channel and with it the whole call: such a decoder leaves 2 KB of LDS per compute unit free (half a
    // KB per walk, but with 1 KB free none of them got onto a unit that held a decoding workgroup) and launches
    // the 120-register kernel while walks are in flight (advance_beside_kernel).  With fewer channels the walks
    // find free units, with more the workgroups are handed out as units come free and a late one costs little:
    // there the 64 tokens of table capacity and the 8 registers are worth more (Stress +2 %, Dynamic +5 %).
    int n_cu_all = 0;
    DCHK(hipDeviceGetAttribute(&n_cu_all, hipDeviceAttributeMultiprocessorCount, g->device));
    d->walk_room = wgs == 1 && cfg->block_threads == 0 && 2 * cfg->num_channels > n_cu_all && cfg->num_channels <= n_cu_all;
    d->walk_room_min_grid = n_cu_all / 2 + 1;
    const int budget = (lds_limit - (d->walk_room ? 2048 : 1024)) / wgs;
    // the lean frame code keeps a commit log per wave next to the tokens' rows (decided with the block size below)
    const int block_guess = cfg->block_threads != 0 ? cfg->block_threads : (wgs >= 4 ? 256 : (wgs >= 2 ? 512 : 1024));
    const int lean_entries = cfg->frame_code == 0 && cfg->table_location != 2 ? cbd::kLeanLogPerWave * (block_guess / 64) : 0;
    auto best_cap = [&](int pdfs_staged) {
      if (cfg->table_location == 2) return 0;
      int want = cfg->lds_token_cap > 0 ? cfg->lds_token_cap : cbd::kLdsTokLimit;
      want = std::min(want, std::min<int>(d->g_tok_cap, cbd::kLdsTokLimit));
      want = std::min(want, (int)(cbd::LogT<true>::kSrcMask * 2 / 3));   // the LDS change log keeps a table slot in 14 bits
      for (int t = want / 64 * 64; t >= 64; t -= 64) {
        cbd::LdsLayout l = cbd::make_layout(pdfs_staged, d->ctx_lds_cap, t, cbd::lds_slots_for(t), cbd::lds_log_for(t),
                                            lean_entries);
        if ((int64_t)l.total <= budget) return t;
      }
      return 0;
    };
    // The frame's log-likelihood row is copied to LDS ahead of the frame only while it is small (4 KB, 1024 pdfs).
    // A 6000-pdf row takes the room of 620 tokens, and reading the scores from device memory (the row stays in
    // L2) costs the lean frame nothing in total: with the room in the tables instead, Stress sends 250 instead of
    // 2000 frames per pass to the tables in device memory and its launches take 5.05 instead of 5.45 ms (Large
    // -1 %, Dynamic +1 %).
    int cap = best_cap(g->P);
    d->stage_rows = 1;
    const bool row_fits = (int64_t)cbd::make_layout(g->P, d->ctx_lds_cap, 0, 0, 0).total <= budget;
    if (!row_fits || (int64_t)g->P * 4 > 4096) {
      d->stage_rows = 0;
      cap = best_cap(0);
    }
    if ((int64_t)cbd::make_layout(d->stage_rows ? g->P : 0, d->ctx_lds_cap, 0, 0, 0).total > lds_limit) {
      return fail(CBD_E_INVALID, "decoder: context list does not fit LDS");
    }
    if (cap == 0 && cfg->table_location == 1) {
      return fail(CBD_E_INVALID, "decoder: no room for token tables in LDS");
    }
    d->lds_tok_cap = cap;
    d->lds_slots = cap ? cbd::lds_slots_for(cap) : 0;
    d->lds_log_cap = cap ? cbd::lds_log_for(cap) : 0;
    d->lean_log_per_wave = cap ? lean_entries / (block_guess / 64) : 0;
    d->lds_bytes = cbd::make_layout(d->stage_rows ? g->P : 0, d->ctx_lds_cap, cap, d->lds_slots, d->lds_log_cap,
                                    cap ? lean_entries : 0).total;
    // workgroup size: the more channels share a compute unit, the smaller the groups
    d->block = wgs >= 4 ? 256 : (wgs >= 2 ? 512 : 1024);
    if (cfg->block_threads != 0) d->block = cfg->block_threads;
    // (the LDS change log keeps a table slot in 14 bits)
    if (d->lds_slots > (int32_t)cbd::LogT<true>::kSrcMask) {
      return fail(CBD_E_INVALID, "decoder: LDS table too large for the change log's slot field");
    }
  }
  DCHK(set_attr(d->block, d->lds_bytes));
  if (cfg->workgroups_per_cu > 1) {
    // the LDS was divided for that many workgroups side by side: registers and waves have to allow them too
    int per_cu = 0;
    DCHK(resident_per_cu(d->block, d->lds_bytes, &per_cu));
    if (per_cu < cfg->workgroups_per_cu)
      return fail(CBD_E_INVALID, "decoder: a compute unit holds " + std::to_string(per_cu) +
                                 " workgroups of this size, fewer than workgroups_per_cu");
  }
  if (cfg->workgroups_per_channel > 1) {
    const int k = cfg->workgroups_per_channel;
    int n_cu = 0;
    DCHK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, g->device));
    // members resident at once: one 1024-thread member per compute unit (it fills the LDS).  (Two 512-thread members
    // per unit were tried for teams of eight: every phase and every wait got longer, 160 instead of 100 us per frame.)
    if ((int64_t)d->C * k > n_cu)
      return fail(CBD_E_INVALID, "decoder: num_channels x workgroups_per_channel exceeds the device's compute units");
    d->team_block = 1024;
    d->team_k = k;
    const int64_t lds_member = (int64_t)lds_limit - 1024;
    // each member's table takes the LDS that the row, the context list and the small arrays leave
    d->team_stage_rows = g->P <= 4096 ? 1 : 0;
    cbd::TeamLayout fixed = cbd::team_layout(d->team_stage_rows ? g->P : 0, d->ctx_lds_cap, 0, d->team_block / 64);
    if ((int64_t)fixed.total + 14 * 1024 > lds_member) {
      d->team_stage_rows = 0;
      fixed = cbd::team_layout(0, d->ctx_lds_cap, 0, d->team_block / 64);
    }
    int slots = (int)((lds_member - (int64_t)fixed.total - 64) / 14) / 64 * 64;
    slots = std::min(slots, 0xFFFF / 2 * 3 / 64 * 64);
    if (slots < 1024) return fail(CBD_E_INVALID, "decoder: no room for a team member's table in LDS");
    d->team_slots = slots;
    d->team_part_cap = slots * 2 / 3 / 64 * 64;
    if ((int64_t)d->team_part_cap * k > d->g_tok_cap)
      d->team_part_cap = d->g_tok_cap / k / 64 * 64;   // (the token arrays are sized by hash_capacity_log2)
    if (d->team_part_cap < 64) return fail(CBD_E_INVALID, "decoder: hash_capacity_log2 too small for a team");
    // (a sender's queue to one owner: in the frame after a reset one member expands a long start row by itself)
    d->team_q_cap = d->team_part_cap + d->team_part_cap / 4;
    d->team_lds = cbd::team_layout(d->team_stage_rows ? g->P : 0, d->ctx_lds_cap, slots, d->team_block / 64).total;
    DCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&cbd::advance_team_kernel<1024>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)d->team_lds));
    {
      // the members wait for one another inside the kernel: the device has to hold all of them at once
      int per_cu = 0;
      DCHK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, cbd::advance_team_kernel<1024>, 1024, d->team_lds));
      if ((int64_t)per_cu * n_cu < (int64_t)d->C * k)
        return fail(CBD_E_INVALID, "decoder: the device cannot hold all members of all teams at once");
    }
    // a frame's records: one block of k shares
    const int64_t bp_team = (int64_t)k * d->team_part_cap * ((int64_t)cfg->max_frames + 1) + d->g_tok_cap;
    if (bp_team > 0x7FFFFFF0) return fail(CBD_E_INVALID, "decoder: back-pointer buffer too large per channel");
    d->bp_cap = std::max(d->bp_cap, (int32_t)bp_team);
  }

  const size_t C = (size_t)d->C;
  DCHK(dmalloc(&d->d_chan, C, &d->bytes));
  DCHK(dmalloc(&d->d_auto_snap, (size_t)cbd_decoder::kSnapRing * C * cbd::kSnapInts, &d->bytes));
  DCHK(dmalloc(&d->d_tok_state, C * d->g_tok_cap, &d->bytes));
  DCHK(dmalloc(&d->d_tok_cost, C * d->g_tok_cap, &d->bytes));
  DCHK(dmalloc(&d->d_tok_row, C * 2 * d->g_tok_cap, &d->bytes));
  DCHK(dmalloc(&d->d_bp, C * (size_t)d->bp_cap, &d->bytes));
  DCHK(dmalloc(&d->d_log, C * (size_t)d->g_log_cap, &d->bytes));
  d->pool = cfg->max_pool_contexts;
  d->pool_used.assign((size_t)d->pool, 0);
  DCHK(dmalloc(&d->d_ctx, (C + d->pool) * (size_t)d->max_ctx, &d->bytes));
  if (d->team_k > 1) {
    const size_t k = (size_t)d->team_k;
    DCHK(dmalloc(&d->d_team, C, &d->bytes));
    DCHK(hipMemsetAsync(d->d_team, 0, sizeof(cbd::TeamChan) * C, d->stream));
    DCHK(dmalloc(&d->d_team_q1, C * k * k * (size_t)d->team_q_cap, &d->bytes));
    DCHK(dmalloc(&d->d_team_q2, C * k * k * (size_t)d->team_q_cap, &d->bytes));
    DCHK(dmalloc(&d->d_team_cwin, C * k * (size_t)d->team_part_cap, &d->bytes));
    DCHK(dmalloc(&d->d_team_pub_key, C * k * (size_t)d->team_slots, &d->bytes));
    DCHK(dmalloc(&d->d_team_pub_lid, C * k * (size_t)d->team_slots, &d->bytes));
    // the graph's long rows, their arcs sorted by owning member (a few thousand rows at most: beyond that the
    // rows are shared out arc by arc through the queues, as are rows this table does not know)
    if (!g->long_rows.empty() && g->long_rows.size() <= 4096) {
      std::vector<int4> rows = g->long_rows;
      int64_t total = 0;
      for (auto &r : rows) { r.w = (int)total; total += r.z; }
      if (total < 0x7FFFFFF0) {
        d->team_n_big_rows = (int32_t)rows.size();
        DCHK(dmalloc(&d->d_team_big_rows, rows.size(), &d->bytes));
        DCHK(dmalloc(&d->d_team_big_group, rows.size() * (k + 1), &d->bytes));
        DCHK(dmalloc(&d->d_team_big_perm, (size_t)total, &d->bytes));
        DCHK(hipMemcpy(d->d_team_big_rows, rows.data(), sizeof(int4) * rows.size(), hipMemcpyHostToDevice));
        hipLaunchKernelGGL(cbd::team_prepare_rows_kernel, dim3((unsigned)rows.size()), dim3(256), 0, d->stream, g->d_arcs,
                           d->d_team_big_rows, d->d_team_big_group, d->d_team_big_perm, d->team_k);
        DCHK(hipGetLastError());
      }
    }
  }
  DCHK(dmalloc(&d->d_ctx_n, C + d->pool, &d->bytes));
  DCHK(dmalloc(&d->d_ctx_off, C + d->pool, &d->bytes));
  DCHK(hipMemsetAsync(d->d_ctx_n, 0, sizeof(int32_t) * (C + d->pool), d->stream));
  DCHK(hipMemsetAsync(d->d_ctx_off, 0, sizeof(float) * (C + d->pool), d->stream));
  DCHK(dmalloc(&d->d_hkey, C * (size_t)d->g_slots, &d->bytes));
  DCHK(dmalloc(&d->d_hval, C * (size_t)d->g_slots, &d->bytes));
  DCHK(dmalloc(&d->d_hidx, C * (size_t)d->g_slots, &d->bytes));
  {
    size_t n = C * (size_t)d->g_slots;
    hipLaunchKernelGGL(cbd::init_tables_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, d->stream,
                       d->d_hkey, d->d_hval, n);
    DCHK(hipGetLastError());
  }
  hipLaunchKernelGGL(cbd::init_chan_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, d->stream, d->d_chan,
                     d->C);
  DCHK(hipGetLastError());
  if (cfg->compact_records_above > 0) {
    DCHK(hipHostMalloc((void **)&d->h_new, sizeof(int2) * C, hipHostMallocDefault));
    memset(d->h_new, 0, sizeof(int2) * C);
    DCHK(hipHostGetDevicePointer((void **)&d->dv_new, d->h_new, 0));
    DCHK(dmalloc(&d->d_due_max, 1, &d->bytes));
    DCHK(hipMemsetAsync(d->d_due_max, 0, sizeof(unsigned long long), d->stream));
  }
  d->h_tmp.reserve(C); d->last_list.reserve(C); d->kept_ids.reserve(C); d->last_ids.reserve(C);
  d->h_static_meta.assign(C * cbd::kMetaInts, 0);
  DCHK(d->ids.init(sizeof(int32_t) * C));
  DCHK(dmalloc(&d->d_ids_kept, C, &d->bytes));
  // context staging: [channels n][list offsets n+1][offsets n][lists ...]
  DCHK(d->ctxs.init(sizeof(int32_t) * (C * 4 + 1 + C * (size_t)d->max_ctx)));
  DCHK(hipStreamSynchronize(d->stream));
#undef DCHK
  guard.d = nullptr;
  *out = d;
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "decoder_create: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("decoder_create: ") + e.what());
}

int32_t cbd_decoder_free(cbd_decoder *d) {
  if (!d) return CBD_OK;
  (void)hipStreamSynchronize(d->stream);
  if (d->side) (void)hipStreamSynchronize(d->side);   // its walks read the records and snapshots freed below
  void *ptrs[] = {d->d_chan, d->d_tok_state, d->d_tok_cost, d->d_tok_row, d->d_bp,
                  d->d_log, d->d_ctx, d->d_ctx_n, d->d_ctx_off, d->d_hkey, d->d_hval, d->d_hidx, d->d_auto_snap,
                  d->d_gc_mark, d->d_gc_prefix, d->d_gc_cross, d->d_fixed_arcs, d->d_fixed_words, d->d_due_max, d->d_ids_kept,
                  d->d_team, d->d_team_q1, d->d_team_q2, d->d_team_cwin, d->d_team_pub_key, d->d_team_pub_lid,
                  d->d_team_big_rows, d->d_team_big_group, d->d_team_big_perm};
  for (void *p : ptrs)
    if (p) (void)hipFree(p);
  if (d->h_new) (void)hipHostFree(d->h_new);
  for (auto &o : d->out) {
    free_out_slot(o);
    if (o.done) (void)hipEventDestroy(o.done);
  }
  if (d->side) (void)hipStreamDestroy(d->side);
  if (d->snap_ev) (void)hipEventDestroy(d->snap_ev);
  d->ids.destroy();
  d->ctxs.destroy();
  delete d;
  return CBD_OK;
}

int32_t cbd_decoder_info(const cbd_decoder *d, int64_t *device_bytes, int32_t *lds_bytes, int32_t *block_threads,
                         int32_t *lds_token_cap) {
  if (!d) return fail(CBD_E_INVALID, "info: null decoder");
  if (device_bytes) *device_bytes = (int64_t)d->bytes;
  if (lds_bytes) *lds_bytes = (int32_t)d->lds_bytes;
  if (block_threads) *block_threads = d->block;
  if (lds_token_cap) *lds_token_cap = d->lds_tok_cap;
  return CBD_OK;
}

int32_t cbd_reset_channels(cbd_decoder *d, const int32_t *channels, int32_t n) try {
  if (!d) return fail(CBD_E_INVALID, "reset: null decoder");
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = stage_channels(d, channels, n, &dev, &slot);
  if (rc != CBD_OK) return rc;
  // a new utterance reuses the back-pointer buffer from its start: let outstanding walks finish first
  for (int k = 1; k < cbd_decoder::kOutSlots; ++k)
    if (d->out[k].pending) HIPCHK(hipStreamWaitEvent(d->stream, d->out[k].done, 0));
  AdvanceParams p = base_params(d);
  p.chan_ids = dev; p.loglikes = nullptr; p.channel_stride = 0; p.n_frames = 0; p.do_reset = 1;
  p.new_records = d->dv_new; p.call_seq = (int32_t)d->adv_calls; p.due_max = d->d_due_max;
  rc = claim_snapshot_slot(d, channels, n, &p);
  if (rc != CBD_OK) return rc;
  HIPCHK(launch_advance(d, p, n));
  if (d->team_k > 1) {
    hipLaunchKernelGGL(cbd::team_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, d->stream, d->d_team, dev, n);
    HIPCHK(hipGetLastError());
  }
  HIPCHK(d->ids.release(slot, d->stream));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "reset_channels: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("reset_channels: ") + e.what());
}

namespace {

// Checks n lists (list i = arc_idx[list_offsets[i] .. list_offsets[i+1])) and turns them into sorted,
// de-duplicated lists in the library's arc order.  Nothing is enqueued here.
int32_t prepare_lists(const cbd_decoder *d, int32_t n, const int32_t *arc_idx, const int32_t *list_offsets,
                      const float *offsets, std::vector<int32_t> &packed, std::vector<int32_t> &new_off,
                      const char *who) {
  const std::string w(who);
  if (list_offsets[0] != 0) return fail(CBD_E_INVALID, w + ": list_offsets[0] != 0");
  for (int32_t i = 0; i < n; ++i) {
    if (list_offsets[i + 1] < list_offsets[i]) return fail(CBD_E_INVALID, w + ": list_offsets not monotone");
    if (!std::isfinite(offsets[i])) return fail(CBD_E_INVALID, w + ": non-finite offset");
  }
  const int32_t total = list_offsets[n];
  if (total > 0 && !arc_idx) return fail(CBD_E_INVALID, w + ": null list");
  // the list is a set: translate to the library's arc order, sort, de-duplicate.  Lists are independent,
  // so large uploads are split over a few host threads (each list is handled in place in `packed`).
  packed.resize((size_t)total);
  new_off.assign((size_t)n + 1, 0);
  std::vector<int32_t> count((size_t)n, 0);
  const int32_t *p2i = d->g->pub2int.data();
  const int32_t num_arcs = d->g->A;
  std::atomic<int> bad{0};
  auto work = [&](int32_t i0, int32_t i1) {
    for (int32_t i = i0; i < i1; ++i) {
      const int32_t b = list_offsets[i], e = list_offsets[i + 1];
      for (int32_t k = b; k < e; ++k) {
        int32_t a = arc_idx[k];
        if (a < 0 || a >= num_arcs) { bad.store(1); return; }
        packed[(size_t)k] = p2i[a];
      }
      std::sort(packed.begin() + b, packed.begin() + e);
      count[(size_t)i] = (int32_t)(std::unique(packed.begin() + b, packed.begin() + e) - (packed.begin() + b));
    }
  };
  const int n_threads = total >= 32768 ? std::min<int>(8, std::max(1u, std::thread::hardware_concurrency())) : 1;
  if (n_threads <= 1) {
    work(0, n);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < n_threads; ++t)
      pool.emplace_back(work, (int32_t)((int64_t)n * t / n_threads), (int32_t)((int64_t)n * (t + 1) / n_threads));
    for (auto &th : pool) th.join();
  }
  if (bad.load()) return fail(CBD_E_INVALID, w + ": arc index out of range");
  int32_t out = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (count[(size_t)i] > d->cfg.max_context_arcs)
      return fail(CBD_E_INVALID, w + ": more than max_context_arcs distinct arcs");
    const int32_t b = list_offsets[i];
    if (out != b) std::copy(packed.begin() + b, packed.begin() + b + count[(size_t)i], packed.begin() + out);
    out += count[(size_t)i];
    new_off[(size_t)i + 1] = out;
  }
  packed.resize((size_t)out);
  return CBD_OK;
}

// Uploads prepared lists into the given store slots (at most C per staging buffer, so in pieces);
// bind != null also switches channel bind[i] to slots[i].
int32_t upload_lists(cbd_decoder *d, int32_t n, const int32_t *slots, const int32_t *bind, const float *offsets,
                     const std::vector<int32_t> &packed, const std::vector<int32_t> &off) {
  for (int32_t i0 = 0; i0 < n; i0 += d->C) {
    const int32_t m = std::min(d->C, n - i0);
    int slot = 0;
    HIPCHK(d->ctxs.acquire(&slot));
    int32_t *h = (int32_t *)d->ctxs.host[slot];
    const size_t mm = (size_t)m;
    const int32_t base = off[(size_t)i0], cnt = off[(size_t)i0 + mm] - base;
    memcpy(h, slots + i0, sizeof(int32_t) * mm);
    if (bind) memcpy(h + mm, bind + i0, sizeof(int32_t) * mm);
    for (size_t k = 0; k <= mm; ++k) h[2 * mm + k] = off[(size_t)i0 + k] - base;
    memcpy(h + 3 * mm + 1, offsets + i0, sizeof(float) * mm);
    if (cnt > 0) memcpy(h + 4 * mm + 1, packed.data() + base, sizeof(int32_t) * (size_t)cnt);
    HIPCHK(d->ctxs.upload(slot, sizeof(int32_t) * (4 * mm + 1 + (size_t)cnt), d->stream));
    const int32_t *dv = (const int32_t *)d->ctxs.dev[slot];
    hipLaunchKernelGGL(cbd::scatter_contexts_kernel, dim3((unsigned)m), dim3(256), 0, d->stream, dv,
                       bind ? dv + mm : (const int32_t *)nullptr, dv + 2 * mm, (const float *)(dv + 3 * mm + 1),
                       dv + 4 * mm + 1, d->d_ctx, d->max_ctx, d->d_ctx_n, d->d_ctx_off, d->d_chan);
    HIPCHK(hipGetLastError());
    HIPCHK(d->ctxs.release(slot, d->stream));
  }
  return CBD_OK;
}

// Checks n lists as given by the caller (offsets, arc numbers in range) without changing anything;
// longest receives the length of the longest list.
int32_t check_raw_lists(const cbd_decoder *d, int32_t n, const int32_t *arc_idx, const int32_t *list_offsets,
                        const float *offsets, const char *who, int32_t *longest) {
  const std::string w(who);
  if (list_offsets[0] != 0) return fail(CBD_E_INVALID, w + ": list_offsets[0] != 0");
  int32_t mx = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (list_offsets[i + 1] < list_offsets[i]) return fail(CBD_E_INVALID, w + ": list_offsets not monotone");
    if (!std::isfinite(offsets[i])) return fail(CBD_E_INVALID, w + ": non-finite offset");
    mx = std::max(mx, list_offsets[i + 1] - list_offsets[i]);
  }
  const int32_t total = list_offsets[n];
  if (total > 0 && !arc_idx) return fail(CBD_E_INVALID, w + ": null list");
  const uint32_t num_arcs = (uint32_t)d->g->A;
  uint32_t bad = 0;
  for (int32_t k = 0; k < total; ++k) bad |= (uint32_t)((uint32_t)arc_idx[k] >= num_arcs);
  if (bad) return fail(CBD_E_INVALID, w + ": arc index out of range");
  *longest = mx;
  return CBD_OK;
}

// Can the device prepare these lists?  (Each must fit its slot even if no entry repeats, and the sort's LDS.)
bool device_can_prepare(const cbd_decoder *d, int32_t longest) {
  return longest <= d->cfg.max_context_arcs && longest <= cbd::kPrepMaxList;
}

// Uploads the caller's lists as they are; the device translates, sorts and de-duplicates them (slots / bind
// as in upload_lists).
int32_t upload_raw_lists(cbd_decoder *d, int32_t n, const int32_t *slots, const int32_t *bind, const float *offsets,
                         const int32_t *arc_idx, const int32_t *list_offsets) {
  for (int32_t i0 = 0; i0 < n; i0 += d->C) {
    const int32_t m = std::min(d->C, n - i0);
    int slot = 0;
    HIPCHK(d->ctxs.acquire(&slot));
    int32_t *h = (int32_t *)d->ctxs.host[slot];
    const size_t mm = (size_t)m;
    const int32_t base = list_offsets[i0], cnt = list_offsets[(size_t)i0 + mm] - base;
    int32_t longest = 0;
    memcpy(h, slots + i0, sizeof(int32_t) * mm);
    if (bind) memcpy(h + mm, bind + i0, sizeof(int32_t) * mm);
    for (size_t k = 0; k <= mm; ++k) h[2 * mm + k] = list_offsets[(size_t)i0 + k] - base;
    for (size_t k = 0; k < mm; ++k) longest = std::max(longest, h[2 * mm + k + 1] - h[2 * mm + k]);
    memcpy(h + 3 * mm + 1, offsets + i0, sizeof(float) * mm);
    if (cnt > 0) memcpy(h + 4 * mm + 1, arc_idx + base, sizeof(int32_t) * (size_t)cnt);
    HIPCHK(d->ctxs.upload(slot, sizeof(int32_t) * (4 * mm + 1 + (size_t)cnt), d->stream));
    const int32_t *dv = (const int32_t *)d->ctxs.dev[slot];
    int pow2 = 1;
    while (pow2 < longest) pow2 <<= 1;
    hipLaunchKernelGGL(cbd::prepare_contexts_kernel, dim3((unsigned)m), dim3(cbd::kPrepThreads),
                       sizeof(int32_t) * (size_t)pow2, d->stream, dv, bind ? dv + mm : (const int32_t *)nullptr,
                       dv + 2 * mm, (const float *)(dv + 3 * mm + 1), dv + 4 * mm + 1, d->g->d_pub2int, d->d_ctx,
                       d->max_ctx, d->d_ctx_n, d->d_ctx_off, d->d_chan);
    HIPCHK(hipGetLastError());
    HIPCHK(d->ctxs.release(slot, d->stream));
  }
  return CBD_OK;
}

int32_t check_channel_list(cbd_decoder *d, const int32_t *channels, int32_t n, const char *who) {
  const std::string w(who);
  if (!channels || n <= 0 || n > d->C) return fail(CBD_E_INVALID, w + ": bad channel count");
  d->h_tmp.assign((size_t)d->C, 0);
  for (int32_t i = 0; i < n; ++i) {
    int32_t c = channels[i];
    if (c < 0 || c >= d->C) return fail(CBD_E_INVALID, w + ": channel out of range");
    if (d->h_tmp[c]) return fail(CBD_E_INVALID, w + ": duplicate channel");
    d->h_tmp[c] = 1;
  }
  return CBD_OK;
}

}  // namespace

int32_t cbd_set_contexts(cbd_decoder *d, const int32_t *channels, int32_t n_channels, const int32_t *arc_idx,
                         const int32_t *list_offsets, const float *offsets) try {
  if (!d || !channels || !list_offsets || !offsets) return fail(CBD_E_INVALID, "set_contexts: null argument");
  // validate everything before anything changes
  int32_t rc = check_channel_list(d, channels, n_channels, "set_contexts");
  if (rc != CBD_OK) return rc;
  int32_t longest = 0;
  rc = check_raw_lists(d, n_channels, arc_idx, list_offsets, offsets, "set_contexts", &longest);
  if (rc != CBD_OK) return rc;
  // a channel's own context lives in store slot `channel`
  if (device_can_prepare(d, longest))
    return upload_raw_lists(d, n_channels, channels, channels, offsets, arc_idx, list_offsets);
  // very long lists, or lists that only fit once their repeats are gone: prepared here
  std::vector<int32_t> packed, off;
  rc = prepare_lists(d, n_channels, arc_idx, list_offsets, offsets, packed, off, "set_contexts");
  if (rc != CBD_OK) return rc;
  return upload_lists(d, n_channels, channels, channels, offsets, packed, off);
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "set_contexts: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("set_contexts: ") + e.what());
}

int32_t cbd_contexts_create(cbd_decoder *d, int32_t n_contexts, const int32_t *arc_idx, const int32_t *list_offsets,
                            const float *offsets, int32_t *context_ids) try {
  if (!d || !list_offsets || !offsets || !context_ids) return fail(CBD_E_INVALID, "contexts_create: null argument");
  if (n_contexts <= 0) return fail(CBD_E_INVALID, "contexts_create: bad count");
  int32_t free_ids = 0;
  for (uint8_t u : d->pool_used) free_ids += !u;
  if (n_contexts > free_ids) return fail(CBD_E_CAPACITY, "contexts_create: context pool full");
  int32_t longest = 0;
  int32_t rc = check_raw_lists(d, n_contexts, arc_idx, list_offsets, offsets, "contexts_create", &longest);
  if (rc != CBD_OK) return rc;
  const bool on_device = device_can_prepare(d, longest);
  std::vector<int32_t> packed, off;
  if (!on_device) {
    rc = prepare_lists(d, n_contexts, arc_idx, list_offsets, offsets, packed, off, "contexts_create");
    if (rc != CBD_OK) return rc;
  }
  std::vector<int32_t> slots((size_t)n_contexts);
  int32_t next = 0;
  for (int32_t i = 0; i < n_contexts; ++i) {
    while (d->pool_used[(size_t)next]) ++next;
    d->pool_used[(size_t)next] = 1;
    context_ids[i] = next;
    slots[(size_t)i] = d->C + next;
  }
  rc = on_device ? upload_raw_lists(d, n_contexts, slots.data(), nullptr, offsets, arc_idx, list_offsets)
                 : upload_lists(d, n_contexts, slots.data(), nullptr, offsets, packed, off);
  if (rc != CBD_OK)
    for (int32_t i = 0; i < n_contexts; ++i) d->pool_used[(size_t)context_ids[i]] = 0;
  return rc;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "contexts_create: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("contexts_create: ") + e.what());
}

int32_t cbd_context_destroy(cbd_decoder *d, int32_t context_id) {
  if (!d) return fail(CBD_E_INVALID, "context_destroy: null decoder");
  if (context_id < 0 || context_id >= d->pool || !d->pool_used[(size_t)context_id])
    return fail(CBD_E_INVALID, "context_destroy: no such context");
  d->pool_used[(size_t)context_id] = 0;
  return CBD_OK;
}

int32_t cbd_use_contexts(cbd_decoder *d, const int32_t *channels, const int32_t *context_ids, int32_t n) try {
  if (!d || !context_ids) return fail(CBD_E_INVALID, "use_contexts: null argument");
  int32_t rc = check_channel_list(d, channels, n, "use_contexts");
  if (rc != CBD_OK) return rc;
  for (int32_t i = 0; i < n; ++i) {
    int32_t id = context_ids[i];
    if (id != -1 && (id < 0 || id >= d->pool || !d->pool_used[(size_t)id]))
      return fail(CBD_E_INVALID, "use_contexts: no such context");
  }
  int slot = 0;
  HIPCHK(d->ctxs.acquire(&slot));
  int32_t *h = (int32_t *)d->ctxs.host[slot];
  for (int32_t i = 0; i < n; ++i) {
    h[i] = channels[i];
    h[(size_t)n + i] = context_ids[i] < 0 ? channels[i] : d->C + context_ids[i];   // -1: the channel's own list
  }
  HIPCHK(d->ctxs.upload(slot, sizeof(int32_t) * 2 * (size_t)n, d->stream));
  const int32_t *dv = (const int32_t *)d->ctxs.dev[slot];
  hipLaunchKernelGGL(cbd::bind_contexts_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, d->stream, dv, dv + n,
                     n, d->d_chan);
  HIPCHK(hipGetLastError());
  HIPCHK(d->ctxs.release(slot, d->stream));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "use_contexts: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("use_contexts: ") + e.what());
}

int32_t cbd_set_context(cbd_decoder *d, int32_t channel, const int32_t *arc_idx, int32_t n, float offset) {
  if (n < 0) return fail(CBD_E_INVALID, "set_context: negative length");
  int32_t lo[2] = {0, n};
  return cbd_set_contexts(d, &channel, 1, arc_idx, lo, &offset);
}

int32_t cbd_advance(cbd_decoder *d, const int32_t *channels, int32_t n_channels, const float *loglikes,
                    int64_t channel_stride, int32_t n_frames) try {
  if (!d) return fail(CBD_E_INVALID, "advance: null decoder");
  if (n_frames < 0) return fail(CBD_E_INVALID, "advance: negative frame count");
  if (n_frames == 0) return CBD_OK;
  if (!loglikes) return fail(CBD_E_INVALID, "advance: null log-likelihoods");
  if (n_channels > 1 && channel_stride < (int64_t)n_frames * d->g->P)
    return fail(CBD_E_INVALID, "advance: channel_stride shorter than a channel's rows");
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = stage_channels(d, channels, n_channels, &dev, &slot);
  if (rc != CBD_OK) return rc;
  if (d->cfg.compact_records_above > 0 && d->adv_calls > 0) {
    // Whether a channel is due is decided on the device, from the counts the previous launch left there: the
    // compaction kernel is enqueued and its workgroups return at once where nothing is to do.  But enqueueing it
    // makes the stream wait for unfinished partial-result walks, which otherwise run beside the decoding.  So each
    // launch also leaves its channels' counts in host memory, and while the counts of one of the last two calls
    // are in and none is over the mark, the kernel is not enqueued at all (the mark may then be overshot by the
    // records of a few calls).  Counts written before the last compaction are recognised by their call number.
    const int32_t mark = d->cfg.compact_records_above;
    // (right after the kernel was enqueued the counts in host memory are still the old ones: nothing can be due)
    bool skip = d->last_compact_call >= 0 && d->adv_calls - d->last_compact_call <= 2;
    for (int32_t i = 0; i < n_channels && !skip; ++i) {
      // (count, call number) as the kernel stored the pair: one 64-bit load, so that a running launch cannot
      // leave an old count beside a new call number
      const uint64_t pair = __atomic_load_n((const uint64_t *)(d->h_new + channels[i]), __ATOMIC_RELAXED);
      const int32_t count = (int32_t)(uint32_t)pair, call = (int32_t)(uint32_t)(pair >> 32);
      const int32_t age = (int32_t)((uint32_t)d->adv_calls - (uint32_t)call);   // (call numbers wrap)
      const bool since_compaction = (int32_t)((uint32_t)call - (uint32_t)d->last_compact_call) >= 0;
      if (!(age >= 1 && age <= 2 && since_compaction && count <= mark)) break;
      if (i == n_channels - 1) skip = true;
    }
    if (!skip) {
      rc = enqueue_compaction(d, dev, n_channels, mark, d->adv_calls - 1);
      if (rc != CBD_OK) return rc;
      d->last_compact_call = d->adv_calls;   // (the number this call is about to take)
    }
  }
  AdvanceParams p = base_params(d);
  p.chan_ids = dev; p.loglikes = loglikes; p.channel_stride = channel_stride; p.n_frames = n_frames; p.do_reset = 0;
  p.new_records = d->dv_new; p.call_seq = (int32_t)d->adv_calls; p.due_max = d->d_due_max;
  if (d->team_k > 1) {
    // (a team leaves no best-token snapshot behind: a request for partial results takes its own)
    d->last_list.clear();
    d->adv_calls++;
    HIPCHK(launch_team(d, p, n_channels));
    HIPCHK(d->ids.release(slot, d->stream));
    return CBD_OK;
  }
  rc = claim_snapshot_slot(d, channels, n_channels, &p);
  if (rc != CBD_OK) return rc;
  HIPCHK(launch_advance(d, p, n_channels));
  HIPCHK(d->ids.release(slot, d->stream));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "advance: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("advance: ") + e.what());
}

int32_t cbd_compact_records(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t min_new_records) try {
  if (!d) return fail(CBD_E_INVALID, "compact_records: null decoder");
  if (min_new_records < 0) return fail(CBD_E_INVALID, "compact_records: negative threshold");
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = stage_channels(d, channels, n, &dev, &slot);
  if (rc != CBD_OK) return rc;
  rc = enqueue_compaction(d, dev, n, min_new_records);
  if (rc != CBD_OK) return rc;
  HIPCHK(d->ids.release(slot, d->stream));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "compact_records: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("compact_records: ") + e.what());
}

}  // extern "C"

namespace {

// tail_only: follow each path down to the beginning that all of the channel's paths share (as the compactions
// have found it) and report how many words and arcs of it precede (n_fixed_*); else whole paths.
int32_t best_paths_impl(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                        int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                        int32_t *status, bool tail_only, int32_t *n_fixed_words, int32_t *n_fixed_arcs,
                        const char *who) {
  if (!d || !words || !n_words || !n_arcs || !cost || !status || (tail_only && (!n_fixed_words || !n_fixed_arcs)))
    return fail(CBD_E_INVALID, std::string(who) + ": null argument");
  if (capacity < 1) return fail(CBD_E_INVALID, std::string(who) + ": capacity < 1");
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = stage_channels(d, channels, n, &dev, &slot);
  if (rc != CBD_OK) return rc;
  cbd_decoder::OutSlot &o = d->out[0];
  rc = size_out_slot(d, o, n, capacity);
  if (rc != CBD_OK) return rc;
  cbd::BestParams bp = best_params(d, o, dev, use_final, capacity, tail_only);
  hipLaunchKernelGGL(cbd::best_path_kernel, dim3((unsigned)n), dim3(cbd::kWalkThreads), 0, d->stream, bp);
  HIPCHK(hipGetLastError());
  HIPCHK(d->ids.release(slot, d->stream));
  return fetch_results(d, o, d->stream, n, capacity, words, arcs, n_words, n_arcs, cost, status, n_fixed_words,
                       n_fixed_arcs);
}

int32_t best_paths_begin_impl(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final,
                              int32_t capacity, int32_t want_arcs, int32_t *ticket, bool tail_only, const char *who) {
  if (!d || !ticket) return fail(CBD_E_INVALID, std::string(who) + ": null argument");
  if (capacity < 1) return fail(CBD_E_INVALID, std::string(who) + ": capacity < 1");
  int t = -1;
  for (int k = 1; k < cbd_decoder::kOutSlots; ++k)
    if (!d->out[k].pending) { t = k; break; }
  if (t < 0) return fail(CBD_E_CAPACITY, std::string(who) + ": too many requests in flight (finish one first)");
  // The decoding kernel leaves each channel's best token behind when it finishes.  A request for the channels
  // of the latest advance / reset call, in the same order and without final costs, walks from those; any other
  // request takes its own snapshot on the decode stream first.
  const bool reuse = !use_final && channels && n > 0 && (size_t)n == d->last_list.size() &&
                     memcmp(channels, d->last_list.data(), sizeof(int32_t) * (size_t)n) == 0;
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = CBD_OK;
  if (!reuse) {
    rc = stage_channels(d, channels, n, &dev, &slot);
    if (rc != CBD_OK) return rc;
  }
  cbd_decoder::OutSlot &o = d->out[t];
  rc = size_out_slot(d, o, n, capacity);
  if (rc != CBD_OK) return rc;
  if (!d->side) HIPCHK(hipStreamCreateWithFlags(&d->side, hipStreamNonBlocking));
  if (!d->snap_ev) HIPCHK(hipEventCreateWithFlags(&d->snap_ev, hipEventDisableTiming));
  if (!o.done) HIPCHK(hipEventCreateWithFlags(&o.done, hipEventDisableTiming));
  cbd::BestParams bp = best_params(d, o, dev, use_final, capacity, tail_only);
  if (reuse) {
    o.snap_slot = (int)((d->adv_calls - 1) % cbd_decoder::kSnapRing);
    bp.snap = d->d_auto_snap + (size_t)o.snap_slot * d->C * cbd::kSnapInts;
  } else {
    o.snap_slot = -1;
    // decode stream: pick the best tokens now, before a later call changes the channels
    hipLaunchKernelGGL(cbd::best_snapshot_kernel, dim3((unsigned)n), dim3(cbd::kSnapThreads), 0, d->stream, bp);
    HIPCHK(hipGetLastError());
    HIPCHK(d->ids.release(slot, d->stream));
  }
  HIPCHK(hipEventRecord(d->snap_ev, d->stream));
  // side stream: the walk reads only records that are already final, so it runs beside later decoding
  HIPCHK(hipStreamWaitEvent(d->side, d->snap_ev, 0));
  hipLaunchKernelGGL(cbd::best_walk_kernel, dim3((unsigned)n), dim3(cbd::kWalkThreads), 0, d->side, bp);
  HIPCHK(hipGetLastError());
  HIPCHK(hipEventRecord(o.done, d->side));
  o.pending = true; o.n = n; o.req_capacity = capacity; o.want_arcs = want_arcs != 0; o.tail_only = tail_only;
  *ticket = t;
  return CBD_OK;
}

int32_t best_paths_finish_impl(cbd_decoder *d, int32_t ticket, int32_t *words, int32_t *arcs, int32_t capacity,
                               int32_t *n_words, int32_t *n_arcs, float *cost, int32_t *status, bool tail_only,
                               int32_t *n_fixed_words, int32_t *n_fixed_arcs, const char *who) {
  if (!d || !words || !n_words || !n_arcs || !cost || !status || (tail_only && (!n_fixed_words || !n_fixed_arcs)))
    return fail(CBD_E_INVALID, std::string(who) + ": null argument");
  if (ticket < 1 || ticket >= cbd_decoder::kOutSlots || !d->out[ticket].pending)
    return fail(CBD_E_INVALID, std::string(who) + ": no such request");
  cbd_decoder::OutSlot &o = d->out[ticket];
  if (o.tail_only != tail_only) return fail(CBD_E_INVALID, std::string(who) + ": the request was begun by the other kind of call");
  if (capacity != o.req_capacity) return fail(CBD_E_INVALID, std::string(who) + ": capacity differs from the request");
  if (arcs && !o.want_arcs) return fail(CBD_E_INVALID, std::string(who) + ": arcs were not requested");
  int32_t rc = fetch_results(d, o, d->side, o.n, capacity, words, arcs, n_words, n_arcs, cost, status, n_fixed_words,
                             n_fixed_arcs);
  o.pending = false;
  return rc;
}

}  // namespace

extern "C" {

int32_t cbd_best_paths(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                       int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                       int32_t *status) try {
  return best_paths_impl(d, channels, n, use_final, words, arcs, capacity, n_words, n_arcs, cost, status, false,
                         nullptr, nullptr, "best_paths");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_paths: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_paths: ") + e.what());
}

int32_t cbd_best_paths_static(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                              int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                              int32_t *status) try {
  if (!d || !words || !n_words || !n_arcs || !cost || !status)
    return fail(CBD_E_INVALID, "best_paths_static: null argument");
  if (capacity < 1) return fail(CBD_E_INVALID, "best_paths_static: capacity < 1");
  if (n < 1 || n > d->C) return fail(CBD_E_INVALID, "best_paths_static: bad channel count");
  // rows in the fixed array: [n] headers, [n][capacity] words, [n][capacity] arcs
  constexpr size_t M = cbd::kMetaInts;
  const size_t need = (size_t)n * (M + 2 * (size_t)capacity);
  if (need > kStaticScratchInts)
    return fail(CBD_E_CAPACITY, "best_paths_static: n * (2 * capacity + 8) exceeds the fixed result area of " +
                                    std::to_string(kStaticScratchInts) + " entries");
  // (looked up when the decoder was created, with its device current; never the array's name itself)
  int32_t *sp = d->g->device >= 0 && d->g->device < kMaxDevices ? g_scratch_ptr[d->g->device] : nullptr;
  if (!sp) return fail(CBD_E_HIP, "best_paths_static: the fixed result area was not set up on this device");
  const int32_t *dev = nullptr;
  int slot = 0;
  int32_t rc = stage_channels(d, channels, n, &dev, &slot);
  if (rc != CBD_OK) return rc;
  cbd_decoder::OutSlot rows;   // (describes the rows only; owns nothing)
  rows.capacity = capacity;
  cbd::BestParams bp = best_params(d, rows, dev, use_final, capacity, false);
  bp.out_meta = sp;
  bp.out_words = sp + (size_t)n * M;
  bp.out_arcs = bp.out_words + (size_t)n * capacity;
  bp.snap = nullptr;
  hipLaunchKernelGGL(cbd::best_path_kernel, dim3((unsigned)n), dim3(cbd::kWalkThreads), 0, d->stream, bp);
  HIPCHK(hipGetLastError());
  HIPCHK(d->ids.release(slot, d->stream));
  int32_t *meta = d->h_static_meta.data();
  HIPCHK(hipMemcpyAsync(meta, bp.out_meta, sizeof(int32_t) * (size_t)n * M, hipMemcpyDeviceToHost, d->stream));
  HIPCHK(hipStreamSynchronize(d->stream));
  int32_t max_na = 0, max_nw = 0;
  for (int32_t i = 0; i < n; ++i) {
    status[i] = meta[(size_t)i * M + 0];
    n_arcs[i] = meta[(size_t)i * M + 1];
    n_words[i] = meta[(size_t)i * M + 2];
    const uint32_t bits = (uint32_t)meta[(size_t)i * M + 3];
    memcpy(&cost[i], &bits, 4);
    if (status[i] != CBD_OK) continue;
    max_na = std::max(max_na, n_arcs[i]);
    max_nw = std::max(max_nw, n_words[i]);
  }
  // as many columns of the rows as the longest result needs, straight into the caller's arrays
  const size_t pitch = sizeof(int32_t) * (size_t)capacity;
  if (max_nw > 0)
    HIPCHK(hipMemcpy2DAsync(words, pitch, bp.out_words, pitch, sizeof(int32_t) * (size_t)max_nw, (size_t)n,
                            hipMemcpyDeviceToHost, d->stream));
  if (arcs && max_na > 0)
    HIPCHK(hipMemcpy2DAsync(arcs, pitch, bp.out_arcs, pitch, sizeof(int32_t) * (size_t)max_na, (size_t)n,
                            hipMemcpyDeviceToHost, d->stream));
  HIPCHK(hipStreamSynchronize(d->stream));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_paths_static: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_paths_static: ") + e.what());
}

int32_t cbd_best_paths_begin(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t capacity,
                             int32_t want_arcs, int32_t *ticket) try {
  return best_paths_begin_impl(d, channels, n, use_final, capacity, want_arcs, ticket, false, "best_paths_begin");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_paths_begin: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_paths_begin: ") + e.what());
}

int32_t cbd_best_paths_finish(cbd_decoder *d, int32_t ticket, int32_t *words, int32_t *arcs, int32_t capacity,
                              int32_t *n_words, int32_t *n_arcs, float *cost, int32_t *status) try {
  return best_paths_finish_impl(d, ticket, words, arcs, capacity, n_words, n_arcs, cost, status, false, nullptr,
                                nullptr, "best_paths_finish");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_paths_finish: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_paths_finish: ") + e.what());
}

int32_t cbd_best_tails(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t *words,
                       int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost,
                       int32_t *status, int32_t *n_fixed_words, int32_t *n_fixed_arcs) try {
  return best_paths_impl(d, channels, n, use_final, words, arcs, capacity, n_words, n_arcs, cost, status, true,
                         n_fixed_words, n_fixed_arcs, "best_tails");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_tails: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_tails: ") + e.what());
}

int32_t cbd_best_tails_begin(cbd_decoder *d, const int32_t *channels, int32_t n, int32_t use_final, int32_t capacity,
                             int32_t want_arcs, int32_t *ticket) try {
  return best_paths_begin_impl(d, channels, n, use_final, capacity, want_arcs, ticket, true, "best_tails_begin");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_tails_begin: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_tails_begin: ") + e.what());
}

int32_t cbd_best_tails_finish(cbd_decoder *d, int32_t ticket, int32_t *words, int32_t *arcs, int32_t capacity,
                              int32_t *n_words, int32_t *n_arcs, float *cost, int32_t *status,
                              int32_t *n_fixed_words, int32_t *n_fixed_arcs) try {
  return best_paths_finish_impl(d, ticket, words, arcs, capacity, n_words, n_arcs, cost, status, true, n_fixed_words,
                                n_fixed_arcs, "best_tails_finish");
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "best_tails_finish: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("best_tails_finish: ") + e.what());
}

int32_t cbd_get_fixed(cbd_decoder *d, int32_t channel, int32_t from_word, int32_t from_arc, int32_t *words,
                      int32_t *arcs, int32_t capacity, int32_t *n_words, int32_t *n_arcs) try {
  if (!d || !n_words || !n_arcs) return fail(CBD_E_INVALID, "get_fixed: null argument");
  if (channel < 0 || channel >= d->C) return fail(CBD_E_INVALID, "get_fixed: channel out of range");
  if (from_word < 0 || from_arc < 0 || capacity < 0) return fail(CBD_E_INVALID, "get_fixed: negative argument");
  HIPCHK(hipStreamSynchronize(d->stream));
  cbd::ChanState cs;
  HIPCHK(hipMemcpy(&cs, d->d_chan + channel, sizeof(cs), hipMemcpyDeviceToHost));
  const int32_t nw = std::max(cs.n_fixed_words - from_word, 0), na = std::max(cs.n_fixed_arcs - from_arc, 0);
  *n_words = nw; *n_arcs = na;
  if ((words && nw > capacity) || (arcs && na > capacity)) return CBD_E_BUFFER;
  if (words && nw > 0)
    HIPCHK(hipMemcpy(words, d->d_fixed_words + (size_t)channel * d->bp_cap + from_word, sizeof(int32_t) * (size_t)nw,
                     hipMemcpyDeviceToHost));
  if (arcs && na > 0)
    HIPCHK(hipMemcpy(arcs, d->d_fixed_arcs + (size_t)channel * d->bp_cap + from_arc, sizeof(int32_t) * (size_t)na,
                     hipMemcpyDeviceToHost));
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "get_fixed: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("get_fixed: ") + e.what());
}

int32_t cbd_best_path(cbd_decoder *d, int32_t channel, int32_t use_final, int32_t *words, int32_t *arcs,
                      int32_t capacity, int32_t *n_words, int32_t *n_arcs, float *cost) {
  if (!n_words || !n_arcs || !cost) return fail(CBD_E_INVALID, "best_path: null argument");
  int32_t nw = 0, na = 0, st = 0;
  float c = 0.0f;
  int32_t rc = cbd_best_paths(d, &channel, 1, use_final, words, arcs, capacity, &nw, &na, &c, &st);
  if (rc != CBD_OK) return rc;
  if (st == CBD_OK || st == CBD_E_BUFFER) { *n_words = nw; *n_arcs = na; *cost = c; }
  return st;
}

int32_t cbd_get_tokens(cbd_decoder *d, int32_t channel, int32_t *states, float *costs, int32_t *arcs,
                       int32_t capacity, int32_t *n) try {
  if (!d || !n) return fail(CBD_E_INVALID, "get_tokens: null argument");
  if (channel < 0 || channel >= d->C) return fail(CBD_E_INVALID, "get_tokens: channel out of range");
  HIPCHK(hipStreamSynchronize(d->stream));
  cbd::ChanState cs;
  HIPCHK(hipMemcpy(&cs, d->d_chan + channel, sizeof(cs), hipMemcpyDeviceToHost));
  if (cs.status != CBD_OK) { *n = 0; return cs.status; }
  const int32_t nt = cs.n_tok;
  std::vector<int32_t> st((size_t)std::max(nt, 1));
  std::vector<float> co((size_t)std::max(nt, 1));
  std::vector<int2> bp((size_t)std::max(nt, 1));
  if (nt > 0) {
    HIPCHK(hipMemcpy(st.data(), d->d_tok_state + (size_t)channel * d->g_tok_cap, sizeof(int32_t) * nt,
                     hipMemcpyDeviceToHost));
    HIPCHK(hipMemcpy(co.data(), d->d_tok_cost + (size_t)channel * d->g_tok_cap, sizeof(float) * nt,
                     hipMemcpyDeviceToHost));
    HIPCHK(hipMemcpy(bp.data(), d->d_bp + (size_t)channel * d->bp_cap + cs.frame_base, sizeof(int2) * nt,
                     hipMemcpyDeviceToHost));
  }
  int32_t k = 0;
  for (int32_t i = 0; i < nt; ++i) {
    if (!(co[i] < INFINITY)) continue;  // dropped by the frame cutoff
    if (k < capacity && states && costs && arcs) {
      states[k] = st[i];
      costs[k] = co[i];
      arcs[k] = (uint32_t)bp[i].x == cbd::kArcNone ? -1 : d->g->int2pub[bp[i].x];
    }
    ++k;
  }
  *n = k;
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "get_tokens: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("get_tokens: ") + e.what());
}

int32_t cbd_get_records(cbd_decoder *d, int32_t channel, int32_t *arcs, int32_t *prev, int32_t capacity,
                        int32_t *n_records, int32_t *frame_base, int32_t *kept_base) try {
  if (!d || !n_records) return fail(CBD_E_INVALID, "get_records: null argument");
  if (channel < 0 || channel >= d->C) return fail(CBD_E_INVALID, "get_records: channel out of range");
  HIPCHK(hipStreamSynchronize(d->stream));
  cbd::ChanState cs;
  HIPCHK(hipMemcpy(&cs, d->d_chan + channel, sizeof(cs), hipMemcpyDeviceToHost));
  *n_records = cs.n_rec;
  if (frame_base) *frame_base = cs.frame_base;
  if (kept_base) *kept_base = cs.gc_base;
  if (!arcs || !prev || capacity < cs.n_rec) return cs.n_rec > 0 && arcs && prev ? CBD_E_BUFFER : CBD_OK;
  std::vector<int2> rec((size_t)std::max(cs.n_rec, 1));
  if (cs.n_rec > 0)
    HIPCHK(hipMemcpy(rec.data(), d->d_bp + (size_t)channel * d->bp_cap, sizeof(int2) * (size_t)cs.n_rec,
                     hipMemcpyDeviceToHost));
  for (int32_t i = 0; i < cs.n_rec; ++i) {
    arcs[i] = (uint32_t)rec[i].x == cbd::kArcNone ? -1 : d->g->int2pub[rec[i].x];
    prev[i] = rec[i].y;
  }
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "get_records: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("get_records: ") + e.what());
}

int32_t cbd_get_stats(cbd_decoder *d, int32_t channel, cbd_stats *out) try {
  if (!d || !out) return fail(CBD_E_INVALID, "get_stats: null argument");
  if (channel < -1 || channel >= d->C) return fail(CBD_E_INVALID, "get_stats: channel out of range");
  HIPCHK(hipStreamSynchronize(d->stream));
  const int32_t lo = channel < 0 ? 0 : channel, hi = channel < 0 ? d->C : channel + 1;
  std::vector<cbd::ChanState> cs((size_t)(hi - lo));
  HIPCHK(hipMemcpy(cs.data(), d->d_chan + lo, sizeof(cbd::ChanState) * cs.size(), hipMemcpyDeviceToHost));
  cbd_stats s{};
  for (const cbd::ChanState &c : cs) {
    s.frames += c.frames; s.active_tokens += c.active_tokens; s.emit_arcs += c.emit_arcs; s.eps_arcs += c.eps_arcs;
    s.candidates += c.candidates; s.improvements += c.improvements; s.tokens += c.tokens;
    s.eps_rounds += c.eps_rounds; s.records += c.n_rec; s.slow_frames += c.slow_frames;
    s.records_dropped += c.gc_dropped; s.compactions += c.gc_runs; s.lean_frames += c.lean_frames;
    if (s.status == CBD_OK && c.status != CBD_OK) s.status = c.status;
    s.max_tokens = std::max(s.max_tokens, c.max_tokens);
  }
  *out = s;
  return CBD_OK;
} catch (const std::bad_alloc &) {
  return fail(CBD_E_NOMEM, "get_stats: host allocation failed");
} catch (const std::exception &e) {
  return fail(CBD_E_HIP, std::string("get_stats: ") + e.what());
}

int32_t cbd_selftest(void) {
  // the decode kernel's wave-level prefix sum and minimum against plain host loops
  int32_t *d_in = nullptr, *d_scan = nullptr;
  uint32_t *d_min = nullptr;
  HIPCHK(hipMalloc((void **)&d_in, 128 * sizeof(int32_t)));
  HIPCHK(hipMalloc((void **)&d_scan, 64 * sizeof(int32_t)));
  HIPCHK(hipMalloc((void **)&d_min, 64 * sizeof(uint32_t)));
  int32_t rc = CBD_OK;
  uint32_t seed = 12345u;
  for (int trial = 0; trial < 8 && rc == CBD_OK; ++trial) {
    int32_t in[128], scan[64];
    uint32_t mn[64];
    for (int i = 0; i < 128; ++i) {
      seed = seed * 1664525u + 1013904223u;
      in[i] = trial == 0 ? 1 : (trial == 1 ? i : (int32_t)(seed >> (i < 64 ? 20 : 0)));
    }
    if (trial == 2) for (int i = 64; i < 128; ++i) in[i] = (i == 64 + 63) ? 7 : 1000 + i;   // minimum in the last lane
    if (trial == 3) for (int i = 64; i < 128; ++i) in[i] = (i == 64) ? 7 : 1000 + i;        // minimum in the first lane
    hipError_t e = hipMemcpy(d_in, in, sizeof(in), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
      hipLaunchKernelGGL(cbd::selftest_kernel, dim3(1), dim3(64), 0, nullptr, d_in, d_scan, d_min);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpy(scan, d_scan, sizeof(scan), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(mn, d_min, sizeof(mn), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { rc = fail(CBD_E_HIP, std::string("selftest: ") + hipGetErrorString(e)); break; }
    int32_t run = 0;
    uint32_t want_min = 0xFFFFFFFFu;
    for (int i = 64; i < 128; ++i) want_min = std::min(want_min, (uint32_t)in[i]);
    for (int i = 0; i < 64; ++i) {
      run += in[i];
      if (scan[i] != run) { rc = fail(CBD_E_HIP, "selftest: wave prefix sum mismatch at lane " + std::to_string(i)); break; }
      if (mn[i] != want_min) { rc = fail(CBD_E_HIP, "selftest: wave minimum mismatch at lane " + std::to_string(i)); break; }
    }
  }
  (void)hipFree(d_in); (void)hipFree(d_scan); (void)hipFree(d_min);
  return rc;
}

#ifdef CBD_PROFILE
// Diagnostic build only: the phase sums a channel's lean frames left (see CBD_STAMP), 15 values, then start, end,
// hardware ids and list place of the workgroup of the channel's last call (ChanState::timeline): 19 values.
int32_t cbd_debug_profile(cbd_decoder *d, int32_t channel, int64_t *out) {
  if (!d || !out || channel < 0 || channel >= d->C) return CBD_E_INVALID;
  HIPCHK(hipStreamSynchronize(d->stream));
  cbd::ChanState cs;
  HIPCHK(hipMemcpy(&cs, d->d_chan + channel, sizeof(cs), hipMemcpyDeviceToHost));
  for (int k = 0; k < 15; ++k) out[k] = cs.spare[k];
  for (int k = 0; k < 4; ++k) out[15 + k] = cs.timeline[k];
  return CBD_OK;
}
#endif

int32_t cbd_synchronize(cbd_decoder *d) {
  if (!d) return fail(CBD_E_INVALID, "synchronize: null decoder");
  HIPCHK(hipStreamSynchronize(d->stream));
  return CBD_OK;
}

}  // extern "C"
