// Communicator: connection FIFOs, flags and semaphores in device memory, instruction tables,
// workgroup placement and kernel launch (Section 6.1 "Point-to-Point Connections" and
// Section 6.2 "Initial Setup" of the paper).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>
#include <mutex>
#include <numeric>
#include <string>
#include <tuple>
#include <vector>

#include "device_tables.h"
#include "plan.h"
#include "program.h"
#include "residency.h"

namespace gc3 {
int launch_interpreter(int dtype, int coherent_user, int mode, bool die_scope, unsigned grid, unsigned block, void* stream,
                       const KParams& p);
int interpreter_occupancy(unsigned block, int kind, int* out);
int static_scratch_ptr(void** out);
int launch_fill_zero(void* ptr, size_t bytes, void* stream);
}  // namespace gc3

using namespace gc3;

namespace {
int dtype_size(int dt) { return dt == GC3_F32 ? 4 : (dt == GC3_F16 || dt == GC3_BF16) ? 2 : 0; }

int hip_fail(hipError_t e, const char* what) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return GC3_ERR_HIP;
}
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);   \
  } while (0)
}  // namespace

struct gc3_comm {
  int device = 0;
  int32_t ranks = 0, in_chunks = 0, out_chunks = 0;
  bool inplace = false;
  bool has_deps = false;    // some instruction waits on another thread block's semaphore
  bool debug_hold = false;  // failure-path test facility
  bool lds_stage = false;   // FIFO payload of the receiving instructions goes through LDS
  bool die_scope = false;   // FIFO payload is read from the L2 of the die both ends of a connection run on
  bool rank_die = false;    // the workgroups of a rank share a die and its user buffers are read through that die's L2
  uint64_t min_lane_bytes = 8192;
  uint64_t ll_max_lane_bytes = 8192;
  uint32_t ll_unit_bytes = 0;
  int max_pushes = 0;
  uint64_t algorithmic_chunks = 0;
  std::vector<int32_t> scratch_chunks;
  gc3_comm_info info{};
  uint64_t spin_limit_ticks = 0;

  // device allocations
  DInstr* d_instrs = nullptr;
  DDep* d_deps = nullptr;
  DWg* d_wgs = nullptr;
  DFiber* d_fibers = nullptr;
  void** d_bufs = nullptr;
  unsigned char* d_fifo = nullptr;
  unsigned char* d_ll_fifo = nullptr;
  uint64_t* d_flags = nullptr;
  uint64_t* d_sems = nullptr;
  uint32_t* d_error = nullptr;
  size_t flags_bytes = 0, sems_bytes = 0;

  // host state
  std::vector<void*> bufs;            // [rank*3 + buffer]
  std::vector<size_t> scratch_bytes;  // capacity bound per rank
  std::vector<char> bound;
  bool poisoned = false;
  hipEvent_t done = nullptr;          // recorded after every launch outside stream capture
  bool done_recorded = false;   // `done` has been recorded at least once
  // The event of the latest run is recorded only when somebody needs it (a status / bind / destroy call, or
  // another communicator's run that has to wait for this one): an event record per run costs a latency-bound
  // collective about 5 us (measured on MI355X: ring AllReduce on 8 ranks at 4 KiB 35 -> 30 us).  Until then the
  // run is known by the stream it was launched on.  Both fields change under the ledger lock only.
  bool event_pending = false;
  hipStream_t last_stream = nullptr;
  hipStream_t aux = nullptr;          // non-blocking stream for the status read-back (stalls no other stream)

  ~gc3_comm() {
    // best effort; errors on teardown are ignored
    for (void* q : {(void*)d_instrs, (void*)d_deps, (void*)d_wgs, (void*)d_fibers, (void*)d_bufs,
                    (void*)d_fifo, (void*)d_ll_fifo, (void*)d_flags, (void*)d_sems, (void*)d_error})
      if (q) (void)hipFree(q);
    if (done) (void)hipEventDestroy(done);
    if (aux) (void)hipStreamDestroy(aux);
  }
};

namespace {

template <class T>
int upload(T** dptr, const std::vector<T>& host) {
  size_t bytes = std::max<size_t>(host.size(), 1) * sizeof(T);
  HIP_TRY(hipMalloc((void**)dptr, bytes));
  if (!host.empty()) HIP_TRY(hipMemcpy(*dptr, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  return GC3_OK;
}

// ---- per-device ledger of runs in flight (see residency.h) -------------------------------------------------
struct LedgerEntry {
  gc3_comm* owner;
  hipStream_t stream;
  int32_t wgs, capacity;
};
constexpr int kMaxLedgerDevices = 64;
std::vector<LedgerEntry> g_ledger[kMaxLedgerDevices];
std::mutex g_ledger_lock;

// Record the event of `c`'s latest run if that is still to be done (the caller holds g_ledger_lock).  Recorded
// later than the run itself, the event also covers whatever was put on that stream in between, which only
// makes a wait for it more conservative.
int settle_event(gc3_comm* c) {
  if (!c->event_pending) return GC3_OK;
  HIP_TRY(hipEventRecord(c->done, c->last_stream));
  c->event_pending = false;
  c->done_recorded = true;
  return GC3_OK;
}

// Wait on the host for `c`'s latest run (not under the ledger lock).  If the event cannot be recorded any more
// (the caller destroyed the run's stream), the whole device is waited for instead.
int wait_for_last_run(gc3_comm* c) {
  int rc;
  {
    std::lock_guard<std::mutex> hold(g_ledger_lock);
    rc = settle_event(c);
    if (rc != GC3_OK) c->event_pending = false;
  }
  if (rc != GC3_OK) {
    (void)hipGetLastError();
    HIP_TRY(hipDeviceSynchronize());
    return GC3_OK;
  }
  if (c->done_recorded) HIP_TRY(hipEventSynchronize(c->done));
  return GC3_OK;
}

void ledger_forget(const gc3_comm* c, int device) {
  if (device < 0 || device >= kMaxLedgerDevices) return;
  std::lock_guard<std::mutex> hold(g_ledger_lock);
  auto& v = g_ledger[device];
  v.erase(std::remove_if(v.begin(), v.end(), [&](const LedgerEntry& e) { return e.owner == c; }), v.end());
}

// Before a launch of `wgs` workgroups on `st` (the caller holds g_ledger_lock from here until it has entered the
// run with ledger_enter): drop finished runs and make `st` wait for the runs on other streams that could not be
// resident beside this one.
int ledger_make_room(const gc3_comm* c, int device, hipStream_t st, int32_t wgs, int32_t capacity) {
  if (device < 0 || device >= kMaxLedgerDevices) return GC3_OK;
  auto& v = g_ledger[device];
  // this communicator's earlier run is ordered before the new one by the caller (runs of one communicator
  // must not overlap); other owners' runs that have completed no longer occupy the device
  v.erase(std::remove_if(v.begin(), v.end(), [&](const LedgerEntry& e) { return e.owner == c; }), v.end());
  for (LedgerEntry& e : v) {
    if (settle_event(e.owner) != GC3_OK) {
      // the other communicator's stream is gone: nothing can be recorded on it any more, so wait for everything
      // the device still runs (its run included) and count that run as finished
      e.owner->event_pending = false;
      (void)hipGetLastError();
      HIP_TRY(hipDeviceSynchronize());
      e.wgs = 0;
    }
  }
  v.erase(std::remove_if(v.begin(), v.end(), [&](const LedgerEntry& e) {
            return e.wgs == 0 || !e.owner->done_recorded || hipEventQuery(e.owner->done) == hipSuccess;
          }), v.end());
  std::vector<InFlightRun> runs;
  for (const LedgerEntry& e : v) runs.push_back({(uint64_t)(uintptr_t)e.stream, e.wgs, e.capacity});
  std::vector<char> wait_on;
  if (residency_waits(runs, (uint64_t)(uintptr_t)st, wgs, capacity, wait_on) > 0)
    for (size_t i = 0; i < v.size(); ++i)
      if (wait_on[i]) HIP_TRY(hipStreamWaitEvent(st, v[i].owner->done, 0));
  return GC3_OK;
}

void ledger_enter(gc3_comm* c, int device, hipStream_t st, int32_t wgs, int32_t capacity) {
  c->last_stream = st;
  c->event_pending = true;
  if (device < 0 || device >= kMaxLedgerDevices) return;
  g_ledger[device].push_back({c, st, wgs, capacity});
}

// What one run launches, as far as it depends on the chunk size only: active lanes, tile, protocol, grid.
struct Launch {
  KParams p{};
  unsigned grid = 0, block = 0;
  bool ll = false;
  int mode = 0;              // kernel variant: 0 general, 1 LL, 2 payload staged through LDS, 3 wavefront-level, 4 wavefront-level LL
  bool die = false;          // FIFO payload at die scope in this run
  uint64_t lane_share = 0;   // largest share a lane has of a chunk, bytes
};

void shape_run_with(const gc3_comm_info& info, uint64_t cb, uint64_t min_lane_bytes, uint64_t ll_max_lane_bytes,
                    bool lds_stage, Launch& L);
void shape_run(const gc3_comm_info& info, uint64_t cb, uint64_t min_lane_bytes, uint64_t ll_max_lane_bytes, bool lds_stage,
               Launch& L);

// The same with the FIFO scope of the run.  Die scope launches bin-major (workgroup = bin x active lanes + lane):
// with a multiple of 8 active lanes, lane w of every thread block then runs on die w mod 8, so both ends of every
// connection share a die; fiber lists must not be split over other lanes' workgroups.
void shape_run(const gc3_comm_info& info, uint64_t cb, uint64_t min_lane_bytes, uint64_t ll_max_lane_bytes, bool lds_stage,
               bool die_scope, Launch& L) {
  shape_run(info, cb, min_lane_bytes, ll_max_lane_bytes, lds_stage, L);
  L.die = die_scope && !L.ll && !lds_stage && L.p.nsplit == 1 && L.p.W_active % 8 == 0;
  L.p.bin_major = L.die ? 1u : 0u;
}

// min_lane_bytes = 0 selects it per run: 8192 (one sweep of a 128-thread workgroup with four 128-bit accesses
// in flight per thread), or 4096 (the same for one wavefront) when the run then uses the wavefront-level
// interpreter - measured on MI355X, ring AllReduce on 8 ranks at 256 KiB: 4 lanes x 8 KiB 45 us, 8 x 4 KiB 38 us.
void shape_run(const gc3_comm_info& info, uint64_t cb, uint64_t min_lane_bytes, uint64_t ll_max_lane_bytes, bool lds_stage,
               Launch& L) {
  if (min_lane_bytes != 0) { shape_run_with(info, cb, min_lane_bytes, ll_max_lane_bytes, lds_stage, L); return; }
  shape_run_with(info, cb, 8192, ll_max_lane_bytes, lds_stage, L);
  if (L.mode != 3 && L.mode != 4) return;
  Launch finer = L;
  shape_run_with(info, cb, 4096, ll_max_lane_bytes, lds_stage, finer);
  if (finer.mode == L.mode) L = finer;
}

void shape_run_with(const gc3_comm_info& info, uint64_t cb, uint64_t min_lane_bytes, uint64_t ll_max_lane_bytes,
                    bool lds_stage, Launch& L) {
  KParams& p = L.p;
  p.chunk_bytes = cb;
  p.W = (uint32_t)info.team_width;
  // small chunks are not worth splitting over all lanes: every active lane gets at least min_lane_bytes
  p.W_active = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(p.W, cb / min_lane_bytes));
  p.slots = (uint32_t)info.fifo_slots;
  p.head_mask = (uint32_t)std::max(1, info.head_stride) - 1;
  p.unit_bytes = (uint32_t)info.tile_bytes;
  // Shares are computed exactly as the kernel does.
  uint64_t lane_share = 0;
  {
    const uint64_t U = cb >> 4, Wa = p.W_active;
    auto begin = [&](uint64_t w) -> uint64_t {
      if (w >= Wa) return U << 4;
      if (U >= 16 * Wa) return (((U >> 4) * w) / Wa) << 8;
      return ((U * w) / Wa) << 4;
    };
    for (uint64_t w = 0; w < Wa; ++w) lane_share = std::max(lane_share, begin(w + 1) - begin(w));
  }
  L.lane_share = lane_share;
  // Tile of this run: about half of the largest lane share (two tiles per chunk keep sender and receiver
  // overlapped), at least 16 KiB, at most the tile the FIFO slots were sized for.
  {
    uint64_t t = ((lane_share + 1) / 2 + 255) & ~255ull;
    t = std::max<uint64_t>(t, 16384);
    p.tile_bytes = (uint32_t)std::min<uint64_t>(t, (uint64_t)info.tile_bytes);
  }
  // Protocol of this run (Section 6.1): LL when forced, or in auto mode when the largest share a lane
  // has of a chunk is small.
  L.ll = info.protocol == 2 || (info.protocol == 3 && lane_share <= ll_max_lane_bytes);
  if (L.ll) p.tile_bytes = (uint32_t)ll_max_lane_bytes;
  // Lane-major grid: the workgroups of the active lanes are a prefix.  When only some lanes own bytes, the
  // workgroups of the others take over part of the work: the fiber list of every (lane, bin) is dealt
  // round-robin to nsplit workgroups, so that on small buffers thread blocks that share a workgroup in the
  // plan run side by side instead.  Never more workgroups than the plan's (resident) grid.
  p.wgs_per_lane = (uint32_t)info.wgs_per_lane;
  p.nsplit = std::max<uint32_t>(1, std::min<uint32_t>(p.W / p.W_active, (uint32_t)info.max_fibers_per_wg));
  L.grid = p.W_active * p.nsplit * p.wgs_per_lane;
  // A lane share of a few KiB is a handful of 128-bit accesses per thread even for one wavefront: such runs are
  // latency-bound, and fewer threads mean less to synchronise per instruction.  When every workgroup runs a
  // single fiber, one wavefront per workgroup needs no synchronisation at all (measured on MI355X: ring
  // AllReduce on 8 ranks up to 1 MiB 44-47 us with 128 threads, 37-39 us with 64); otherwise two wavefronts
  // (2-3 % faster than four up to 8 KiB per lane, slower above).
  L.block = (unsigned)info.wg_size;
  const bool single_fiber = (uint32_t)info.max_fibers_per_wg <= p.nsplit;
  if (lane_share <= 8192 && (L.ll || !lds_stage) && single_fiber) L.block = 64;
  else if (L.block > 128 && lane_share <= 8192) L.block = 128;
  // Instantiation: LL, or payload staged through LDS, or - for workgroups of one wavefront that each run one
  // fiber - the wavefront-level interpreter (simple or LL protocol), or the general one.
  L.mode = 0;
  if (L.ll) L.mode = (L.block == 64 && single_fiber) ? 4 : 1;
  else if (lds_stage) L.mode = 2;
  else if (L.block == 64 && single_fiber) L.mode = 3;
}

}  // namespace

extern "C" {

int gc3_comm_create(const gc3_program* prog, const gc3_comm_config* cfg_in, gc3_comm** out) {
  if (!prog || !out) { set_error("null argument"); return GC3_ERR_ARG; }
  *out = nullptr;
  gc3_comm_config cfg{};
  std::string msg;
  int rc = resolve_config(cfg_in, cfg, msg);
  if (rc != GC3_OK) { set_error(msg); return rc; }

  gc3_comm* c = new gc3_comm();
  struct Guard { gc3_comm* c; ~Guard() { delete c; } } guard{c};
  HIP_TRY(hipGetDevice(&c->device));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, c->device));
  int occ = 0;
  {
    int e = interpreter_occupancy((unsigned)cfg.wg_size, cfg.lds_stage ? 1 : cfg.fifo_scope == 2 ? 2 : 0, &occ);
    if (e != 0) return hip_fail((hipError_t)e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
  }
  // all workgroups wait on each other, so the whole grid has to be resident at once (Section 6.2)
  Plan plan;
  rc = make_plan(*prog, cfg, prop.multiProcessorCount, (long)occ * prop.multiProcessorCount, plan, msg);
  if (rc != GC3_OK) { set_error(msg); return rc; }

  const int R = prog->ranks;
  const int W = plan.info.team_width;
  c->flags_bytes = std::max<size_t>(1, (size_t)plan.nconn * W * 2) * kFlagStrideWords * sizeof(uint64_t);
  c->sems_bytes = std::max<size_t>(1, (size_t)plan.ntb * W) * kFlagStrideWords * sizeof(uint64_t);
  if ((rc = upload(&c->d_instrs, plan.instrs)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_deps, plan.deps)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_wgs, plan.wgs)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_fibers, plan.fibers)) != GC3_OK) return rc;
  HIP_TRY(hipMalloc((void**)&c->d_bufs, (size_t)R * 3 * sizeof(void*)));
  HIP_TRY(hipMalloc((void**)&c->d_fifo, plan.info.fifo_bytes));
  if (plan.info.ll_fifo_bytes) {
    // LL slots must never hold anything but (data, flag) pairs: start from zero, flags start at 1
    HIP_TRY(hipMalloc((void**)&c->d_ll_fifo, plan.info.ll_fifo_bytes));
    HIP_TRY(hipMemset(c->d_ll_fifo, 0, plan.info.ll_fifo_bytes));
  }
  HIP_TRY(hipMalloc((void**)&c->d_flags, c->flags_bytes));
  HIP_TRY(hipMalloc((void**)&c->d_sems, c->sems_bytes));
  HIP_TRY(hipMalloc((void**)&c->d_error, 256));
  HIP_TRY(hipMemset(c->d_flags, 0, c->flags_bytes));
  HIP_TRY(hipMemset(c->d_sems, 0, c->sems_bytes));
  HIP_TRY(hipMemset(c->d_error, 0, 256));
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipEventCreateWithFlags(&c->done, hipEventDisableTiming));
  HIP_TRY(hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking));

  c->ranks = R;
  c->in_chunks = prog->in_chunks;
  c->out_chunks = prog->inplace ? prog->in_chunks : prog->out_chunks;
  c->inplace = prog->inplace;
  c->algorithmic_chunks = plan.algorithmic_chunks;
  c->has_deps = !plan.deps.empty();
  c->debug_hold = cfg.debug_hold != 0;
  c->lds_stage = cfg.lds_stage != 0;
  c->die_scope = cfg.fifo_scope == 2;
  c->rank_die = cfg.user_scope == 2;
  c->min_lane_bytes = (uint64_t)cfg.min_lane_bytes;
  c->ll_max_lane_bytes = (uint64_t)cfg.ll_max_lane_bytes;
  c->ll_unit_bytes = (uint32_t)(2ull * (uint64_t)cfg.ll_max_lane_bytes);
  c->max_pushes = plan.max_pushes;
  for (int r = 0; r < R; ++r) c->scratch_chunks.push_back(prog->rank[r].scratch_chunks);
  c->bufs.assign((size_t)R * 3, nullptr);
  c->scratch_bytes.assign(R, 0);
  c->bound.assign(R, 0);
  c->spin_limit_ticks = cfg.spin_limit_us * 100ull;  // wall clock runs at 100 MHz
  c->info = plan.info;
  guard.c = nullptr;
  *out = c;
  return GC3_OK;
}

int gc3_comm_info_get(const gc3_comm* comm, gc3_comm_info* out) {
  if (!comm || !out) { set_error("null argument"); return GC3_ERR_ARG; }
  *out = comm->info;
  return GC3_OK;
}

int gc3_comm_bind(gc3_comm* comm, int rank, void* input, void* output, void* scratch, size_t scratch_bytes) {
  if (!comm) { set_error("null communicator"); return GC3_ERR_ARG; }
  if (rank < 0 || rank >= comm->ranks) { set_error("rank out of range"); return GC3_ERR_ARG; }
  if (!input) { set_error("input buffer is null"); return GC3_ERR_ARG; }
  if (comm->inplace) {
    if (output && output != input) { set_error("in-place program: output must alias input"); return GC3_ERR_ARG; }
    output = input;
  } else if (!output || output == input) {
    set_error("out-of-place program needs a separate output buffer");
    return GC3_ERR_ARG;
  }
  if (comm->scratch_chunks[rank] > 0 && !scratch) { set_error("rank uses scratch chunks but scratch is null"); return GC3_ERR_ARG; }
  for (void* p : {input, output, scratch})
    if ((uintptr_t)p % 16) { set_error("buffers must be 16-byte aligned"); return GC3_ERR_ARG; }
  // The device-side pointer table is updated here, synchronously, so that a run has nothing to copy and
  // its kernel arguments never change; an earlier run of this communicator still reads the table, so it is
  // waited for first.
  int wrc = wait_for_last_run(comm);
  if (wrc != GC3_OK) return wrc;
  void* triple[3] = {input, output, scratch};
  HIP_TRY(hipMemcpy(comm->d_bufs + (size_t)rank * 3, triple, sizeof(triple), hipMemcpyHostToDevice));
  comm->bufs[(size_t)rank * 3 + 0] = input;
  comm->bufs[(size_t)rank * 3 + 1] = output;
  comm->bufs[(size_t)rank * 3 + 2] = scratch;
  comm->scratch_bytes[rank] = scratch ? scratch_bytes : 0;
  comm->bound[rank] = 1;
  return GC3_OK;
}

static int chunk_bytes_of(const gc3_comm* comm, size_t elems, int dtype, uint64_t* out) {
  int es = dtype_size(dtype);
  if (!es) { set_error("unknown dtype"); return GC3_ERR_ARG; }
  if (elems % (size_t)comm->in_chunks) { set_error("elems_per_rank is not a multiple of the program's chunk count"); return GC3_ERR_SIZE; }
  uint64_t cb = (uint64_t)(elems / comm->in_chunks) * es;
  if (cb % 16) { set_error("chunk size is not a multiple of 16 bytes"); return GC3_ERR_SIZE; }
  if (cb >> 40) { set_error("chunks of 1 TiB and more are not supported"); return GC3_ERR_SIZE; }
  *out = cb;
  return GC3_OK;
}

int gc3_comm_algorithmic_bytes(const gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, uint64_t* out) {
  if (!comm || !out) { set_error("null argument"); return GC3_ERR_ARG; }
  uint64_t cb = 0;
  int rc = chunk_bytes_of(comm, elems_per_rank, dtype, &cb);
  if (rc != GC3_OK) return rc;
  *out = comm->algorithmic_chunks * cb;
  return GC3_OK;
}

int gc3_comm_launch_info(const gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, gc3_launch_info* out) {
  if (!comm || !out) { set_error("null argument"); return GC3_ERR_ARG; }
  uint64_t cb = 0;
  int rc = chunk_bytes_of(comm, elems_per_rank, dtype, &cb);
  if (rc != GC3_OK) return rc;
  Launch L;
  shape_run(comm->info, cb, comm->min_lane_bytes, comm->ll_max_lane_bytes, comm->lds_stage, comm->die_scope, L);
  *out = gc3_launch_info{};
  out->grid = (elems_per_rank == 0 || comm->info.grid == 0) ? 0 : (int32_t)L.grid;
  out->wg_size = (int32_t)L.block;
  out->active_lanes = (int32_t)L.p.W_active;
  out->split = (int32_t)L.p.nsplit;
  out->tile_bytes = (int32_t)L.p.tile_bytes;
  out->kernel = L.mode;
  out->die_scope = L.die ? 1 : 0;
  out->lane_bytes = L.lane_share;
  return GC3_OK;
}

int gc3_comm_run(gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, gc3_redop op, void* hip_stream) {
  if (!comm) { set_error("null communicator"); return GC3_ERR_ARG; }
  if (op != GC3_SUM) { set_error("unknown reduction"); return GC3_ERR_ARG; }
  if (comm->poisoned) { set_error("an earlier run failed; call gc3_comm_reset"); return GC3_ERR_POISONED; }
  uint64_t cb = 0;
  int rc = chunk_bytes_of(comm, elems_per_rank, dtype, &cb);
  if (rc != GC3_OK) return rc;
  for (int r = 0; r < comm->ranks; ++r) {
    if (!comm->bound[r]) { set_error("rank " + std::to_string(r) + " has no buffers bound"); return GC3_ERR_UNBOUND; }
    if ((uint64_t)comm->scratch_chunks[r] * cb > comm->scratch_bytes[r]) {
      set_error("rank " + std::to_string(r) + ": scratch buffer too small for this size");
      return GC3_ERR_SIZE;
    }
  }
  if (elems_per_rank == 0 || comm->info.grid == 0) return GC3_OK;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != comm->device) { set_error("communicator belongs to another device"); return GC3_ERR_ARG; }
  hipStream_t st = (hipStream_t)hip_stream;
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  HIP_TRY(hipStreamIsCapturing(st, &capture));
  const bool capturing = capture != hipStreamCaptureStatusNone;
  Launch L;
  KParams& p = L.p;
  p.instrs = comm->d_instrs;
  p.deps = comm->d_deps;
  p.wgs = comm->d_wgs;
  p.fibers = comm->d_fibers;
  p.bufs = comm->d_bufs;
  p.fifo = comm->d_fifo;
  p.flags = comm->d_flags;
  p.sems = comm->d_sems;
  p.error = comm->d_error;
  p.hold = comm->debug_hold ? comm->d_error + 32 : nullptr;   // a word of the zeroed error block nobody writes
  p.spin_limit_ticks = comm->spin_limit_ticks;
  shape_run(comm->info, cb, comm->min_lane_bytes, comm->ll_max_lane_bytes, comm->lds_stage, comm->die_scope, L);
  p.ll_fifo = comm->d_ll_fifo;
  p.ll_unit_bytes = comm->ll_unit_bytes;
  if (L.ll) {
    // an upper bound of the messages one connection carries in this run: the same for every run of one size, so
    // the kernel's arguments stay constant (the fibers keep the running message number in device memory)
    const uint64_t tiles = (L.lane_share + p.tile_bytes - 1) / p.tile_bytes;
    const uint64_t messages = (uint64_t)comm->max_pushes * tiles + 1;
    if (messages >= (1ull << 31)) { set_error("too many tiles for the LL protocol"); return GC3_ERR_SIZE; }
    p.ll_msgs = (uint32_t)messages;
  }
  // Outside capture the run enters the device's ledger: its stream first waits for runs of other communicators
  // on other streams beside which this grid could not be resident.  A captured launch is replayed at times
  // the library does not see: keeping such launches apart from other communicators' runs is the caller's job.
  std::unique_lock<std::mutex> ledger(g_ledger_lock, std::defer_lock);
  if (!capturing) {
    ledger.lock();
    rc = ledger_make_room(comm, comm->device, st, (int32_t)L.grid, comm->info.max_resident_wgs);
    if (rc != GC3_OK) return rc;
  }
  // die-scope user buffers: the thread blocks of a rank meet in one L2, so their accesses need not bypass it
  // (with die-scope FIFOs the placement is by lanes and holds in the runs that use it; the others fall back to
  // device scope for both)
  const bool user_die = comm->rank_die && (!comm->die_scope || L.die);
  p.rank_die = user_die ? 1u : 0u;
  int e = launch_interpreter((int)dtype, user_die ? 2 : comm->has_deps ? 1 : 0, L.mode, L.die, L.grid, L.block, hip_stream, p);
  if (e != 0) return hip_fail((hipError_t)e, "interpreter launch");
  if (!capturing) {
    ledger_enter(comm, comm->device, st, (int32_t)L.grid, comm->info.max_resident_wgs);
  }
  return GC3_OK;
}

int gc3_comm_status(gc3_comm* comm) {
  if (!comm) { set_error("null communicator"); return GC3_ERR_ARG; }
  // wait for this communicator's last run only, and read the error word on a stream of its own: no other
  // stream of the process is stalled
  int wrc = wait_for_last_run(comm);
  if (wrc != GC3_OK) return wrc;
  uint32_t err = 0;
  HIP_TRY(hipMemcpyAsync(&err, comm->d_error, sizeof(err), hipMemcpyDeviceToHost, comm->aux));
  HIP_TRY(hipStreamSynchronize(comm->aux));
  if (err != 0) {
    comm->poisoned = true;
    if (-(int)err == GC3_ERR_PLACEMENT)
      set_error(comm->rank_die && comm->die_scope
                    ? "die-scope FIFOs and user buffers: workgroups that have to share a die did not (results not valid); use fifo_scope 1 and user_scope 1"
                    : comm->rank_die ? "die-scope user buffers: the workgroups of a rank did not share a die (results not valid); use user_scope 1"
                                     : "die-scope FIFOs: a receiving workgroup did not run on the die of its sender (run abandoned); use fifo_scope 1");
    else
      set_error("a workgroup waited longer than the spin limit (run abandoned)");
    return -(int)err;
  }
  return GC3_OK;
}

int gc3_comm_reset(gc3_comm* comm) {
  if (!comm) { set_error("null communicator"); return GC3_ERR_ARG; }
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemset(comm->d_flags, 0, comm->flags_bytes));
  HIP_TRY(hipMemset(comm->d_sems, 0, comm->sems_bytes));
  // (the semaphore lines also hold the LL message numbers, which restart: no LL slot may keep a flag of the past)
  if (comm->d_ll_fifo) HIP_TRY(hipMemset(comm->d_ll_fifo, 0, comm->info.ll_fifo_bytes));
  HIP_TRY(hipMemset(comm->d_error, 0, 256));
  HIP_TRY(hipDeviceSynchronize());
  comm->poisoned = false;
  return GC3_OK;
}

void gc3_comm_destroy(gc3_comm* comm) {
  if (!comm) return;
  // the last run launched through the library must have left the device before its state is freed (a run
  // replayed from a captured graph is the caller's to wait for)
  (void)wait_for_last_run(comm);
  ledger_forget(comm, comm->device);
  delete comm;
}

int gc3_comm_tune(const gc3_program* prog, const gc3_comm_config* base, size_t elems_per_rank, gc3_dtype dtype,
                  void* hip_stream, gc3_comm_config* best, gc3_tune_report* report) {
  if (!prog || !best) { set_error("null argument"); return GC3_ERR_ARG; }
  gc3_comm_config cfg0{};
  if (base) cfg0 = *base;
  if (report) std::memset(report, 0, sizeof(*report));
  gc3_program_info pi{};
  int rc = gc3_program_info_get(prog, &pi);
  if (rc != GC3_OK) return rc;
  const int es = dtype_size(dtype);
  if (!es) { set_error("unknown dtype"); return GC3_ERR_ARG; }
  if (elems_per_rank == 0 || elems_per_rank % (size_t)pi.in_chunks) {
    set_error("elems_per_rank must be a positive multiple of the program's chunk count");
    return GC3_ERR_SIZE;
  }
  const uint64_t cb = (uint64_t)(elems_per_rank / pi.in_chunks) * es;
  if (cb % 16) { set_error("chunk size is not a multiple of 16 bytes"); return GC3_ERR_SIZE; }

  // stand-in buffers of the real sizes, one allocation: per rank input, output, scratch; filled with a non-zero
  // byte (0x3c3c3c3c is a small normal number in every supported type): all-zero data moves measurably faster
  // on this hardware and would not rank the plans as real data does
  const uint64_t in_b = cb * pi.in_chunks, out_b = pi.inplace ? 0 : cb * pi.out_chunks;
  std::vector<uint64_t> off(pi.ranks * 3 + 1, 0);
  uint64_t total = 0;
  auto place = [&](int slot, uint64_t bytes) { off[slot] = total; total += (bytes + 255) & ~255ull; };
  for (int r = 0; r < pi.ranks; ++r) {
    int sc = 0;
    rc = gc3_program_scratch_chunks(prog, r, &sc);
    if (rc != GC3_OK) return rc;
    place(r * 3 + 0, in_b);
    place(r * 3 + 1, out_b);
    place(r * 3 + 2, cb * (uint64_t)sc);
  }
  off[pi.ranks * 3] = total;
  struct DeviceBlock { void* p = nullptr; ~DeviceBlock() { if (p) (void)hipFree(p); } } block;
  constexpr int kTimed = 5;
  struct Events {
    hipEvent_t a[kTimed] = {}, b[kTimed] = {};
    ~Events() { for (int i = 0; i < kTimed; ++i) { if (a[i]) (void)hipEventDestroy(a[i]); if (b[i]) (void)hipEventDestroy(b[i]); } }
  } ev;
  HIP_TRY(hipMalloc(&block.p, std::max<uint64_t>(total, 256)));
  HIP_TRY(hipMemset(block.p, 0x3c, std::max<uint64_t>(total, 256)));
  for (int i = 0; i < kTimed; ++i) {
    HIP_TRY(hipEventCreate(&ev.a[i]));
    HIP_TRY(hipEventCreate(&ev.b[i]));
  }
  // Bandwidth-bound sizes are timed the way a collective is used: every run finds inputs that something else has
  // just written (here a fill of the input buffers, outside the timed window), not the cache state its own previous
  // run left behind - the two rank some plans differently by a few per cent.  Latency-bound sizes are timed back
  // to back, where the dispatch gap of a bracketed single run would drown the differences.
  const bool fresh_inputs = in_b * (uint64_t)pi.ranks >= (32ull << 20);
  hipStream_t st = (hipStream_t)hip_stream;

  std::vector<std::tuple<int, int, int>> seen;   // (team width, grid, slot tile) of plans already timed
  double best_ms = 0;
  bool have = false, first_only = false;   // first_only: the best so far is still the caller's configuration
  int last_err = GC3_OK;
  std::string last_msg;
  int best_tile = 0;
  // Times one configuration; returns GC3_OK also when the plan was skipped (does not fit, seen before).
  auto try_config = [&](const gc3_comm_config& cfg) -> int {
    gc3_comm* c = nullptr;
    int rc = gc3_comm_create(prog, &cfg, &c);
    if (rc != GC3_OK) { last_err = rc; last_msg = gc3_last_error(); return GC3_OK; }
    struct CommGuard { gc3_comm* c; ~CommGuard() { gc3_comm_destroy(c); } } cg{c};
    std::tuple<int, int, int> key(c->info.team_width, c->info.grid, c->info.tile_bytes);
    if (std::find(seen.begin(), seen.end(), key) != seen.end()) return GC3_OK;
    seen.push_back(key);
    unsigned char* basep = (unsigned char*)block.p;
    for (int r = 0; r < pi.ranks && rc == GC3_OK; ++r) {
      void* in = basep + off[r * 3];
      void* outp = pi.inplace ? in : (void*)(basep + off[r * 3 + 1]);
      uint64_t sb = off[r * 3 + 3] - off[r * 3 + 2];
      rc = gc3_comm_bind(c, r, in, outp, basep + off[r * 3 + 2], sb);
    }
    // the first plan timed also pays for cold code and freshly mapped stand-in buffers: warm it longer
    const int warm = seen.size() == 1 ? 8 : 2, timed = kTimed;
    auto refill = [&]() -> int {
      for (int r = 0; r < pi.ranks; ++r) HIP_TRY(hipMemsetAsync(basep + off[r * 3], 0x3c, in_b, st));
      return GC3_OK;
    };
    for (int i = 0; i < warm && rc == GC3_OK; ++i) {
      if (fresh_inputs) rc = refill();
      if (rc == GC3_OK) rc = gc3_comm_run(c, elems_per_rank, dtype, GC3_SUM, st);
    }
    if (rc == GC3_OK && !fresh_inputs) {
      HIP_TRY(hipEventRecord(ev.a[0], st));
      for (int i = 0; i < timed && rc == GC3_OK; ++i) rc = gc3_comm_run(c, elems_per_rank, dtype, GC3_SUM, st);
      HIP_TRY(hipEventRecord(ev.b[0], st));
    }
    for (int i = 0; fresh_inputs && i < timed && rc == GC3_OK; ++i) {
      rc = refill();
      if (rc != GC3_OK) break;
      HIP_TRY(hipEventRecord(ev.a[i], st));
      rc = gc3_comm_run(c, elems_per_rank, dtype, GC3_SUM, st);
      HIP_TRY(hipEventRecord(ev.b[i], st));
    }
    if (rc == GC3_OK) rc = gc3_comm_status(c);   // synchronises
    if (rc != GC3_OK) {
      last_err = rc; last_msg = gc3_last_error();
      if (rc == GC3_ERR_TIMEOUT || rc == GC3_ERR_HIP) { set_error("tuning run failed: " + last_msg); return rc; }
      return GC3_OK;
    }
    float ms = 0;
    if (fresh_inputs) {
      for (int i = 0; i < timed; ++i) {
        float one = 0;
        HIP_TRY(hipEventElapsedTime(&one, ev.a[i], ev.b[i]));
        ms += one;
      }
    } else {
      HIP_TRY(hipEventElapsedTime(&ms, ev.a[0], ev.b[0]));
    }
    const double per = (double)ms / timed;
    // the caller's configuration is timed first and is replaced only by a plan that is faster by more than
    // the run-to-run noise (2 %); after that every strictly faster plan wins
    const bool better = !have || (first_only ? per < 0.98 * best_ms : per < best_ms);
    if (report && report->count < GC3_TUNE_MAX_TRIED) {
      auto& e = report->tried[report->count];
      e.team_width = c->info.team_width; e.target_wgs = cfg.target_wgs; e.grid = c->info.grid;
      e.active_wgs = c->info.active_wgs; e.tile_bytes = c->info.tile_bytes; e.wg_size = c->info.wg_size; e.fifo_scope = cfg.fifo_scope == 2 ? 2 : 1; e.protocol = c->info.protocol; e.min_lane_bytes = cfg.min_lane_bytes; e.fifo_slots = c->info.fifo_slots; e.user_scope = c->info.user_scope; e.ms = per;
      if (better) report->best = report->count;
      ++report->count;
    }
    if (better) {
      first_only = !have;
      have = true; best_ms = per;
      *best = cfg;
      best_tile = c->info.tile_bytes;
    }
    return GC3_OK;
  };
  // pass 1: team width x workgroup target, the caller's configuration as given first
  static const int widths[] = {0, 4, 8, 16, 32, 64};
  static const int targets[] = {0, 512, 768};
  for (int w : widths)
    for (int t : targets) {
      gc3_comm_config cfg = cfg0;
      if (w != 0 || t != 0) {
        if ((cfg0.team_width && w) || (cfg0.target_wgs && t)) continue;   // fixed by the caller
        if (w) cfg.team_width = w;
        if (t) cfg.target_wgs = t;
      }
      if ((rc = try_config(cfg)) != GC3_OK) return rc;
    }
  // pass 2: the slot tile of the winner (it bounds the tile of a run and sets the FIFO footprint)
  if (have && cfg0.tile_bytes == 0) {
    const gc3_comm_config winner = *best;
    for (int tile : {16384, 32768, 65536}) {
      if (tile == best_tile) continue;
      gc3_comm_config cfg = winner;
      cfg.tile_bytes = tile;
      if ((rc = try_config(cfg)) != GC3_OK) return rc;
    }
  }
  // pass 3: smaller workgroups for the winner (less to synchronise per instruction)
  if (have && cfg0.wg_size == 0) {
    gc3_comm_config cfg = *best;
    cfg.wg_size = 128;
    seen.clear();        // a plan of another workgroup size is a different plan even if W, grid and tile agree
    seen.emplace_back(-1, -1, -1);   // (keeps the longer warm-up for the very first plan only)
    if ((rc = try_config(cfg)) != GC3_OK) return rc;
    // and as many 128-thread workgroups as the device holds, for programs whose thread blocks wait on each other a
    // lot (All Pairs AllReduce at 64 MiB: 128 lanes, 3072 workgroups, 6.4 -> 6.65 TB/s on MI355X)
    for (int w : {64, 128}) {
      if ((cfg0.team_width && cfg0.team_width != w) || cfg0.target_wgs) continue;
      gc3_comm_config wide = cfg0;
      wide.wg_size = 128;
      wide.team_width = w;
      wide.target_wgs = 3584;
      if (cfg0.tile_bytes == 0) wide.tile_bytes = 16384;
      if ((rc = try_config(wide)) != GC3_OK) return rc;
    }
  }
  // pass 4: workgroups of one wavefront.  Where every workgroup then runs a single fiber the wavefront-level
  // interpreter is used (no barriers); four times as many workgroups fit the device, so wider teams and larger
  // workgroup targets come into reach (All Pairs AllReduce at 64 MiB: 4.8 -> 6.2 TB/s on MI355X).
  if (have && cfg0.wg_size == 0) {
    seen.clear();
    seen.emplace_back(-1, -1, -1);
    // besides 16, 32 and 64 lanes: the widest team with which every thread block still gets workgroups of its own
    // (the planner shares nothing then), for programs with many thread blocks (AllToNext on 3 x 8 ranks: 396 thread
    // blocks x 10 lanes, 6.36 -> 6.68 TB/s on MI355X)
    int widths64[4] = {16, 32, 64, 0};
    if (pi.num_tbs > 0) {
      const int w1 = 4096 / pi.num_tbs;
      if (w1 >= 2 && w1 < 64 && w1 != 16 && w1 != 32) widths64[3] = w1;
    }
    for (int w : widths64)
      for (int t : {2048, 4096}) {
        if (w == 0 || (w == widths64[3] && t != 4096)) continue;
        if ((cfg0.team_width && cfg0.team_width != w) || (cfg0.target_wgs && cfg0.target_wgs != t)) continue;
        gc3_comm_config cfg = cfg0;
        cfg.wg_size = 64;
        cfg.team_width = w;
        cfg.target_wgs = t;
        if ((rc = try_config(cfg)) != GC3_OK) return rc;
      }
    if (best->wg_size == 64 && cfg0.tile_bytes == 0) {
      const gc3_comm_config winner = *best;
      const int winner_tile = best_tile;
      for (int tile : {16384, 32768, 65536}) {
        if (tile == winner_tile) continue;
        gc3_comm_config cfg = winner;
        cfg.tile_bytes = tile;
        if ((rc = try_config(cfg)) != GC3_OK) return rc;
      }
    }
  }
  // pass 5: die-scope FIFOs (payload read from the L2 of the die both ends of a connection run on): small slot
  // tiles so that a die's slots fit its L2, hence more and smaller workgroups.  On MI355X the ring AllReduce
  // gains 12 % at 64 MiB per rank and 35 % at 16 MiB, programs with many connections (hierarchical) lose.
  if (have && cfg0.fifo_scope == 0 && cfg0.protocol <= 1 && cfg0.lds_stage == 0) {
    seen.clear();
    seen.emplace_back(-1, -1, -1);
    struct Shape { int wg, target; };
    for (Shape sh : {Shape{64, 4096}, Shape{128, 2048}, Shape{256, 0}}) {
      if (cfg0.wg_size && cfg0.wg_size != sh.wg) continue;
      for (int w : {8, 16, 32, 64, 128, 256}) {
        // 256 threads: 8 .. 64 lanes; 128 threads: 16, 32, 64; one wavefront: 16 .. 256 (programs with few thread
        // blocks need that many lanes to fill the device; plans that do not fit are skipped).  Die scope can pay
        // even when the slots are far larger than the L2s: plain stores instead of write-through ones (Two-Step
        // AllToAll on 3 x 8 ranks, 256 threads x 32 lanes: 6.7 -> 7.0 TB/s on MI355X).
        if (sh.wg == 256 ? w > 64 : (w < 16 || (sh.wg == 128 && w > 64))) continue;
        if (cfg0.team_width && cfg0.team_width != w) continue;
        gc3_comm_config cfg = cfg0;
        cfg.fifo_scope = 2;
        cfg.wg_size = sh.wg;
        cfg.team_width = w;
        if (cfg0.target_wgs == 0) cfg.target_wgs = sh.target;
        if ((rc = try_config(cfg)) != GC3_OK) return rc;
        // (the die-scope default tile is small, for slots that fit the L2s; 256 threads want a large one)
        if (sh.wg == 256 && cfg0.tile_bytes == 0) {
          cfg.tile_bytes = 32768;
          if ((rc = try_config(cfg)) != GC3_OK) return rc;
        }
      }
      seen.clear();
      seen.emplace_back(-1, -1, -1);
    }
    if (best->fifo_scope == 2 && cfg0.tile_bytes == 0) {
      const gc3_comm_config winner = *best;
      const int winner_tile = best_tile;
      for (int tile : {8192, 16384, 32768}) {
        if (tile == winner_tile) continue;
        gc3_comm_config cfg = winner;
        cfg.tile_bytes = tile;
        if ((rc = try_config(cfg)) != GC3_OK) return rc;
      }
    }
  }
  // pass 6: the LL protocol (Section 6.1) with workgroups of one wavefront, for runs that are latency-bound.  A hop
  // is then one flagged store and the polling load that finds it.  On MI355X this pays where consecutive steps of
  // a chain are spread over several thread blocks, which then wait ahead of time (one ring over four channels, 4 KiB
  // to 256 KiB: 34 -> 25-28 us), and gains little or loses where one thread block executes them back to back, so it
  // is decided by measurement.
  if (have && cfg0.protocol == 0 && cfg0.lds_stage == 0 && cfg0.fifo_scope != 2 && best_ms < 0.1 &&
      (cfg0.wg_size == 0 || cfg0.wg_size == 64)) {
    seen.clear();
    seen.emplace_back(-1, -1, -1);
    for (int slots : {0, 8}) {                // eight slots: a push hardly ever has to look at the head flag
      if (cfg0.fifo_slots && slots) continue;
      for (int mlb : {0, 1024}) {
        if (cfg0.min_lane_bytes && mlb) continue;
        for (int w : {16, 64}) {
          if (cfg0.team_width && cfg0.team_width != w) continue;
          gc3_comm_config cfg = cfg0;
          cfg.protocol = 2;
          cfg.wg_size = 64;
          cfg.team_width = w;
          if (mlb) cfg.min_lane_bytes = mlb;
          if (slots) cfg.fifo_slots = slots;
          if ((rc = try_config(cfg)) != GC3_OK) return rc;
        }
        seen.clear();
        seen.emplace_back(-1, -1, -1);
      }
    }
  }
  // pass 7: die-scope user buffers - the workgroups of a rank on one die, its buffers read through that die's L2 -
  // for programs whose thread blocks wait on each other: the plan chosen so far, placed that way.  It shortens chains
  // of dependent instructions (All Pairs AllReduce on 8 ranks up to 256 KiB: 21-24 -> 17-19 us back to back on
  // MI355X) and loses where it leaves dies idle (rank counts that are no multiple of 8).
  bool has_deps = false;
  for (const auto& rk : prog->rank)
    for (const auto& tb : rk.tbs)
      for (const auto& in : tb.instrs) has_deps = has_deps || !in.deps.empty();
  if (have && has_deps && cfg0.user_scope == 0 && best->fifo_scope != 2) {
    seen.clear();
    seen.emplace_back(-1, -1, -1);
    gc3_comm_config cfg = *best;
    cfg.user_scope = 2;
    if ((rc = try_config(cfg)) != GC3_OK) return rc;
    // and the shapes that suit such programs, whichever of them won above: as many 128-thread workgroups as the
    // device holds, and workgroups of one wavefront (All Pairs AllReduce at 64 MiB: the 128-thread plan gains 6 %
    // from this placement, the one-wavefront plan loses 4 %, and without it the two are within noise of each other)
    if (cfg0.wg_size == 0 && cfg0.target_wgs == 0) {
      for (int w : {64, 128}) {
        if (cfg0.team_width && cfg0.team_width != w) continue;
        gc3_comm_config wide = cfg0;
        wide.wg_size = 128;
        wide.team_width = w;
        wide.target_wgs = 3584;
        wide.user_scope = 2;
        if (cfg0.tile_bytes == 0) wide.tile_bytes = 16384;
        if ((rc = try_config(wide)) != GC3_OK) return rc;
      }
      seen.clear();
      seen.emplace_back(-1, -1, -1);
      for (int w : {16, 64}) {
        if (cfg0.team_width && cfg0.team_width != w) continue;
        gc3_comm_config one = cfg0;
        one.wg_size = 64;
        one.team_width = w;
        one.target_wgs = 4096;
        one.user_scope = 2;
        if ((rc = try_config(one)) != GC3_OK) return rc;
      }
    }
  }
  if (!have) {
    set_error("no configuration could be timed: " + last_msg);
    return last_err != GC3_OK ? last_err : GC3_ERR_ARG;
  }
  return GC3_OK;
}

}  // extern "C"

// ---- one run for callers that cannot allocate device memory ---------------------------------------------------

namespace {
// What gc3_run_static needs to know of a device, looked up once per device.
struct StaticDevice {
  bool ready = false;
  void* scratch = nullptr;      // this device's copy of the static array
  int cus = 0;
  int occupancy[3][4] = {};     // [plain, LDS-staged, die-scope FIFOs][64, 128, 256, 512 threads]: workgroups per compute unit
};
constexpr int kMaxStaticDevices = 64;
StaticDevice g_static[kMaxStaticDevices];
std::mutex g_static_lock;

int static_device(int dev, const StaticDevice** out) {
  if (dev < 0 || dev >= kMaxStaticDevices) { set_error("device index out of range"); return GC3_ERR_ARG; }
  std::lock_guard<std::mutex> hold(g_static_lock);
  StaticDevice& d = g_static[dev];
  if (!d.ready) {
    void* ptr = nullptr;
    int e = static_scratch_ptr(&ptr);
    if (e != 0) return hip_fail((hipError_t)e, "hipGetSymbolAddress(static scratch)");
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    for (int kind = 0; kind < 3; ++kind) {
      int k = 0;
      for (unsigned block : {64u, 128u, 256u, 512u}) {
        e = interpreter_occupancy(block, kind, &d.occupancy[kind][k++]);
        if (e != 0) return hip_fail((hipError_t)e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
      }
    }
    d.scratch = ptr;
    d.cus = cus;
    d.ready = true;
  }
  *out = &d;
  return GC3_OK;
}

uint64_t align256(uint64_t v) { return (v + 255) & ~255ull; }
}  // namespace

extern "C" int gc3_run_static(const gc3_program* prog, const gc3_comm_config* cfg_in, void* const* inputs,
                              void* const* outputs, void* const* scratch_bufs, const size_t* scratch_bytes,
                              size_t elems_per_rank, gc3_dtype dtype, gc3_redop op, void* hip_stream) {
  if (!prog || !inputs) { set_error("null argument"); return GC3_ERR_ARG; }
  if (op != GC3_SUM) { set_error("unknown reduction"); return GC3_ERR_ARG; }
  const int es = dtype_size(dtype);
  if (!es) { set_error("unknown dtype"); return GC3_ERR_ARG; }
  gc3_comm_config cfg{};
  std::string msg;
  int rc = resolve_config(cfg_in, cfg, msg);
  if (rc != GC3_OK) { set_error(msg); return rc; }
  if (cfg.protocol > 1) { set_error("gc3_run_static runs the simple protocol only"); return GC3_ERR_ARG; }
  cfg.protocol = 1;
  const int R = prog->ranks;
  if (prog->in_chunks <= 0 || elems_per_rank % (size_t)prog->in_chunks) {
    set_error("elems_per_rank is not a multiple of the program's chunk count");
    return GC3_ERR_SIZE;
  }
  const uint64_t cb = (uint64_t)(elems_per_rank / prog->in_chunks) * es;
  if (cb % 16) { set_error("chunk size is not a multiple of 16 bytes"); return GC3_ERR_SIZE; }
  if (cb >> 40) { set_error("chunks of 1 TiB and more are not supported"); return GC3_ERR_SIZE; }
  if (!prog->inplace && !outputs) { set_error("out-of-place program needs output buffers"); return GC3_ERR_ARG; }
  std::vector<void*> bufs((size_t)R * 3, nullptr);
  for (int r = 0; r < R; ++r) {
    void* in = inputs[r];
    void* out = prog->inplace ? in : outputs[r];
    if (prog->inplace && outputs && outputs[r] && outputs[r] != in) {
      set_error("in-place program: output must alias input");
      return GC3_ERR_ARG;
    }
    const int sc = prog->rank[r].scratch_chunks;
    void* sb = (sc > 0 && scratch_bufs) ? scratch_bufs[r] : nullptr;
    if (!in || !out || (!prog->inplace && out == in)) { set_error("rank " + std::to_string(r) + ": bad input / output buffer"); return GC3_ERR_ARG; }
    if (sc > 0 && (!sb || !scratch_bytes)) { set_error("rank " + std::to_string(r) + " uses scratch chunks but has no scratch buffer"); return GC3_ERR_ARG; }
    if (sc > 0 && (uint64_t)sc * cb > scratch_bytes[r]) { set_error("rank " + std::to_string(r) + ": scratch buffer too small for this size"); return GC3_ERR_SIZE; }
    for (void* q : {in, out, sb})
      if ((uintptr_t)q % 16) { set_error("buffers must be 16-byte aligned"); return GC3_ERR_ARG; }
    bufs[(size_t)r * 3 + 0] = in;
    bufs[(size_t)r * 3 + 1] = out;
    bufs[(size_t)r * 3 + 2] = sb;
  }

  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  const StaticDevice* sd = nullptr;
  if ((rc = static_device(dev, &sd)) != GC3_OK) return rc;
  const int occ = sd->occupancy[cfg.lds_stage ? 1 : cfg.fifo_scope == 2 ? 2 : 0][cfg.wg_size == 64 ? 0 : cfg.wg_size == 128 ? 1 : cfg.wg_size == 256 ? 2 : 3];

  // Plan with the FIFOs bounded by what the static array can hold; tables, flags and semaphores are small and
  // get a fixed reserve that is checked exactly below.
  Plan plan;
  const uint64_t reserve = 8ull << 20;
  rc = make_plan(*prog, cfg, sd->cus, (long)occ * sd->cus, plan, msg, kStaticScratchBytes - reserve);
  if (rc != GC3_OK) { set_error("gc3_run_static: " + msg); return rc; }
  if (elems_per_rank == 0 || plan.info.grid == 0) return GC3_OK;

  // Layout: [error block | flags | semaphores] (cleared every call) [pointer table | instructions |
  // dependencies | workgroup headers | fibers] (copied every call) [FIFOs].
  const int W = plan.info.team_width;
  const uint64_t flags_bytes = std::max<uint64_t>(1, (uint64_t)plan.nconn * W * 2) * kFlagStrideWords * sizeof(uint64_t);
  const uint64_t sems_bytes = std::max<uint64_t>(1, (uint64_t)plan.ntb * W) * kFlagStrideWords * sizeof(uint64_t);
  const uint64_t off_flags = 256, off_sems = off_flags + flags_bytes, off_tables = align256(off_sems + sems_bytes);
  const uint64_t t_bufs = 0;
  const uint64_t t_instrs = align256(t_bufs + bufs.size() * sizeof(void*));
  const uint64_t t_deps = align256(t_instrs + plan.instrs.size() * sizeof(DInstr));
  const uint64_t t_wgs = align256(t_deps + plan.deps.size() * sizeof(DDep));
  const uint64_t t_fibers = align256(t_wgs + plan.wgs.size() * sizeof(DWg));
  const uint64_t tables_bytes = align256(t_fibers + plan.fibers.size() * sizeof(DFiber));
  const uint64_t off_fifo = off_tables + tables_bytes;
  const uint64_t need = off_fifo + plan.info.fifo_bytes;
  if (need > kStaticScratchBytes) {
    set_error("gc3_run_static: this program needs " + std::to_string(need) + " bytes of device state, the static array holds " +
              std::to_string((uint64_t)kStaticScratchBytes) + " (use a communicator instead)");
    return GC3_ERR_SIZE;
  }
  std::vector<unsigned char> tables(tables_bytes, 0);
  std::memcpy(tables.data() + t_bufs, bufs.data(), bufs.size() * sizeof(void*));
  if (!plan.instrs.empty()) std::memcpy(tables.data() + t_instrs, plan.instrs.data(), plan.instrs.size() * sizeof(DInstr));
  if (!plan.deps.empty()) std::memcpy(tables.data() + t_deps, plan.deps.data(), plan.deps.size() * sizeof(DDep));
  if (!plan.wgs.empty()) std::memcpy(tables.data() + t_wgs, plan.wgs.data(), plan.wgs.size() * sizeof(DWg));
  if (!plan.fibers.empty()) std::memcpy(tables.data() + t_fibers, plan.fibers.data(), plan.fibers.size() * sizeof(DFiber));

  // `base` is the device address obtained from hipGetSymbolAddress: the array's name is never used here.
  unsigned char* const base = (unsigned char*)sd->scratch;
  hipStream_t st = (hipStream_t)hip_stream;
  // the error word the previous call on this device left, then this call's tables; the host copies of both
  // die with this call, so the stream is drained before going on
  uint32_t previous_error = 0;
  HIP_TRY(hipMemcpyAsync(&previous_error, base, sizeof(previous_error), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipMemcpyAsync(base + off_tables, tables.data(), tables_bytes, hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));
  // flags, semaphores and the error word of whatever ran here before must start at zero
  int e = launch_fill_zero(base, off_tables, hip_stream);
  if (e != 0) return hip_fail((hipError_t)e, "fill launch");
  if (previous_error != 0) {
    set_error("the previous gc3_run_static on this device was abandoned (a wait exceeded the spin limit); its outputs are "
              "incomplete and this call did not run");
    return -(int)previous_error;
  }

  Launch L;
  KParams& p = L.p;
  p.bufs = (void* const*)(base + off_tables + t_bufs);
  p.instrs = (const DInstr*)(base + off_tables + t_instrs);
  p.deps = (const DDep*)(base + off_tables + t_deps);
  p.wgs = (const DWg*)(base + off_tables + t_wgs);
  p.fibers = (const DFiber*)(base + off_tables + t_fibers);
  p.fifo = base + off_fifo;
  p.flags = (uint64_t*)(base + off_flags);
  p.sems = (uint64_t*)(base + off_sems);
  p.error = (uint32_t*)base;
  p.hold = cfg.debug_hold ? (const uint32_t*)(base + 128) : nullptr;
  p.spin_limit_ticks = cfg.spin_limit_us * 100ull;
  shape_run(plan.info, cb, (uint64_t)cfg.min_lane_bytes, (uint64_t)cfg.ll_max_lane_bytes, cfg.lds_stage != 0,
            cfg.fifo_scope == 2, L);
  // (epochs were cleared with the flags: every call is the first run)
  const bool user_die = cfg.user_scope == 2 && (cfg.fifo_scope != 2 || L.die);
  p.rank_die = user_die ? 1u : 0u;
  e = launch_interpreter((int)dtype, user_die ? 2 : plan.deps.empty() ? 0 : 1, L.mode, L.die, L.grid, L.block, hip_stream, p);
  if (e != 0) return hip_fail((hipError_t)e, "interpreter launch");
  return GC3_OK;
}

// ---- selection by buffer size (Section 6, introduction) -----------------------------------------------

struct gc3_selector {
  struct Entry { gc3_comm* comm; uint64_t lo, hi; };
  std::vector<Entry> entries;
};

extern "C" {

int gc3_selector_create(gc3_selector** out) {
  if (!out) { set_error("null argument"); return GC3_ERR_ARG; }
  *out = new gc3_selector();
  return GC3_OK;
}

int gc3_selector_add(gc3_selector* sel, gc3_comm* comm, uint64_t min_bytes, uint64_t max_bytes) {
  if (!sel || !comm) { set_error("null argument"); return GC3_ERR_ARG; }
  if (max_bytes != 0 && max_bytes < min_bytes) { set_error("empty size range"); return GC3_ERR_ARG; }
  if (!sel->entries.empty()) {
    const gc3_comm* first = sel->entries.front().comm;
    if (first->ranks != comm->ranks || first->inplace != comm->inplace) {
      set_error("entries of a selector must agree in rank count and in being in place or not");
      return GC3_ERR_ARG;
    }
  }
  sel->entries.push_back({comm, min_bytes, max_bytes == 0 ? UINT64_MAX : max_bytes});
  return GC3_OK;
}

int gc3_selector_run(gc3_selector* sel, size_t elems_per_rank, gc3_dtype dtype, gc3_redop op, void* hip_stream,
                     int* chosen) {
  if (!sel) { set_error("null selector"); return GC3_ERR_ARG; }
  const int es = dtype_size(dtype);
  if (!es) { set_error("unknown dtype"); return GC3_ERR_ARG; }
  const uint64_t bytes = (uint64_t)elems_per_rank * (uint64_t)es;
  for (size_t i = 0; i < sel->entries.size(); ++i) {
    const auto& e = sel->entries[i];
    if (bytes < e.lo || bytes > e.hi) continue;
    if (chosen) *chosen = (int)i;
    return gc3_comm_run(e.comm, elems_per_rank, dtype, op, hip_stream);
  }
  set_error("no program is registered for " + std::to_string(bytes) + " bytes per rank");
  return GC3_ERR_SIZE;
}

void gc3_selector_destroy(gc3_selector* sel) { delete sel; }

}  // extern "C"
