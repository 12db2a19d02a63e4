// Communicator: connection FIFOs, flags and semaphores in device memory, instruction tables,
// workgroup placement and kernel launch (Section 6.1 "Point-to-Point Connections" and
// Section 6.2 "Initial Setup" of the paper).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <numeric>
#include <string>
#include <tuple>
#include <vector>

#include "device_tables.h"
#include "program.h"

namespace gc3 {
int launch_interpreter(int dtype, bool coherent_user, unsigned grid, unsigned block, void* stream, const KParams& p);
int interpreter_occupancy(unsigned block, int* out);
}  // namespace gc3

using namespace gc3;

namespace {
constexpr int kXcds = 8;  // MI355X: 8 accelerator dies, workgroup i is dispatched to die i mod 8

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
  bool has_deps = false;  // some instruction waits on another thread block's semaphore
  uint64_t algorithmic_chunks = 0;
  std::vector<int32_t> scratch_chunks;
  gc3_comm_info info{};
  uint64_t spin_limit_ticks = 0;

  // device allocations
  DTb* d_tbs = nullptr;
  DInstr* d_instrs = nullptr;
  DDep* d_deps = nullptr;
  uint32_t* d_wgmap = nullptr;
  void** d_bufs = nullptr;
  unsigned char* d_fifo = nullptr;
  uint64_t* d_flags = nullptr;
  uint64_t* d_sems = nullptr;
  uint32_t* d_error = nullptr;
  size_t flags_bytes = 0, sems_bytes = 0;

  // host state
  std::vector<void*> bufs;            // [rank*3 + buffer]
  std::vector<size_t> scratch_bytes;  // capacity bound per rank
  std::vector<char> bound;
  bool bufs_dirty = true;
  bool poisoned = false;
  uint64_t run_number = 0;

  ~gc3_comm() {
    // best effort; errors on teardown are ignored
    for (void* q : {(void*)d_tbs, (void*)d_instrs, (void*)d_deps, (void*)d_wgmap, (void*)d_bufs,
                    (void*)d_fifo, (void*)d_flags, (void*)d_sems, (void*)d_error})
      if (q) (void)hipFree(q);
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

// Union-find over thread blocks: blocks joined by a connection or a dependency form one group.
struct Dsu {
  std::vector<int> p;
  explicit Dsu(int n) : p(n) { std::iota(p.begin(), p.end(), 0); }
  int find(int x) { while (p[x] != x) x = p[x] = p[p[x]]; return x; }
  void join(int a, int b) { p[find(a)] = find(b); }
};

}  // namespace

extern "C" {

int gc3_comm_create(const gc3_program* prog, const gc3_comm_config* cfg_in, gc3_comm** out) {
  if (!prog || !out) { set_error("null argument"); return GC3_ERR_ARG; }
  *out = nullptr;
  gc3_comm_config cfg{};
  if (cfg_in) cfg = *cfg_in;
  if (cfg.fifo_slots == 0) cfg.fifo_slots = 4;
  if (cfg.tile_bytes == 0) cfg.tile_bytes = 32768;
  if (cfg.wg_size == 0) cfg.wg_size = 256;
  if (cfg.spin_limit_us == 0) cfg.spin_limit_us = 10ull * 1000 * 1000;
  if (cfg.fifo_slots < 1 || cfg.fifo_slots > 8) { set_error("fifo_slots must be 1..8"); return GC3_ERR_ARG; }
  if (cfg.tile_bytes < 16 || cfg.tile_bytes % 16 || cfg.tile_bytes > (1 << 20)) {
    set_error("tile_bytes must be a multiple of 16 in [16, 1 MiB]");
    return GC3_ERR_ARG;
  }
  if (cfg.wg_size != 64 && cfg.wg_size != 128 && cfg.wg_size != 256 && cfg.wg_size != 512) {
    set_error("wg_size must be 64, 128, 256 or 512");
    return GC3_ERR_ARG;
  }
  if (cfg.team_width < 0 || cfg.team_width > 256) { set_error("team_width must be 0..256"); return GC3_ERR_ARG; }
  if (cfg.xcd_placement < 0 || cfg.xcd_placement > 2) { set_error("xcd_placement must be 0, 1 or 2"); return GC3_ERR_ARG; }

  std::string msg;
  int rc = validate(*prog, cfg.fifo_slots, msg);
  if (rc != GC3_OK) { set_error(msg); return rc; }

  // ---- flatten the program -------------------------------------------------------------------
  const int R = prog->ranks;
  std::vector<int> tb_base(R + 1, 0);
  for (int r = 0; r < R; ++r) tb_base[r + 1] = tb_base[r] + (int)prog->rank[r].tbs.size();
  const int ntb = tb_base[R];
  if (ntb == 0) { set_error("program has no thread blocks"); return GC3_ERR_INVALID_PROGRAM; }
  std::map<std::tuple<int, int, int>, int> conn_id;
  auto conn_of = [&](int src, int dst, int ch) {
    auto key = std::make_tuple(src, dst, ch);
    auto it = conn_id.find(key);
    if (it != conn_id.end()) return it->second;
    int id = (int)conn_id.size();
    conn_id[key] = id;
    return id;
  };
  std::vector<DTb> tbs(ntb);
  std::vector<DInstr> instrs;
  std::vector<DDep> deps;
  Dsu groups(ntb);
  std::map<int, int> conn_first_tb;
  int max_count = 1;
  uint64_t alg_chunks = 0;
  for (int r = 0; r < R; ++r) {
    for (size_t b = 0; b < prog->rank[r].tbs.size(); ++b) {
      const ThreadBlock& tb = prog->rank[r].tbs[b];
      const int g = tb_base[r] + (int)b;
      DTb& d = tbs[g];
      d = DTb{};
      d.rank = (uint32_t)r;
      d.instr_begin = (uint32_t)instrs.size();
      d.ninstr = (uint32_t)tb.instrs.size();
      d.send_conn = d.recv_conn = -1;
      for (const Instr& in : tb.instrs) {
        if (op_pushes(in.op)) d.send_conn = conn_of(r, tb.send, tb.chan);
        if (op_pops(in.op)) d.recv_conn = conn_of(tb.recv, r, tb.chan);
        DInstr di{};
        di.op = in.op;
        di.srcbuf = (in.srcbuf == BUF_OUT && prog->inplace) ? (uint32_t)BUF_IN : in.srcbuf;
        di.dstbuf = (in.dstbuf == BUF_OUT && prog->inplace) ? (uint32_t)BUF_IN : in.dstbuf;
        di.srcidx = (uint32_t)in.srcidx;
        di.dstidx = (uint32_t)in.dstidx;
        di.count = (uint32_t)in.count;
        di.dep_begin = (uint32_t)deps.size();
        di.ndeps_hasdep = ((uint32_t)in.deps.size() << 1) | (in.hasdep ? 1u : 0u);
        for (auto& dp : in.deps) {
          DDep dd{};
          dd.tb = (uint32_t)(tb_base[r] + dp.first);
          dd.step = (uint32_t)dp.second;
          dd.ninstr = (uint32_t)prog->rank[r].tbs[dp.first].instrs.size();
          deps.push_back(dd);
          groups.join(g, (int)dd.tb);
        }
        instrs.push_back(di);
        max_count = std::max(max_count, in.count);
        alg_chunks += (uint64_t)op_traffic(in.op) * (uint64_t)in.count;
      }
      for (int c : {d.send_conn, d.recv_conn}) {
        if (c < 0) continue;
        auto it = conn_first_tb.find(c);
        if (it == conn_first_tb.end()) conn_first_tb[c] = g;
        else groups.join(g, it->second);
      }
    }
  }
  const int nconn = (int)conn_id.size();

  // ---- device, team width, residency -----------------------------------------------------------
  gc3_comm* c = new gc3_comm();
  struct Guard { gc3_comm* c; ~Guard() { delete c; } } guard{c};
  HIP_TRY(hipGetDevice(&c->device));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, c->device));
  const int cus = prop.multiProcessorCount;
  int occ = 0;
  {
    int e = interpreter_occupancy((unsigned)cfg.wg_size, &occ);
    if (e != 0) return hip_fail((hipError_t)e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
  }
  const long resident = (long)occ * cus;
  int W = cfg.team_width;
  if (W == 0) {
    // about four workgroups per compute unit (enough bytes in flight to cover memory latency),
    // never beyond residency
    long target = std::min<long>(4L * cus, resident);
    W = (int)std::max<long>(1, std::min<long>(64, target / ntb));
  }
  const long active = (long)ntb * W;

  // ---- placement: workgroup index -> (thread block, lane) ------------------------------------------
  std::vector<uint32_t> wgmap;
  if (cfg.xcd_placement == 2) {
    wgmap.resize(active);
    for (long i = 0; i < active; ++i) wgmap[i] = (uint32_t)i;
  } else {
    // groups of thread blocks that talk to each other, one copy per lane, spread over the dies
    std::map<int, std::vector<int>> members;
    for (int g = 0; g < ntb; ++g) members[groups.find(g)].push_back(g);
    std::vector<std::vector<uint32_t>> per_xcd(kXcds);
    std::vector<std::pair<size_t, int>> order;  // (size, root), large groups first
    for (auto& kv : members) order.emplace_back(kv.second.size(), kv.first);
    std::stable_sort(order.begin(), order.end(), [](auto& a, auto& b) { return a.first > b.first; });
    // no die takes more than its fair share, so a group larger than that spills onto the next die
    const size_t fair = (size_t)((active + kXcds - 1) / kXcds);
    auto least_loaded = [&]() {
      int best = 0;
      for (int x = 1; x < kXcds; ++x)
        if (per_xcd[x].size() < per_xcd[best].size()) best = x;
      return best;
    };
    for (auto& o : order) {
      for (int w = 0; w < W; ++w) {
        int cur = least_loaded();
        for (int g : members[o.second]) {
          if (per_xcd[cur].size() >= fair) cur = least_loaded();
          per_xcd[cur].push_back((uint32_t)(g * W + w));
        }
      }
    }
    size_t longest = 0;
    for (auto& v : per_xcd) longest = std::max(longest, v.size());
    wgmap.assign(longest * kXcds, kIdleWg);
    for (int x = 0; x < kXcds; ++x)
      for (size_t k = 0; k < per_xcd[x].size(); ++k) wgmap[k * kXcds + x] = per_xcd[x][k];
  }
  const long grid = (long)wgmap.size();
  if (grid > resident) {
    set_error("program needs " + std::to_string(grid) + " resident workgroups of " + std::to_string(cfg.wg_size) +
              " threads, the device holds " + std::to_string(resident));
    return GC3_ERR_RESIDENCY;
  }

  // ---- allocate ---------------------------------------------------------------------------------
  const uint64_t slot_bytes = (uint64_t)max_count * (uint64_t)cfg.tile_bytes;
  const uint64_t fifo_bytes = std::max<uint64_t>(16, (uint64_t)nconn * W * cfg.fifo_slots * slot_bytes);
  if (slot_bytes > (1ull << 30) || fifo_bytes > (64ull << 30)) { set_error("FIFO memory too large"); return GC3_ERR_SIZE; }
  c->flags_bytes = std::max<size_t>(1, (size_t)nconn * W * 2) * kFlagStrideWords * sizeof(uint64_t);
  c->sems_bytes = (size_t)ntb * W * kFlagStrideWords * sizeof(uint64_t);
  if ((rc = upload(&c->d_tbs, tbs)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_instrs, instrs)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_deps, deps)) != GC3_OK) return rc;
  if ((rc = upload(&c->d_wgmap, wgmap)) != GC3_OK) return rc;
  HIP_TRY(hipMalloc((void**)&c->d_bufs, (size_t)R * 3 * sizeof(void*)));
  HIP_TRY(hipMalloc((void**)&c->d_fifo, fifo_bytes));
  HIP_TRY(hipMalloc((void**)&c->d_flags, c->flags_bytes));
  HIP_TRY(hipMalloc((void**)&c->d_sems, c->sems_bytes));
  HIP_TRY(hipMalloc((void**)&c->d_error, 256));
  HIP_TRY(hipMemset(c->d_flags, 0, c->flags_bytes));
  HIP_TRY(hipMemset(c->d_sems, 0, c->sems_bytes));
  HIP_TRY(hipMemset(c->d_error, 0, 256));
  HIP_TRY(hipDeviceSynchronize());

  c->ranks = R;
  c->in_chunks = prog->in_chunks;
  c->out_chunks = prog->inplace ? prog->in_chunks : prog->out_chunks;
  c->inplace = prog->inplace;
  c->algorithmic_chunks = alg_chunks;
  c->has_deps = !deps.empty();
  for (int r = 0; r < R; ++r) c->scratch_chunks.push_back(prog->rank[r].scratch_chunks);
  c->bufs.assign((size_t)R * 3, nullptr);
  c->scratch_bytes.assign(R, 0);
  c->bound.assign(R, 0);
  c->spin_limit_ticks = cfg.spin_limit_us * 100ull;  // wall clock runs at 100 MHz
  c->info.team_width = W;
  c->info.wg_size = cfg.wg_size;
  c->info.grid = (int32_t)grid;
  c->info.active_wgs = (int32_t)active;
  c->info.max_resident_wgs = (int32_t)std::min<long>(resident, INT32_MAX);
  c->info.fifo_slots = cfg.fifo_slots;
  c->info.tile_bytes = cfg.tile_bytes;
  c->info.slot_bytes = (int32_t)slot_bytes;
  c->info.fifo_bytes = fifo_bytes;
  c->info.compute_units = cus;
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
  comm->bufs[(size_t)rank * 3 + 0] = input;
  comm->bufs[(size_t)rank * 3 + 1] = output;
  comm->bufs[(size_t)rank * 3 + 2] = scratch;
  comm->scratch_bytes[rank] = scratch ? scratch_bytes : 0;
  comm->bound[rank] = 1;
  comm->bufs_dirty = true;
  return GC3_OK;
}

static int chunk_bytes_of(const gc3_comm* comm, size_t elems, int dtype, uint64_t* out) {
  int es = dtype_size(dtype);
  if (!es) { set_error("unknown dtype"); return GC3_ERR_ARG; }
  if (elems % (size_t)comm->in_chunks) { set_error("elems_per_rank is not a multiple of the program's chunk count"); return GC3_ERR_SIZE; }
  uint64_t cb = (uint64_t)(elems / comm->in_chunks) * es;
  if (cb % 16) { set_error("chunk size is not a multiple of 16 bytes"); return GC3_ERR_SIZE; }
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
  if (elems_per_rank == 0) return GC3_OK;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != comm->device) { set_error("communicator belongs to another device"); return GC3_ERR_ARG; }
  hipStream_t st = (hipStream_t)hip_stream;
  if (comm->bufs_dirty) {
    HIP_TRY(hipMemcpyAsync(comm->d_bufs, comm->bufs.data(), comm->bufs.size() * sizeof(void*), hipMemcpyHostToDevice, st));
    // the host table may change right after this call returns: make the copy complete first
    HIP_TRY(hipStreamSynchronize(st));
    comm->bufs_dirty = false;
  }
  KParams p{};
  p.tbs = comm->d_tbs;
  p.instrs = comm->d_instrs;
  p.deps = comm->d_deps;
  p.wgmap = comm->d_wgmap;
  p.bufs = comm->d_bufs;
  p.fifo = comm->d_fifo;
  p.flags = comm->d_flags;
  p.sems = comm->d_sems;
  p.error = comm->d_error;
  p.run_base = (++comm->run_number) << 32;
  p.chunk_bytes = cb;
  p.spin_limit_ticks = comm->spin_limit_ticks;
  p.W = (uint32_t)comm->info.team_width;
  p.slots = (uint32_t)comm->info.fifo_slots;
  p.tile_bytes = (uint32_t)comm->info.tile_bytes;
  p.slot_bytes = (uint32_t)comm->info.slot_bytes;
  int e = launch_interpreter((int)dtype, comm->has_deps, (unsigned)comm->info.grid, (unsigned)comm->info.wg_size, hip_stream, p);
  if (e != 0) return hip_fail((hipError_t)e, "interpreter launch");
  return GC3_OK;
}

int gc3_comm_status(gc3_comm* comm) {
  if (!comm) { set_error("null communicator"); return GC3_ERR_ARG; }
  HIP_TRY(hipDeviceSynchronize());
  uint32_t err = 0;
  HIP_TRY(hipMemcpy(&err, comm->d_error, sizeof(err), hipMemcpyDeviceToHost));
  if (err != 0) {
    comm->poisoned = true;
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
  HIP_TRY(hipMemset(comm->d_error, 0, 256));
  HIP_TRY(hipDeviceSynchronize());
  comm->poisoned = false;
  return GC3_OK;
}

void gc3_comm_destroy(gc3_comm* comm) {
  if (!comm) return;
  (void)hipDeviceSynchronize();
  delete comm;
}

}  // extern "C"
