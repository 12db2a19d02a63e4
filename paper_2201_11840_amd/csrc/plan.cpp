// Planning of a GC3-IR program for the interpreter kernel (host only, no device calls).
//
// The paper's runtime launches one thread block per IR thread block (Section 6.2) and relies on the
// user's parallelize(N) directive for parallelism (Section 5.1).  Here the runtime itself splits
// every IR thread block into W lanes (each lane = the program applied to 1/W of every chunk) and
// lets lightly loaded thread blocks of one rank share a workgroup, so that the number of busy
// workgroups matches the device whatever the program's thread-block count is.
#include "plan.h"

#include <algorithm>
#include <cmath>
#include <map>
#include <numeric>
#include <tuple>

namespace gc3 {

int resolve_config(const gc3_comm_config* cfg_in, gc3_comm_config& cfg, std::string& msg) {
  cfg = gc3_comm_config{};
  if (cfg_in) cfg = *cfg_in;
  if (cfg.fifo_slots == 0) cfg.fifo_slots = 2;
  if (cfg.wg_size == 0) cfg.wg_size = 256;
  if (cfg.spin_limit_us == 0) cfg.spin_limit_us = 10ull * 1000 * 1000;
  if (cfg.fifo_slots < 1 || cfg.fifo_slots > 8) { msg = "fifo_slots must be 1..8"; return GC3_ERR_ARG; }
  if (cfg.tile_bytes != 0 && (cfg.tile_bytes < 16 || cfg.tile_bytes % 16 || cfg.tile_bytes > (1 << 20))) {
    msg = "tile_bytes must be a multiple of 16 in [16, 1 MiB]";
    return GC3_ERR_ARG;
  }
  if (cfg.wg_size != 64 && cfg.wg_size != 128 && cfg.wg_size != 256 && cfg.wg_size != 512) {
    msg = "wg_size must be 64, 128, 256 or 512";
    return GC3_ERR_ARG;
  }
  if (cfg.team_width < 0 || cfg.team_width > 256) { msg = "team_width must be 0..256"; return GC3_ERR_ARG; }

  if (cfg.target_wgs < 0) { msg = "target_wgs must not be negative"; return GC3_ERR_ARG; }
  if (cfg.lds_stage < 0 || cfg.lds_stage > 1) { msg = "lds_stage must be 0 or 1"; return GC3_ERR_ARG; }
  if (cfg.debug_hold < 0 || cfg.debug_hold > 1) { msg = "debug_hold must be 0 or 1"; return GC3_ERR_ARG; }
  if (cfg.protocol < 0 || cfg.protocol > 3) { msg = "protocol must be 0..3"; return GC3_ERR_ARG; }
  if (cfg.fifo_scope < 0 || cfg.fifo_scope > 2) { msg = "fifo_scope must be 0, 1 or 2"; return GC3_ERR_ARG; }
  if (cfg.user_scope == 0) cfg.user_scope = 1;
  if (cfg.user_scope != 1 && cfg.user_scope != 2) { msg = "user_scope must be 0, 1 (device) or 2 (die)"; return GC3_ERR_ARG; }
  if (cfg.fifo_scope == 2 && (cfg.lds_stage || cfg.protocol > 1)) {
    msg = "die-scope FIFOs run the simple protocol through registers (protocol 0 or 1, lds_stage 0)";
    return GC3_ERR_ARG;
  }
  if (cfg.ll_max_lane_bytes == 0) cfg.ll_max_lane_bytes = 8192;
  if (cfg.ll_max_lane_bytes < 16 || cfg.ll_max_lane_bytes % 16 || cfg.ll_max_lane_bytes > 65536) {
    msg = "ll_max_lane_bytes must be a multiple of 16 in [16, 65536]";
    return GC3_ERR_ARG;
  }
  // (0 stays 0 = automatic: 8192, or 4096 for runs of the wavefront-level interpreter; decided per run)
  if (cfg.min_lane_bytes != 0 && (cfg.min_lane_bytes < 16 || cfg.min_lane_bytes % 16)) { msg = "min_lane_bytes must be a positive multiple of 16"; return GC3_ERR_ARG; }
  return GC3_OK;
}

int make_plan(const gc3_program& prog, const gc3_comm_config& cfg, int cus, long resident, Plan& plan, std::string& msg,
              uint64_t fifo_limit) {
  if (cus < 1 || resident < 1) { msg = "device size must be positive"; return GC3_ERR_ARG; }
  int rc = validate(prog, cfg.fifo_slots, msg);
  if (rc != GC3_OK) return rc;
  plan.cfg = cfg;
  // A receiver that announces freed slots only after every h-th message saves flag stores on the path of a hop.
  // A sender can then count on s - h + 1 slots only (it sees the receiver's count rounded down to a multiple
  // of h), and may find up to s: if the program completes with s - h + 1 slots it completes under this rule too
  // (take the order of events of a complete execution with s - h + 1 slots: the first of them that has not
  // happened yet is always enabled - its message has been sent, or at most as many messages are in flight as
  // then, or its semaphore has been set).
  int head_stride = 1;
  if (cfg.fifo_slots >= 4) {
    const int h = cfg.fifo_slots >= 8 ? 4 : 2;
    std::string unused;
    if (validate(prog, cfg.fifo_slots - h + 1, unused) == GC3_OK) head_stride = h;
  }

  // ---- flatten the program -------------------------------------------------------------------
  const int R = prog.ranks;
  std::vector<int> tb_base(R + 1, 0);
  for (int r = 0; r < R; ++r) tb_base[r + 1] = tb_base[r] + (int)prog.rank[r].tbs.size();
  const int ntb = tb_base[R];
  std::map<std::tuple<int, int, int>, int> conn_id;
  auto conn_of = [&](int src, int dst, int ch) {
    auto key = std::make_tuple(src, dst, ch);
    auto it = conn_id.find(key);
    if (it != conn_id.end()) return it->second;
    int id = (int)conn_id.size();
    conn_id[key] = id;
    return id;
  };
  std::vector<int> conn_sender;   // global thread-block index of the sending end of every connection
  std::vector<uint32_t> conn_count;   // largest `count` of an instruction that uses the connection
  auto note_end = [&](std::vector<int>& ends, int conn, int tb) {
    if ((int)ends.size() <= conn) ends.resize(conn + 1, -1);
    ends[conn] = tb;
  };
  std::vector<DTb>& tbs = plan.tbs;
  std::vector<DInstr>& instrs = plan.instrs;
  std::vector<DDep>& deps = plan.deps;
  tbs.assign(ntb, DTb{});
  instrs.clear();
  deps.clear();
  int max_count = 1;
  uint64_t alg_chunks = 0;
  for (int r = 0; r < R; ++r) {
    for (size_t b = 0; b < prog.rank[r].tbs.size(); ++b) {
      const ThreadBlock& tb = prog.rank[r].tbs[b];
      const int g = tb_base[r] + (int)b;
      DTb& d = tbs[g];
      d = DTb{};
      d.rank = (uint32_t)r;
      d.instr_begin = (uint32_t)instrs.size();
      d.ninstr = (uint32_t)tb.instrs.size();
      d.send_conn = d.recv_conn = -1;
      for (const Instr& in : tb.instrs) {
        auto note_count = [&](int conn) {
          if ((int)conn_count.size() <= conn) conn_count.resize(conn + 1, 1);
          conn_count[conn] = std::max<uint32_t>(conn_count[conn], (uint32_t)in.count);
        };
        if (op_pushes(in.op)) { d.send_conn = conn_of(r, tb.send, tb.chan); note_end(conn_sender, d.send_conn, g); note_count(d.send_conn); }
        if (op_pops(in.op)) { d.recv_conn = conn_of(tb.recv, r, tb.chan); note_count(d.recv_conn); }
        DInstr di{};
        di.op = in.op;
        di.srcbuf = (in.srcbuf == BUF_OUT && prog.inplace) ? (uint32_t)BUF_IN : in.srcbuf;
        di.dstbuf = (in.dstbuf == BUF_OUT && prog.inplace) ? (uint32_t)BUF_IN : in.dstbuf;
        di.srcidx = (uint32_t)in.srcidx;
        di.dstidx = (uint32_t)in.dstidx;
        di.count = (uint32_t)in.count;
        di.dep_begin = (uint32_t)deps.size();
        di.ndeps_hasdep = ((uint32_t)in.deps.size() << 1) | (in.hasdep ? 1u : 0u);
        for (auto& dp : in.deps) {
          DDep dd{};
          dd.tb = (uint32_t)(tb_base[r] + dp.first);
          dd.step = (uint32_t)dp.second;
          dd.ninstr = (uint32_t)prog.rank[r].tbs[dp.first].instrs.size();
          deps.push_back(dd);
        }
        instrs.push_back(di);
        max_count = std::max(max_count, in.count);
        alg_chunks += (uint64_t)op_traffic(in.op) * (uint64_t)in.count;
      }
    }
  }
  const int nconn = (int)conn_id.size();
  // FIFO memory is laid out connection by connection, each with slots of its own size
  conn_count.resize(nconn, 1);
  std::vector<uint32_t> units_before(nconn + 1, 0);
  for (int c = 0; c < nconn; ++c) units_before[c + 1] = units_before[c] + conn_count[c];
  const uint64_t total_units = units_before[nconn];


  // about four workgroups per compute unit give enough bytes in flight to cover memory latency
  long target = cfg.target_wgs > 0 ? cfg.target_wgs : 4L * cus;
  target = std::max<long>(1, std::min<long>(target, resident));

  // ---- schedule: team width W and which thread blocks share a workgroup -----------------------------
  // A workgroup multiplexes the lanes (fibers) of several thread blocks of one rank.  The weight of
  // a thread block is its traffic per tile; the thread blocks of a rank are packed into k bins
  // (largest first into the lightest bin) and every (bin, lane) pair becomes one workgroup.  W and
  // the bin counts are chosen to minimise the heaviest workgroup's traffic, bin weight / W, with at
  // most `target` workgroups.
  std::vector<uint64_t> weight(ntb, 0);
  for (int r = 0; r < R; ++r)
    for (size_t b = 0; b < prog.rank[r].tbs.size(); ++b)
      for (const Instr& in : prog.rank[r].tbs[b].instrs)
        weight[tb_base[r] + b] += (uint64_t)op_traffic(in.op) * (uint64_t)in.count;
  uint64_t total_weight = 0;
  for (uint64_t w : weight) total_weight += std::max<uint64_t>(w, 1);
  auto pack = [&](int W, bool round_up, std::vector<std::vector<int>>* bins_out, double* heaviest) -> long {
    // returns the number of workgroups, or -1 when a workgroup would exceed the fiber limit
    const double ideal = (double)total_weight * W / (double)target;   // traffic of one workgroup if perfectly spread
    // Workgroups of one wavefront run best with one fiber each (the wavefront-level interpreter: no barrier, no
    // state in LDS): when every thread block can have workgroups of its own within the target, nothing is shared.
    const bool singletons = cfg.wg_size == 64 && (long)ntb * W <= target;
    long wgs = 0;
    double worst = 0;
    for (int r = 0; r < R; ++r) {
      const int n = tb_base[r + 1] - tb_base[r];
      if (n == 0) continue;
      std::vector<int> order(n);
      std::iota(order.begin(), order.end(), tb_base[r]);
      std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return weight[a] > weight[b]; });
      double rank_weight = 0;
      for (int g : order) rank_weight += (double)std::max<uint64_t>(weight[g], 1);
      const double cap = std::max(ideal, (double)std::max<uint64_t>(weight[order[0]], 1));
      int k = round_up ? (int)std::ceil(rank_weight / cap - 1e-9) : (int)std::floor(rank_weight / cap + 1e-9);
      k = std::max(1, std::min(k, n));
      k = std::max(k, (n + kMaxFibersPerWg - 1) / kMaxFibersPerWg);
      if (singletons) k = n;
      std::vector<std::vector<int>> bins(k);
      std::vector<double> load(k, 0.0);
      for (int g : order) {
        int best = -1;
        for (int i = 0; i < k; ++i)
          if ((int)bins[i].size() < kMaxFibersPerWg && (best < 0 || load[i] < load[best])) best = i;
        if (best < 0) return -1;
        bins[best].push_back(g);
        load[best] += (double)std::max<uint64_t>(weight[g], 1);
      }
      for (int i = 0; i < k; ++i) {
        worst = std::max(worst, load[i]);
        std::sort(bins[i].begin(), bins[i].end());   // program order inside a workgroup
        if (bins_out) bins_out->push_back(bins[i]);
      }
      wgs += (long)k * W;
    }
    if (heaviest) *heaviest = worst;
    return wgs;
  };
  int W = cfg.team_width;
  bool round_up = true;
  if (ntb == 0) {
    W = std::max(W, 1);   // a program without thread blocks is a valid no-op (e.g. AllToNext on one rank)
  } else if (W == 0) {
    double best_cost = 0;
    for (int cand : {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64}) {
      for (bool up : {true, false}) {
        double heaviest = 0;
        long wgs = pack(cand, up, nullptr, &heaviest);
        if (wgs < 0 || wgs > target) continue;
        double cost = heaviest / cand;
        // fewer lanes mean larger shares per lane and less FIFO memory: take more only for a clear gain
        if (W == 0 || cost < best_cost * 0.97) { W = cand; round_up = up; best_cost = cost; }
      }
    }
    if (W == 0) { W = 1; round_up = false; }
  } else {
    // explicit team width: use the sharing that gives the lighter heaviest workgroup within the target
    double h_up = 0, h_dn = 0;
    long n_up = pack(W, true, nullptr, &h_up), n_dn = pack(W, false, nullptr, &h_dn);
    if (n_up < 0 || n_up > target) round_up = false;
    else if (n_dn >= 0 && h_dn < h_up) round_up = false;
  }
  std::vector<std::vector<int>> bins;
  {
    long wgs = pack(W, round_up, &bins, nullptr);
    if (wgs < 0) { msg = "a workgroup would have to multiplex too many thread blocks"; return GC3_ERR_RESIDENCY; }
  }
  if (cfg.user_scope == 2 && cfg.fifo_scope != 2) {
    // Die-scope user buffers (with die-scope FIFOs the lanes are placed on dies instead, which serves both): bin index = row * (rank count rounded up to a multiple of 8) + rank, with empty bins
    // where a rank has fewer than the others.  The grid is lane-major with this many bins per lane, so workgroup
    // index mod 8 = rank mod 8 whatever the number of active lanes, and consecutive workgroups go to consecutive
    // dies: all workgroups of a rank run on one die.
    const int width = (R + 7) / 8 * 8;
    std::vector<std::vector<std::vector<int>>> of_rank(R);
    for (auto& b : bins) of_rank[tbs[b.front()].rank].push_back(b);
    size_t rows = 0;
    for (auto& v : of_rank) rows = std::max(rows, v.size());
    std::vector<std::vector<int>> placed;
    for (size_t i = 0; i < rows; ++i)
      for (int r = 0; r < width; ++r)
        placed.push_back(r < R && i < of_rank[r].size() ? of_rank[r][i] : std::vector<int>());
    bins.swap(placed);
  }
  long nonempty = 0;
  for (auto& b : bins) nonempty += b.empty() ? 0 : 1;
  const long active = nonempty * W;   // (empty workgroups leave at once and hold no place)
  if (active > resident) {
    msg = "program needs " + std::to_string(active) + " resident workgroups of " + std::to_string(cfg.wg_size) +
          " threads, the device holds " + std::to_string(resident);
    return GC3_ERR_RESIDENCY;
  }

  // ---- grid order: lane-major ------------------------------------------------------------------------
  // Workgroup index = lane * bins + bin.  A run whose chunks are too small to be worth W lanes uses only
  // the first lanes and launches just that prefix of the grid.  Consecutive workgroups are dispatched
  // round-robin over the 8 dies (XCDs), so every prefix is spread evenly.  (Placing connected thread
  // blocks on one die was measured and makes no difference: FIFO payload and flags bypass the
  // per-die L2 by design, so nothing is shared through it.)
  // The instruction table is reordered by bin (then thread block, then step), so that the instructions a
  // workgroup needs are one contiguous range it can fetch without first reading its thread blocks' records.
  {
    std::vector<DInstr> ordered;
    ordered.reserve(instrs.size());
    for (auto& bin : bins)
      for (int g : bin) {
        const uint32_t from = tbs[g].instr_begin;
        tbs[g].instr_begin = (uint32_t)ordered.size();
        ordered.insert(ordered.end(), instrs.begin() + from, instrs.begin() + from + tbs[g].ninstr);
      }
    instrs.swap(ordered);
  }
  std::vector<DWg>& wgs = plan.wgs;
  std::vector<DFiber>& fibers = plan.fibers;
  wgs.clear();
  fibers.clear();
  int max_fibers = 0;
  for (int w = 0; w < W; ++w)
    for (size_t b = 0; b < bins.size(); ++b) {
      DWg h{};
      h.fiber_begin = (uint32_t)fibers.size();
      h.nfibers = (uint32_t)bins[b].size();
      h.instr_begin = bins[b].empty() ? 0u : tbs[bins[b].front()].instr_begin;
      for (int g : bins[b]) {
        DFiber f{};
        f.fid = (uint32_t)(g * W + w);
        f.instr_begin = tbs[g].instr_begin;
        f.ninstr = tbs[g].ninstr;
        f.send_conn = tbs[g].send_conn;
        f.recv_conn = tbs[g].recv_conn;
        f.recv_from_tb = (tbs[g].recv_conn >= 0 && (size_t)tbs[g].recv_conn < conn_sender.size())
                             ? (uint32_t)conn_sender[tbs[g].recv_conn] : 0xffffffffu;
        if (f.send_conn >= 0) { f.send_units_before = units_before[f.send_conn]; f.send_count = conn_count[f.send_conn]; }
        if (f.recv_conn >= 0) { f.recv_units_before = units_before[f.recv_conn]; f.recv_count = conn_count[f.recv_conn]; }
        fibers.push_back(f);
        h.ninstr += tbs[g].ninstr;
        h.rank = tbs[g].rank;
        h.rank_first_tb = (uint32_t)tb_base[tbs[g].rank];
      }
      wgs.push_back(h);
      max_fibers = std::max(max_fibers, (int)bins[b].size());
    }
  const long grid = (long)wgs.size();


  // Largest tile (= what a FIFO slot holds per chunk): 64 KiB unless given; halved (not below 16 KiB)
  // while all FIFOs together exceed 256 MiB, the size of the memory-side cache they should stay in.
  // A run uses a tile of about half a lane's share of a chunk, within [16 KiB, this].
  int tile_bytes = cfg.tile_bytes;
  if (tile_bytes == 0) {
    tile_bytes = 65536;
    // device scope: the FIFOs should stay in the 256 MiB memory-side cache; die scope: in the dies' L2s (8 x 4 MiB,
    // shared with the user data that streams through)
    const uint64_t soft = fifo_limit ? fifo_limit : cfg.fifo_scope == 2 ? (16ull << 20) : (256ull << 20);
    const int floor_bytes = fifo_limit ? 1024 : cfg.fifo_scope == 2 ? 4096 : 16384;
    while (tile_bytes > floor_bytes && total_units * W * cfg.fifo_slots * (uint64_t)tile_bytes > soft)
      tile_bytes /= 2;
  }
  plan.cfg.tile_bytes = tile_bytes;
  const uint64_t slot_bytes = (uint64_t)max_count * (uint64_t)tile_bytes;
  const uint64_t fifo_bytes = std::max<uint64_t>(16, total_units * W * cfg.fifo_slots * (uint64_t)tile_bytes);
  if (slot_bytes > (1ull << 30) || fifo_bytes > (64ull << 30)) { msg = "FIFO memory too large"; return GC3_ERR_SIZE; }
  if (fifo_limit && fifo_bytes > fifo_limit) {
    msg = "the connections' FIFOs need " + std::to_string(fifo_bytes) + " bytes, " + std::to_string(fifo_limit) + " are available";
    return GC3_ERR_SIZE;
  }
  int protocol = cfg.protocol;
  if (cfg.fifo_scope == 2) protocol = 1;
  if (protocol == 0) protocol = prog.protocol == "simple" ? 1 : (prog.protocol == "ll" || prog.protocol == "ll128") ? 2 : 3;
  const uint64_t ll_slot_bytes = 2ull * max_count * (uint64_t)cfg.ll_max_lane_bytes;
  const uint64_t ll_fifo_bytes =
      protocol == 1 ? 0 : std::max<uint64_t>(16, total_units * W * cfg.fifo_slots * 2ull * (uint64_t)cfg.ll_max_lane_bytes);
  if (protocol != 1 && (ll_slot_bytes > (1ull << 30) || ll_fifo_bytes > (64ull << 30))) {
    msg = "LL FIFO memory too large";
    return GC3_ERR_SIZE;
  }
  int max_pushes = 0;
  for (int r = 0; r < R; ++r)
    for (auto& tb : prog.rank[r].tbs) {
      int n = 0;
      for (auto& in : tb.instrs) n += op_pushes(in.op) ? 1 : 0;
      max_pushes = std::max(max_pushes, n);
    }
  plan.max_pushes = max_pushes;
  plan.nconn = nconn;
  plan.ntb = ntb;
  plan.max_count = max_count;
  plan.algorithmic_chunks = alg_chunks;
  plan.info = gc3_comm_info{};
  plan.info.team_width = W;
  plan.info.wg_size = cfg.wg_size;
  plan.info.grid = (int32_t)grid;
  plan.info.wgs_per_lane = (int32_t)bins.size();
  plan.info.active_wgs = (int32_t)active;
  plan.info.max_resident_wgs = (int32_t)std::min<long>(resident, INT32_MAX);
  plan.info.fifo_slots = cfg.fifo_slots;
  plan.info.tile_bytes = tile_bytes;
  plan.info.slot_bytes = (int32_t)slot_bytes;
  plan.info.fifo_bytes = fifo_bytes;
  plan.info.compute_units = cus;
  plan.info.max_fibers_per_wg = max_fibers;
  plan.info.protocol = protocol;
  plan.info.ll_fifo_bytes = ll_fifo_bytes;
  plan.info.head_stride = head_stride;
  plan.info.user_scope = cfg.user_scope;
  return GC3_OK;
}

}  // namespace gc3

extern "C" int gc3_program_plan(const gc3_program* prog, const gc3_comm_config* cfg_in, int compute_units,
                                int max_resident_wgs, gc3_comm_info* out) {
  if (!prog || !out) { gc3::set_error("null argument"); return GC3_ERR_ARG; }
  gc3_comm_config cfg{};
  std::string msg;
  int rc = gc3::resolve_config(cfg_in, cfg, msg);
  gc3::Plan plan;
  if (rc == GC3_OK) rc = gc3::make_plan(*prog, cfg, compute_units, max_resident_wgs, plan, msg);
  if (rc != GC3_OK) { gc3::set_error(msg); return rc; }
  *out = plan.info;
  return GC3_OK;
}
