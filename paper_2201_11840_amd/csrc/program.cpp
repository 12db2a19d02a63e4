// GC3-IR text loader and validator (host only; no device code).
//
// Section 6.2 "Initial Setup": programs are parsed when the runtime initialises.  The checks in
// validate() are the properties the paper's compiler guarantees for every IR it emits
// (Section 5: one send / one receive peer per thread block, one sending and one receiving
// thread block per connection; Section 5.2: dependencies and absence of deadlock; Section 6.1:
// never more than s outstanding sends), re-derived here because this runtime accepts IR from
// any producer.
#include "program.h"

#include <cstring>
#include <deque>
#include <map>
#include <sstream>
#include <tuple>

namespace gc3 {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }

namespace {

const char* kOpNames[] = {"send", "recv", "copy", "reduce", "rrc", "rcs", "rrcs", "rrs"};

bool parse_int(const std::string& s, long long lo, long long hi, int32_t* out) {
  if (s.empty() || s.size() > 12) return false;
  size_t i = 0;
  bool neg = false;
  if (s[0] == '-') { neg = true; i = 1; }
  if (i >= s.size()) return false;
  long long v = 0;
  for (; i < s.size(); ++i) {
    if (s[i] < '0' || s[i] > '9') return false;
    v = v * 10 + (s[i] - '0');
  }
  if (neg) v = -v;
  if (v < lo || v > hi) return false;
  *out = static_cast<int32_t>(v);
  return true;
}

bool parse_buf(const std::string& s, uint8_t* out) {
  if (s == "i") *out = BUF_IN;
  else if (s == "o") *out = BUF_OUT;
  else if (s == "s") *out = BUF_SCRATCH;
  else if (s == "-") *out = BUF_NONE;
  else return false;
  return true;
}

std::vector<std::string> tokens(const std::string& line) {
  std::vector<std::string> t;
  size_t i = 0, n = line.size();
  while (i < n) {
    while (i < n && (line[i] == ' ' || line[i] == '\t' || line[i] == '\r')) ++i;
    if (i >= n || line[i] == '#') break;
    size_t j = i;
    while (j < n && line[j] != ' ' && line[j] != '\t' && line[j] != '\r' && line[j] != '#') ++j;
    t.emplace_back(line, i, j - i);
    i = j;
  }
  return t;
}

constexpr int kMaxRanks = 4096, kMaxTbs = 4096, kMaxOps = 65536, kMaxChunks = 1 << 20, kMaxChan = 1 << 16;

}  // namespace

static int parse(const char* text, size_t len, gc3_program& p, std::string& msg) {
  std::string all(text, len);
  std::istringstream in(all);
  std::string line;
  int ln = 0;
  bool seen_version = false, ended = false, seen_ranks = false, seen_chunks = false;
  int32_t want_tbs = 0, want_ops = 0;
  RankProgram* cur_rank = nullptr;
  ThreadBlock* cur_tb = nullptr;
  auto fail = [&](const std::string& what) {
    msg = "line " + std::to_string(ln) + ": " + what;
    return (int)GC3_ERR_PARSE;
  };
  auto rank_complete = [&]() {
    if (!cur_rank) return true;
    if ((int32_t)cur_rank->tbs.size() != want_tbs) return false;
    if (cur_tb && (int32_t)cur_tb->instrs.size() != want_ops) return false;
    return true;
  };
  while (std::getline(in, line)) {
    ++ln;
    std::vector<std::string> t = tokens(line);
    if (t.empty()) continue;
    if (ended) return fail("text after end");
    const std::string& k = t[0];
    if (!seen_version && k != "gc3ir") return fail("missing gc3ir header");
    if (k == "gc3ir") {
      if (t.size() != 2 || t[1] != "1") return fail("unsupported gc3ir version");
      seen_version = true;
    } else if (k == "name" || k == "collective" || k == "protocol") {
      if (t.size() != 2) return fail("expected one token after " + k);
      (k == "name" ? p.name : k == "collective" ? p.collective : p.protocol) = t[1];
      if (k == "protocol" && t[1] != "simple" && t[1] != "ll" && t[1] != "ll128" && t[1] != "auto")
        return fail("protocol must be simple, ll, ll128 or auto");
    } else if (k == "inplace") {
      int32_t v;
      if (t.size() != 2 || !parse_int(t[1], 0, 1, &v)) return fail("inplace takes 0 or 1");
      p.inplace = v != 0;
    } else if (k == "ranks") {
      if (seen_ranks || t.size() != 2 || !parse_int(t[1], 1, kMaxRanks, &p.ranks)) return fail("bad ranks statement");
      seen_ranks = true;
      p.rank.reserve(p.ranks);
    } else if (k == "chunks") {
      if (t.size() != 3 || !parse_int(t[1], 1, kMaxChunks, &p.in_chunks) ||
          !parse_int(t[2], 1, kMaxChunks, &p.out_chunks))
        return fail("bad chunks statement");
      seen_chunks = true;
    } else if (k == "rank") {
      int32_t r, sc, nt;
      if (!seen_ranks || !seen_chunks) return fail("rank before ranks/chunks");
      if (t.size() != 6 || t[2] != "scratch" || t[4] != "tbs" || !parse_int(t[1], 0, kMaxRanks, &r) ||
          !parse_int(t[3], 0, kMaxChunks, &sc) || !parse_int(t[5], 0, kMaxTbs, &nt))
        return fail("bad rank statement");
      if (r != (int32_t)p.rank.size() || r >= p.ranks) return fail("ranks must appear in order 0..R-1");
      if (!rank_complete()) return fail("previous rank is incomplete");
      p.rank.emplace_back();
      cur_rank = &p.rank.back();
      cur_rank->scratch_chunks = sc;
      cur_rank->tbs.reserve(nt);
      cur_tb = nullptr;
      want_tbs = nt;
      want_ops = 0;
    } else if (k == "tb") {
      int32_t id, s, r, c, n;
      if (!cur_rank) return fail("tb outside a rank");
      if (t.size() != 10 || t[2] != "send" || t[4] != "recv" || t[6] != "chan" || t[8] != "ops" ||
          !parse_int(t[1], 0, kMaxTbs, &id) || !parse_int(t[3], -1, kMaxRanks, &s) ||
          !parse_int(t[5], -1, kMaxRanks, &r) || !parse_int(t[7], 0, kMaxChan, &c) ||
          !parse_int(t[9], 0, kMaxOps, &n))
        return fail("bad tb statement");
      if (cur_tb && (int32_t)cur_tb->instrs.size() != want_ops) return fail("previous tb is incomplete");
      if (id != (int32_t)cur_rank->tbs.size() || id >= want_tbs) return fail("tb ids must appear in order");
      cur_rank->tbs.emplace_back();
      cur_tb = &cur_rank->tbs.back();
      cur_tb->rank = (int32_t)p.rank.size() - 1;
      cur_tb->send = s;
      cur_tb->recv = r;
      cur_tb->chan = c;
      cur_tb->instrs.reserve(n);
      want_ops = n;
    } else if (k == "op") {
      if (!cur_tb) return fail("op outside a tb");
      if ((int32_t)cur_tb->instrs.size() >= want_ops) return fail("more ops than the tb declared");
      if (t.size() < 9) return fail("op needs 8 fields");
      Instr ins;
      int op = -1;
      for (int i = 0; i < 8; ++i)
        if (t[1] == kOpNames[i]) op = i;
      if (op < 0) return fail("unknown opcode " + t[1]);
      ins.op = (uint8_t)op;
      int32_t hd, nd;
      if (!parse_buf(t[2], &ins.srcbuf) || !parse_int(t[3], 0, kMaxChunks, &ins.srcidx) ||
          !parse_buf(t[4], &ins.dstbuf) || !parse_int(t[5], 0, kMaxChunks, &ins.dstidx) ||
          !parse_int(t[6], 1, kMaxChunks, &ins.count) || !parse_int(t[7], 0, 1, &hd) ||
          !parse_int(t[8], 0, 1024, &nd))
        return fail("bad op field");
      ins.hasdep = hd != 0;
      if ((int32_t)t.size() != 9 + 2 * nd) return fail("dependency list length mismatch");
      for (int i = 0; i < nd; ++i) {
        int32_t b, s;
        if (!parse_int(t[9 + 2 * i], 0, kMaxTbs, &b) || !parse_int(t[10 + 2 * i], 0, kMaxOps, &s))
          return fail("bad dependency");
        ins.deps.emplace_back(b, s);
      }
      cur_tb->instrs.push_back(std::move(ins));
    } else if (k == "end") {
      if (t.size() != 1) return fail("bad end statement");
      ended = true;
    } else {
      return fail("unknown statement " + k);
    }
  }
  ++ln;
  if (!ended) return fail("missing end");
  if (!seen_ranks || !seen_chunks) return fail("missing ranks/chunks");
  if ((int32_t)p.rank.size() != p.ranks) return fail("fewer rank sections than ranks");
  if (!rank_complete()) return fail("last rank is incomplete");
  return GC3_OK;
}

int validate(const gc3_program& p, int fifo_slots, std::string& msg) {
  auto bad = [&](const std::string& m) { msg = m; return (int)GC3_ERR_INVALID_PROGRAM; };
  if (fifo_slots < 1 || fifo_slots > 8) { msg = "fifo_slots must be 1..8"; return GC3_ERR_ARG; }
  const int R = p.ranks;
  using Conn = std::tuple<int, int, int>;  // (source rank, destination rank, channel)
  std::map<Conn, std::pair<int, int>> sender, receiver;  // -> (rank, tb)
  for (int r = 0; r < R; ++r) {
    const RankProgram& rp = p.rank[r];
    for (size_t b = 0; b < rp.tbs.size(); ++b) {
      const ThreadBlock& tb = rp.tbs[b];
      std::string where = "rank " + std::to_string(r) + " tb " + std::to_string(b);
      if (tb.send >= R || tb.recv >= R) return bad(where + ": peer out of range");
      if (tb.send == r || tb.recv == r) return bad(where + ": a rank cannot be its own peer");
      bool pushes = false, pops = false;
      for (size_t s = 0; s < tb.instrs.size(); ++s) {
        const Instr& in = tb.instrs[s];
        std::string at = where + " step " + std::to_string(s);
        if (op_pushes(in.op)) {
          pushes = true;
          if (tb.send < 0) return bad(at + ": sends without a send peer");
        }
        if (op_pops(in.op)) {
          pops = true;
          if (tb.recv < 0) return bad(at + ": receives without a receive peer");
        }
        auto check_operand = [&](bool used, uint8_t buf, int idx, const char* which) -> bool {
          if (!used) return true;
          int limit = buf == BUF_IN ? p.in_chunks : buf == BUF_OUT ? (p.inplace ? p.in_chunks : p.out_chunks)
                      : buf == BUF_SCRATCH ? rp.scratch_chunks : -1;
          if (limit < 0) { msg = at + ": missing " + which + " buffer"; return false; }
          if (idx + in.count > limit) { msg = at + ": " + which + " chunks out of range"; return false; }
          return true;
        };
        if (!check_operand(op_uses_src(in.op), in.srcbuf, in.srcidx, "source")) return GC3_ERR_INVALID_PROGRAM;
        if (!check_operand(op_uses_dst(in.op), in.dstbuf, in.dstidx, "destination")) return GC3_ERR_INVALID_PROGRAM;
        for (auto& d : in.deps) {
          if (d.first >= (int)rp.tbs.size()) return bad(at + ": depends on a thread block that does not exist");
          if (d.first == (int)b) return bad(at + ": depends on its own thread block");
          const ThreadBlock& dt = rp.tbs[d.first];
          if (d.second >= (int)dt.instrs.size()) return bad(at + ": depends on a step that does not exist");
          if (!dt.instrs[d.second].hasdep) return bad(at + ": depends on a step whose has-dependent flag is not set");
        }
      }
      if (pushes) {
        Conn c(r, tb.send, tb.chan);
        if (sender.count(c)) return bad(where + ": a second sending thread block on one connection");
        sender[c] = {r, (int)b};
      }
      if (pops) {
        Conn c(tb.recv, r, tb.chan);
        if (receiver.count(c)) return bad(where + ": a second receiving thread block on one connection");
        receiver[c] = {r, (int)b};
      }
    }
  }
  for (auto& kv : sender)
    if (!receiver.count(kv.first))
      return bad("connection " + std::to_string(std::get<0>(kv.first)) + "->" + std::to_string(std::get<1>(kv.first)) +
                 " chan " + std::to_string(std::get<2>(kv.first)) + " has no receiving thread block");
  for (auto& kv : receiver)
    if (!sender.count(kv.first))
      return bad("connection " + std::to_string(std::get<0>(kv.first)) + "->" + std::to_string(std::get<1>(kv.first)) +
                 " chan " + std::to_string(std::get<2>(kv.first)) + " has no sending thread block");

  // Bounded-FIFO execution of one tile iteration.  A network of sequential processes joined by
  // bounded FIFOs is determinate: whether it completes does not depend on the order in which
  // runnable processes are stepped, so one sweep order decides it.  Later tile iterations repeat
  // the same pattern from empty FIFOs.
  std::map<Conn, std::deque<int>> q;  // message sizes in flight
  std::vector<std::vector<int>> pc(R);
  long remaining = 0;
  for (int r = 0; r < R; ++r) {
    pc[r].assign(p.rank[r].tbs.size(), 0);
    for (auto& tb : p.rank[r].tbs) remaining += (long)tb.instrs.size();
  }
  bool progressed = true;
  while (remaining > 0 && progressed) {
    progressed = false;
    for (int r = 0; r < R; ++r) {
      for (size_t b = 0; b < p.rank[r].tbs.size(); ++b) {
        const ThreadBlock& tb = p.rank[r].tbs[b];
        while (pc[r][b] < (int)tb.instrs.size()) {
          const Instr& in = tb.instrs[pc[r][b]];
          bool ok = true;
          for (auto& d : in.deps)
            if (pc[r][d.first] <= d.second) ok = false;
          std::deque<int>* rq = nullptr;
          std::deque<int>* sq = nullptr;
          if (ok && op_pops(in.op)) {
            rq = &q[Conn(tb.recv, r, tb.chan)];
            if (rq->empty()) ok = false;
          }
          if (ok && op_pushes(in.op)) {
            sq = &q[Conn(r, tb.send, tb.chan)];
            if ((int)sq->size() >= fifo_slots) ok = false;
          }
          if (!ok) break;
          if (rq) {
            if (rq->front() != in.count)
              return bad("rank " + std::to_string(r) + " tb " + std::to_string(b) + " step " +
                         std::to_string(pc[r][b]) + ": receives " + std::to_string(in.count) +
                         " chunks but the matching send carries " + std::to_string(rq->front()));
            rq->pop_front();
          }
          if (sq) sq->push_back(in.count);
          ++pc[r][b];
          --remaining;
          progressed = true;
        }
      }
    }
  }
  if (remaining > 0) {
    for (int r = 0; r < R; ++r)
      for (size_t b = 0; b < p.rank[r].tbs.size(); ++b)
        if (pc[r][b] < (int)p.rank[r].tbs[b].instrs.size()) {
          msg = "deadlock with " + std::to_string(fifo_slots) + " FIFO slot(s): rank " + std::to_string(r) + " tb " +
                std::to_string(b) + " cannot pass step " + std::to_string(pc[r][b]);
          return GC3_ERR_DEADLOCK;
        }
  }
  for (auto& kv : q)
    if (!kv.second.empty())
      return bad("connection " + std::to_string(std::get<0>(kv.first)) + "->" + std::to_string(std::get<1>(kv.first)) +
                 " chan " + std::to_string(std::get<2>(kv.first)) + ": messages sent but never received");
  return GC3_OK;
}

}  // namespace gc3

extern "C" {

const char* gc3_last_error(void) { return gc3::g_last_error.c_str(); }

int gc3_program_load(const char* text, size_t len, gc3_program** out) {
  if (!text || !out) { gc3::set_error("null argument"); return GC3_ERR_ARG; }
  *out = nullptr;
  gc3_program* p = new gc3_program();
  std::string msg;
  int rc = gc3::parse(text, len, *p, msg);
  if (rc != GC3_OK) {
    delete p;
    gc3::set_error(msg);
    return rc;
  }
  *out = p;
  return GC3_OK;
}

void gc3_program_free(gc3_program* prog) { delete prog; }

int gc3_program_validate(const gc3_program* prog, int fifo_slots, char* err, size_t errlen) {
  if (!prog) { gc3::set_error("null program"); return GC3_ERR_ARG; }
  std::string msg;
  int rc = gc3::validate(*prog, fifo_slots, msg);
  if (rc != GC3_OK) gc3::set_error(msg);
  if (err && errlen) {
    std::strncpy(err, msg.c_str(), errlen - 1);
    err[errlen - 1] = 0;
  }
  return rc;
}

int gc3_program_info_get(const gc3_program* prog, gc3_program_info* out) {
  if (!prog || !out) { gc3::set_error("null argument"); return GC3_ERR_ARG; }
  gc3_program_info i{};
  i.ranks = prog->ranks;
  i.in_chunks = prog->in_chunks;
  i.out_chunks = prog->out_chunks;
  i.inplace = prog->inplace ? 1 : 0;
  i.max_count = 1;
  std::map<std::tuple<int, int, int>, int> conns;
  for (int r = 0; r < prog->ranks; ++r) {
    const gc3::RankProgram& rp = prog->rank[r];
    i.num_tbs += (int32_t)rp.tbs.size();
    i.max_tbs_per_rank = std::max<int32_t>(i.max_tbs_per_rank, (int32_t)rp.tbs.size());
    i.max_scratch_chunks = std::max<int32_t>(i.max_scratch_chunks, rp.scratch_chunks);
    for (auto& tb : rp.tbs) {
      for (auto& in : tb.instrs) {
        ++i.num_instructions;
        i.max_count = std::max(i.max_count, in.count);
        i.algorithmic_chunks += (uint64_t)gc3::op_traffic(in.op) * (uint64_t)in.count;
        if (gc3::op_pushes(in.op)) conns[{r, tb.send, tb.chan}] = 1;
        if (gc3::op_pops(in.op)) conns[{tb.recv, r, tb.chan}] = 1;
      }
    }
  }
  i.num_connections = (int32_t)conns.size();
  *out = i;
  return GC3_OK;
}

int gc3_program_scratch_chunks(const gc3_program* prog, int rank, int* out) {
  if (!prog || !out || rank < 0 || rank >= prog->ranks) { gc3::set_error("bad argument"); return GC3_ERR_ARG; }
  *out = prog->rank[rank].scratch_chunks;
  return GC3_OK;
}

}  // extern "C"
