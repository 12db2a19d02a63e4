// Host-side representation of a parsed GC3-IR program (Section 5, "GC3-IR").
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "gc3.h"

namespace gc3 {

enum Buf : uint8_t { BUF_IN = 0, BUF_OUT = 1, BUF_SCRATCH = 2, BUF_NONE = 3 };

struct Instr {
  uint8_t op = 0;          // gc3_opcode
  uint8_t srcbuf = BUF_NONE, dstbuf = BUF_NONE;
  bool hasdep = false;     // another thread block waits on this step
  int32_t srcidx = 0, dstidx = 0, count = 1;
  std::vector<std::pair<int32_t, int32_t>> deps;  // (thread block of the same rank, step)
};

struct ThreadBlock {
  int32_t rank = 0, send = -1, recv = -1, chan = 0;
  std::vector<Instr> instrs;
};

struct RankProgram {
  int32_t scratch_chunks = 0;
  std::vector<ThreadBlock> tbs;
};

inline bool op_pops(int op) {
  return op == GC3_OP_RECV || op == GC3_OP_RRC || op == GC3_OP_RCS || op == GC3_OP_RRCS || op == GC3_OP_RRS;
}
inline bool op_pushes(int op) {
  return op == GC3_OP_SEND || op == GC3_OP_RCS || op == GC3_OP_RRCS || op == GC3_OP_RRS;
}
inline bool op_uses_src(int op) {
  return op == GC3_OP_SEND || op == GC3_OP_COPY || op == GC3_OP_REDUCE || op == GC3_OP_RRC ||
         op == GC3_OP_RRCS || op == GC3_OP_RRS;
}
inline bool op_uses_dst(int op) {
  return op == GC3_OP_RECV || op == GC3_OP_COPY || op == GC3_OP_REDUCE || op == GC3_OP_RRC ||
         op == GC3_OP_RCS || op == GC3_OP_RRCS;
}
// global-memory traffic of one instruction in chunk units (loads + stores)
inline int op_traffic(int op) {
  switch (op) {
    case GC3_OP_SEND: case GC3_OP_RECV: case GC3_OP_COPY: return 2;
    case GC3_OP_RRCS: return 4;
    default: return 3;
  }
}

void set_error(const std::string& msg);

}  // namespace gc3

struct gc3_program {
  std::string name, collective, protocol;
  bool inplace = false;
  int32_t ranks = 0, in_chunks = 0, out_chunks = 0;
  std::vector<gc3::RankProgram> rank;
};

namespace gc3 {
// Structural checks plus a bounded-FIFO execution; fills `msg` on failure.
int validate(const gc3_program& p, int fifo_slots, std::string& msg);
}  // namespace gc3
