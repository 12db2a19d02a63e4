// Device-resident tables of a communicator: the parsed program flattened for the interpreter
// kernel (Section 6.2, "Instruction Data Structure": step, opcode, source/destination buffer and
// chunk offset, count, dependency lists, has-dependent flag).
#pragma once
#include <cstdint>

namespace gc3 {

constexpr int kMaxFibersPerWg = 32;  // lanes of IR thread blocks one workgroup may multiplex
constexpr int kFlagStrideWords = 16;  // one 64-bit flag per 128-byte line
constexpr int kLdsInstrs = 192;       // instructions (of all its fibers together) a workgroup keeps in LDS
// Size of the per-GPU static array that serves callers who cannot allocate device memory: flags, semaphores,
// instruction tables and FIFOs of one run must fit.
constexpr unsigned long long kStaticScratchBytes = 64ull << 20;

struct DInstr {            // 32 bytes
  uint32_t op;             // gc3_opcode
  uint32_t srcbuf, dstbuf; // 0 input, 1 output, 2 scratch (3 unused)
  uint32_t srcidx, dstidx; // chunk index inside the buffer
  uint32_t count;          // consecutive chunks
  uint32_t dep_begin;      // first entry in the dependency table
  uint32_t ndeps_hasdep;   // (number of dependencies << 1) | has-dependent flag
};

struct DDep {              // 16 bytes
  uint32_t tb;             // global thread-block index of the dependee
  uint32_t step;           // its step
  uint32_t ninstr;         // instruction count of the dependee (semaphore values advance by this per tile)
  uint32_t pad;
};

struct DTb {               // 32 bytes (host side: one per IR thread block)
  uint32_t rank;
  uint32_t instr_begin, ninstr;
  int32_t send_conn, recv_conn;  // connection index or -1
  uint32_t pad[3];
};

// What a workgroup needs to start, laid out so that it is two dependent loads away from the kernel
// arguments: its own header, then - side by side - its fiber records, the instructions of its bin (the
// instruction table is ordered by bin, so they are one contiguous range) and its rank's buffer pointers.
struct DWg {               // 32 bytes, one per (lane, bin) of the plan
  uint32_t fiber_begin, nfibers;     // range in the fiber table
  uint32_t instr_begin, ninstr;      // range of the bin's instructions in the instruction table
  uint32_t rank;                     // all fibers of a workgroup belong to one rank
  uint32_t rank_first_tb;            // global index of the rank's first thread block (its semaphore lines hold the
                                     // words in which the rank's workgroups agree, lane by lane, on their die)
  uint32_t pad[2];
};

struct DFiber {            // 48 bytes: one lane of one IR thread block
  uint32_t fid;            // global thread-block index * W + lane
  uint32_t instr_begin, ninstr;
  int32_t send_conn, recv_conn;  // connection index or -1
  uint32_t recv_from_tb;   // global index of the thread block at the sending end of recv_conn (die-scope FIFOs:
                           // the receiver checks that it runs on the sender's die), 0xffffffff if none
  // Where the connections' slots are.  A slot of connection c holds count(c) units (count(c) = the largest `count`
  // of an instruction that uses c; a unit = the slot tile of the plan); the connections follow one another in FIFO
  // memory, `before` = the sum of count over the connections in front of this one.
  uint32_t send_units_before, send_count;
  uint32_t recv_units_before, recv_count;
  uint32_t pad[2];
};

struct KParams {
  const DInstr* instrs;    // ordered by bin, then thread block, then step
  const DDep* deps;
  const DWg* wgs;          // [W * wgs_per_lane], lane-major
  const DFiber* fibers;
  void* const* bufs;       // [rank*3 + buffer] user buffers
  unsigned char* fifo;     // connection c, lane, slot at ((before(c) * W + lane * count(c)) * slots + slot * count(c)) * unit_bytes
  unsigned char* ll_fifo;  // the same for the LL protocol with ll_unit_bytes (data + flag pairs only)
  uint64_t* flags;         // [((conn*W + lane)*2 + {0 tail, 1 head}) * kFlagStrideWords]
  uint64_t* sems;          // [(tb*W + lane) * kFlagStrideWords]: word 0 the semaphore, word 1 the fiber's epoch
                           // (runs it has completed); flag values of a run lie above (epoch + 1) << 32;
                           // word 2 (die-scope FIFOs) the die the fiber runs on in this run, as run base + die + 1;
                           // word 3 (LL protocol) LL message numbers the fiber's past runs have used up;
                           // word 4 (first thread block of a rank; die-scope user buffers) the die the workgroups of
                           // this lane of the rank run on in this run, as run base + die + 1
  uint32_t* error;         // 0 = fine, else a gc3_status (negated) set by the first failing workgroup
  const uint32_t* hold;    // null, or a start word every workgroup waits for (failure-path tests)
  uint64_t chunk_bytes;
  uint64_t spin_limit_ticks;  // of the 100 MHz wall clock
  uint32_t W, slots, tile_bytes;
  uint32_t head_mask;      // a receiver stores the head flag when (messages taken & head_mask) == 0: the plan's
                           // head stride (a power of two) minus one
  uint32_t unit_bytes;     // what a slot holds per unit of `count`: the slot tile of the plan (>= tile_bytes)
  uint32_t ll_unit_bytes;  // 2 * LL tile bytes
  uint32_t ll_msgs;        // LL protocol: an upper bound of the messages one connection carries in this run.  Every
                           // fiber keeps the number of LL messages of its past runs next to its epoch (word 3 of its
                           // semaphore line); message k of this run carries flag = low 32 bits of that number + k + 1
  uint32_t W_active;       // lanes that own bytes in this run (<= W); the others own nothing and finish at once
  uint32_t wgs_per_lane;   // workgroups per lane of the static plan (the grid is lane-major)
  uint32_t nsplit;         // in this run the fiber list of every (lane, bin) is dealt round-robin to this many
                           // workgroups (1 = as planned); uses the workgroups of lanes that own no bytes
  uint32_t rank_die;       // 1: the plan placed the workgroups of rank r on die r mod 8 and the run relies on it (user
                           // buffers of dependent thread blocks meet in that die's L2): every workgroup checks it
  uint32_t bin_major;      // 0: workgroup = (sub * W_active + lane) * wgs_per_lane + bin.  1 (die-scope FIFOs, needs
                           // W_active a multiple of 8 and nsplit 1): workgroup = bin * W_active + lane, so that lane w of
                           // every thread block runs on die w mod 8 (consecutive workgroups go to consecutive dies)
};

}  // namespace gc3
