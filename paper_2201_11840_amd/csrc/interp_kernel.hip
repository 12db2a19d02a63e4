// The GC3-IR interpreter kernel for gfx950 (Section 6.2 of the paper, figure "GC3 interpreter").
//
// A workgroup executes one or a few FIBERS.  A fiber is one lane of one IR thread block: it walks
// that thread block's instruction list once per tile (outer loop = chunk tiling, inner loop =
// instructions), waits for the instruction's cross-thread-block dependencies and FIFO slots, moves
// one tile of each of the instruction's chunks with 128-bit accesses, then publishes FIFO flags and
// its semaphore.  Lightly loaded thread blocks of one rank share a workgroup, which visits its
// fibers round-robin (see the comment at the kernel).
//
// A thread block is split into W lanes; lane w owns the w-th 1/W of every chunk and has FIFO slots,
// flags and a semaphore of its own, so lanes never synchronise with each other.  All instructions
// are element-wise, hence this is Section 5.1's parallelize(W) applied by the runtime: values and
// reduction order are those of the program.
//
// Flag protocol (Section 6.1, remote buffers with s slots).  All flags are 64-bit and only grow:
// value = run_base + n, where run_base = (epoch + 1) << 32 and the epoch of a fiber is the number of runs it
// has completed, kept in device memory next to its semaphore (a fiber reads it when it starts and stores
// epoch + 1 when it is done).  The fibers of one lane take part in exactly the same runs, so both ends of a
// connection and both ends of a dependency agree on the epoch without the host passing a run number: the
// kernel's arguments are the same for every run of one size, which lets a launch be captured in a graph.
//   tail[conn, lane]  written by the sender:   messages published in this run
//   head[conn, lane]  written by the receiver: messages consumed in this run
//   sem[tb, lane]     written by the thread block: tile * ninstr + step + 1 of the latest
//                     instruction with dependents that it finished (the listing in the paper
//                     stores the bare step; the tile term and the +1 make the value monotone and
//                     distinguish "step 0 done" from the initial 0)
// A sender waits for head >= run_base + k + 1 - s before its k-th push (k >= s), a receiver for
// tail >= run_base + k + 1 before its k-th pop.  Publishing is: every wavefront waits (s_waitcnt) until
// its device-scope stores have completed, workgroup barrier, then one thread stores the flags with
// relaxed agent-scope atomics; waiting is relaxed agent-scope loads by the first wavefront, then a
// workgroup barrier, then device-scope loads of the payload.
#include <hip/hip_runtime.h>

#include <mutex>

#include "device_tables.h"
#include "gc3.h"

namespace gc3 {

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

template <int DT>
__device__ __forceinline__ uint32_t add_word(uint32_t a, uint32_t b);

template <>
__device__ __forceinline__ uint32_t add_word<GC3_F32>(uint32_t a, uint32_t b) {
  return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
}
// two fp16 values per word: one correctly rounded add each (round to nearest even, subnormals kept)
template <>
__device__ __forceinline__ uint32_t add_word<GC3_F16>(uint32_t a, uint32_t b) {
  half2_t x = __builtin_bit_cast(half2_t, a), y = __builtin_bit_cast(half2_t, b);
  return __builtin_bit_cast(uint32_t, (half2_t)(x + y));
}
// two bf16 values per word: widen to fp32 (exact), add, round to nearest even back to bf16
template <>
__device__ __forceinline__ uint32_t add_word<GC3_BF16>(uint32_t a, uint32_t b) {
  float2_t x, y;
  x.x = __uint_as_float(a << 16);
  x.y = __uint_as_float(a & 0xffff0000u);
  y.x = __uint_as_float(b << 16);
  y.y = __uint_as_float(b & 0xffff0000u);
  float2_t s = x + y;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(s, bf16x2_t));
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ u32x4 add_vec(u32x4 a, u32x4 b) {
  u32x4 r;
  r.x = add_word<DT>(a.x, b.x);
  r.y = add_word<DT>(a.y, b.y);
  r.z = add_word<DT>(a.z, b.z);
  r.w = add_word<DT>(a.w, b.w);
  return r;
}

// Cache policy of a 128-bit access: the sc0 / nt / sc1 bits of gfx950 buffer instructions.
// MI355X has one L2 per die (XCD) and these L2s are not kept coherent with each other, so data that a
// workgroup on another die wrote, or will read, must not be served from / parked in the local L2:
//   sc1 (device scope) store: written through, complete at device scope when its counter retires;
//   sc1 load: never served from a stale line.
// FIFO payload always moves with sc1.  User buffers are streamed once (nt = non-temporal); they need
// device scope only in programs with cross-thread-block dependencies, where one workgroup reads
// chunks another one wrote in the same run (template parameter COH).  With these policies no bulk L2
// write-back / invalidate (agent-scope fence) is needed anywhere in the kernel.
constexpr int kPolNt = 2, kPolSc1 = 16;   // (bit 0 would be sc0)
constexpr int kSlotLd = kPolSc1, kSlotSt = kPolSc1;
constexpr int kUserLd = kPolNt, kUserSt = kPolSc1;
constexpr int kUserLdCoh = kPolSc1 | kPolNt, kUserStCoh = kPolSc1 | kPolNt;
// How a program's thread blocks see each other's writes to their rank's buffers (template parameter COH):
// kCohNone - they never read them (no cross-thread-block dependencies); kCohDevice - through the memory system;
// kCohDie - through the L2 of the die that all workgroups of the rank run on (loads that bypass only the compute
// unit's L1, plain stores: complete, for a reader on the same die, when the store counter retires).
constexpr int kCohNone = 0, kCohDevice = 1, kCohDie = 2;
constexpr int kUserStDie = 0;
constexpr int kUnroll = 4;                // 128-bit loads per stream in flight before the adds and stores
constexpr uint32_t kStageBytes = 16384;   // LDS staging area per workgroup (staged variant only): one sweep of 256 threads

typedef __amdgpu_buffer_rsrc_t rsrc_t;

// Buffer descriptor over [base, base + bytes): accesses beyond it are dropped by the hardware
// (loads return 0), which also makes the ragged last sweep of a tile safe without predicates.
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// out0[i] (and out1[i]) = in0[i] (+ in1[i]) for i in [0, nvec), 16 bytes per element.  Element i is
// always handled by thread i mod nthreads, so a location is touched by the same thread in every
// instruction of a thread block.
template <bool IN1, bool OUT1, int DT, int P_IN0, int P_IN1, int P_OUT0, int P_OUT1>
__device__ __forceinline__ void move_tile(rsrc_t in0, rsrc_t in1, rsrc_t out0, rsrc_t out1,
                                          uint32_t nvec, uint32_t tid, uint32_t nthreads) {
  const uint32_t step = nthreads * kUnroll;
  for (uint32_t base = tid; base < nvec; base += step) {
    u32x4 a[kUnroll], b[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      a[u] = __builtin_amdgcn_raw_buffer_load_b128(in0, (base + u * nthreads) << 4, 0, P_IN0);
    if (IN1) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        b[u] = __builtin_amdgcn_raw_buffer_load_b128(in1, (base + u * nthreads) << 4, 0, P_IN1);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) a[u] = add_vec<DT>(a[u], b[u]);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      __builtin_amdgcn_raw_buffer_store_b128(a[u], out0, (base + u * nthreads) << 4, 0, P_OUT0);
      if (OUT1) __builtin_amdgcn_raw_buffer_store_b128(a[u], out1, (base + u * nthreads) << 4, 0, P_OUT1);
    }
  }
}

// Same contract as move_tile, but in0 (a FIFO slot) is first brought into LDS by direct-to-LDS loads:
// wavefront w's k-th load writes elements [k*nthreads + 64w, +64) to consecutive 16-byte LDS cells, so
// element i sits at LDS byte 16*i and thread i mod nthreads reads back only what its own wavefront
// loaded (no workgroup barrier, just the wait for the loads).
template <bool IN1, bool OUT1, int DT, int P_IN0, int P_IN1, int P_OUT0, int P_OUT1>
__device__ __forceinline__ void move_tile_staged(rsrc_t in0, rsrc_t in1, rsrc_t out0, rsrc_t out1, uint32_t nvec,
                                                 uint32_t tid, uint32_t nthreads, unsigned char* stage) {
  typedef __attribute__((address_space(3))) void lds_void;
  const uint32_t cap = kStageBytes >> 4;                       // elements per staging round
  const uint32_t wave_first = tid & ~63u;
  for (uint32_t r0 = 0; r0 < nvec; r0 += cap) {
    const uint32_t n = nvec - r0 < cap ? nvec - r0 : cap;
    for (uint32_t k = 0; k < n; k += nthreads)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(in0, (lds_void*)(stage + ((k + wave_first) << 4)), 16,
                                               (r0 + k + tid) << 4, 0, 0, P_IN0);
    const uint32_t step = nthreads * kUnroll;
    for (uint32_t base = tid; base < n; base += step) {
      u32x4 a[kUnroll], b[kUnroll];
      if (IN1) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          b[u] = __builtin_amdgcn_raw_buffer_load_b128(in1, (r0 + base + u * nthreads) << 4, 0, P_IN1);
      }
      __builtin_amdgcn_s_waitcnt(0);                           // staged loads (and in1) have landed
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t i = base + u * nthreads;
        a[u] = i < n ? *(const u32x4*)(stage + (i << 4)) : u32x4{0, 0, 0, 0};
        if (IN1) a[u] = add_vec<DT>(a[u], b[u]);
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        __builtin_amdgcn_raw_buffer_store_b128(a[u], out0, (r0 + base + u * nthreads) << 4, 0, P_OUT0);
        if (OUT1) __builtin_amdgcn_raw_buffer_store_b128(a[u], out1, (r0 + base + u * nthreads) << 4, 0, P_OUT1);
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();                           // this wavefront's cells may be reused
  }
}

// ---- LL protocol (Section 6.1, "Protocols": lowest latency, half the bandwidth) -------------------------
// A message is not announced by a separate flag: every 8 bytes in the FIFO slot are 4 bytes of data plus
// a 4-byte flag (an 8-byte store is indivisible), so a 16-byte element occupies 32 bytes
// {d0 f d1 f | d2 f d3 f}.  The receiver polls the data itself until all four flags carry the
// message's number; the sender needs neither a completion wait nor a barrier.  LL slots live in a
// region of their own that only ever holds such pairs, so a stale word can never pass for a flag.
//
// out[i] = (POP ? unpack(in_ll[i]) : src[i]) (+ src[i] if POP && ADD); optionally stored to dst and/or
// packed into out_ll with flag `fout`.  Returns false when the wait for data exceeded the spin limit.
template <bool POP, bool ADD, bool OUT0, bool PUSH, int DT, int P_SRC, int P_DST>
__device__ __forceinline__ bool move_tile_ll(rsrc_t in_ll, rsrc_t src, rsrc_t dst, rsrc_t out_ll, uint32_t nvec,
                                             uint32_t tid, uint32_t nthreads, uint32_t fin, uint32_t fout,
                                             const KParams& p) {
  constexpr int UN = 2;
  bool ok = true;
  const uint32_t step = nthreads * UN;
  for (uint32_t base = tid; base < nvec && ok; base += step) {
    u32x4 v[UN], b[UN];
    if (ADD || !POP) {
#pragma unroll
      for (int u = 0; u < UN; ++u) b[u] = __builtin_amdgcn_raw_buffer_load_b128(src, (base + u * nthreads) << 4, 0, P_SRC);
    }
    if (POP) {
      uint64_t start = 0;                              // wall clock at the first periodic check (reading it costs ~0.1 us)
      uint32_t spins = 0;
      for (;;) {
        bool all = true;
        asm volatile("" ::: "memory");                   // the slot is re-read in every iteration, never hoisted
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const uint32_t i = base + u * nthreads;
          const u32x4 lo = __builtin_amdgcn_raw_buffer_load_b128(in_ll, i << 5, 0, kPolSc1);
          const u32x4 hi = __builtin_amdgcn_raw_buffer_load_b128(in_ll, (i << 5) + 16, 0, kPolSc1);
          if (i < nvec && (lo.y != fin || lo.w != fin || hi.y != fin || hi.w != fin)) all = false;
          v[u] = u32x4{lo.x, lo.z, hi.x, hi.z};
        }
        if (all) break;
        if ((++spins & 1023u) == 0) {
          const uint64_t now = wall_clock64();
          if (start == 0) start = now;
          if (__hip_atomic_load(p.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 ||
              now - start > p.spin_limit_ticks) {
            atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_TIMEOUT));
            ok = false;
            break;
          }
        }
      }
      if (ADD) {
#pragma unroll
        for (int u = 0; u < UN; ++u) v[u] = add_vec<DT>(v[u], b[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < UN; ++u) v[u] = b[u];
    }
    if (!ok) break;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const uint32_t i = base + u * nthreads;
      if (OUT0) __builtin_amdgcn_raw_buffer_store_b128(v[u], dst, i << 4, 0, P_DST);
      if (PUSH) {
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{v[u].x, fout, v[u].y, fout}, out_ll, i << 5, 0, kPolSc1);
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{v[u].z, fout, v[u].w, fout}, out_ll, (i << 5) + 16, 0, kPolSc1);
      }
    }
  }
  return ok;
}

__device__ __forceinline__ uint64_t load_flag(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_flag(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// First byte of lane w's share of a chunk of `chunk_bytes` split over W lanes (w = W gives the chunk's end).
// Shares are cut at 256-byte boundaries when every lane can get at least that much, else at 16-byte
// boundaries.  32-bit arithmetic: the host admits chunks below 2^40 bytes only, and
// floor(n * w / W) = (n / W) * w + floor((n % W) * w / W).
__device__ __forceinline__ uint64_t lane_begin(uint64_t chunk_bytes, uint32_t w, uint32_t W) {
  if (w >= W) return chunk_bytes;
  const uint64_t U = chunk_bytes >> 4;
  if (U >= 16ull * W) {
    const uint32_t n = (uint32_t)(U >> 4);
    return ((uint64_t)(n / W) * w + ((n % W) * w) / W) << 8;
  }
  return (uint64_t)(((uint32_t)U * w) / W) << 4;
}

}  // namespace

constexpr uint32_t kFiberDone = 0xffffffffu;

__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uni64(uint64_t v) { return ((uint64_t)uni((uint32_t)(v >> 32)) << 32) | uni((uint32_t)v); }

namespace {

// Protocol / payload path of an interpreter instantiation.
constexpr int kSimple = 0;   // payload, completion wait, separate flag; payload moves through registers
constexpr int kLL = 1;       // every 8 bytes carry 4 bytes of data and a 4-byte flag
constexpr int kStaged = 2;   // simple protocol, FIFO payload of the receiving instructions staged through LDS
constexpr int kDie = 3;      // simple protocol, FIFO payload kept in the L2 of the die both ends of a connection run on

// Die-scope FIFO payload.  Such a run is launched bin-major with a multiple of 8 active lanes, so that the two ends
// of every connection - always the same lane of two thread blocks - run on one die (XCD), whose L2 all its compute
// units share.  The sender writes slots with plain stores - through the compute unit's L1 into that L2, complete
// when the store counter retires - and the receiver reads them with non-temporal loads, which never hit in its L1
// (MISS_EVICT policy) and find the line in the shared L2: FIFO reads no longer cross the fabric (measured: 94 % of
// them with 2 MiB of slots per die; the writes are still written back to memory).  A line evicted in between is
// simply fetched again.  Flags stay device-scope atomics.  Because a receiver on another die would silently read
// stale memory, every fiber publishes the die it runs on and every receiver checks it against its own before its
// first pop.
constexpr int kDieSlotLd = kPolNt, kDieSlotSt = 0;

__device__ __forceinline__ uint32_t this_die() {
  // XCC_ID hardware register (id 20), bits 3:0
  return (uint32_t)__builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & 0xfu;
}

__device__ __forceinline__ uint64_t* flag_of(const KParams& p, int32_t conn, uint32_t lane, uint32_t which) {
  return p.flags + ((uint64_t)((uint32_t)conn * p.W + lane) * 2 + which) * kFlagStrideWords;
}
__device__ __forceinline__ uint64_t* sem_of(const KParams& p, uint32_t tb, uint32_t lane) {
  return p.sems + (uint64_t)(tb * p.W + lane) * kFlagStrideWords;
}

// LL message numbers of a run.  A fiber's past runs have used up `used` of them (kept in its semaphore line, the
// same value at both ends of a connection because the fibers of one lane take part in the same runs); this run may
// use `msgs`.  The low 32 bits are the flags that travel with the payload and 0 is what untouched slot memory holds,
// so a run's range never crosses a multiple of 2^32.  Returns the number the run starts from.
__device__ __forceinline__ uint64_t ll_run_start(uint64_t used, uint32_t msgs) {
  return ((used + msgs) >> 32) != (used >> 32) ? ((used >> 32) + 1) << 32 : used;
}

// Failure-path test facility: wait (bounded by the spin limit) for a start word that the host never sets.
// Called by one thread; returns false when the run is abandoned.
// Die-scope user buffers: the workgroups that run lane w of a rank's thread blocks - they wait on each other and
// read what the others wrote of the lane's share of the rank's buffers - must share a die.  Each of them raises the
// word of (rank, lane) to (run base + its die + 1) at its start and looks at what it found when it ends: a different
// value of this run means two of them ran on different dies (whichever came second sees it), and the run is marked
// as failed.  (The fibers of one lane have all completed the same runs, so they agree on the run base; other lanes
// may have sat out runs on small buffers.)
__device__ __forceinline__ uint64_t rank_die_enter(const KParams& p, uint32_t rank_first_tb, uint32_t lane, uint64_t run_base) {
  uint64_t* const word = p.sems + ((uint64_t)rank_first_tb * p.W + lane) * kFlagStrideWords + 4;
  return __hip_atomic_fetch_max(word, run_base + this_die() + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void rank_die_leave(const KParams& p, uint64_t found, uint64_t run_base) {
  if (found > run_base && found != run_base + this_die() + 1) atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_PLACEMENT));
}

__device__ __forceinline__ bool hold_wait(const KParams& p) {
  const uint64_t start = wall_clock64();
  while (__hip_atomic_load(p.hold, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
    __builtin_amdgcn_s_sleep(8);
    if (__hip_atomic_load(p.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return false;
    if (wall_clock64() - start > p.spin_limit_ticks) {
      atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_TIMEOUT));
      return false;
    }
  }
  return true;
}

// The waits of one instruction, taken by the lanes of ONE wavefront (all 64 call this): lane 0 polls the tail
// flag of the receive connection (tail_recv, may be null), lane 1 the head flag of the send connection
// (head_send, may be null), lanes 2.. one dependency's semaphore each, in rounds of 64 when an instruction has
// more than 62 dependencies.  block: spin (bounded by the spin limit) until every flag has reached its value;
// otherwise a single look.  Returns 1 = ready, 0 = not ready, -1 = the run is abandoned.  `seen` is the last
// value this lane loaded (lane 1: the head flag, meaningful when ndeps <= 62).
__device__ __forceinline__ int poll_flags(const KParams& p, uint32_t lane_id, bool block,
                                          const uint64_t* tail_recv, uint64_t want_tail,
                                          const uint64_t* head_send, uint64_t want_head,
                                          uint32_t dep_begin, uint32_t ndeps, uint32_t lane,
                                          uint64_t run_base, uint32_t t, uint64_t& seen) {
  int res = 1;
  seen = 0;
  const uint32_t total = 2 + ndeps;
  for (uint32_t it0 = 0; it0 < total && res == 1; it0 += 64) {
    const uint32_t it = it0 + lane_id;
    const uint64_t* ptr = nullptr;
    uint64_t want = 0;
    if (it == 0) {
      ptr = tail_recv; want = want_tail;
    } else if (it == 1) {
      ptr = head_send; want = want_head;
    } else if (it < total) {
      const DDep d = p.deps[dep_begin + it - 2];
      ptr = sem_of(p, d.tb, lane);
      want = run_base + (uint64_t)t * d.ninstr + d.step + 1;
    }
    bool pending = ptr != nullptr;
    uint64_t start = 0;                                // wall clock at the first periodic check (reading it costs ~0.1 us)
    uint32_t spins = 0;
    for (;;) {
      if (pending) {
        seen = load_flag(ptr);
        if (seen >= want) pending = false;
      }
      if (!__any(pending)) break;
      if (!block) { res = 0; break; }
      if (++spins > 16) __builtin_amdgcn_s_sleep(1);     // poll hard first, politely later
      if ((spins & 255u) == 0) {
        if (__hip_atomic_load(p.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { res = -1; break; }
        const uint64_t now = wall_clock64();
        if (start == 0) start = now;
        if (now - start > p.spin_limit_ticks) {
          atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_TIMEOUT));
          res = -1;
          break;
        }
      }
    }
  }
  return res;
}

// One tile of one instruction under the simple protocol: `count` pieces of `len` bytes, piece j at
// srcb / dstb + j * chunk_bytes in the user buffers and packed back to back in the FIFO slots.
template <int DT, int COH, bool STAGE, bool DIE>
__device__ __forceinline__ void move_simple(uint32_t op, uint32_t count, unsigned char* srcb, unsigned char* dstb,
                                            unsigned char* rslot, unsigned char* sslot, uint32_t len,
                                            uint64_t chunk_bytes, uint32_t tid, uint32_t nthreads, unsigned char* stage) {
  constexpr int UL = COH == kCohDevice ? kUserLdCoh : kUserLd, US = COH == kCohDevice ? kUserStCoh : COH == kCohDie ? kUserStDie : kUserSt;
  constexpr int SL = DIE ? kDieSlotLd : kSlotLd, SS = DIE ? kDieSlotSt : kSlotSt;
  const uint32_t nvec = len >> 4;
  for (uint32_t j = 0; j < count; ++j) {
    const rsrc_t src = make_rsrc(srcb + (uint64_t)j * chunk_bytes, srcb ? len : 0);
    const rsrc_t dst = make_rsrc(dstb + (uint64_t)j * chunk_bytes, dstb ? len : 0);
    const rsrc_t rs = make_rsrc(rslot + (uint64_t)j * len, rslot ? len : 0);
    const rsrc_t ss = make_rsrc(sslot + (uint64_t)j * len, sslot ? len : 0);
    switch (op) {
      case GC3_OP_SEND:   move_tile<false, false, DT, UL, 0, SS, 0>(src, src, ss, ss, nvec, tid, nthreads); break;
      case GC3_OP_COPY:   move_tile<false, false, DT, UL, 0, US, 0>(src, src, dst, dst, nvec, tid, nthreads); break;
      case GC3_OP_REDUCE: move_tile<true, false, DT, UL, UL, US, 0>(dst, src, dst, dst, nvec, tid, nthreads); break;
      default:
        if (STAGE) {
          switch (op) {
            case GC3_OP_RECV: move_tile_staged<false, false, DT, SL, 0, US, 0>(rs, rs, dst, dst, nvec, tid, nthreads, stage); break;
            case GC3_OP_RRC:  move_tile_staged<true, false, DT, SL, UL, US, 0>(rs, src, dst, dst, nvec, tid, nthreads, stage); break;
            case GC3_OP_RCS:  move_tile_staged<false, true, DT, SL, 0, US, SS>(rs, rs, dst, ss, nvec, tid, nthreads, stage); break;
            case GC3_OP_RRCS: move_tile_staged<true, true, DT, SL, UL, US, SS>(rs, src, dst, ss, nvec, tid, nthreads, stage); break;
            case GC3_OP_RRS:  move_tile_staged<true, false, DT, SL, UL, SS, 0>(rs, src, ss, ss, nvec, tid, nthreads, stage); break;
            default: break;
          }
        } else {
          switch (op) {
            case GC3_OP_RECV: move_tile<false, false, DT, SL, 0, US, 0>(rs, rs, dst, dst, nvec, tid, nthreads); break;
            case GC3_OP_RRC:  move_tile<true, false, DT, SL, UL, US, 0>(rs, src, dst, dst, nvec, tid, nthreads); break;
            case GC3_OP_RCS:  move_tile<false, true, DT, SL, 0, US, SS>(rs, rs, dst, ss, nvec, tid, nthreads); break;
            case GC3_OP_RRCS: move_tile<true, true, DT, SL, UL, US, SS>(rs, src, dst, ss, nvec, tid, nthreads); break;
            case GC3_OP_RRS:  move_tile<true, false, DT, SL, UL, SS, 0>(rs, src, ss, ss, nvec, tid, nthreads); break;
            default: break;
          }
        }
    }
  }
}

__device__ __forceinline__ bool op_pops(uint32_t op) {
  return op == GC3_OP_RECV || op == GC3_OP_RRC || op == GC3_OP_RCS || op == GC3_OP_RRCS || op == GC3_OP_RRS;
}
__device__ __forceinline__ bool op_pushes(uint32_t op) {
  return op == GC3_OP_SEND || op == GC3_OP_RCS || op == GC3_OP_RRCS || op == GC3_OP_RRS;
}

}  // namespace

// A workgroup runs a short list of FIBERS.  A fiber is one lane of one IR thread block: its own
// tile counter, step counter and FIFO sequence numbers.  The workgroup visits its unfinished
// fibers round-robin and advances each as far as its waits allow; while more than one fiber is
// unfinished a wait is a single poll (a fiber that is not ready yields to the next one, so thread
// blocks sharing a workgroup can never block each other), and the last unfinished fiber waits by
// spinning.  One fiber per workgroup is the paper's one-thread-block-per-block execution.
template <int DT, int COH, int MODE>
__global__ void __launch_bounds__(512) gc3_interpreter(KParams p) {
  constexpr bool LL = MODE == kLL;
  constexpr bool STAGE = MODE == kStaged;
  constexpr bool DIE = MODE == kDie;
  __shared__ uint32_t f_id[kMaxFibersPerWg], f_t[kMaxFibersPerWg], f_s[kMaxFibersPerWg];
  __shared__ uint32_t f_send[kMaxFibersPerWg], f_recv[kMaxFibersPerWg];
  // messages of this run the fiber's receiver is known to have consumed (last head flag value seen): a push
  // polls the head flag only when this does not already show a free slot
  __shared__ uint32_t f_head[kMaxFibersPerWg];
  __shared__ uint32_t f_epoch[kMaxFibersPerWg];    // runs the fiber has completed before this one
  __shared__ uint64_t f_ll[LL ? kMaxFibersPerWg : 1];   // LL message number the fiber's run starts from
  __shared__ uint32_t f_from[kMaxFibersPerWg];     // thread block at the sending end of the fiber's receive connection
  __shared__ uint32_t s_headv[2];
  __shared__ uint64_t f_off0[kMaxFibersPerWg], f_share[kMaxFibersPerWg];
  // per fiber: its thread block's record and the three buffer pointers of its rank, fetched once
  __shared__ uint32_t f_ibeg[kMaxFibersPerWg], f_ninstr[kMaxFibersPerWg], f_ilds[kMaxFibersPerWg];
  __shared__ int32_t f_sconn[kMaxFibersPerWg], f_rconn[kMaxFibersPerWg];
  // slots of the fiber's connections: position of its first slot in units of `count` x slot tile, units per slot
  __shared__ uint64_t f_sfirst[kMaxFibersPerWg], f_rfirst[kMaxFibersPerWg];
  __shared__ uint32_t f_scount[kMaxFibersPerWg], f_rcount[kMaxFibersPerWg];
  __shared__ uint64_t s_buf[3];
  // the instruction lists of this workgroup's fibers, when they fit (else they are read from global memory
  // every time): an instruction is fetched once per tile, and a fetch is a dependent global access on the
  // critical path of every hop
  __shared__ uint32_t s_instr[kLdsInstrs * 8];
  __shared__ int s_res[2];
  __shared__ __attribute__((aligned(16))) unsigned char s_stage[STAGE ? kStageBytes : 16];
  const uint32_t tid = threadIdx.x, nthreads = blockDim.x;
  // blockIdx = (sub * W_active + lane) * wgs_per_lane + bin: this workgroup takes entries sub, sub + nsplit, ...
  // of the fiber list the plan gives (lane, bin); or, bin-major, blockIdx = bin * W_active + lane
  const uint32_t slot = p.bin_major ? blockIdx.x % p.W_active : blockIdx.x / p.wgs_per_lane;
  const uint32_t bin = p.bin_major ? blockIdx.x / p.W_active : blockIdx.x % p.wgs_per_lane;
  const uint32_t sub = slot / p.W_active, nsplit = p.nsplit;
  const DWg hdr = p.wgs[(slot % p.W_active) * p.wgs_per_lane + bin];
  const uint32_t nf = hdr.nfibers > sub ? (hdr.nfibers - sub + nsplit - 1) / nsplit : 0;
  if (nf == 0) return;
  if (p.hold) {
    if (tid == 0) s_res[0] = hold_wait(p) ? 1 : -1;
    __syncthreads();
    if (s_res[0] < 0) return;
    __syncthreads();
  }
  const uint32_t W = p.W;
  const uint32_t tile = p.tile_bytes;
  uint64_t rank_die_found = 0, rank_die_base = 0;      // (thread 0 only)
  // fiber records, the bin's instructions and the rank's buffer pointers: independent loads, one barrier
  if (tid < nf) {
    const DFiber f = p.fibers[hdr.fiber_begin + sub + tid * nsplit];
    const uint32_t lane = f.fid % W;
    const uint64_t o = lane_begin(p.chunk_bytes, lane, p.W_active);
    f_id[tid] = f.fid;
    f_t[tid] = 0;
    f_s[tid] = 0;
    f_send[tid] = 0;
    f_recv[tid] = 0;
    f_head[tid] = 0;
    const uint32_t epoch = (uint32_t)load_flag(p.sems + (uint64_t)f.fid * kFlagStrideWords + 1);
    f_epoch[tid] = epoch;
    if (p.rank_die && tid == 0) {
      rank_die_base = (uint64_t)(epoch + 1) << 32;
      rank_die_found = rank_die_enter(p, hdr.rank_first_tb, lane, rank_die_base);
    }
    if (LL) f_ll[tid] = ll_run_start(load_flag(p.sems + (uint64_t)f.fid * kFlagStrideWords + 3), p.ll_msgs);
    f_from[tid] = f.recv_from_tb;
    if (DIE) store_flag(p.sems + (uint64_t)f.fid * kFlagStrideWords + 2, ((uint64_t)(epoch + 1) << 32) + this_die() + 1);
    f_off0[tid] = o;
    f_share[tid] = lane_begin(p.chunk_bytes, lane + 1, p.W_active) - o;
    f_ninstr[tid] = f.ninstr;
    f_ibeg[tid] = f.instr_begin;
    f_ilds[tid] = f.instr_begin - hdr.instr_begin;
    f_sconn[tid] = f.send_conn;
    f_rconn[tid] = f.recv_conn;
    f_sfirst[tid] = ((uint64_t)f.send_units_before * W + (uint64_t)lane * f.send_count) * p.slots;
    f_rfirst[tid] = ((uint64_t)f.recv_units_before * W + (uint64_t)lane * f.recv_count) * p.slots;
    f_scount[tid] = f.send_count;
    f_rcount[tid] = f.recv_count;
  }
  if (tid >= 32 && tid < 35) s_buf[tid - 32] = (uint64_t)p.bufs[hdr.rank * 3 + (tid - 32)];
  const bool instr_in_lds = hdr.ninstr <= (uint32_t)kLdsInstrs;
  if (instr_in_lds) {
    const uint32_t* gi = (const uint32_t*)(p.instrs + hdr.instr_begin);
    for (uint32_t k = tid; k < hdr.ninstr * 8; k += nthreads) s_instr[k] = gi[k];
  }
  uint32_t live = nf, phase = 0;
  uint64_t last_progress = wall_clock64();

  while (live) {
    bool any_progress = false;
    for (uint32_t fi = 0; fi < nf; ++fi) {
      __syncthreads();                                   // state written in the previous visit is visible
      uint32_t t = uni(f_t[fi]);
      if (t == kFiberDone) continue;
      const uint32_t fid = uni(f_id[fi]);
      const uint32_t tbi = fid / W, lane = fid % W;
      const uint32_t tb_instr_begin = uni(f_ibeg[fi]), tb_ninstr = uni(f_ninstr[fi]);
      const int32_t send_conn = (int32_t)uni((uint32_t)f_sconn[fi]), recv_conn = (int32_t)uni((uint32_t)f_rconn[fi]);
      const uint32_t ilds = uni(f_ilds[fi]) * 8;
      const uint32_t epoch = uni(f_epoch[fi]);
      const uint64_t run_base = (uint64_t)(epoch + 1) << 32;
      const uint64_t off0 = ((uint64_t)uni((uint32_t)(f_off0[fi] >> 32)) << 32) | uni((uint32_t)f_off0[fi]);
      const uint64_t share = ((uint64_t)uni((uint32_t)(f_share[fi] >> 32)) << 32) | uni((uint32_t)f_share[fi]);
      const uint32_t ntiles = (uint32_t)((share + tile - 1) / tile);
      uint32_t s = uni(f_s[fi]), send_seq = uni(f_send[fi]), recv_seq = uni(f_recv[fi]);
      uint32_t head_known = uni(f_head[fi]);
      const uint64_t ll_start = LL ? uni64(f_ll[fi]) : 0;
      const uint32_t ll_base = (uint32_t)ll_start;

      uint64_t* const tail_send = send_conn >= 0 ? flag_of(p, send_conn, lane, 0) : nullptr;
      uint64_t* const head_send = send_conn >= 0 ? flag_of(p, send_conn, lane, 1) : nullptr;
      uint64_t* const tail_recv = recv_conn >= 0 ? flag_of(p, recv_conn, lane, 0) : nullptr;
      uint64_t* const head_recv = recv_conn >= 0 ? flag_of(p, recv_conn, lane, 1) : nullptr;
      unsigned char* const fifo_base = LL ? p.ll_fifo : p.fifo;            // LL slots have a region of their own
      const uint32_t unit_bytes = LL ? p.ll_unit_bytes : p.unit_bytes;
      const uint32_t sslot_bytes = uni(f_scount[fi]) * unit_bytes, rslot_bytes = uni(f_rcount[fi]) * unit_bytes;
      unsigned char* const fifo_send = send_conn >= 0 ? fifo_base + uni64(f_sfirst[fi]) * unit_bytes : nullptr;
      unsigned char* const fifo_recv = recv_conn >= 0 ? fifo_base + uni64(f_rfirst[fi]) * unit_bytes : nullptr;
      uint64_t* const my_sem = sem_of(p, tbi, lane);

      bool progressed = false;
      while (t < ntiles && s < tb_ninstr) {              // tile loop outside, instruction loop inside
        const uint64_t toff = (uint64_t)t * tile;
        const uint32_t len = (uint32_t)(share - toff < tile ? share - toff : tile);   // bytes of this tile, per chunk
        const uint32_t nvec = len >> 4;
        DInstr ins;
        if (instr_in_lds) {
          const uint32_t* w = s_instr + ilds + s * 8;
          ins.op = uni(w[0]); ins.srcbuf = uni(w[1]); ins.dstbuf = uni(w[2]); ins.srcidx = uni(w[3]);
          ins.dstidx = uni(w[4]); ins.count = uni(w[5]); ins.dep_begin = uni(w[6]); ins.ndeps_hasdep = uni(w[7]);
        } else {
          ins = p.instrs[tb_instr_begin + s];
        }
        const uint32_t op = ins.op;
        const bool pops = op_pops(op), pushes = op_pushes(op);
        const uint32_t ndeps = ins.ndeps_hasdep >> 1;
        const bool hasdep = ins.ndeps_hasdep & 1;
        const bool wait_slot = pushes && send_seq >= head_known + p.slots;

        // ---- wait for dependencies, for a message, for a free slot -----------------------------
        // LL: the message's number doubles as the flag carried by every 8 bytes of its payload
        const uint32_t ll_fin = ll_base + recv_seq + 1, ll_fout = ll_base + send_seq + 1;
        const bool block = live == 1;
        // (in LL mode a blocking receive needs no announcement: every thread polls its own data)
        if ((pops && !(LL && block)) || wait_slot || ndeps) {
          if (tid < 64) {
            uint64_t seen;
            int res = poll_flags(p, tid, block, (pops && !LL) ? tail_recv : nullptr, run_base + recv_seq + 1,
                                 wait_slot ? head_send : nullptr, run_base + send_seq + 1 - p.slots,
                                 ins.dep_begin, ndeps, lane, run_base, t, seen);
            // (only more than 62 dependencies would take the polling past its first round, in which lane 1
            // polls the head flag)
            if (tid == 1 && wait_slot && res == 1 && ndeps <= 62) s_headv[phase & 1] = (uint32_t)(seen - run_base);
            if (DIE && pops && recv_seq == 0 && res == 1 && tid == 0) {
              // first message of this run on this connection: the sender published its die before the message
              if (load_flag(sem_of(p, uni(f_from[fi]), lane) + 2) != run_base + this_die() + 1) {
                atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_PLACEMENT));
                res = -1;
              }
            }
            if (LL && pops && !block && res == 1) {
              // non-blocking readiness probe: has the first element of the message arrived?
              const uint32_t* first = (const uint32_t*)(fifo_recv + (uint64_t)(recv_seq % p.slots) * rslot_bytes);
              if (__hip_atomic_load(first + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != ll_fin) res = 0;
            }
            if (tid == 0) s_res[phase & 1] = res;
          }
          __syncthreads();
          const int res_all = s_res[phase & 1];
          ++phase;
          if (res_all < 0) return;     // the run is abandoned; every workgroup leaves the same way
          if (res_all == 0) break;     // not ready: yield to the next fiber
          if (wait_slot && ndeps <= 62) head_known = uni(s_headv[(phase - 1) & 1]);
        }

        // ---- move the tile --------------------------------------------------------------------
        const uint64_t coff = off0 + toff;   // byte offset inside each chunk
        unsigned char* const srcb = ins.srcbuf < 3 ? (unsigned char*)uni64(s_buf[ins.srcbuf]) + (uint64_t)ins.srcidx * p.chunk_bytes + coff : nullptr;
        unsigned char* const dstb = ins.dstbuf < 3 ? (unsigned char*)uni64(s_buf[ins.dstbuf]) + (uint64_t)ins.dstidx * p.chunk_bytes + coff : nullptr;
        unsigned char* const rslot = pops ? fifo_recv + (uint64_t)(recv_seq % p.slots) * rslot_bytes : nullptr;
        unsigned char* const sslot = pushes ? fifo_send + (uint64_t)(send_seq % p.slots) * sslot_bytes : nullptr;
        bool data_ok = true;
        if (LL && (pops || pushes)) {
          constexpr int UL = COH == kCohDevice ? kUserLdCoh : kUserLd, US = COH == kCohDevice ? kUserStCoh : COH == kCohDie ? kUserStDie : kUserSt;
          for (uint32_t j = 0; j < ins.count; ++j) {
            const rsrc_t src = make_rsrc(srcb + (uint64_t)j * p.chunk_bytes, srcb ? len : 0);
            const rsrc_t dst = make_rsrc(dstb + (uint64_t)j * p.chunk_bytes, dstb ? len : 0);
            const rsrc_t rl = make_rsrc(rslot + (uint64_t)j * len * 2, rslot ? len * 2 : 0);
            const rsrc_t sl = make_rsrc(sslot + (uint64_t)j * len * 2, sslot ? len * 2 : 0);
            switch (op) {
              case GC3_OP_SEND: move_tile_ll<false, false, false, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              case GC3_OP_RECV: data_ok &= move_tile_ll<true, false, true, false, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              case GC3_OP_RRC:  data_ok &= move_tile_ll<true, true, true, false, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              case GC3_OP_RCS:  data_ok &= move_tile_ll<true, false, true, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              case GC3_OP_RRCS: data_ok &= move_tile_ll<true, true, true, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              case GC3_OP_RRS:  data_ok &= move_tile_ll<true, true, false, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, nthreads, ll_fin, ll_fout, p); break;
              default: break;
            }
          }
        } else {
          move_simple<DT, COH, STAGE, DIE>(op, ins.count, srcb, dstb, rslot, sslot, len, p.chunk_bytes, tid, nthreads, s_stage);
        }

        // ---- publish: slot filled, slot freed, semaphore ----------------------------------------
        if (pushes) ++send_seq;
        if (pops) ++recv_seq;
        // Simple protocol: a push publishes tail, a pop publishes head.  LL: payload carries its own flag,
        // so only head (slot free again) and semaphores are published, and only a semaphore - which
        // covers plain user-buffer stores - needs the stores to have completed.
        if (LL ? (pops || hasdep) : (pushes || pops || hasdep)) {
          // Every wavefront waits until its own stores have completed at device scope (the store counter
          // retires a device-scope store only then) BEFORE the barrier: a workgroup-scope barrier alone
          // does not wait for outstanding global stores on this target, and the flag written below
          // must never overtake the payload.
          if (!LL || hasdep) __builtin_amdgcn_s_waitcnt(0);
          if (LL) {
            if (__syncthreads_or(data_ok ? 0 : 1)) return;     // a thread gave up waiting for data
          } else {
            __syncthreads();
          }
          if (tid == 0) {
            if (pushes && !LL) store_flag(tail_send, run_base + send_seq);
            if (pops && (recv_seq & p.head_mask) == 0) store_flag(head_recv, run_base + recv_seq);
            if (hasdep) store_flag(my_sem, run_base + (uint64_t)t * tb_ninstr + s + 1);
          }
        }
        progressed = true;
        if (++s == tb_ninstr) { s = 0; ++t; }
      }

      const bool finished = t >= ntiles || tb_ninstr == 0;   // also true for a lane that owns no bytes
      if (progressed || finished) {
        any_progress = true;
        __syncthreads();                                 // every wavefront has read this fiber's old state
        if (tid == 0) {
          f_t[fi] = finished ? kFiberDone : t;
          f_s[fi] = s;
          f_send[fi] = send_seq;
          f_recv[fi] = recv_seq;
          f_head[fi] = head_known;
          if (finished) {
            store_flag(my_sem + 1, (uint64_t)epoch + 1);   // this fiber has completed one more run
            if (LL) store_flag(my_sem + 3, ll_start + p.ll_msgs);
          }
        }
      }
      if (finished) --live;
    }
    if (live && !any_progress) {
      // a whole sweep without progress: back off, and give up when nothing moved for the spin limit
      if (tid == 0) {
        int res = 1;
        if (__hip_atomic_load(p.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
          res = -1;
        } else if (wall_clock64() - last_progress > p.spin_limit_ticks) {
          atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_TIMEOUT));
          res = -1;
        }
        s_res[phase & 1] = res;
      }
      __syncthreads();
      const int res_all = s_res[phase & 1];
      ++phase;
      if (res_all < 0) return;
      __builtin_amdgcn_s_sleep(2);
    } else {
      last_progress = wall_clock64();
    }
  }
  if (p.rank_die && tid == 0) rank_die_leave(p, rank_die_found, rank_die_base);
}

// The same interpreter for workgroups of ONE wavefront that run ONE fiber (simple protocol): tile, step and
// sequence counters live in registers, waits and publishes are wavefront-level - the lanes poll, the wavefront
// waits for its own stores, lane 0 stores the flags - and there is no workgroup barrier and no state in LDS
// anywhere on the path of a hop.  This is the instantiation for latency-bound sizes, where a lane's share of a
// chunk is a few 128-bit accesses per thread.
//
// WM selects the protocol / payload path as for the general kernel: kSimple, kDie, or kLL - there a message needs
// no tail flag, no completion wait and no separate load of the payload, so a hop is one store and the polling
// load that finds it (the receiver's loads have completed when it has seen the flags, so the head flag needs no
// wait either).
constexpr int kWaveLdsInstrs = 64;
template <int DT, int COH, int WM>
__global__ void __launch_bounds__(64) gc3_interpreter_wave(KParams p) {
  constexpr bool DIE = WM == kDie, LL = WM == kLL;
  __shared__ uint32_t s_instr[kWaveLdsInstrs * 8];
  const uint32_t tid = threadIdx.x;
  const uint32_t slot = p.bin_major ? blockIdx.x % p.W_active : blockIdx.x / p.wgs_per_lane;
  const uint32_t bin = p.bin_major ? blockIdx.x / p.W_active : blockIdx.x % p.wgs_per_lane;
  const uint32_t sub = slot / p.W_active;
  const DWg hdr = p.wgs[(slot % p.W_active) * p.wgs_per_lane + bin];
  if (hdr.nfibers <= sub) return;                     // (the host launches this kernel only when nfibers <= nsplit)
  if (p.hold) {
    int ok = 1;
    if (tid == 0) ok = hold_wait(p) ? 1 : 0;
    if (!uni((uint32_t)ok)) return;
  }
  const uint32_t W = p.W, tile = p.tile_bytes;
  const DFiber f = p.fibers[hdr.fiber_begin + sub];
  const uint32_t fid = uni(f.fid), tb_ninstr = uni(f.ninstr), tb_instr_begin = uni(f.instr_begin);
  const int32_t send_conn = (int32_t)uni((uint32_t)f.send_conn), recv_conn = (int32_t)uni((uint32_t)f.recv_conn);
  const uint32_t tbi = fid / W, lane = fid % W;
  uint64_t* const my_sem = sem_of(p, tbi, lane);
  const uint32_t epoch = uni((uint32_t)load_flag(my_sem + 1));
  const uint64_t run_base = (uint64_t)(epoch + 1) << 32;
  uint64_t rank_die_found = 0;
  if (p.rank_die && tid == 0) rank_die_found = rank_die_enter(p, hdr.rank_first_tb, lane, run_base);
  const uint32_t recv_from_tb = uni(f.recv_from_tb);
  const uint64_t ll_start = LL ? uni64(ll_run_start(load_flag(my_sem + 3), p.ll_msgs)) : 0;
  const uint32_t ll_base = (uint32_t)ll_start;
  if (DIE && tid == 0) store_flag(my_sem + 2, run_base + this_die() + 1);
  unsigned char* bufs[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) bufs[k] = (unsigned char*)uni64((uint64_t)p.bufs[hdr.rank * 3 + k]);
  const bool instr_in_lds = tb_ninstr <= (uint32_t)kWaveLdsInstrs;
  if (instr_in_lds) {
    const uint32_t* gi = (const uint32_t*)(p.instrs + tb_instr_begin);
    for (uint32_t k = tid; k < tb_ninstr * 8; k += 64) s_instr[k] = gi[k];
    __syncthreads();                                   // one wavefront: only orders the LDS writes before the reads
  }
  const uint64_t off0 = lane_begin(p.chunk_bytes, lane, p.W_active);
  const uint64_t share = lane_begin(p.chunk_bytes, lane + 1, p.W_active) - off0;
  const uint32_t ntiles = (uint32_t)((share + tile - 1) / tile);
  uint64_t* const tail_send = send_conn >= 0 ? flag_of(p, send_conn, lane, 0) : nullptr;
  uint64_t* const head_send = send_conn >= 0 ? flag_of(p, send_conn, lane, 1) : nullptr;
  uint64_t* const tail_recv = recv_conn >= 0 ? flag_of(p, recv_conn, lane, 0) : nullptr;
  uint64_t* const head_recv = recv_conn >= 0 ? flag_of(p, recv_conn, lane, 1) : nullptr;
  unsigned char* const fifo_base = LL ? p.ll_fifo : p.fifo;
  const uint32_t unit_bytes = LL ? p.ll_unit_bytes : p.unit_bytes;
  const uint32_t send_count = uni(f.send_count), recv_count = uni(f.recv_count);
  const uint32_t sslot_bytes = send_count * unit_bytes, rslot_bytes = recv_count * unit_bytes;
  unsigned char* const fifo_send = send_conn >= 0
      ? fifo_base + ((uint64_t)uni(f.send_units_before) * W + (uint64_t)lane * send_count) * p.slots * unit_bytes : nullptr;
  unsigned char* const fifo_recv = recv_conn >= 0
      ? fifo_base + ((uint64_t)uni(f.recv_units_before) * W + (uint64_t)lane * recv_count) * p.slots * unit_bytes : nullptr;
  uint32_t send_seq = 0, recv_seq = 0, head_known = 0;

  for (uint32_t t = 0; t < ntiles; ++t) {               // tile loop outside, instruction loop inside
    const uint64_t toff = (uint64_t)t * tile;
    const uint32_t len = (uint32_t)(share - toff < tile ? share - toff : tile);
    for (uint32_t s = 0; s < tb_ninstr; ++s) {
      DInstr ins;
      if (instr_in_lds) {
        const uint32_t* w = s_instr + s * 8;
        ins.op = uni(w[0]); ins.srcbuf = uni(w[1]); ins.dstbuf = uni(w[2]); ins.srcidx = uni(w[3]);
        ins.dstidx = uni(w[4]); ins.count = uni(w[5]); ins.dep_begin = uni(w[6]); ins.ndeps_hasdep = uni(w[7]);
      } else {
        ins = p.instrs[tb_instr_begin + s];
      }
      const uint32_t op = ins.op;
      const bool pops = op_pops(op), pushes = op_pushes(op);
      const uint32_t ndeps = ins.ndeps_hasdep >> 1;
      const bool hasdep = ins.ndeps_hasdep & 1;
      const bool wait_slot = pushes && send_seq >= head_known + p.slots;
      if ((pops && !LL) || wait_slot || ndeps) {
        uint64_t seen;
        const int res = poll_flags(p, tid, true, (pops && !LL) ? tail_recv : nullptr, run_base + recv_seq + 1,
                                   wait_slot ? head_send : nullptr, run_base + send_seq + 1 - p.slots,
                                   ins.dep_begin, ndeps, lane, run_base, t, seen);
        if (res < 0) return;                           // (the same value in every lane: decided by wavefront votes)
        if (wait_slot && ndeps <= 62) head_known = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(seen - run_base), 1);
        if (DIE && pops && recv_seq == 0) {
          // first message of this run on this connection: the sender published its die before the message
          uint32_t same = 1;
          if (tid == 0) {
            same = load_flag(sem_of(p, recv_from_tb, lane) + 2) == run_base + this_die() + 1 ? 1u : 0u;
            if (!same) atomicCAS(p.error, 0u, (uint32_t)(-GC3_ERR_PLACEMENT));
          }
          if (!uni(same)) return;
        }
      }
      const uint64_t coff = off0 + toff;
      unsigned char* const srcb = ins.srcbuf < 3 ? bufs[ins.srcbuf] + (uint64_t)ins.srcidx * p.chunk_bytes + coff : nullptr;
      unsigned char* const dstb = ins.dstbuf < 3 ? bufs[ins.dstbuf] + (uint64_t)ins.dstidx * p.chunk_bytes + coff : nullptr;
      unsigned char* const rslot = pops ? fifo_recv + (uint64_t)(recv_seq % p.slots) * rslot_bytes : nullptr;
      unsigned char* const sslot = pushes ? fifo_send + (uint64_t)(send_seq % p.slots) * sslot_bytes : nullptr;
      if (LL && (pops || pushes)) {
        constexpr int UL = COH == kCohDevice ? kUserLdCoh : kUserLd, US = COH == kCohDevice ? kUserStCoh : COH == kCohDie ? kUserStDie : kUserSt;
        const uint32_t ll_fin = ll_base + recv_seq + 1, ll_fout = ll_base + send_seq + 1, nvec = len >> 4;
        bool data_ok = true;
        for (uint32_t j = 0; j < ins.count; ++j) {
          const rsrc_t src = make_rsrc(srcb + (uint64_t)j * p.chunk_bytes, srcb ? len : 0);
          const rsrc_t dst = make_rsrc(dstb + (uint64_t)j * p.chunk_bytes, dstb ? len : 0);
          const rsrc_t rl = make_rsrc(rslot + (uint64_t)j * len * 2, rslot ? len * 2 : 0);
          const rsrc_t sl = make_rsrc(sslot + (uint64_t)j * len * 2, sslot ? len * 2 : 0);
          switch (op) {
            case GC3_OP_SEND: move_tile_ll<false, false, false, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            case GC3_OP_RECV: data_ok &= move_tile_ll<true, false, true, false, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            case GC3_OP_RRC:  data_ok &= move_tile_ll<true, true, true, false, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            case GC3_OP_RCS:  data_ok &= move_tile_ll<true, false, true, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            case GC3_OP_RRCS: data_ok &= move_tile_ll<true, true, true, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            case GC3_OP_RRS:  data_ok &= move_tile_ll<true, true, false, true, DT, UL, US>(rl, src, dst, sl, nvec, tid, 64, ll_fin, ll_fout, p); break;
            default: break;
          }
        }
        if (__any(!data_ok)) return;                     // a lane gave up waiting for data: the run is abandoned
      } else {
        move_simple<DT, COH, false, DIE>(op, ins.count, srcb, dstb, rslot, sslot, len, p.chunk_bytes, tid, 64, nullptr);
      }
      if (pushes) ++send_seq;
      if (pops) ++recv_seq;
      if (LL ? (pops || hasdep) : (pushes || pops || hasdep)) {
        // the wavefront's own device-scope stores have completed when its counter reaches zero; all of the
        // fiber's stores are this wavefront's, so nothing else has to be waited for before the flags.  (LL: only a
        // semaphore, which covers plain user-buffer stores, needs that.)
        if (!LL || hasdep) __builtin_amdgcn_s_waitcnt(0);
        if (tid == 0) {
          if (pushes && !LL) store_flag(tail_send, run_base + send_seq);
          if (pops && (recv_seq & p.head_mask) == 0) store_flag(head_recv, run_base + recv_seq);
          if (hasdep) store_flag(my_sem, run_base + (uint64_t)t * tb_ninstr + s + 1);
        }
      }
    }
  }
  if (tid == 0) {
    if (p.rank_die) rank_die_leave(p, rank_die_found, run_base);
    store_flag(my_sem + 1, (uint64_t)epoch + 1);   // this fiber has completed one more run
    if (LL) store_flag(my_sem + 3, ll_start + p.ll_msgs);
  }
}

// Host-callable launcher; returns the hipError_t of the launch.  `coherent_user`: 0 for programs without
// cross-thread-block dependencies, 1 with (user buffers at device scope), 2 with die-scope user buffers; `mode`: 0 simple, 1 LL, 2 simple with the
// FIFO payload staged through LDS, 3 the one-wavefront one-fiber interpreter (block must be 64), 4 the same under
// the LL protocol; `die_scope` (modes 0 and 3): FIFO payload kept in the L2 of the die both ends of a connection
// run on.
template <int DT>
static int launch_dt(int coh, int mode, bool die, unsigned grid, unsigned block, hipStream_t st, const KParams& p) {
#define GC3_LAUNCH(K) hipLaunchKernelGGL((K), dim3(grid), dim3(block), 0, st, p)
  if (die && mode != 0 && mode != 3) return (int)hipErrorInvalidValue;
  int variant = mode;                       // 0..3 as above, 4 die-scope general, 5 die-scope wavefront, 6 LL wavefront
  if (die) variant = mode == 3 ? 5 : 4;
  else if (mode == 4) variant = 6;
  switch (variant * 3 + coh) {
    case 0: GC3_LAUNCH((gc3_interpreter<DT, kCohNone, kSimple>)); break;
    case 1: GC3_LAUNCH((gc3_interpreter<DT, kCohDevice, kSimple>)); break;
    case 2: GC3_LAUNCH((gc3_interpreter<DT, kCohDie, kSimple>)); break;
    case 3: GC3_LAUNCH((gc3_interpreter<DT, kCohNone, kLL>)); break;
    case 4: GC3_LAUNCH((gc3_interpreter<DT, kCohDevice, kLL>)); break;
    case 5: GC3_LAUNCH((gc3_interpreter<DT, kCohDie, kLL>)); break;
    case 6: GC3_LAUNCH((gc3_interpreter<DT, kCohNone, kStaged>)); break;
    case 7: GC3_LAUNCH((gc3_interpreter<DT, kCohDevice, kStaged>)); break;
    case 8: GC3_LAUNCH((gc3_interpreter<DT, kCohDie, kStaged>)); break;
    case 9: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohNone, kSimple>)); break;
    case 10: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDevice, kSimple>)); break;
    case 11: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDie, kSimple>)); break;
    case 12: GC3_LAUNCH((gc3_interpreter<DT, kCohNone, kDie>)); break;
    case 13: GC3_LAUNCH((gc3_interpreter<DT, kCohDevice, kDie>)); break;
    case 14: GC3_LAUNCH((gc3_interpreter<DT, kCohDie, kDie>)); break;
    case 15: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohNone, kDie>)); break;
    case 16: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDevice, kDie>)); break;
    case 17: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDie, kDie>)); break;
    case 18: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohNone, kLL>)); break;
    case 19: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDevice, kLL>)); break;
    case 20: GC3_LAUNCH((gc3_interpreter_wave<DT, kCohDie, kLL>)); break;
    default: return (int)hipErrorInvalidValue;
  }
#undef GC3_LAUNCH
  return (int)hipGetLastError();
}

int launch_interpreter(int dtype, int coherent_user, int mode, bool die_scope, unsigned grid, unsigned block, void* stream,
                       const KParams& p) {
  if (coherent_user < kCohNone || coherent_user > kCohDie) return (int)hipErrorInvalidValue;
  hipStream_t st = (hipStream_t)stream;
  if ((mode == 3 || mode == 4) && block != 64) return (int)hipErrorInvalidValue;
  switch (dtype) {
    case GC3_F32: return launch_dt<GC3_F32>(coherent_user, mode, die_scope, grid, block, st, p);
    case GC3_F16: return launch_dt<GC3_F16>(coherent_user, mode, die_scope, grid, block, st, p);
    case GC3_BF16: return launch_dt<GC3_BF16>(coherent_user, mode, die_scope, grid, block, st, p);
    default: return (int)hipErrorInvalidValue;
  }
}

// Occupancy of the interpreter (workgroups of `block` threads per compute unit), minimum over the instantiations
// that a communicator of this kind may launch.  kind 0: simple and LL protocol through registers, device-scope
// FIFOs (and the wavefront-level kernel for 64 threads); 1: FIFO payload staged through LDS; 2: die-scope FIFOs
// (and, for runs that fall back to it, device scope).
int interpreter_occupancy(unsigned block, int kind, int* out) {
  int best = 1 << 30;
#define GC3_ALL_DT(K, C, M) (const void*)K<GC3_F32, C, M>, (const void*)K<GC3_F16, C, M>, (const void*)K<GC3_BF16, C, M>
  const void* plain[] = {GC3_ALL_DT(gc3_interpreter, kCohNone, kSimple), GC3_ALL_DT(gc3_interpreter, kCohDevice, kSimple),
                         GC3_ALL_DT(gc3_interpreter, kCohDie, kSimple), GC3_ALL_DT(gc3_interpreter, kCohNone, kLL),
                         GC3_ALL_DT(gc3_interpreter, kCohDevice, kLL), GC3_ALL_DT(gc3_interpreter, kCohDie, kLL)};
  const void* die[] = {GC3_ALL_DT(gc3_interpreter, kCohNone, kDie), GC3_ALL_DT(gc3_interpreter, kCohDevice, kDie),
                       GC3_ALL_DT(gc3_interpreter, kCohDie, kDie)};
  const void* with_stage[] = {GC3_ALL_DT(gc3_interpreter, kCohNone, kStaged), GC3_ALL_DT(gc3_interpreter, kCohDevice, kStaged),
                              GC3_ALL_DT(gc3_interpreter, kCohDie, kStaged)};
  const void* wave[] = {GC3_ALL_DT(gc3_interpreter_wave, kCohNone, kSimple), GC3_ALL_DT(gc3_interpreter_wave, kCohDevice, kSimple),
                        GC3_ALL_DT(gc3_interpreter_wave, kCohDie, kSimple)};
  const void* wave_ll[] = {GC3_ALL_DT(gc3_interpreter_wave, kCohNone, kLL), GC3_ALL_DT(gc3_interpreter_wave, kCohDevice, kLL),
                           GC3_ALL_DT(gc3_interpreter_wave, kCohDie, kLL)};
  const void* wave_die[] = {GC3_ALL_DT(gc3_interpreter_wave, kCohNone, kDie), GC3_ALL_DT(gc3_interpreter_wave, kCohDevice, kDie),
                            GC3_ALL_DT(gc3_interpreter_wave, kCohDie, kDie)};
#undef GC3_ALL_DT
  auto take = [&](const void* const* fns, int n) -> int {
    for (int i = 0; i < n; ++i) {
      int occ = 0;
      hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fns[i], (int)block, 0);
      if (e != hipSuccess) return (int)e;
      if (occ < best) best = occ;
    }
    return 0;
  };
  int e = kind == 1 ? take(with_stage, 9) : take(plain, 18);
  if (e == 0 && kind != 1 && block == 64) e = take(wave, 9);
  if (e == 0 && kind != 1 && block == 64) e = take(wave_ll, 9);
  if (e == 0 && kind == 2) e = take(die, 9);
  if (e == 0 && kind == 2 && block == 64) e = take(wave_die, 9);
  if (e != 0) return e;
  *out = best;
  return 0;
}

}  // namespace gc3

// ---- device memory for callers that cannot allocate ---------------------------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// stand-in for the symbol, not a device address: its address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to kernels and copies.
static __device__ __align__(256) unsigned char scratch[gc3::kStaticScratchBytes];

namespace gc3 {

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // per device, set once under the lock
std::mutex g_scratch_lock;

__global__ void __launch_bounds__(256) gc3_fill_zero(u32x4* dst, uint32_t nvec) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nvec) dst[i] = u32x4{0, 0, 0, 0};
}
}  // namespace

// Address of the current device's copy of the static scratch array (resolved on the first call per device).
int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!ptr) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

// Zero [ptr, ptr + bytes) with a kernel on `stream` (bytes a multiple of 16, ptr 16-byte aligned): a fill
// kernel, not a memset node, so that the call may be recorded into a graph.
int launch_fill_zero(void* ptr, size_t bytes, void* stream) {
  const uint32_t nvec = (uint32_t)(bytes >> 4);
  if (nvec == 0) return 0;
  hipLaunchKernelGGL(gc3_fill_zero, dim3((nvec + 255) / 256), dim3(256), 0, (hipStream_t)stream, (u32x4*)ptr, nvec);
  return (int)hipGetLastError();
}

}  // namespace gc3
