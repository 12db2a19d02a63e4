/*
 * gc3.h - C ABI of the MI355X (gfx950) runtime that executes GC3-IR collective programs.
 *
 * The library implements the runtime of the paper's Section 6: programs in GC3-IR (Section 5,
 * "GC3-IR": GPU programs -> thread blocks -> sequential instruction lists, one send and one
 * receive connection per thread block, identified with a channel) are parsed and stored in GPU
 * memory, their point-to-point connections (Section 6.1: remote buffers of s FIFO slots) are set
 * up, and a collective is executed by one interpreter kernel (Section 6.2) in which every thread
 * block walks its own instruction list tile by tile.
 *
 * The R ranks of a program are VIRTUAL ranks: disjoint buffers in the memory of one GPU.  A
 * connection is a FIFO in that GPU's memory guarded by flags; no second GPU and no collective
 * library is involved.
 *
 * Conventions
 *  - Every function returns a gc3_status (0 = success, negative = error) unless stated
 *    otherwise; nothing throws across this boundary.  gc3_last_error() gives a message for the
 *    last failure on the calling thread.
 *  - "host" / "device" says where a pointer must point.  The library never takes ownership of a
 *    caller's buffer; objects it returns (gc3_program, gc3_comm) are owned by the library and
 *    released with the matching free / destroy call.
 *  - Calls on one gc3_comm must not overlap in time (from several threads or streams): the
 *    FIFOs, flags and semaphores of a communicator are shared by its runs.
 *  - Runs of DIFFERENT communicators may be launched on different streams.  All workgroups of a run
 *    wait on each other, so every grid in flight has to be resident at once (Section 6.2); the
 *    library keeps a per-device ledger of the runs it launched and makes a new run's stream wait
 *    for earlier runs on other streams when they would not fit the device together (see
 *    gc3_residency_plan for the rule).  The ledger sees only launches made through gc3_comm_run
 *    outside stream capture: kernels of other libraries that fill the device for longer than the
 *    spin limit, and replays of captured launches, are the caller's to keep apart.
 */
#ifndef GC3_H
#define GC3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gc3_program gc3_program;
typedef struct gc3_comm gc3_comm;

typedef enum gc3_status {
  GC3_OK = 0,
  GC3_ERR_PARSE = -1,            /* text is not well-formed GC3-IR */
  GC3_ERR_INVALID_PROGRAM = -2,  /* structurally invalid (see gc3_program_validate) */
  GC3_ERR_DEADLOCK = -3,         /* cannot complete with the given number of FIFO slots */
  GC3_ERR_UNBOUND = -4,          /* a rank has no buffers bound */
  GC3_ERR_SIZE = -5,             /* element count / chunk size / scratch size not acceptable */
  GC3_ERR_RESIDENCY = -6,        /* the grid cannot be co-resident on the device */
  GC3_ERR_TIMEOUT = -7,          /* a wait inside the kernel exceeded the spin limit */
  GC3_ERR_HIP = -8,              /* a HIP runtime call failed */
  GC3_ERR_ARG = -9,              /* bad argument (null pointer, out-of-range value) */
  GC3_ERR_POISONED = -10,        /* communicator had a failed run; call gc3_comm_reset */
  GC3_ERR_PLACEMENT = -11        /* die-scope FIFOs: the two ends of a connection did not run on one die */
} gc3_status;

typedef enum gc3_dtype { GC3_F32 = 0, GC3_F16 = 1, GC3_BF16 = 2 } gc3_dtype;

/* The paper's reduction is element-wise and addition is the only operator it names (Section 3.1);
 * only the sum is built. */
typedef enum gc3_redop { GC3_SUM = 0 } gc3_redop;

/* Opcodes of Section 4.2 (instruction generation and fusion). */
typedef enum gc3_opcode {
  GC3_OP_SEND = 0, GC3_OP_RECV = 1, GC3_OP_COPY = 2, GC3_OP_REDUCE = 3,
  GC3_OP_RRC = 4, GC3_OP_RCS = 5, GC3_OP_RRCS = 6, GC3_OP_RRS = 7
} gc3_opcode;

typedef struct gc3_program_info {
  int32_t ranks;
  int32_t in_chunks;          /* chunks per rank in the input buffer */
  int32_t out_chunks;         /* chunks per rank in the output buffer */
  int32_t inplace;            /* 1: output aliases input (Section 3.2) */
  int32_t num_tbs;            /* thread blocks, all ranks */
  int32_t max_tbs_per_rank;
  int32_t num_connections;    /* distinct (source rank, destination rank, channel) */
  int32_t num_instructions;
  int32_t max_count;          /* largest `count` of any instruction (aggregation, Section 5.1) */
  int32_t max_scratch_chunks; /* largest scratch chunk count of any rank */
  uint64_t algorithmic_chunks;/* global-memory traffic of one run in units of one chunk:
                                 count x (send 2, recv 2, copy 2, reduce 3, rrc 3, rcs 3, rrcs 4, rrs 3) */
} gc3_program_info;

/* Tunables of a communicator.  Zero in any field selects the default. */
typedef struct gc3_comm_config {
  int32_t fifo_slots;      /* s of Section 6.1, 1..8; default 2 (with 4 or more a receiver may announce freed slots
                              less often than after every message, see gc3_comm_info.head_stride) */
  int32_t tile_bytes;      /* largest number of bytes of one chunk a workgroup moves per tile (Section 6.2,
                              chunk tiling); multiple of 16, at most 1 MiB; default 65536, halved (not
                              below 16384) while all FIFOs together exceed 256 MiB.  A FIFO slot of a
                              connection holds tile_bytes x the largest `count` of the instructions that use
                              that connection.  A run tiles with about half a lane's share of a
                              chunk, at least 16 KiB and at most this. */
  int32_t team_width;      /* W: lanes per IR thread block; lane w owns the w-th 1/W of every chunk and
                              has FIFO slots, flags and a semaphore of its own (the runtime applying
                              Section 5.1's parallelize(W)).  Lightly loaded thread blocks of one
                              rank may share a workgroup (not with 64-thread workgroups when thread
                              blocks x W stays within target_wgs: every lane then has a workgroup of its
                              own).  0 = choose W and the sharing so that the heaviest workgroup is
                              lightest */
  int32_t wg_size;         /* threads per workgroup: 64, 128, 256 or 512; default 256.  A run whose lanes get
                              at most 8 KiB of a chunk launches fewer: 64 when every workgroup executes a
                              single thread-block lane, else at most 128.  Workgroups of 64 threads with a
                              single thread-block lane each run the wavefront-level interpreter (under either
                              protocol): no workgroup barrier and no LDS state on the path of a hop */
  int32_t lds_stage;       /* 1 = the receiving instructions (recv, rrc, rcs, rrcs, rrs) bring the FIFO payload into LDS
                              with direct-to-LDS 128-bit loads and read it back from there, so loads in flight
                              hold no registers; 0 (default) = through registers.  Same results; on MI355X the
                              register path is as fast or faster, the option exists for measurement */
  int32_t target_wgs;      /* workgroups the schedule aims at (never more than can be resident);
                              0 = four per compute unit */
  uint64_t spin_limit_us;  /* longest a workgroup waits on one flag before the run is abandoned
                              with GC3_ERR_TIMEOUT; default 10 s */
  int32_t debug_hold;      /* test facility for the failure path: 1 = every workgroup first waits for a
                              start word that nobody sets, so each run ends, after spin_limit_us, with
                              GC3_ERR_TIMEOUT and all workgroups leaving through the error path */
  int32_t min_lane_bytes;  /* a run splits a chunk over at most chunk bytes / min_lane_bytes lanes (at least
                              one): small chunks are not worth spreading; multiple of 16.  0 = automatic: 8192, or
                              4096 for runs of the wavefront-level interpreter.  The workgroups of
                              the lanes left without bytes then share the thread blocks of the active ones */
  int32_t protocol;        /* Section 6.1 "Protocols".  0 = what the program's `protocol` line says:
                              `simple` (payload, then a separate flag), `ll` (every 8 bytes carry 4 bytes of
                              data and a 4-byte flag: lowest latency, half the bandwidth) or `auto` (LL when
                              a lane's share of a chunk is at most ll_max_lane_bytes); 1 = force simple,
                              2 = force LL, 3 = force auto */
  int32_t ll_max_lane_bytes; /* `auto` switches to LL up to this many bytes per lane and chunk; also the LL
                              tile size; multiple of 16, at most 65536; default 8192 */
  int32_t fifo_scope;      /* where FIFO payload lives (Section 6.1: the remote buffer of a connection).
                              0 or 1 = device scope: slots are written through to the memory system and read from
                              there, valid wherever the two ends of a connection run.
                              2 = die scope: consecutive workgroups run on consecutive dies (XCDs) round-robin,
                              so a run whose number of active lanes is a multiple of 8 is launched bin-major
                              (workgroup = bin x active lanes + lane): lane w of every thread block then runs on die
                              w mod 8, both ends of every connection share a die, and the payload is read from
                              that die's L2 (plain stores, loads that bypass the compute unit's L1) instead of
                              from the memory system.  It pays while the slots of a die fit its 4 MiB L2, so the
                              slot tile defaults to the largest of 64 ... 4 KiB with which all FIFOs together stay
                              within 16 MiB.  Simple protocol only; runs with another number of active lanes, or
                              that split fiber lists over idle lanes' workgroups (small chunks), use device scope.
                              Every receiver checks at run time that it shares its sender's die and abandons the
                              run with GC3_ERR_PLACEMENT otherwise */
  int32_t user_scope;      /* how thread blocks of one rank see each other's writes to the rank's buffers (Section 5.2:
                              the dependencies between thread blocks of a GPU).  0 or 1 = device scope: in programs
                              with such dependencies every access to a user buffer bypasses the dies' L2s.
                              2 = die scope: the workgroups of rank r all run on die r mod 8 (the plan orders its
                              workgroups so that workgroup index mod 8 = rank mod 8, padding with empty workgroups
                              where ranks have unequal numbers of them or the rank count is no multiple of 8), so
                              the thread blocks of a rank meet in one L2: reads are served from it (loads that
                              bypass only the compute unit's L1, plain stores).  A chain of dependent
                              instructions gets shorter by a trip to memory per link (All Pairs AllReduce, 8 ranks,
                              4 - 256 KiB: 21 - 24 -> 17 - 19 us back to back on MI355X).  Together with
                              fifo_scope 2 the lanes are placed on dies instead (lane w of every thread block of
                              every rank on die w mod 8, which serves both), in the runs that use die-scope FIFOs;
                              the others use device scope for both.  Every workgroup checks at
                              run time that its rank's workgroups share a die; a run where they do not ends with
                              GC3_ERR_PLACEMENT and its results are not to be used */
} gc3_comm_config;

typedef struct gc3_comm_info {
  int32_t team_width;        /* W in use */
  int32_t wg_size;
  int32_t grid;              /* workgroups of a run that uses all lanes: team_width x wgs_per_lane */
  int32_t active_wgs;        /* workgroups that execute at least one thread-block lane */
  int32_t max_resident_wgs;  /* occupancy x compute units */
  int32_t fifo_slots;
  int32_t tile_bytes;
  int32_t slot_bytes;        /* the largest slot: max_count x tile_bytes (a connection's slots are sized for the
                                largest `count` among its own instructions) */
  uint64_t fifo_bytes;       /* device memory held by all FIFOs */
  int32_t compute_units;
  int32_t max_fibers_per_wg; /* most thread-block lanes multiplexed by one workgroup (1 = none shared) */
  int32_t wgs_per_lane;      /* a run launches active lanes x split x wgs_per_lane workgroups: on small chunks only
                                some lanes own bytes, and the fiber lists are then dealt to up to
                                team_width / active lanes workgroups each (split) */
  int32_t protocol;          /* 1 simple, 2 LL, 3 auto (after applying the configuration's override) */
  uint64_t ll_fifo_bytes;    /* device memory held by the LL slots */
  int32_t head_stride;       /* a receiver announces freed slots after every head_stride-th message it has taken: 1, or
                                - with 4 or more slots - 2 (4 with 8 slots) when the program is also free of
                                deadlock with fifo_slots - head_stride + 1 slots, which is what a sender can then
                                count on (Section 6.1: a sender may be up to s messages ahead) */
  int32_t user_scope;        /* 1 device, 2 die (see gc3_comm_config) */
} gc3_comm_info;

/* Message for the most recent error on this thread.  host; owned by the library; never null. */
const char* gc3_last_error(void);

/* ---- programs (Section 5, GC3-IR; Section 6.2 "Initial Setup": programs are parsed at init) ---- */

/* Parse GC3-IR text (`text`: host, `len` bytes, need not be NUL-terminated).  On success *out is
 * a new program.  The text format is line oriented:
 *   gc3ir 1 / name T / collective T / inplace 0|1 / protocol simple|ll|ll128|auto / ranks R / chunks IN OUT
 *   rank r scratch N tbs K            (ranks in order)
 *   tb id send P recv Q chan C ops n  (ids in order; -1 = no peer)
 *   op OPCODE SRCBUF SRCIDX DSTBUF DSTIDX COUNT HASDEP NDEPS {TB STEP}...
 *   end
 * with OPCODE in send recv copy reduce rrc rcs rrcs rrs and buffers i, o, s or - (unused).
 * Errors: GC3_ERR_PARSE, GC3_ERR_ARG. */
int gc3_program_load(const char* text, size_t len, gc3_program** out);

void gc3_program_free(gc3_program* prog);

/* Check the constraints the paper's compiler guarantees (Section 5 and 5.2): peers in range,
 * every send-type instruction in a thread block with a send peer (same for receive), one sending
 * and one receiving thread block per connection, matching message sizes on both ends of a
 * connection, chunk indices inside the buffers, dependencies on existing steps of the same rank
 * whose has-dependent flag is set; then execute the program with `fifo_slots` slots per
 * connection (Section 6.1) to prove it terminates.  `err`/`errlen`: optional host buffer for a
 * message.  Errors: GC3_ERR_INVALID_PROGRAM, GC3_ERR_DEADLOCK, GC3_ERR_ARG. */
int gc3_program_validate(const gc3_program* prog, int fifo_slots, char* err, size_t errlen);

/* Shape of a parsed program (Section 3.1: number of ranks and chunks per buffer are fixed by the program, the
 * buffer size is not; Section 5: thread blocks, connections, instructions).  Errors: GC3_ERR_ARG. */
int gc3_program_info_get(const gc3_program* prog, gc3_program_info* out);

/* Scratch chunks rank `rank` needs (Section 3.2: deduced from the highest index used). */
int gc3_program_scratch_chunks(const gc3_program* prog, int rank, int* out);

/* ---- communicators (Section 6.1 connections, Section 6.2 interpreter) ---- */

/* Validate `prog`, allocate its connections' FIFOs, flags and the thread-block semaphores in
 * device memory of the current HIP device, upload the instruction tables and check that all
 * workgroups can be resident at once (Section 6.2: all thread blocks must run concurrently).
 * `cfg` may be null (defaults).  The program may be freed afterwards.
 * Errors: validation errors, GC3_ERR_RESIDENCY, GC3_ERR_HIP, GC3_ERR_ARG. */
int gc3_comm_create(const gc3_program* prog, const gc3_comm_config* cfg, gc3_comm** out);

/* The plan in use: team width, grid, tile and slot sizes, FIFO memory (Section 6.1: b and s are properties of the
 * connection set-up).  Errors: GC3_ERR_ARG. */
int gc3_comm_info_get(const gc3_comm* comm, gc3_comm_info* out);

/* What gc3_comm_tune tried. */
#define GC3_TUNE_MAX_TRIED 96
typedef struct gc3_tune_entry {
  int32_t team_width;      /* W of the plan */
  int32_t target_wgs;      /* as passed to the planner (0 = default) */
  int32_t grid;            /* workgroups of the plan */
  int32_t active_wgs;      /* of them, workgroups that hold work */
  int32_t tile_bytes;      /* slot tile of the plan */
  int32_t wg_size;         /* threads per workgroup */
  int32_t fifo_scope;      /* 1 device, 2 die */
  int32_t protocol;        /* 1 simple, 2 LL, 3 chosen per run */
  int32_t min_lane_bytes;  /* as passed to the planner (0 = chosen per run) */
  int32_t fifo_slots;      /* s of the plan */
  int32_t user_scope;      /* 1 device, 2 die */
  int32_t reserved;
  double ms;               /* mean duration of one run */
} gc3_tune_entry;
typedef struct gc3_tune_report {
  int32_t count;           /* entries filled */
  int32_t best;            /* index of the fastest */
  gc3_tune_entry tried[GC3_TUNE_MAX_TRIED];
} gc3_tune_report;

/* Pick team width and workgroup target for `prog` at one buffer size by measurement (Section 7: the
 * parallelization of every algorithm is tuned for the system and the buffer size; this does it for the
 * parallelization the runtime applies).  For the configuration in `base` (may be null) and for team
 * widths 4..64 x workgroup targets {default, 512, 768}, then for the fastest of them the slot tiles 16, 32
 * and 64 KiB, then workgroups of 128 threads (the winner's plan; team widths 64 and 128 with as many workgroups as
 * the device holds and a 16 KiB tile), then workgroups of one wavefront (64 threads) with team widths
 * 16..64 (and the widest with which no two thread blocks share a workgroup) x workgroup targets {2048, 4096} and
 * again the slot tiles, then die-scope FIFOs with 64, 128 and 256
 * threads x team widths 8..64 and their slot tiles, then - when the fastest run so far takes under 0.1 ms and `base`
 * leaves the protocol to the program - the LL protocol (Section 6.1) with workgroups of one wavefront, team widths
 * 16 and 64, lane shares of at least 4 KiB or 1 KiB and the default number of slots or 8, then - for programs with
 * dependencies between thread blocks - die-scope user buffers for the plan chosen so far, for 64 and 128 lanes of
 * 128-thread workgroups and for 16 and 64 lanes of one-wavefront workgroups - only over fields `base` leaves 0 - it creates
 * a communicator on the current device, binds stand-in buffers of the real sizes (non-zero filler) that it
 * allocates and frees itself, times 5 runs after 2 warm-up runs (8 for the first plan) on `hip_stream` - back to back
 * when all inputs together are under 32 MiB, else each run on its own after a fill of the input buffers, so that a run
 * finds freshly written inputs as it does in use -, and writes the
 * chosen configuration to `*best` (ready for gc3_comm_create): the fastest one if it beats `base`,
 * which is timed first (report entry 0), by more than 2 %, else `base`.  `report` may be null.
 * Synchronises the device.  Plans that do not fit the device are skipped.
 * Errors: GC3_ERR_SIZE (size not a multiple of the chunk count / 16 bytes, or zero), validation errors,
 * GC3_ERR_TIMEOUT or GC3_ERR_HIP from a tuning run, GC3_ERR_ARG. */
int gc3_comm_tune(const gc3_program* prog, const gc3_comm_config* base, size_t elems_per_rank, gc3_dtype dtype,
                  void* hip_stream, gc3_comm_config* best, gc3_tune_report* report);

/* The plan gc3_comm_create would make for `prog` on a device with `compute_units` compute units that
 * holds `max_resident_wgs` workgroups of cfg->wg_size threads at once, without touching any device
 * (host only): team width, grid, sharing of workgroups, FIFO memory (Section 6.2, "Initial Setup":
 * an IR must fit the device).  Errors: as gc3_comm_create, except GC3_ERR_HIP. */
int gc3_program_plan(const gc3_program* prog, const gc3_comm_config* cfg, int compute_units,
                     int max_resident_wgs, gc3_comm_info* out);

/* Bind the three named buffers of one rank (Section 3.1): device pointers, 16-byte aligned,
 * owned by the caller and alive for every later run.  For an in-place program `output` must be
 * null or equal `input`.  `scratch` may be null iff the rank uses no scratch chunk;
 * `scratch_bytes` is its capacity, checked against the run's chunk size.  The device-side pointer table is
 * updated before the call returns (a small synchronous copy, after waiting for this communicator's last run),
 * so binding is set-up work: not for use under stream capture.
 * Errors: GC3_ERR_ARG, GC3_ERR_HIP. */
int gc3_comm_bind(gc3_comm* comm, int rank, void* input, void* output, void* scratch, size_t scratch_bytes);

/* What gc3_comm_run launches for one size (host only). */
typedef struct gc3_launch_info {
  int32_t grid;           /* workgroups (0 = nothing is launched) */
  int32_t wg_size;        /* threads per workgroup of this run */
  int32_t active_lanes;   /* lanes that own bytes: min(team width, chunk bytes / min_lane_bytes), at least 1 */
  int32_t split;          /* workgroups that share the fiber list of one (lane, bin) of the plan */
  int32_t tile_bytes;     /* bytes of one chunk a fiber moves per tile in this run */
  int32_t kernel;         /* 0 general interpreter, 1 LL protocol, 2 FIFO payload staged through LDS,
                             3 wavefront-level interpreter (one wavefront, one thread-block lane per workgroup),
                             4 wavefront-level interpreter under the LL protocol */
  int32_t die_scope;      /* 1 = this run reads FIFO payload from the dies' L2s (fifo_scope 2, active lanes a
                             multiple of 8, no split) and is launched bin-major */
  int32_t reserved;
  uint64_t lane_bytes;    /* largest share a lane has of one chunk */
} gc3_launch_info;

/* The launch gc3_comm_run would make for `elems_per_rank` elements of `dtype`: how the runtime's own
 * parallelization (Section 5.1 applied by the runtime) and tiling (Section 6.2) turn out for this chunk size.
 * Touches no device.  Errors: GC3_ERR_SIZE, GC3_ERR_ARG. */
int gc3_comm_launch_info(const gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, gc3_launch_info* out);

/* Run the collective once, asynchronously on `hip_stream` (a hipStream_t, null = default stream): one launch
 * of the interpreter kernel (Section 6.2), in which every thread block executes its instruction list tile by
 * tile.  `elems_per_rank` is the element count of every rank's INPUT buffer; a chunk is
 * elems_per_rank / in_chunks elements (Section 3.1: the chunk size is known only at run time),
 * the output buffer holds out_chunks chunks.  The chunk must be a whole number of elements and
 * of 16-byte units.  elems_per_rank = 0 is a no-op.  Errors: GC3_ERR_UNBOUND, GC3_ERR_SIZE,
 * GC3_ERR_POISONED, GC3_ERR_HIP, GC3_ERR_ARG.  A GC3_ERR_TIMEOUT inside the kernel is reported by
 * gc3_comm_status.
 * Stream capture: the kernel's arguments depend only on the communicator, the size and the data type (the run
 * counters and the LL message numbers live in device memory), the call copies nothing and waits for nothing, so
 * under either protocol it may be recorded into a HIP graph and replayed any number of times, also interleaved
 * with eager runs of the same communicator (never overlapping them).  A communicator serves 2^32 - 1 runs between
 * resets.
 * The call records no event of its own (that costs a latency-bound collective several microseconds): the library
 * remembers `hip_stream` and records an event on it when the run has to be waited for - in gc3_comm_status,
 * gc3_comm_bind, gc3_comm_destroy, or when a run of another communicator must not overlap this one.  Keep the
 * stream alive until then; if it is gone, the whole device is waited for instead. */
int gc3_comm_run(gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, gc3_redop op, void* hip_stream);

/* Bytes the method itself loads and stores through global memory in one run of this size: the sum over all
 * instructions of count x chunk bytes x (send 2, recv 2, copy 2, reduce 3, rrc 3, rcs 3, rrcs 4, rrs 3) -
 * every instruction of Section 4.2 reads each of its operands once and writes each of its results once;
 * flags, semaphores and instruction fetches are not counted.  This is the numerator of the throughput the
 * benchmark reports.  Errors: GC3_ERR_SIZE, GC3_ERR_ARG. */
int gc3_comm_algorithmic_bytes(const gc3_comm* comm, size_t elems_per_rank, gc3_dtype dtype, uint64_t* out);

/* Wait for this communicator's last run launched outside stream capture (its completion event; no other stream
 * of the process is stalled) and report whether any run since the last reset was abandoned because a wait
 * inside the kernel - for a semaphore, a message or a free slot, Section 6.2 - exceeded the spin limit
 * (GC3_ERR_TIMEOUT; the communicator is then poisoned) or GC3_OK.  After replaying a captured run, synchronise
 * the stream it ran on first.  Errors: GC3_ERR_TIMEOUT, GC3_ERR_HIP, GC3_ERR_ARG. */
int gc3_comm_status(gc3_comm* comm);

/* Clear all flags, semaphores, run counters and the error state, as after the initial set-up of Section 6.2
 * (synchronises the device).  Errors: GC3_ERR_HIP, GC3_ERR_ARG. */
int gc3_comm_reset(gc3_comm* comm);

/* Wait for the communicator's last run launched outside capture and release its connections (FIFOs, flags),
 * semaphores and tables (the teardown of what Section 6.2's initial set-up created). */
void gc3_comm_destroy(gc3_comm* comm);

/* One run in flight, as the per-device ledger sees it. */
typedef struct gc3_inflight {
  uint64_t stream;    /* identity of the stream it was launched on */
  int32_t wgs;        /* workgroups of the run */
  int32_t capacity;   /* workgroups of that size the device holds at once */
} gc3_inflight;

/* The rule gc3_comm_run applies before a launch, as a host-only function (no device is touched): given the runs
 * in flight on a device, oldest first, and a new run of `wgs` workgroups (device capacity `capacity`) on
 * `stream`, set wait_on[i] = 1 for the runs the new run's stream must wait for and 0 for the others.  A run's
 * share of the device is wgs / capacity; runs on `stream` itself never overlap the new one; the oldest runs on
 * other streams are waited for until the shares of the rest plus the new run's are at most the whole device
 * (Section 6.2: all thread blocks of a program must be able to run concurrently).
 * Returns the number of runs to wait for (>= 0), or GC3_ERR_ARG. */
int gc3_residency_plan(const gc3_inflight* inflight, int n, uint64_t stream, int32_t wgs, int32_t capacity,
                       int32_t* wait_on);

/* For callers that cannot allocate device memory - code under HIP graph capture rules that forbid hipMalloc,
 * tight serving loops, harnesses that ban allocation: one complete run of `prog` without a communicator and
 * without any hipMalloc / hipFree.  Everything a communicator would allocate (flags, semaphores, instruction
 * tables, FIFOs) is laid out, for the duration of the call's kernels, in a static device array of
 * GC3_STATIC_SCRATCH_BYTES (64 MiB) that every GPU the library runs on holds until the process ends.
 *   inputs / outputs / scratch: host arrays of `ranks` device pointers (16-byte aligned, owned by the caller);
 *     `outputs` may be null for an in-place program (else outputs[r] must be null or equal inputs[r]);
 *     `scratch` / `scratch_bytes` (capacities) may be null when no rank uses scratch chunks.
 *   cfg: as for gc3_comm_create (null = defaults); the simple protocol only (protocol must be 0 or 1).  The
 *     slot tile defaults to the largest of 64 KiB ... 1 KiB with which the FIFOs fit.
 * The results are those of gc3_comm_run on the same program and buffers, bit for bit.
 * The call plans the program on the host, copies the tables (and waits for `hip_stream` once, because the host
 * copy dies with the call), clears flags and semaphores with a fill kernel and launches the interpreter, all on
 * `hip_stream`; it returns without waiting for the run.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (several streams or threads) race and are not allowed; calls on one stream are safe.
 * A run abandoned inside the kernel (spin limit) is reported by the NEXT call on that device, which returns
 * GC3_ERR_TIMEOUT without running.
 * Errors: GC3_ERR_SIZE when the program's state does not fit the static array (or the element count / scratch
 * capacity is unacceptable, as for gc3_comm_run), validation errors, GC3_ERR_RESIDENCY, GC3_ERR_ARG, GC3_ERR_HIP. */
#define GC3_STATIC_SCRATCH_BYTES (64u << 20)
int gc3_run_static(const gc3_program* prog, const gc3_comm_config* cfg, void* const* inputs, void* const* outputs,
                   void* const* scratch, const size_t* scratch_bytes, size_t elems_per_rank, gc3_dtype dtype,
                   gc3_redop op, void* hip_stream);

/* ---- selection by buffer size (Section 6, introduction) ---- */

/* A program may be fast only for a range of buffer sizes, so the paper's runtime picks the algorithm
 * from user-configured size ranges (and otherwise falls back to the vendor library, which does not exist
 * here: a size outside every range is an error).  A selector is an ordered list of (communicator, size
 * range) entries for one collective; it does not own the communicators, which must outlive it and have
 * their buffers bound by the caller. */
typedef struct gc3_selector gc3_selector;

int gc3_selector_create(gc3_selector** out);

/* Append an entry: `comm` serves runs whose per-rank INPUT size in bytes lies in [min_bytes, max_bytes]
 * (max_bytes = 0: no upper limit).  All entries must agree in the number of ranks and in being in place
 * or not.  Errors: GC3_ERR_ARG. */
int gc3_selector_add(gc3_selector* sel, gc3_comm* comm, uint64_t min_bytes, uint64_t max_bytes);

/* gc3_comm_run on the first entry whose range holds elems_per_rank x element size; `chosen` (may be null)
 * receives its index.  Errors: GC3_ERR_SIZE when no range matches, else those of gc3_comm_run. */
int gc3_selector_run(gc3_selector* sel, size_t elems_per_rank, gc3_dtype dtype, gc3_redop op, void* hip_stream,
                     int* chosen);

void gc3_selector_destroy(gc3_selector* sel);

#ifdef __cplusplus
}
#endif
#endif /* GC3_H */
