"""ctypes binding of libgc3.so: the same entry points as include/gc3.h, argument marshalling only.

Every step of the collective runs inside the library's kernels.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# GC3_LIB_PATH selects another build of the same library (a tuning variant); there is no other path.
LIB_PATH = os.environ.get("GC3_LIB_PATH") or os.path.join(_HERE, "lib", "libgc3.so")

GC3_OK = 0
GC3_ERR_PARSE = -1
GC3_ERR_INVALID_PROGRAM = -2
GC3_ERR_DEADLOCK = -3
GC3_ERR_UNBOUND = -4
GC3_ERR_SIZE = -5
GC3_ERR_RESIDENCY = -6
GC3_ERR_TIMEOUT = -7
GC3_ERR_HIP = -8
GC3_ERR_ARG = -9
GC3_ERR_POISONED = -10
GC3_ERR_PLACEMENT = -11
FIFO_DEVICE, FIFO_DIE = 1, 2

GC3_F32, GC3_F16, GC3_BF16 = 0, 1, 2
GC3_SUM = 0
PROTO_PROGRAM, PROTO_SIMPLE, PROTO_LL, PROTO_AUTO = 0, 1, 2, 3
DTYPE_CODE = {"f32": GC3_F32, "f16": GC3_F16, "bf16": GC3_BF16}

EXPORTS = ("gc3_last_error", "gc3_program_load", "gc3_program_free", "gc3_program_validate",
           "gc3_program_info_get", "gc3_program_scratch_chunks", "gc3_program_plan", "gc3_comm_create", "gc3_comm_info_get",
           "gc3_comm_bind", "gc3_comm_launch_info", "gc3_comm_run", "gc3_comm_algorithmic_bytes", "gc3_comm_status",
           "gc3_comm_reset", "gc3_comm_destroy", "gc3_comm_tune", "gc3_run_static", "gc3_residency_plan",
           "gc3_selector_create", "gc3_selector_add", "gc3_selector_run", "gc3_selector_destroy")


class ProgramInfo(C.Structure):
    _fields_ = [("ranks", C.c_int32), ("in_chunks", C.c_int32), ("out_chunks", C.c_int32),
                ("inplace", C.c_int32), ("num_tbs", C.c_int32), ("max_tbs_per_rank", C.c_int32),
                ("num_connections", C.c_int32), ("num_instructions", C.c_int32), ("max_count", C.c_int32),
                ("max_scratch_chunks", C.c_int32), ("algorithmic_chunks", C.c_uint64)]


class CommConfig(C.Structure):
    _fields_ = [("fifo_slots", C.c_int32), ("tile_bytes", C.c_int32), ("team_width", C.c_int32),
                ("wg_size", C.c_int32), ("lds_stage", C.c_int32), ("target_wgs", C.c_int32),
                ("spin_limit_us", C.c_uint64), ("debug_hold", C.c_int32), ("min_lane_bytes", C.c_int32),
                ("protocol", C.c_int32), ("ll_max_lane_bytes", C.c_int32), ("fifo_scope", C.c_int32),
                ("user_scope", C.c_int32)]


def make_config(fifo_slots: int = 0, tile_bytes: int = 0, team_width: int = 0, wg_size: int = 0,
                spin_limit_us: int = 0, target_wgs: int = 0, debug_hold: int = 0,
                min_lane_bytes: int = 0, protocol: int = 0, ll_max_lane_bytes: int = 0, lds_stage: int = 0,
                fifo_scope: int = 0, user_scope: int = 0) -> CommConfig:
    """A gc3_comm_config; zero fields select the library's defaults."""
    return CommConfig(fifo_slots, tile_bytes, team_width, wg_size, lds_stage, target_wgs, spin_limit_us,
                      debug_hold, min_lane_bytes, protocol, ll_max_lane_bytes, fifo_scope, user_scope)


class CommInfo(C.Structure):
    _fields_ = [("team_width", C.c_int32), ("wg_size", C.c_int32), ("grid", C.c_int32),
                ("active_wgs", C.c_int32), ("max_resident_wgs", C.c_int32), ("fifo_slots", C.c_int32),
                ("tile_bytes", C.c_int32), ("slot_bytes", C.c_int32), ("fifo_bytes", C.c_uint64),
                ("compute_units", C.c_int32), ("max_fibers_per_wg", C.c_int32),
                ("wgs_per_lane", C.c_int32), ("protocol", C.c_int32), ("ll_fifo_bytes", C.c_uint64),
                ("head_stride", C.c_int32), ("user_scope", C.c_int32)]


GC3_TUNE_MAX_TRIED = 96


class LaunchInfo(C.Structure):
    _fields_ = [("grid", C.c_int32), ("wg_size", C.c_int32), ("active_lanes", C.c_int32), ("split", C.c_int32),
                ("tile_bytes", C.c_int32), ("kernel", C.c_int32), ("die_scope", C.c_int32), ("reserved", C.c_int32),
                ("lane_bytes", C.c_uint64)]


KERNEL_GENERAL, KERNEL_LL, KERNEL_STAGED, KERNEL_WAVE, KERNEL_WAVE_LL = 0, 1, 2, 3, 4


class InFlight(C.Structure):
    _fields_ = [("stream", C.c_uint64), ("wgs", C.c_int32), ("capacity", C.c_int32)]


class TuneEntry(C.Structure):
    _fields_ = [("team_width", C.c_int32), ("target_wgs", C.c_int32), ("grid", C.c_int32),
                ("active_wgs", C.c_int32), ("tile_bytes", C.c_int32), ("wg_size", C.c_int32), ("fifo_scope", C.c_int32),
                ("protocol", C.c_int32), ("min_lane_bytes", C.c_int32),
                ("fifo_slots", C.c_int32), ("user_scope", C.c_int32), ("reserved", C.c_int32), ("ms", C.c_double)]


class TuneReport(C.Structure):
    _fields_ = [("count", C.c_int32), ("best", C.c_int32), ("tried", TuneEntry * GC3_TUNE_MAX_TRIED)]


class Gc3Error(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gc3 status {status}: {message}")
        self.status = status
        self.message = message


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py build` "
                               "(or paper_2201_11840_amd.build.build()) first")
        L = C.CDLL(LIB_PATH)
        L.gc3_last_error.restype = C.c_char_p
        L.gc3_last_error.argtypes = []
        L.gc3_program_load.argtypes = [C.c_char_p, C.c_size_t, C.POINTER(C.c_void_p)]
        L.gc3_program_free.argtypes = [C.c_void_p]
        L.gc3_program_free.restype = None
        L.gc3_program_validate.argtypes = [C.c_void_p, C.c_int, C.c_char_p, C.c_size_t]
        L.gc3_program_info_get.argtypes = [C.c_void_p, C.POINTER(ProgramInfo)]
        L.gc3_program_scratch_chunks.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int)]
        L.gc3_program_plan.argtypes = [C.c_void_p, C.POINTER(CommConfig), C.c_int, C.c_int, C.POINTER(CommInfo)]
        L.gc3_comm_create.argtypes = [C.c_void_p, C.POINTER(CommConfig), C.POINTER(C.c_void_p)]
        L.gc3_comm_info_get.argtypes = [C.c_void_p, C.POINTER(CommInfo)]
        L.gc3_comm_bind.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
        L.gc3_comm_launch_info.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(LaunchInfo)]
        L.gc3_comm_run.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p]
        L.gc3_comm_algorithmic_bytes.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_uint64)]
        L.gc3_comm_status.argtypes = [C.c_void_p]
        L.gc3_comm_reset.argtypes = [C.c_void_p]
        L.gc3_comm_destroy.argtypes = [C.c_void_p]
        L.gc3_comm_destroy.restype = None
        L.gc3_comm_tune.argtypes = [C.c_void_p, C.POINTER(CommConfig), C.c_size_t, C.c_int, C.c_void_p,
                                    C.POINTER(CommConfig), C.POINTER(TuneReport)]
        L.gc3_run_static.argtypes = [C.c_void_p, C.POINTER(CommConfig), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                     C.POINTER(C.c_void_p), C.POINTER(C.c_size_t), C.c_size_t, C.c_int, C.c_int, C.c_void_p]
        L.gc3_residency_plan.argtypes = [C.POINTER(InFlight), C.c_int, C.c_uint64, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        L.gc3_selector_create.argtypes = [C.POINTER(C.c_void_p)]
        L.gc3_selector_add.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64]
        L.gc3_selector_run.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_int)]
        L.gc3_selector_destroy.argtypes = [C.c_void_p]
        L.gc3_selector_destroy.restype = None
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != GC3_OK:
        raise Gc3Error(status, gc3_last_error())


def gc3_last_error() -> str:
    return lib().gc3_last_error().decode()


def gc3_program_load(text: str) -> C.c_void_p:
    raw = text.encode()
    h = C.c_void_p()
    _check(lib().gc3_program_load(raw, len(raw), C.byref(h)))
    return h


def gc3_program_free(prog: C.c_void_p) -> None:
    lib().gc3_program_free(prog)


def gc3_program_validate(prog: C.c_void_p, fifo_slots: int) -> None:
    buf = C.create_string_buffer(512)
    _check(lib().gc3_program_validate(prog, fifo_slots, buf, len(buf)))


def gc3_program_info_get(prog: C.c_void_p) -> ProgramInfo:
    info = ProgramInfo()
    _check(lib().gc3_program_info_get(prog, C.byref(info)))
    return info


def gc3_program_scratch_chunks(prog: C.c_void_p, rank: int) -> int:
    n = C.c_int()
    _check(lib().gc3_program_scratch_chunks(prog, rank, C.byref(n)))
    return n.value


def gc3_program_plan(prog: C.c_void_p, cfg: Optional[CommConfig], compute_units: int, max_resident_wgs: int) -> CommInfo:
    info = CommInfo()
    _check(lib().gc3_program_plan(prog, C.byref(cfg) if cfg is not None else None, compute_units,
                                  max_resident_wgs, C.byref(info)))
    return info


def gc3_comm_create(prog: C.c_void_p, cfg: Optional[CommConfig] = None) -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().gc3_comm_create(prog, C.byref(cfg) if cfg is not None else None, C.byref(h)))
    return h


def gc3_comm_info_get(comm: C.c_void_p) -> CommInfo:
    info = CommInfo()
    _check(lib().gc3_comm_info_get(comm, C.byref(info)))
    return info


def gc3_comm_bind(comm: C.c_void_p, rank: int, input_ptr: int, output_ptr: Optional[int],
                  scratch_ptr: Optional[int], scratch_bytes: int) -> None:
    _check(lib().gc3_comm_bind(comm, rank, C.c_void_p(input_ptr), C.c_void_p(output_ptr or 0),
                               C.c_void_p(scratch_ptr or 0), scratch_bytes))


def gc3_comm_launch_info(comm: C.c_void_p, elems_per_rank: int, dtype: int) -> LaunchInfo:
    info = LaunchInfo()
    _check(lib().gc3_comm_launch_info(comm, elems_per_rank, dtype, C.byref(info)))
    return info


def gc3_comm_run(comm: C.c_void_p, elems_per_rank: int, dtype: int, op: int = GC3_SUM, stream: int = 0) -> None:
    _check(lib().gc3_comm_run(comm, elems_per_rank, dtype, op, C.c_void_p(stream)))


def gc3_comm_algorithmic_bytes(comm: C.c_void_p, elems_per_rank: int, dtype: int) -> int:
    n = C.c_uint64()
    _check(lib().gc3_comm_algorithmic_bytes(comm, elems_per_rank, dtype, C.byref(n)))
    return n.value


def gc3_comm_status(comm: C.c_void_p) -> None:
    _check(lib().gc3_comm_status(comm))


def gc3_comm_reset(comm: C.c_void_p) -> None:
    _check(lib().gc3_comm_reset(comm))


def gc3_comm_destroy(comm: C.c_void_p) -> None:
    lib().gc3_comm_destroy(comm)


def gc3_comm_tune(prog: C.c_void_p, base: Optional[CommConfig], elems_per_rank: int, dtype: int,
                  stream: int = 0) -> Tuple[CommConfig, TuneReport]:
    best, report = CommConfig(), TuneReport()
    _check(lib().gc3_comm_tune(prog, C.byref(base) if base is not None else None, elems_per_rank, dtype,
                               C.c_void_p(stream), C.byref(best), C.byref(report)))
    return best, report


def gc3_run_static(prog: C.c_void_p, cfg: Optional[CommConfig], inputs, outputs, scratch, scratch_bytes,
                   elems_per_rank: int, dtype: int, op: int = GC3_SUM, stream: int = 0) -> None:
    """inputs / outputs / scratch: sequences of device addresses (ints; None entries = null), outputs and scratch
    may be None; scratch_bytes: sequence of capacities or None."""
    n = len(inputs)
    ptrs = lambda seq: None if seq is None else (C.c_void_p * n)(*[C.c_void_p(a or 0) for a in seq])
    sizes = None if scratch_bytes is None else (C.c_size_t * n)(*scratch_bytes)
    _check(lib().gc3_run_static(prog, C.byref(cfg) if cfg is not None else None, ptrs(inputs), ptrs(outputs),
                                ptrs(scratch), sizes, elems_per_rank, dtype, op, C.c_void_p(stream)))


def gc3_residency_plan(inflight, stream: int, wgs: int, capacity: int):
    """inflight: sequence of (stream, wgs, capacity), oldest first.  Returns the list of 0/1 marks."""
    n = len(inflight)
    arr = (InFlight * max(n, 1))(*[InFlight(*e) for e in inflight])
    marks = (C.c_int32 * max(n, 1))()
    rc = lib().gc3_residency_plan(arr, n, stream, wgs, capacity, marks)
    if rc < 0:
        raise Gc3Error(rc, gc3_last_error())
    return list(marks)[:n]


def gc3_selector_create() -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().gc3_selector_create(C.byref(h)))
    return h


def gc3_selector_add(sel: C.c_void_p, comm: C.c_void_p, min_bytes: int, max_bytes: int) -> None:
    _check(lib().gc3_selector_add(sel, comm, min_bytes, max_bytes))


def gc3_selector_run(sel: C.c_void_p, elems_per_rank: int, dtype: int, op: int = GC3_SUM, stream: int = 0) -> int:
    chosen = C.c_int(-1)
    _check(lib().gc3_selector_run(sel, elems_per_rank, dtype, op, C.c_void_p(stream), C.byref(chosen)))
    return chosen.value


def gc3_selector_destroy(sel: C.c_void_p) -> None:
    lib().gc3_selector_destroy(sel)
