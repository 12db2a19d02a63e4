"""Device-memory plumbing around the C-ABI: PyTorch supplies buffers and streams, nothing else.

`Collective` owns one communicator and the per-rank device buffers (raw byte tensors) of one
workload; `run()` is a single gc3_comm_run on torch's current stream.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .inputs import ITEMSIZE, SENTINEL16, STORAGE


make_config = B.make_config


class Collective:
    def __init__(self, ir_text: str, dtype: str, elems_per_rank: int, cfg: Optional[B.CommConfig] = None,
                 device: str = "cuda:0", tune: bool = False, share_buffers_with: Optional["Collective"] = None):
        """`tune=True` lets gc3_comm_tune pick team width and workgroup target for this size first.
        `share_buffers_with`: use that object's input / output tensors (another program of the same collective on
        the same data, e.g. for a Selector) instead of allocating new ones; scratch is always this object's own."""
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the GC3 runtime has no CPU path")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.dtype = dtype
        self.code = B.DTYPE_CODE[dtype]
        self.elems = elems_per_rank
        prog = B.gc3_program_load(ir_text)
        try:
            self.pinfo = B.gc3_program_info_get(prog)
            self.scratch_chunks = [B.gc3_program_scratch_chunks(prog, r) for r in range(self.pinfo.ranks)]
            self.tune_report = None
            if tune and elems_per_rank:
                cfg, self.tune_report = B.gc3_comm_tune(prog, cfg, elems_per_rank, self.code,
                                                        torch.cuda.current_stream().cuda_stream)
            self.cfg = cfg
            self.comm = B.gc3_comm_create(prog, cfg)
        finally:
            B.gc3_program_free(prog)
        self.info = B.gc3_comm_info_get(self.comm)
        self.ranks = self.pinfo.ranks
        self.inplace = bool(self.pinfo.inplace)
        es = ITEMSIZE[dtype]
        if elems_per_rank % self.pinfo.in_chunks:
            raise ValueError("elems_per_rank must be a multiple of the program's chunk count")
        self.chunk_bytes = elems_per_rank // self.pinfo.in_chunks * es
        in_bytes = elems_per_rank * es
        out_bytes = self.chunk_bytes * self.pinfo.out_chunks
        alloc = lambda n: torch.empty(max(n, 16), dtype=torch.uint8, device=self.device)
        if share_buffers_with is not None:
            o = share_buffers_with
            if (o.ranks, o.inplace) != (self.ranks, self.inplace) or o.inputs[0].numel() < in_bytes \
                    or o.outputs[0].numel() < out_bytes:
                raise ValueError("cannot share buffers: different rank count / in-place kind, or buffers too small")
            self.inputs, self.outputs = o.inputs, o.outputs
        else:
            self.inputs = [alloc(in_bytes) for _ in range(self.ranks)]
            self.outputs = self.inputs if self.inplace else [alloc(out_bytes) for _ in range(self.ranks)]
        self.scratch = [alloc(self.scratch_chunks[r] * self.chunk_bytes) if self.scratch_chunks[r] else None
                        for r in range(self.ranks)]
        self.in_bytes, self.out_bytes = in_bytes, out_bytes
        for r in range(self.ranks):
            s = self.scratch[r]
            B.gc3_comm_bind(self.comm, r, self.inputs[r].data_ptr(),
                            None if self.inplace else self.outputs[r].data_ptr(),
                            s.data_ptr() if s is not None else None,
                            self.scratch_chunks[r] * self.chunk_bytes)
        self.algorithmic_bytes = (B.gc3_comm_algorithmic_bytes(self.comm, elems_per_rank, self.code)
                                  if elems_per_rank else 0)

    def resize(self, elems_per_rank: int) -> None:
        """Use a smaller element count on the same communicator and buffers."""
        es = ITEMSIZE[self.dtype]
        if elems_per_rank % self.pinfo.in_chunks:
            raise ValueError("elems_per_rank must be a multiple of the program's chunk count")
        cb = elems_per_rank // self.pinfo.in_chunks * es
        if elems_per_rank * es > self.inputs[0].numel() or cb * self.pinfo.out_chunks > self.outputs[0].numel():
            raise ValueError("larger than the buffers this object allocated")
        self.elems, self.chunk_bytes = elems_per_rank, cb
        self.in_bytes, self.out_bytes = elems_per_rank * es, cb * self.pinfo.out_chunks
        self.algorithmic_bytes = (B.gc3_comm_algorithmic_bytes(self.comm, elems_per_rank, self.code)
                                  if elems_per_rank else 0)

    # -- data movement between host arrays and the device buffers (not part of the collective) --
    def upload(self, inputs: Sequence[np.ndarray], outputs: Optional[Sequence[np.ndarray]] = None) -> None:
        for r in range(self.ranks):
            if self.in_bytes:
                self.inputs[r][:self.in_bytes].copy_(torch.from_numpy(inputs[r].view(np.uint8)))
            if outputs is not None and not self.inplace and self.out_bytes:
                self.outputs[r][:self.out_bytes].copy_(torch.from_numpy(outputs[r].view(np.uint8)))
        torch.cuda.synchronize()

    def fill_outputs_with_sentinel(self) -> None:
        if self.inplace:
            return
        for r in range(self.ranks):
            self.outputs[r].view(torch.int16).fill_(SENTINEL16)
        torch.cuda.synchronize()

    def download(self, which: str = "out") -> List[np.ndarray]:
        torch.cuda.synchronize()
        bufs, n = (self.outputs, self.out_bytes) if which == "out" else (self.inputs, self.in_bytes)
        st = STORAGE[self.dtype]
        return [b[:n].cpu().numpy().view(st).copy() for b in bufs]

    @property
    def launch(self) -> B.LaunchInfo:
        """What a run of the current size launches (grid, workgroup size, kernel variant ...)."""
        return B.gc3_comm_launch_info(self.comm, self.elems, self.code)

    def run(self) -> None:
        """One collective, asynchronous on torch's current stream."""
        B.gc3_comm_run(self.comm, self.elems, self.code, B.GC3_SUM, torch.cuda.current_stream().cuda_stream)

    def status(self) -> None:
        B.gc3_comm_status(self.comm)

    def reset(self) -> None:
        B.gc3_comm_reset(self.comm)

    def close(self) -> None:
        if getattr(self, "comm", None) is not None:
            B.gc3_comm_destroy(self.comm)
            self.comm = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Selector:
    """Several programs of one collective on the same per-rank buffers, each with the range of per-rank input
    sizes (bytes) it serves; run(elems) executes the first whose range holds the size (gc3_selector_run)."""

    def __init__(self, entries: Sequence[tuple], dtype: str, max_elems_per_rank: int, tune: bool = False,
                 device: str = "cuda:0"):
        """entries: (ir_text, min_bytes, max_bytes [, cfg]); max_bytes 0 = unbounded.  With `tune`, every entry is
        tuned at the largest size of its range (bounded by max_elems_per_rank)."""
        self.dtype = dtype
        self.code = B.DTYPE_CODE[dtype]
        es = ITEMSIZE[dtype]
        self.colls: List[Collective] = []
        self.sel = B.gc3_selector_create()
        first: Optional[Collective] = None
        for e in entries:
            text, lo, hi = e[0], e[1], e[2]
            cfg = e[3] if len(e) > 3 else None
            if tune:
                top = max_elems_per_rank if hi == 0 else min(max_elems_per_rank, hi // es)
                cfg = self._tuned_cfg(text, top, cfg)
            c = Collective(text, dtype, max_elems_per_rank, cfg, device, share_buffers_with=first)
            first = first or c
            self.colls.append(c)
            B.gc3_selector_add(self.sel, c.comm, lo, hi)
        self.inputs, self.outputs = first.inputs, first.outputs
        self.chosen = -1

    def _tuned_cfg(self, text: str, top_elems: int, cfg: Optional[B.CommConfig]) -> Optional[B.CommConfig]:
        prog = B.gc3_program_load(text)
        try:
            chunks = B.gc3_program_info_get(prog).in_chunks
            top_elems -= top_elems % chunks
            if top_elems <= 0:
                return cfg
            best, _ = B.gc3_comm_tune(prog, cfg, top_elems, self.code, torch.cuda.current_stream().cuda_stream)
            return best
        finally:
            B.gc3_program_free(prog)

    def run(self, elems_per_rank: int) -> int:
        self.chosen = B.gc3_selector_run(self.sel, elems_per_rank, self.code, B.GC3_SUM,
                                         torch.cuda.current_stream().cuda_stream)
        return self.chosen

    def status(self) -> None:
        for c in self.colls:
            c.status()

    def close(self) -> None:
        if getattr(self, "sel", None) is not None:
            B.gc3_selector_destroy(self.sel)
            self.sel = None
        for c in self.colls:
            c.close()
