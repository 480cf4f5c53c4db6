"""Table sweeps: the same layers evaluated against a sequence of multiplier tables that arrive
from host memory, with the upload of the next tables overlapping the layers that run on the
current ones.

Evaluating many candidate approximate multipliers on one network is what the emulator is for
(paper, Sec. I and Sec. V).  A table is 128 KB; copied on the compute stream it would sit
between two layer calls.  Here the copies run on a second stream into one of two device staging
buffers, and events order them against the compute stream:

    upload stream :  wait(free[b])   copy tables of chunk c into staging[b]     record(ready[b])
    compute stream:  wait(ready[b])  prepare + run every layer on staging[b]    record(free[b])

with b = c mod 3, so the copy of chunk c + 1 proceeds while chunk c is being computed.  Three
staging buffers rather than two: the host, not the upload stream, waits for free[b] (see run), and
with three it waits for the chunk before the one the device is working on, so the device never
runs out of enqueued work while the host waits.  An
upload chunk holds several tables (eight by default) even when every layer call takes one table:
an event wait between two streams costs far more than the copy it orders (about 0.1 ms against
a few microseconds per table on this machine), so it is paid once per eight tables.  Only
stream plumbing happens here (torch provides streams, events and memory; both streams have the
default priority); preparing the tables and running the layers are the library's ax_layer_*
calls.  Host tables should be in page-locked memory (torch.Tensor.pin_memory() on a new
tensor), otherwise the copies are not asynchronous.
"""

from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as ax


class TableSweep:
    """layers: sequence of (desc, q, x, w) with desc an ax_conv_desc_t, q the quantization
    parameters, x / w device tensors.  chunk: tables per layer call (1 = one call per table and
    layer; more = the tiles of `chunk` tables share one grid).  tables_per_upload: tables per
    host-to-device copy and per pair of stream synchronizations (a multiple of chunk)."""

    NBUF = 3  # staging buffers

    def __init__(self, layers: Sequence, chunk: int = 1, tables_per_upload: Optional[int] = None, device="cuda"):
        self.layers = list(layers)
        self.chunk = int(chunk)
        self.per_upload = int(tables_per_upload) if tables_per_upload else max(self.chunk, 8)
        if self.per_upload % self.chunk:
            raise ValueError("tables_per_upload must be a multiple of chunk")
        self.device = torch.device(device)
        self.upload = torch.cuda.Stream(device=self.device)
        self._handles = {}   # (layer index, tables per call) -> AxLayer
        self._blocks = {}    # (layer index, tables per call, buffer) -> prepared block
        self._ws = {}        # (layer index, tables per call) -> workspace
        self.staging = [torch.empty((self.per_upload, 65536), dtype=torch.int16, device=self.device) for _ in range(self.NBUF)]
        self.ready = [torch.cuda.Event() for _ in range(self.NBUF)]
        self.free = [torch.cuda.Event() for _ in range(self.NBUF)]

    def _handle(self, li: int, n: int) -> ax.AxLayer:
        key = (li, n)
        if key not in self._handles:
            desc, q, _, _ = self.layers[li]
            h = ax.AxLayer(desc, q, num_luts=n)
            self._handles[key] = h
            for b in range(2):
                self._blocks[key + (b,)] = torch.empty(max(256, h.prepared_bytes), dtype=torch.uint8,
                                                       device=self.device)
            self._ws[key] = torch.empty(max(256, h.workspace_bytes), dtype=torch.uint8, device=self.device)
        return self._handles[key]

    def out_shape(self, li: int, num_tables: int):
        desc = self.layers[li][0]
        OH, OW = ax._out_hw(desc)
        return (num_tables, desc.N, OH, OW, desc.Cout)

    def run(self, host_tables: torch.Tensor, acc_out: Optional[List[torch.Tensor]] = None,
            y_out: Optional[List[torch.Tensor]] = None, overlap: bool = True):
        """host_tables: int16 / uint16 CPU tensor [T, 65536] (page-locked for asynchronous copies).
        acc_out / y_out: per layer a device tensor [T, N, OH, OW, Cout] (allocated when None; pass
        False to skip).  overlap=False enqueues the copies on the compute stream instead (the
        serialized form, for comparison).  Returns (acc_out, y_out).  The device is not waited for at
        the end, but with overlap the host paces itself: before it enqueues the copy of upload unit
        u it waits until unit u - 3 has finished on the device."""
        T = int(host_tables.shape[0])
        if host_tables.dim() != 2 or host_tables.shape[1] != 65536 or host_tables.dtype not in (torch.int16, torch.uint16):
            raise ValueError("host_tables must be a 16-bit integer tensor [T, 65536]")
        if host_tables.dtype == torch.uint16:
            host_tables = host_tables.view(torch.int16)
        L = len(self.layers)
        if acc_out is None:
            acc_out = [torch.empty(self.out_shape(li, T), dtype=torch.int32, device=self.device) for li in range(L)]
        if y_out is None:
            y_out = [torch.empty(self.out_shape(li, T), dtype=torch.float32, device=self.device) for li in range(L)]
        compute = torch.cuda.current_stream(self.device)
        units = [(t0, min(self.per_upload, T - t0)) for t0 in range(0, T, self.per_upload)]
        for _, nu in units:  # handles, blocks and workspaces exist before anything is enqueued
            for t in range(0, nu, self.chunk):
                for li in range(L):
                    self._handle(li, min(self.chunk, nu - t))

        def enqueue_upload(u):
            t0, n = units[u]
            b = u % self.NBUF
            if not overlap:
                self.staging[b][:n].copy_(host_tables[t0:t0 + n], non_blocking=True)
                return
            if u >= self.NBUF:
                # Unit u - 3 must have stopped reading this staging buffer.  The host waits for that
                # here rather than the upload stream on the device: a queue that sits blocked on an
                # event slows every kernel launch of the other queue (measured: 40 us per launch).
                # This copy is enqueued before the launches of unit u - 1, so the device is then
                # still working on unit u - 2 and has that unit's launches ahead of it.
                self.free[b].synchronize()
            with torch.cuda.stream(self.upload):
                self.staging[b][:n].copy_(host_tables[t0:t0 + n], non_blocking=True)
                self.ready[b].record(self.upload)

        if overlap:
            self.upload.wait_stream(compute)  # whatever filled or read the staging buffers before this call
            enqueue_upload(0)
        for u, (t0, nu) in enumerate(units):
            b = u % self.NBUF
            if overlap:
                if u + 1 < len(units):
                    enqueue_upload(u + 1)
                compute.wait_event(self.ready[b])
            else:
                enqueue_upload(u)
            for c, t in enumerate(range(0, nu, self.chunk)):
                n = min(self.chunk, nu - t)
                for li in range(L):
                    _, _, x, w = self.layers[li]
                    h = self._handle(li, n)
                    # two prepared blocks per layer, used in turn: preparing the next tables does
                    # not wait for anything but the stream's own order
                    h.prepare(w, self.staging[b][t:t + n], prepared=self._blocks[(li, n, c % 2)])
                    a = False if acc_out is False else acc_out[li][t0 + t:t0 + t + n]
                    y = False if y_out is False else y_out[li][t0 + t:t0 + t + n]
                    if n == 1:
                        a = a if a is False else a[0]
                        y = y if y is False else y[0]
                    h.run(x, a, y, workspace=self._ws[(li, n)])
            if overlap:
                self.free[b].record(compute)
        if overlap:
            compute.wait_stream(self.upload)
        return acc_out, y_out

    def close(self):
        for h in self._handles.values():
            h.close()
        self._handles.clear()
        self._blocks.clear()
        self._ws.clear()
