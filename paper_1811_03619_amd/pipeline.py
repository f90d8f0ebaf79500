"""Buffer plumbing for a simulated Pipe-SGD job on one GPU: allocates the p
workers' gradient, payload, model and momentum buffers with PyTorch and strings
the library calls together in the order of Algorithm 1 (arXiv 1811.03619).
No arithmetic happens in this file.

Iteration t (width K; K = 2 is the paper's optimal pipeline, K = 1 synchronous):
    A[t]  = AllReduce(g_local[t])              -> slot[t % K]
    w[t]  = Update(w[t-1], slot[(t-K+1) % K])     (slots start as zero)
The two calls touch disjoint buffers, which is what lets the paper overlap
them; here they are enqueued back to back on one stream.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B

_PAYLOAD_TORCH = {B.NONE: torch.float32, B.TRUNC16: torch.int16, B.QUANT8: torch.int8}
_PAYLOAD_NUMPY = {B.NONE: np.float32, B.TRUNC16: np.uint16, B.QUANT8: np.int8}


def payload_empty(mode: int, n: int, device) -> torch.Tensor:
    return torch.zeros(max(n, 1), dtype=_PAYLOAD_TORCH[mode], device=device)[:n]


# Placement.  PyTorch hands out large buffers at multiples of 2 MiB; the library's
# pipesgd_placement_offset says where within a 4 KiB page each buffer should start so that
# the streams a workgroup touches together do not queue on one HBM channel.
def staggered_zeros(count: int, dtype: torch.dtype, device, kind: int, r: int, workers: int,
                    stagger: bool = True) -> torch.Tensor:
    """count zero elements of dtype, starting at the advised offset within a 4 KiB page
    (stagger=False: at the page start)."""
    itemsize = torch.empty(0, dtype=dtype).element_size()
    nbytes = count * itemsize
    raw = torch.zeros(nbytes + 2 * 4096, dtype=torch.uint8, device=device)
    off = (-raw.data_ptr()) % 4096 + (B.placement_offset(kind, r, workers) if stagger else 0)
    return raw[off:off + nbytes].view(dtype)


def payload_to_numpy(mode: int, t: torch.Tensor) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(_PAYLOAD_NUMPY[mode]) if mode == B.TRUNC16 else a


class PipeSgdSim:
    """p simulated workers on one device."""

    def __init__(self, mode: int, workers: int, n: int, lr: float, momentum: float = 0.0,
                 grad_scale: float = 1.0, width: int = 2, buckets: Optional[Sequence[Tuple[int, int]]] = None,
                 schedule: int = B.STEPWISE, device="cuda:0", stagger: bool = True):
        assert 1 <= width <= 7
        self.mode, self.p, self.n = mode, workers, n
        self.lr, self.momentum, self.grad_scale, self.width = lr, momentum, grad_scale, width
        self.schedule = schedule
        self.device = torch.device(device)
        self.buckets = list(buckets) if buckets else None
        dev = self.device
        ns = B.num_scales(mode, n)
        f32, pay_t = torch.float32, _PAYLOAD_TORCH[mode]
        z = lambda count, dtype, kind, r: staggered_zeros(count, dtype, dev, kind, r, workers, stagger)
        self.g_local = [z(n, f32, B.BUF_GRADIENT, r) for r in range(workers)]
        self.w = [z(n, f32, B.BUF_W, r) for r in range(workers)]
        self.v = [z(n, f32, B.BUF_V, r) for r in range(workers)]
        nslots = width                                  # Alg. 1 keeps K result buffers
        self.slots = [[z(n, pay_t, B.BUF_SLOT_A + (i % 2), r) for r in range(workers)] for i in range(nslots)]
        self.slot_scales = [[z(ns, f32, B.BUF_SCALES_A + (i % 2), r) for r in range(workers)] for i in range(nslots)]
        self.rings = [B.make_ring(mode, n, self.g_local, self.slots[i],
                                  self.slot_scales[i] if mode == B.QUANT8 else None, self.buckets)
                      for i in range(nslots)]
        self.updates = [B.UpdateArgs(self.slots[i], self.slot_scales[i] if mode == B.QUANT8 else None,
                                     self.w, self.v if momentum != 0.0 else None)
                        for i in range(nslots)]
        self.stage = self.stage_scales = self.partial = None
        if schedule in (B.DIRECT, B.HALVING_DOUBLING):  # send buffers of the one-exchange / halving-doubling schedules
            self.stage = [z(n, pay_t, B.BUF_STAGE, r) for r in range(workers)]
            self.stage_scales = [z(ns, f32, B.BUF_STAGE_SC, r) for r in range(workers)]
        if schedule == B.HALVING_DOUBLING and workers > 2:      # fp32 partial sums between halving rounds
            self.partial = [z(n, f32, B.BUF_PARTIAL, r) for r in range(workers)]
        if self.stage is not None and workers > 1:              # sizes as the library states them
            ws = B.workspace_bytes(B.WS_DIRECT if schedule == B.DIRECT else B.WS_HALVING_DOUBLING, mode, n, workers)
            assert ws[0] == self.stage[0].numel() * self.stage[0].element_size()
            assert ws[1] == (self.stage_scales[0].numel() * 4 if mode == B.QUANT8 else 0)
            assert ws[2] == (self.partial[0].numel() * 4 if self.partial is not None else 0)
        self.workspace = None
        if self.stage is not None:
            self.workspace = B.make_workspace(self.stage, self.stage_scales if mode == B.QUANT8 else None, self.partial)
        self.t = 0

    # -- data in / out (host <-> device copies; plumbing) --
    def set_gradients(self, grads: Sequence[np.ndarray]) -> None:
        for r, g in enumerate(grads):
            self.g_local[r].copy_(torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)))

    def set_model(self, w0: np.ndarray) -> None:
        t = torch.from_numpy(np.ascontiguousarray(w0, dtype=np.float32))
        for r in range(self.p):
            self.w[r].copy_(t)

    def model(self, r: int = 0) -> np.ndarray:
        return self.w[r].detach().cpu().numpy()

    def velocity(self, r: int = 0) -> np.ndarray:
        return self.v[r].detach().cpu().numpy()

    def result(self, r: int, which: Optional[int] = None):
        """(payload, scales) of the most recent AllReduce on worker r."""
        i = self._last if which is None else which
        pay = payload_to_numpy(self.mode, self.slots[i][r])
        sc = self.slot_scales[i][r].detach().cpu().numpy() if self.mode == B.QUANT8 else None
        return pay, sc

    # -- the path --
    def allreduce(self, stream=None) -> int:
        """Enqueue the AllReduce of the current gradients; returns the slot index."""
        i = (self.t + 1) % len(self.rings)
        if self.schedule == B.DIRECT:
            B.allreduce_direct(self.rings[i], self.workspace, stream)
        elif self.schedule == B.HALVING_DOUBLING:
            B.allreduce_halving_doubling(self.rings[i], self.workspace, stream)
        else:
            B.allreduce_sim(self.rings[i], B.FUSED if self.schedule == B.ONE_LAUNCH else self.schedule, stream)
        self._last = i
        return i

    def update_from(self, slot: int, stream=None) -> None:
        B.apply_update_multi(self.mode, self.updates[slot], self.n, self.lr, self.momentum, self.grad_scale, stream)

    def capture_pair(self):
        """Record two consecutive iterations (one ping and one pong of the slot
        sets) into a HIP graph and return it; ``graph.replay()`` then enqueues
        both with one host call.  Launch-bound (small or many-bucket) models are
        limited by per-launch host and queue latency, not by the kernels.  The
        library's calls only launch kernels (no memset, no allocation), so they
        capture as they are; warm the kernels up once before capturing."""
        assert self.width == 2 and self.t % 2 == 0, "capture at an even iteration count"
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.iteration()
            self.iteration()
        return g

    def iteration(self, stream=None) -> None:
        """One pass of the hot path: AllReduce of g_local[t] and the update that
        yields w[t] (from the previous AllReduce's slot when width is 2)."""
        if self.schedule == B.ONE_LAUNCH:
            assert self.width == 2
            cur = (self.t + 1) % 2
            B.iteration_fused(self.rings[cur], self.updates[1 - cur], self.lr, self.momentum, self.grad_scale, stream)
            self._last = cur
            self.t += 1
            return
        cur = self.allreduce(stream)
        self.update_from((cur + 1) % self.width, stream)        # the slot written width-1 iterations ago
        self.t += 1
