"""ctypes front-end of the scalar C oracle (``pipesgd_oracle.c``) plus the
host-integer parts of the path (bucket plan, pipelined driver loop).

TEST INFRASTRUCTURE ONLY -- see the header of ``pipesgd_oracle.c``.

Notation follows the paper (arXiv 1811.03619): ``p`` workers, ``n`` elements
per gradient vector, ``g_local`` / ``g_sum`` local and aggregated gradients,
``w`` the model, ``gamma`` = ``lr`` the step size, pipeline width ``K``
(Algorithm 1's "iteration dependency"; called ``width`` here because the
workload descriptions use K for the worker count).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

NONE, TRUNC16, QUANT8 = 0, 1, 2
QBLOCK = 4096

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pipesgd_oracle.c")
_LIB = os.path.join(_HERE, "libpipesgd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc.  One rounding per written operation:
    no contraction, no fast-math; -mfma only so that fmaf() is the hardware
    single-rounding instruction instead of the (equally exact) soft routine."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-mfma", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        # PIPESGD_ORACLE_LIB: a deliberately broken build of the oracle, used by
        # the test that checks that the pins notice planted mistakes.
        override = os.environ.get("PIPESGD_ORACLE_LIB")
        if not override:
            build()
        L = C.CDLL(override or _LIB)
        vp, sz, i32, u64, f32 = C.c_void_p, C.c_size_t, C.c_int, C.c_uint64, C.c_float
        L.orc_chunk_elems.restype = sz
        L.orc_chunk_elems.argtypes = [sz, i32]
        L.orc_payload_bytes.restype = sz
        L.orc_payload_bytes.argtypes = [i32, sz]
        L.orc_num_scales.restype = sz
        L.orc_num_scales.argtypes = [i32, sz]
        L.orc_compress.restype = None
        L.orc_compress.argtypes = [i32, vp, sz, vp, vp]
        L.orc_decompress.restype = None
        L.orc_decompress.argtypes = [i32, vp, vp, sz, vp]
        L.orc_ring_new.restype = vp
        L.orc_ring_new.argtypes = [i32, i32, sz, vp]
        L.orc_ring_free.restype = None
        L.orc_ring_free.argtypes = [vp]
        for name in ("orc_ring_reduce_scatter_step", "orc_ring_allgather_step"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [vp, i32]
        L.orc_ring_seal.restype = None
        L.orc_ring_seal.argtypes = [vp]
        L.orc_ring_owner_chunk.restype = i32
        L.orc_ring_owner_chunk.argtypes = [vp, i32]
        for name in ("orc_ring_work", "orc_ring_result_payload", "orc_ring_result_scales"):
            getattr(L, name).restype = vp
            getattr(L, name).argtypes = [vp, i32]
        L.orc_ring_rounds.restype = i32
        L.orc_ring_rounds.argtypes = [vp]
        for name in ("orc_ring_elems_sent", "orc_ring_elems_reduced", "orc_ring_bytes_sent"):
            getattr(L, name).restype = u64
            getattr(L, name).argtypes = [vp, i32]
        L.orc_allreduce.restype = None
        L.orc_allreduce.argtypes = [i32, i32, sz, vp, vp, vp]
        L.orc_allreduce_direct.restype = None
        L.orc_allreduce_direct.argtypes = [i32, i32, sz, vp, vp, vp, vp]
        L.orc_allreduce_hd.restype = i32
        L.orc_allreduce_hd.argtypes = [i32, i32, sz, vp, vp, vp, vp]
        L.orc_sgd_update.restype = None
        L.orc_sgd_update.argtypes = [i32, vp, vp, sz, vp, vp, f32, f32, f32]
        _lib = L
    return _lib


# ------------------------------------------------------------------ helpers --

_PAYLOAD_DTYPE = {NONE: np.float32, TRUNC16: np.uint16, QUANT8: np.int8}


def payload_dtype(mode: int):
    return _PAYLOAD_DTYPE[mode]


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    T = C.c_void_p * len(arrs)
    return T(*[None if a is None else a.ctypes.data for a in arrs])


def chunk_elems(n: int, p: int) -> int:
    return int(lib().orc_chunk_elems(n, p))


def chunk_range(n: int, p: int, c: int) -> Tuple[int, int]:
    ce = chunk_elems(n, p)
    return min(n, c * ce), min(n, (c + 1) * ce)


def num_scales(mode: int, n: int) -> int:
    return int(lib().orc_num_scales(mode, n))


def payload_bytes(mode: int, n: int) -> int:
    """Bytes on the wire for n elements, scales included."""
    return int(lib().orc_payload_bytes(mode, n)) + 4 * num_scales(mode, n)


# ------------------------------------------------------------------- codecs --

def compress(mode: int, x) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    x = _f32(x).ravel()
    pay = np.empty(x.size, dtype=_PAYLOAD_DTYPE[mode])
    sc = np.empty(num_scales(mode, x.size), dtype=np.float32) if mode == QUANT8 else None
    lib().orc_compress(mode, _ptr(x), x.size, _ptr(pay), _ptr(sc))
    return pay, sc


def decompress(mode: int, payload: np.ndarray, scales: Optional[np.ndarray] = None) -> np.ndarray:
    payload = np.ascontiguousarray(payload, dtype=_PAYLOAD_DTYPE[mode]).ravel()
    if mode == QUANT8:
        scales = _f32(scales).ravel()
        assert scales.size == num_scales(mode, payload.size)
    out = np.empty(payload.size, dtype=np.float32)
    lib().orc_decompress(mode, _ptr(payload), _ptr(scales), payload.size, _ptr(out))
    return out


# --------------------------------------------------------------------- ring --

class Ring:
    """Step-by-step ring AllReduce over p simulated workers (Sec. 3.1)."""

    def __init__(self, mode: int, g_local: Sequence[np.ndarray]):
        self.mode, self.p = mode, len(g_local)
        self._g = [_f32(g).ravel() for g in g_local]
        self.n = self._g[0].size
        assert all(g.size == self.n for g in self._g)
        self.ce = chunk_elems(self.n, self.p)
        self._h = lib().orc_ring_new(mode, self.p, self.n, _ptr_array(self._g))

    def close(self):
        if self._h:
            lib().orc_ring_free(self._h)
            self._h = None

    __del__ = close

    def reduce_scatter_step(self, s: int):
        assert 0 <= s <= self.p - 2
        lib().orc_ring_reduce_scatter_step(self._h, s)

    def seal(self):
        lib().orc_ring_seal(self._h)

    def allgather_step(self, s: int):
        assert 0 <= s <= self.p - 2
        lib().orc_ring_allgather_step(self._h, s)

    def run(self):
        for s in range(self.p - 1):
            self.reduce_scatter_step(s)
        self.seal()
        for s in range(self.p - 1):
            self.allgather_step(s)
        return self

    def owner_chunk(self, r: int) -> int:
        return int(lib().orc_ring_owner_chunk(self._h, r))

    def work(self, r: int) -> np.ndarray:
        """Worker r's fp32 working vector (local gradient with the blocks it
        has reduced into replaced by partial sums)."""
        addr = lib().orc_ring_work(self._h, r)
        return np.ctypeslib.as_array(C.cast(addr, C.POINTER(C.c_float)), shape=(self.n,)).copy() \
            if self.n else np.empty(0, np.float32)

    def result(self, r: int) -> Tuple[np.ndarray, Optional[np.ndarray]]:
        """Worker r's aggregated gradient in compressed format."""
        dt = np.dtype(_PAYLOAD_DTYPE[self.mode])
        if self.n == 0:
            return np.empty(0, dt), (np.empty(0, np.float32) if self.mode == QUANT8 else None)
        addr = lib().orc_ring_result_payload(self._h, r)
        buf = (C.c_char * (self.n * dt.itemsize)).from_address(addr)
        pay = np.frombuffer(buf, dtype=dt, count=self.n).copy()
        sc = None
        if self.mode == QUANT8:
            ns = num_scales(self.mode, self.n)
            saddr = lib().orc_ring_result_scales(self._h, r)
            sc = np.ctypeslib.as_array(C.cast(saddr, C.POINTER(C.c_float)), shape=(ns,)).copy()
        return pay, sc

    @property
    def rounds(self) -> int:
        return int(lib().orc_ring_rounds(self._h))

    def elems_sent(self, r): return int(lib().orc_ring_elems_sent(self._h, r))
    def elems_reduced(self, r): return int(lib().orc_ring_elems_reduced(self._h, r))
    def bytes_sent(self, r): return int(lib().orc_ring_bytes_sent(self._h, r))


def allreduce(mode: int, g_local: Sequence[np.ndarray]):
    """Alg. 1 communication thread line 4.  Returns, per worker, the
    aggregated gradient in compressed format: [(payload, scales|None)] * p."""
    g = [_f32(x).ravel() for x in g_local]
    p, n = len(g), g[0].size
    pays = [np.zeros(n, dtype=_PAYLOAD_DTYPE[mode]) for _ in range(p)]
    scs = [np.zeros(num_scales(mode, n), dtype=np.float32) if mode == QUANT8 else None for _ in range(p)]
    lib().orc_allreduce(mode, p, n, _ptr_array(g), _ptr_array(pays), _ptr_array(scs))
    return list(zip(pays, scs))


def allreduce_direct(mode: int, g_local: Sequence[np.ndarray], counters: Optional[np.ndarray] = None):
    """The one-exchange schedule: every block is reduced on its owner from the
    other workers' compressed blocks and sent back once.  Same return shape as
    ``allreduce``.  ``counters``: optional uint64[3] (rounds, elements sent by
    worker 0, elements reduced by worker 0)."""
    g = [_f32(x).ravel() for x in g_local]
    p, n = len(g), g[0].size
    pays = [np.zeros(n, dtype=_PAYLOAD_DTYPE[mode]) for _ in range(p)]
    scs = [np.zeros(num_scales(mode, n), dtype=np.float32) if mode == QUANT8 else None for _ in range(p)]
    lib().orc_allreduce_direct(mode, p, n, _ptr_array(g), _ptr_array(pays), _ptr_array(scs), _ptr(counters))
    return list(zip(pays, scs))


def allreduce_hd(mode: int, g_local: Sequence[np.ndarray], counters: Optional[np.ndarray] = None):
    """Recursive halving (reduce-scatter) and doubling (all-gather); the number
    of workers must be a power of two.  Same return shape as ``allreduce``.
    ``counters``: optional uint64[3] (rounds, elements sent by worker 0,
    elements worker 0 received and added)."""
    g = [_f32(x).ravel() for x in g_local]
    p, n = len(g), g[0].size
    pays = [np.zeros(n, dtype=_PAYLOAD_DTYPE[mode]) for _ in range(p)]
    scs = [np.zeros(num_scales(mode, n), dtype=np.float32) if mode == QUANT8 else None for _ in range(p)]
    rc = lib().orc_allreduce_hd(mode, p, n, _ptr_array(g), _ptr_array(pays), _ptr_array(scs), _ptr(counters))
    if rc != 0:
        raise ValueError("recursive halving-doubling needs a power-of-two number of workers")
    return list(zip(pays, scs))


def sgd_update(mode: int, g_sum_c: np.ndarray, scales: Optional[np.ndarray],
               w: np.ndarray, v: Optional[np.ndarray],
               lr: float, momentum: float = 0.0, grad_scale: float = 1.0) -> None:
    """Alg. 1 compute thread lines 4-5 on one replica, in place on w (and v)."""
    assert w.dtype == np.float32 and w.flags.c_contiguous
    if momentum != 0.0:
        assert v is not None and v.dtype == np.float32 and v.flags.c_contiguous and v.size == w.size
    g_sum_c = np.ascontiguousarray(g_sum_c, dtype=_PAYLOAD_DTYPE[mode])
    assert g_sum_c.size == w.size
    lib().orc_sgd_update(mode, _ptr(g_sum_c), _ptr(scales), w.size, _ptr(w), _ptr(v),
                         C.c_float(lr), C.c_float(momentum), C.c_float(grad_scale))


# ------------------------------------------------------------- bucket plan --

def bucket_plan(numels: Sequence[int], bucket_elems: int = 1 << 20):
    """Greedy small-tensor fusion (workload definition, not in the paper, which
    communicates the gradient as one segment -- Sec. 3.1, L = 1 in Eq. 6).

    Tensors are taken in declaration order; a bucket is closed when the next
    tensor would push it past ``bucket_elems``; a tensor larger than that is
    a bucket by itself.  Every bucket starts at a multiple of 4096 elements
    of the packed buffer.  Returns (buckets, tensor_offsets, n_packed) with
    buckets = [(start, n)], tensor_offsets[i] = offset of tensor i in the
    packed buffer."""
    buckets: List[Tuple[int, int]] = []
    offs: List[int] = []
    start, fill = 0, 0
    for ne in numels:
        if fill > 0 and fill + ne > bucket_elems:
            buckets.append((start, fill))
            start = (start + fill + QBLOCK - 1) // QBLOCK * QBLOCK
            fill = 0
        offs.append(start + fill)
        fill += ne
    if fill > 0 or not buckets:
        buckets.append((start, fill))
    n_packed = (buckets[-1][0] + buckets[-1][1] + QBLOCK - 1) // QBLOCK * QBLOCK
    return buckets, offs, n_packed


def single_bucket(n: int):
    return [(0, n)]


def pack(tensors: Sequence[np.ndarray], offs: Sequence[int], n_packed: int) -> np.ndarray:
    flat = np.zeros(n_packed, dtype=np.float32)
    for t, o in zip(tensors, offs):
        flat[o:o + t.size] = np.asarray(t, dtype=np.float32).ravel()
    return flat


def allreduce_bucketed(mode: int, g_packed: Sequence[np.ndarray], buckets):
    """Each bucket is ring-reduced as a vector of its own, with its own p
    blocks.  Results are laid back into packed-buffer coordinates; padding
    between buckets stays zero."""
    p, N = len(g_packed), g_packed[0].size
    pays = [np.zeros(N, dtype=_PAYLOAD_DTYPE[mode]) for _ in range(p)]
    scs = [np.zeros(num_scales(mode, N), dtype=np.float32) if mode == QUANT8 else None for _ in range(p)]
    for (st, nb) in buckets:
        res = allreduce(mode, [g[st:st + nb] for g in g_packed])
        for r, (pay, sc) in enumerate(res):
            pays[r][st:st + nb] = pay
            if sc is not None:
                scs[r][st // QBLOCK: st // QBLOCK + sc.size] = sc
    return list(zip(pays, scs))


# ------------------------------------------------------- pipelined driver --

def pipe_sgd_run(mode: int, grad_fn, w0: np.ndarray, p: int, iters: int, lr: float,
                 momentum: float = 0.0, grad_scale: float = 1.0, width: int = 2,
                 buckets=None):
    """Algorithm 1 with the two threads serialised.

    Indexing used by the whole project: for t = 1..T
        g_local[t] on every worker is evaluated at w[t-1];
        A[t]  = AllReduce(g_local[t]);
        w[t]  = Update(w[t-1], A[t-(width-1)])      (A[<=0] = 0)
    width = 2 is the paper's optimal pipeline (staleness 1: the update that
    produces w[t] applies the gradient aggregated one iteration earlier);
    width = 1 is decentralised synchronous SGD.  ``grad_fn(r, w, t)`` returns
    worker r's fp32 gradient.  All p replicas are stepped; returns
    (list of w per replica, list of v per replica)."""
    n = w0.size
    ws = [w0.astype(np.float32).copy() for _ in range(p)]
    vs = [np.zeros(n, np.float32) for _ in range(p)]
    zero = (np.zeros(n, dtype=_PAYLOAD_DTYPE[mode]),
            np.zeros(num_scales(mode, n), np.float32) if mode == QUANT8 else None)
    pending = [[zero] * p for _ in range(width - 1)]     # slots for iterations <= 0
    for t in range(1, iters + 1):
        g = [grad_fn(r, ws[r], t) for r in range(p)]
        A = allreduce_bucketed(mode, g, buckets) if buckets is not None else allreduce(mode, g)
        pending.append(A)
        use = pending.pop(0)
        for r in range(p):
            sgd_update(mode, use[r][0], use[r][1], ws[r], vs[r] if momentum != 0.0 else None,
                       lr, momentum, grad_scale)
    return ws, vs
