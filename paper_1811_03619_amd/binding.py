"""ctypes binding of ``libpipesgd.so``: same names as the C ABI
(``include/pipesgd.h``), argument marshalling only.  Device memory and streams
come from PyTorch; every computation runs in the library's HIP kernels.

There is no fallback: if the library cannot be loaded, or a call fails, a
``PipeSgdError`` is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

from . import buildlib

NONE, TRUNC16, QUANT8 = 0, 1, 2
STEPWISE, FUSED = 0, 1
ONE_LAUNCH = 2          # pipeline.PipeSgdSim only: pipesgd_iteration_fused
DIRECT = 3              # pipeline.PipeSgdSim only: pipesgd_allreduce_direct
HALVING_DOUBLING = 4    # pipeline.PipeSgdSim only: pipesgd_allreduce_halving_doubling
MAX_WORKERS = 16
MAX_BUCKETS = 64
QBLOCK = 4096

EXPORTS = [
    "pipesgd_strerror", "pipesgd_version", "pipesgd_chunk_elems", "pipesgd_payload_bytes",
    "pipesgd_num_scales", "pipesgd_compress", "pipesgd_decompress", "pipesgd_ring_first_send",
    "pipesgd_ring_reduce_scatter_step", "pipesgd_ring_allgather_step", "pipesgd_allreduce_sim",
    "pipesgd_apply_update", "pipesgd_apply_update_multi", "pipesgd_bucket_plan",
    "pipesgd_segments_prepare", "pipesgd_pack", "pipesgd_unpack",
    "pipesgd_set_launch_config", "pipesgd_get_launch_config",
    "pipesgd_overlap_create", "pipesgd_overlap_destroy", "pipesgd_allreduce_pipelined",
    "pipesgd_runtime_create", "pipesgd_runtime_destroy", "pipesgd_runtime_iteration", "pipesgd_runtime_sync",
    "pipesgd_runtime_stream", "pipesgd_runtime_update_time", "pipesgd_synthetic_compute",
    "pipesgd_model_sync_time", "pipesgd_model_pipe_ideal_time", "pipesgd_model_pipe_time",
    "pipesgd_model_ring_comm_time", "pipesgd_model_scaling_efficiency", "pipesgd_iteration_fused", "pipesgd_allreduce_direct",
    "pipesgd_allreduce_halving_doubling", "pipesgd_workspace_bytes", "pipesgd_placement_offset",
    "pipesgd_allreduce_direct_static", "pipesgd_probe_stream",
]
PROBE_READ, PROBE_WRITE, PROBE_MIXED, PROBE_COPY = range(4)
STATIC_SCRATCH_BYTES = 32 << 20
K_FIRST_SEND, K_REDUCE_SCATTER, K_ALLGATHER, K_FUSED, K_UPDATE, K_COMPRESS, K_DECOMPRESS, K_DIRECT_REDUCE = range(8)


class PipeSgdError(RuntimeError):
    pass


class Bucket(C.Structure):
    _fields_ = [("start", C.c_uint64), ("n", C.c_uint64)]


class RingStruct(C.Structure):
    _fields_ = [
        ("workers", C.c_int32),
        ("mode", C.c_int32),
        ("n", C.c_uint64),
        ("num_buckets", C.c_uint32),
        ("reserved", C.c_uint32),
        ("buckets", C.POINTER(Bucket)),
        ("g_local", C.c_void_p * MAX_WORKERS),
        ("g_sum_c", C.c_void_p * MAX_WORKERS),
        ("scales", C.c_void_p * MAX_WORKERS),
    ]


RT_TIME_UPDATE = 1


class RuntimeIter(C.Structure):
    _fields_ = [
        ("ring", C.POINTER(RingStruct)),
        ("schedule", C.c_int32), ("width", C.c_int32), ("replicas", C.c_int32), ("compute_workgroups", C.c_int32),
        ("compute_us", C.c_float), ("wire_us", C.c_float), ("lr", C.c_float), ("momentum", C.c_float),
        ("grad_scale", C.c_float), ("flags", C.c_int32),
        ("stale_g_sum_c", C.c_void_p), ("stale_scales", C.c_void_p),
        ("fresh_g_sum_c", C.c_void_p), ("fresh_scales", C.c_void_p),
        ("w", C.c_void_p), ("v", C.c_void_p),
    ]


class Workspace(C.Structure):
    _fields_ = [("stage", C.c_void_p), ("stage_scales", C.c_void_p), ("partial", C.c_void_p),
                ("stage_bytes", C.c_uint64), ("stage_scales_bytes", C.c_uint64), ("partial_bytes", C.c_uint64)]


class Segment(C.Structure):
    _fields_ = [("tensor", C.c_void_p), ("packed", C.c_void_p), ("numel", C.c_uint64),
                ("first_tile", C.c_uint64)]


_lib = None


def lib():
    """Open libpipesgd.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("PIPESGD_LIB")            # a tuning variant built elsewhere
    if not path:
        path = buildlib.LIB_PATH
        if not os.path.exists(path):
            buildlib.build(force=True)
    try:
        L = C.CDLL(path)
    except OSError as e:                                    # pragma: no cover
        raise PipeSgdError(f"cannot load {path}: {e}") from e
    vp, u64, i32, f32 = C.c_void_p, C.c_uint64, C.c_int, C.c_float
    L.pipesgd_strerror.restype = C.c_char_p
    L.pipesgd_strerror.argtypes = [i32]
    L.pipesgd_version.restype = i32
    L.pipesgd_version.argtypes = []
    L.pipesgd_chunk_elems.restype = u64
    L.pipesgd_chunk_elems.argtypes = [u64, i32]
    L.pipesgd_payload_bytes.restype = u64
    L.pipesgd_payload_bytes.argtypes = [i32, u64]
    L.pipesgd_num_scales.restype = u64
    L.pipesgd_num_scales.argtypes = [i32, u64]
    L.pipesgd_compress.restype = i32
    L.pipesgd_compress.argtypes = [i32, vp, u64, vp, vp, vp]
    L.pipesgd_decompress.restype = i32
    L.pipesgd_decompress.argtypes = [i32, vp, vp, u64, vp, vp]
    L.pipesgd_ring_first_send.restype = i32
    L.pipesgd_ring_first_send.argtypes = [C.POINTER(RingStruct), vp]
    L.pipesgd_ring_reduce_scatter_step.restype = i32
    L.pipesgd_ring_reduce_scatter_step.argtypes = [C.POINTER(RingStruct), i32, vp]
    L.pipesgd_ring_allgather_step.restype = i32
    L.pipesgd_ring_allgather_step.argtypes = [C.POINTER(RingStruct), i32, vp]
    L.pipesgd_allreduce_sim.restype = i32
    L.pipesgd_allreduce_sim.argtypes = [C.POINTER(RingStruct), i32, vp]
    L.pipesgd_apply_update.restype = i32
    L.pipesgd_apply_update.argtypes = [i32, vp, vp, u64, vp, vp, f32, f32, f32, vp]
    L.pipesgd_apply_update_multi.restype = i32
    L.pipesgd_apply_update_multi.argtypes = [i32, i32, vp, vp, u64, vp, vp, f32, f32, f32, vp]
    L.pipesgd_bucket_plan.restype = i32
    L.pipesgd_bucket_plan.argtypes = [C.POINTER(u64), u64, u64, C.POINTER(Bucket), u64,
                                      C.POINTER(u64), C.POINTER(u64)]
    L.pipesgd_segments_prepare.restype = i32
    L.pipesgd_segments_prepare.argtypes = [C.POINTER(Segment), u64, C.POINTER(u64)]
    L.pipesgd_pack.restype = i32
    L.pipesgd_pack.argtypes = [vp, u64, u64, vp]
    L.pipesgd_unpack.restype = i32
    L.pipesgd_unpack.argtypes = [vp, u64, u64, vp]
    L.pipesgd_overlap_create.restype = i32
    L.pipesgd_overlap_create.argtypes = [C.POINTER(vp)]
    L.pipesgd_overlap_destroy.restype = None
    L.pipesgd_overlap_destroy.argtypes = [vp]
    L.pipesgd_allreduce_pipelined.restype = i32
    L.pipesgd_allreduce_pipelined.argtypes = [C.POINTER(RingStruct), C.POINTER(Workspace), i32, i32, f32, vp, vp, vp]
    L.pipesgd_runtime_create.restype = i32
    L.pipesgd_runtime_create.argtypes = [C.POINTER(vp)]
    L.pipesgd_runtime_destroy.restype = None
    L.pipesgd_runtime_destroy.argtypes = [vp]
    L.pipesgd_runtime_iteration.restype = i32
    L.pipesgd_runtime_iteration.argtypes = [vp, C.POINTER(RuntimeIter)]
    L.pipesgd_runtime_sync.restype = i32
    L.pipesgd_runtime_sync.argtypes = [vp]
    L.pipesgd_runtime_update_time.restype = i32
    L.pipesgd_runtime_update_time.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    L.pipesgd_runtime_stream.restype = vp
    L.pipesgd_runtime_stream.argtypes = [vp, i32]
    L.pipesgd_synthetic_compute.restype = i32
    L.pipesgd_synthetic_compute.argtypes = [f32, i32, vp]
    dbl = C.c_double
    for name, nargs in (("pipesgd_model_sync_time", 4), ("pipesgd_model_pipe_ideal_time", 5),
                        ("pipesgd_model_pipe_time", 4), ("pipesgd_model_scaling_efficiency", 3)):
        getattr(L, name).restype = dbl
        getattr(L, name).argtypes = [dbl] * nargs
    L.pipesgd_model_ring_comm_time.restype = dbl
    L.pipesgd_model_ring_comm_time.argtypes = [i32, dbl, dbl, dbl, dbl, dbl, i32]
    L.pipesgd_allreduce_direct.restype = i32
    L.pipesgd_allreduce_direct.argtypes = [C.POINTER(RingStruct), C.POINTER(Workspace), vp]
    L.pipesgd_allreduce_direct_static.restype = i32
    L.pipesgd_allreduce_direct_static.argtypes = [C.POINTER(RingStruct), vp]
    L.pipesgd_probe_stream.restype = i32
    L.pipesgd_probe_stream.argtypes = [i32, i32, i32, vp, vp, vp, u64, i32, i32, i32, vp]
    L.pipesgd_placement_offset.restype = u64
    L.pipesgd_placement_offset.argtypes = [i32, i32, i32]
    L.pipesgd_workspace_bytes.restype = i32
    L.pipesgd_workspace_bytes.argtypes = [i32, i32, u64, i32, C.POINTER(C.c_uint64)]
    L.pipesgd_allreduce_halving_doubling.restype = i32
    L.pipesgd_allreduce_halving_doubling.argtypes = [C.POINTER(RingStruct), C.POINTER(Workspace), vp]
    L.pipesgd_iteration_fused.restype = i32
    L.pipesgd_iteration_fused.argtypes = [C.POINTER(RingStruct), vp, vp, vp, vp, f32, f32, f32, vp]
    L.pipesgd_set_launch_config.restype = i32
    L.pipesgd_set_launch_config.argtypes = [i32, i32, i32, i32, i32]
    L.pipesgd_get_launch_config.restype = i32
    L.pipesgd_get_launch_config.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    _lib = L
    return L


def strerror(rc: int) -> str:
    return lib().pipesgd_strerror(rc).decode()


def check(rc: int, what: str = "pipesgd") -> None:
    if rc != 0:
        raise PipeSgdError(f"{what}: {strerror(rc)} ({rc})")


# --------------------------------------------------------------- marshalling --

def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, or a raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr_array(items: Sequence) -> C.Array:
    arr = (C.c_void_p * len(items))()
    for i, t in enumerate(items):
        arr[i] = _ptr(t)
    return arr


def version() -> int:
    return int(lib().pipesgd_version())


def chunk_elems(n: int, workers: int) -> int:
    return int(lib().pipesgd_chunk_elems(n, workers))


def payload_bytes(mode: int, n: int) -> int:
    return int(lib().pipesgd_payload_bytes(mode, n))


def num_scales(mode: int, n: int) -> int:
    return int(lib().pipesgd_num_scales(mode, n))


WS_RING, WS_PIPELINED, WS_DIRECT, WS_HALVING_DOUBLING = 0, 1, 2, 3
(BUF_GRADIENT, BUF_W, BUF_V, BUF_SLOT_A, BUF_SLOT_B, BUF_SCALES_A, BUF_SCALES_B, BUF_STAGE, BUF_STAGE_SC,
 BUF_PARTIAL) = range(10)


def placement_offset(kind: int, worker: int, workers: int) -> int:
    """Byte offset within a 4 KiB page at which this buffer should start (advisory)."""
    return int(lib().pipesgd_placement_offset(kind, worker, workers))


def workspace_bytes(schedule: int, mode: int, n: int, workers: int) -> Tuple[int, int, int]:
    """(payload staging, scales staging, fp32 partial sums) bytes per worker."""
    out = (C.c_uint64 * 3)()
    check(lib().pipesgd_workspace_bytes(schedule, mode, n, workers, out), "pipesgd_workspace_bytes")
    return int(out[0]), int(out[1]), int(out[2])


def compress(mode: int, src, n: int, payload, scales=None, stream=None) -> None:
    check(lib().pipesgd_compress(mode, _ptr(src), n, _ptr(payload), _ptr(scales), _stream(stream)),
          "pipesgd_compress")


def decompress(mode: int, payload, scales, n: int, dst, stream=None) -> None:
    check(lib().pipesgd_decompress(mode, _ptr(payload), _ptr(scales), n, _ptr(dst), _stream(stream)),
          "pipesgd_decompress")


def make_ring(mode: int, n: int, g_local: Sequence, g_sum_c: Sequence, scales: Optional[Sequence] = None,
              buckets: Optional[Sequence[Tuple[int, int]]] = None) -> RingStruct:
    """Fill a pipesgd_ring.  The returned struct keeps the bucket table alive."""
    p = len(g_local)
    if p > MAX_WORKERS:
        raise PipeSgdError("too many workers")
    R = RingStruct()
    R.workers, R.mode, R.n, R.reserved = p, mode, n, 0
    if buckets:
        tab = (Bucket * len(buckets))(*[Bucket(int(s), int(m)) for s, m in buckets])
        R._bucket_keepalive = tab
        R.buckets = C.cast(tab, C.POINTER(Bucket))
        R.num_buckets = len(buckets)
    else:
        R.num_buckets = 0
        R.buckets = None
    for r in range(p):
        R.g_local[r] = _ptr(g_local[r])
        R.g_sum_c[r] = _ptr(g_sum_c[r])
        R.scales[r] = _ptr(scales[r]) if scales is not None else None
    return R


def ring_first_send(ring: RingStruct, stream=None) -> None:
    check(lib().pipesgd_ring_first_send(C.byref(ring), _stream(stream)), "pipesgd_ring_first_send")


def ring_reduce_scatter_step(ring: RingStruct, step: int, stream=None) -> None:
    check(lib().pipesgd_ring_reduce_scatter_step(C.byref(ring), step, _stream(stream)),
          "pipesgd_ring_reduce_scatter_step")


def ring_allgather_step(ring: RingStruct, step: int, stream=None) -> None:
    check(lib().pipesgd_ring_allgather_step(C.byref(ring), step, _stream(stream)),
          "pipesgd_ring_allgather_step")


def allreduce_sim(ring: RingStruct, schedule: int = STEPWISE, stream=None) -> None:
    check(lib().pipesgd_allreduce_sim(C.byref(ring), schedule, _stream(stream)), "pipesgd_allreduce_sim")


def _nbytes(t) -> int:
    """Bytes of a torch tensor; a raw address says nothing about its size."""
    return t.numel() * t.element_size()


def make_workspace(stage: Optional[Sequence] = None, stage_scales: Optional[Sequence] = None,
                   partial: Optional[Sequence] = None, sizes: Optional[Tuple[int, int, int]] = None) -> Workspace:
    """Fill a pipesgd_workspace from lists of torch tensors (or raw addresses,
    then `sizes` = bytes of each stage / stage_scales / partial buffer must be
    given).  The returned struct keeps the pointer tables alive."""
    ws = Workspace()
    tabs = []
    for name, items in (("stage", stage), ("stage_scales", stage_scales), ("partial", partial)):
        if items is None:
            setattr(ws, name, None)
            tabs.append(None)
        else:
            arr = _ptr_array(items)
            tabs.append(arr)
            setattr(ws, name, C.cast(arr, C.c_void_p))
    ws._keepalive = tabs
    if sizes is None:
        def smallest(items):
            known = [_nbytes(t) for t in (items or []) if t is not None and not isinstance(t, int)]
            return min(known) if known else 0
        sizes = (smallest(stage), smallest(stage_scales), smallest(partial))
    ws.stage_bytes, ws.stage_scales_bytes, ws.partial_bytes = (int(x) for x in sizes)
    return ws


def _ws_arg(ws: Optional[Workspace]):
    return C.byref(ws) if ws is not None else None


def allreduce_direct(ring: RingStruct, ws: Optional[Workspace], stream=None) -> None:
    check(lib().pipesgd_allreduce_direct(C.byref(ring), _ws_arg(ws), _stream(stream)), "pipesgd_allreduce_direct")


def allreduce_direct_static(ring: RingStruct, stream=None) -> None:
    check(lib().pipesgd_allreduce_direct_static(C.byref(ring), _stream(stream)), "pipesgd_allreduce_direct_static")


def allreduce_halving_doubling(ring: RingStruct, ws: Optional[Workspace], stream=None) -> None:
    check(lib().pipesgd_allreduce_halving_doubling(C.byref(ring), _ws_arg(ws), _stream(stream)),
          "pipesgd_allreduce_halving_doubling")


class Overlap:
    """Owner of a pipesgd_overlap handle (HIP events of the two-stream schedule)."""

    def __init__(self):
        h = C.c_void_p()
        check(lib().pipesgd_overlap_create(C.byref(h)), "pipesgd_overlap_create")
        self.handle = h

    def close(self):
        if self.handle and _lib is not None:
            _lib.pipesgd_overlap_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def allreduce_pipelined(ring: RingStruct, ws: Optional[Workspace], segments: int,
                        overlap: Overlap, compute_stream=None, wire_stream=None, wire_workgroups: int = 0,
                        link_us_per_mib: float = 0.0) -> None:
    check(lib().pipesgd_allreduce_pipelined(C.byref(ring), _ws_arg(ws), segments, wire_workgroups, link_us_per_mib,
                                            overlap.handle, _stream(compute_stream), _stream(wire_stream)),
          "pipesgd_allreduce_pipelined")


class Runtime:
    """Owner of a pipesgd_runtime handle (Algorithm 1's two threads as two streams)."""

    def __init__(self):
        h = C.c_void_p()
        check(lib().pipesgd_runtime_create(C.byref(h)), "pipesgd_runtime_create")
        self.handle = h

    def iteration(self, ring: RingStruct, stale: "UpdateArgs", fresh: Optional["UpdateArgs"], schedule: int,
                  width: int, lr: float, momentum: float, grad_scale: float = 1.0, compute_us: float = 0.0,
                  compute_workgroups: int = 1, wire_us: float = 0.0, time_update: bool = False) -> None:
        it = RuntimeIter()
        it.ring = C.pointer(ring)
        it.schedule, it.width, it.replicas, it.compute_workgroups = schedule, width, stale.replicas, compute_workgroups
        it.compute_us, it.wire_us, it.lr, it.momentum, it.grad_scale = compute_us, wire_us, lr, momentum, grad_scale
        it.flags = RT_TIME_UPDATE if time_update else 0
        it.stale_g_sum_c = C.cast(stale.g_sum_c, C.c_void_p)
        it.stale_scales = C.cast(stale.scales, C.c_void_p) if stale.scales is not None else None
        if fresh is not None:
            it.fresh_g_sum_c = C.cast(fresh.g_sum_c, C.c_void_p)
            it.fresh_scales = C.cast(fresh.scales, C.c_void_p) if fresh.scales is not None else None
        it.w = C.cast(stale.w, C.c_void_p)
        it.v = C.cast(stale.v, C.c_void_p) if stale.v is not None else None
        check(lib().pipesgd_runtime_iteration(self.handle, C.byref(it)), "pipesgd_runtime_iteration")

    def sync(self) -> None:
        check(lib().pipesgd_runtime_sync(self.handle), "pipesgd_runtime_sync")

    def update_time(self) -> Tuple[float, int]:
        """(summed milliseconds, count) of the update launches timed since the last call."""
        ms, k = C.c_double(), C.c_uint64()
        check(lib().pipesgd_runtime_update_time(self.handle, C.byref(ms), C.byref(k)), "pipesgd_runtime_update_time")
        return float(ms.value), int(k.value)

    def stream(self, which: int) -> int:
        return lib().pipesgd_runtime_stream(self.handle, which)

    def close(self):
        if self.handle and _lib is not None:
            _lib.pipesgd_runtime_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def synthetic_compute(duration_us: float, workgroups: int = 1, stream=None) -> None:
    check(lib().pipesgd_synthetic_compute(duration_us, workgroups, _stream(stream)), "pipesgd_synthetic_compute")


def apply_update(mode: int, g_sum_c, scales, n: int, w, v, lr: float, momentum: float = 0.0,
                 grad_scale: float = 1.0, stream=None) -> None:
    check(lib().pipesgd_apply_update(mode, _ptr(g_sum_c), _ptr(scales), n, _ptr(w), _ptr(v),
                                     lr, momentum, grad_scale, _stream(stream)), "pipesgd_apply_update")


class UpdateArgs:
    """Pre-marshalled pointer tables for pipesgd_apply_update_multi, so that a
    timed loop does not rebuild them on every call."""

    def __init__(self, g_sum_c: Sequence, scales: Optional[Sequence], w: Sequence, v: Optional[Sequence]):
        self.replicas = len(w)
        self.g_sum_c = _ptr_array(g_sum_c)
        self.scales = _ptr_array(scales) if scales is not None else None
        self.w = _ptr_array(w)
        self.v = _ptr_array(v) if v is not None else None


def apply_update_multi(mode: int, args: UpdateArgs, n: int, lr: float, momentum: float = 0.0,
                       grad_scale: float = 1.0, stream=None) -> None:
    check(lib().pipesgd_apply_update_multi(mode, args.replicas, args.g_sum_c, args.scales, n, args.w, args.v,
                                           lr, momentum, grad_scale, _stream(stream)),
          "pipesgd_apply_update_multi")


def probe_stream(kind: int, mode: int, args: UpdateArgs, n: int, threads: int, quads: int, lds_bytes: int = 0,
                 stream=None) -> None:
    """Measurement aid: the update's memory streams without its arithmetic (overwrites w / v)."""
    check(lib().pipesgd_probe_stream(kind, mode, args.replicas, args.g_sum_c, args.w, args.v, n, threads, quads,
                                     lds_bytes, _stream(stream)), "pipesgd_probe_stream")


def set_launch_config(kernel: int, mode: int, threads: int, quads: int, lds_bytes: int = 0) -> None:
    check(lib().pipesgd_set_launch_config(kernel, mode, threads, quads, lds_bytes), "pipesgd_set_launch_config")


def get_launch_config(kernel: int, mode: int) -> Tuple[int, int, int]:
    t, q, l = C.c_int(), C.c_int(), C.c_int()
    check(lib().pipesgd_get_launch_config(kernel, mode, C.byref(t), C.byref(q), C.byref(l)),
          "pipesgd_get_launch_config")
    return t.value, q.value, l.value


def model_sync_time(T, l_up, l_comp, l_comm):
    return lib().pipesgd_model_sync_time(T, l_up, l_comp, l_comm)


def model_pipe_ideal_time(T, K, l_up, l_comp, l_comm):
    return lib().pipesgd_model_pipe_ideal_time(T, K, l_up, l_comp, l_comm)


def model_pipe_time(T, l_up, l_comp, l_comm):
    return lib().pipesgd_model_pipe_time(T, l_up, l_comp, l_comm)


def model_ring_comm_time(p, n_bytes, alpha, beta, gamma, S=0.0, L=1):
    return lib().pipesgd_model_ring_comm_time(p, n_bytes, alpha, beta, gamma, S, L)


def model_scaling_efficiency(l_up, l_comp, l_comm):
    return lib().pipesgd_model_scaling_efficiency(l_up, l_comp, l_comm)


def iteration_fused(ring: RingStruct, stale: UpdateArgs, lr: float, momentum: float = 0.0,
                    grad_scale: float = 1.0, stream=None) -> None:
    check(lib().pipesgd_iteration_fused(C.byref(ring), stale.g_sum_c, stale.scales, stale.w, stale.v,
                                        lr, momentum, grad_scale, _stream(stream)), "pipesgd_iteration_fused")


def bucket_plan(numels: Sequence[int], bucket_elems: int = 1 << 20, max_buckets: int = MAX_BUCKETS):
    """Host planner.  Returns (buckets [(start, n)], tensor_offsets, n_packed)."""
    nt = len(numels)
    arr = (C.c_uint64 * max(nt, 1))(*numels)
    out_b = (Bucket * max_buckets)()
    out_o = (C.c_uint64 * max(nt, 1))()
    n_packed = C.c_uint64(0)
    rc = lib().pipesgd_bucket_plan(arr, nt, bucket_elems, out_b, max_buckets, out_o, C.byref(n_packed))
    if rc < 0:
        check(rc, "pipesgd_bucket_plan")
    return ([(int(out_b[i].start), int(out_b[i].n)) for i in range(rc)],
            [int(out_o[i]) for i in range(nt)], int(n_packed.value))


def segments_prepare(tensor_ptrs: Sequence[int], packed_ptrs: Sequence[int], numels: Sequence[int]):
    """Returns (ctypes table ready to be copied to the device, total_tiles)."""
    num = len(numels)
    tab = (Segment * max(num, 1))()
    for i in range(num):
        tab[i].tensor, tab[i].packed, tab[i].numel, tab[i].first_tile = tensor_ptrs[i], packed_ptrs[i], numels[i], 0
    total = C.c_uint64(0)
    check(lib().pipesgd_segments_prepare(tab, num, C.byref(total)), "pipesgd_segments_prepare")
    return tab, int(total.value)


def pack(segments_dev, num: int, total_tiles: int, stream=None) -> None:
    check(lib().pipesgd_pack(_ptr(segments_dev), num, total_tiles, _stream(stream)), "pipesgd_pack")


def unpack(segments_dev, num: int, total_tiles: int, stream=None) -> None:
    check(lib().pipesgd_unpack(_ptr(segments_dev), num, total_tiles, _stream(stream)), "pipesgd_unpack")
