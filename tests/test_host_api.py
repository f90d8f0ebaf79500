"""Host-side checks of libpipesgd that need no GPU: the library loads, exports
every symbol the header declares, its size rules and bucket planner agree with
the oracle's, and argument validation rejects bad calls before anything is
launched.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1811_03619_amd import binding as B
from paper_1811_03619_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pipesgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pipesgd_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 17
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names
    assert B.version() == 100
    assert B.strerror(0) == "ok" and "aligned" in B.strerror(-2)


def test_ring_struct_layout_matches_header():
    # int32 x2, uint64, uint32 x2, pointer, 3 arrays of 16 pointers
    assert C.sizeof(B.RingStruct) == 4 + 4 + 8 + 4 + 4 + 8 + 3 * 16 * 8
    assert C.sizeof(B.Segment) == 32 and C.sizeof(B.Bucket) == 16
    assert B.RingStruct.g_local.offset == 32


@pytest.mark.parametrize("n", [0, 1, 4095, 4096, 4097, 648010, 1 << 20, 60965224, 138357544, 25557032])
@pytest.mark.parametrize("p", [1, 2, 3, 4, 7, 16])
def test_size_rules_agree_with_oracle(orc, n, p):
    assert B.chunk_elems(n, p) == orc.chunk_elems(n, p)
    for mode in (0, 1, 2):
        assert B.num_scales(mode, n) == orc.num_scales(mode, n)
        assert B.payload_bytes(mode, n) + 4 * B.num_scales(mode, n) == orc.payload_bytes(mode, n)
    assert B.chunk_elems(n, 0) == 0 and B.payload_bytes(9, n) == 0


@pytest.mark.parametrize("cap", [1, 4096, 16384, 1 << 20, 1 << 40])
def test_bucket_plan_agrees_with_oracle(orc, cap):
    cases = [
        [10, 20, 5000, 3, 2_000_000, 7, 1 << 20, 1],
        [t.numel for t in W.config_tensors(2)],
        [t.numel for t in W.config_tensors(3)],
        [1],
        [4096, 4096, 4096],
    ]
    if cap >= 16384:
        cases.append([t.numel for t in W.config_tensors(5)])
    for numels in cases:
        want = orc.bucket_plan(numels, cap)
        if len(want[0]) > B.MAX_BUCKETS:
            with pytest.raises(B.PipeSgdError):
                B.bucket_plan(numels, cap)
            got = B.bucket_plan(numels, cap, max_buckets=len(want[0]))
        else:
            got = B.bucket_plan(numels, cap)
        assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2]


def test_bucket_plan_rejects_bad_arguments():
    L = B.lib()
    n_packed = C.c_uint64()
    out_b = (B.Bucket * 4)()
    out_o = (C.c_uint64 * 4)()
    arr = (C.c_uint64 * 4)(1, 2, 3, 4)
    assert L.pipesgd_bucket_plan(arr, 4, 0, out_b, 4, out_o, C.byref(n_packed)) == -1
    assert L.pipesgd_bucket_plan(None, 4, 10, out_b, 4, out_o, C.byref(n_packed)) == -1
    assert L.pipesgd_bucket_plan(arr, 4, 1, out_b, 2, out_o, C.byref(n_packed)) == -4
    assert L.pipesgd_bucket_plan(arr, 0, 10, out_b, 4, out_o, C.byref(n_packed)) == 1     # one empty bucket
    assert (out_b[0].start, out_b[0].n, n_packed.value) == (0, 0, 0)


def test_segments_prepare():
    tab, total = B.segments_prepare([4096, 8192, 16384], [65536, 65540, 131072], [1, 4096, 4097])
    assert total == 1 + 1 + 2
    assert [tab[i].first_tile for i in range(3)] == [0, 1, 2]
    with pytest.raises(B.PipeSgdError):
        B.segments_prepare([4097], [65536], [8])            # not 4-byte aligned
    with pytest.raises(B.PipeSgdError):
        B.segments_prepare([0], [65536], [8])               # null tensor


# Validation happens before any HIP call, so these run without a GPU.  The
# "device" addresses below are never dereferenced.

def fake_ring(p=4, mode=B.NONE, n=8192, buckets=None, g=0x10000, pay=0x20000, sc=0x30000):
    return B.make_ring(mode, n, [g] * p, [pay] * p, [sc] * p, buckets)


def test_ring_validation_errors():
    L = B.lib()
    call = lambda R, step=0: L.pipesgd_ring_reduce_scatter_step(C.byref(R), step, None)
    assert L.pipesgd_ring_reduce_scatter_step(None, 0, None) == -1
    assert call(fake_ring(mode=7)) == -3
    R = fake_ring(); R.workers = 0
    assert call(R) == -1
    R = fake_ring(); R.workers = 17
    assert call(R) == -4
    R = fake_ring(); R.reserved = 1
    assert call(R) == -1
    assert call(fake_ring(g=0x10004)) == -2
    assert call(fake_ring(pay=0x20008)) == -2
    assert call(fake_ring(g=0)) == -1
    assert call(fake_ring(mode=B.QUANT8, sc=0)) == -1
    assert call(fake_ring(), step=3) == -1                  # rounds are 0..p-2
    assert call(fake_ring(), step=-1) == -1
    assert call(fake_ring(p=1), step=0) == -1               # a single worker has no rounds
    assert call(fake_ring(buckets=[(100, 50)])) == -2       # bucket start not a multiple of 4096
    assert call(fake_ring(buckets=[(0, 5000), (4096, 100)])) == -1    # overlap
    assert call(fake_ring(buckets=[(4096, 8192)])) == -1    # runs past n
    R = fake_ring(buckets=[(0, 10)]); R.num_buckets = 65
    assert call(R) == -4
    assert L.pipesgd_allreduce_sim(C.byref(fake_ring()), 5, None) == -3
    # an empty vector is valid and enqueues nothing
    assert L.pipesgd_allreduce_sim(C.byref(fake_ring(n=0, g=0, pay=0, sc=0)), 0, None) == 0
    assert L.pipesgd_ring_first_send(C.byref(fake_ring(n=0, g=0, pay=0, sc=0)), None) == 0


def fake_workspace(p=4, mode=B.NONE, n=8192, schedule=None, stage=0x40000, stage_sc=0x48000, partial=0x50000,
                   shrink=(0, 0, 0)):
    """A workspace of never-dereferenced addresses, sized as the library asks
    for `schedule` minus `shrink` bytes per table."""
    need = B.workspace_bytes(schedule, mode, n, p)
    arr = lambda v: None if v is None else [v] * p
    return B.make_workspace(arr(stage), arr(stage_sc), arr(partial),
                            sizes=tuple(max(0, a - b) for a, b in zip(need, shrink)))


def test_extra_schedules_validate_before_launching():
    # every call below is rejected (or is a no-op) on the host: nothing is enqueued
    L = B.lib()
    hd = lambda ring, ws: L.pipesgd_allreduce_halving_doubling(C.byref(ring) if ring is not None else None,
                                                               C.byref(ws) if ws is not None else None, None)
    HD, DI, PI = B.WS_HALVING_DOUBLING, B.WS_DIRECT, B.WS_PIPELINED
    assert hd(None, fake_workspace(schedule=HD)) == -1
    for p in (3, 5, 6, 12):                                 # worker count must be a power of two
        assert hd(fake_ring(p=p), fake_workspace(p=p, schedule=HD)) == -1
    assert hd(fake_ring(), None) == -1                                                  # no workspace at all
    assert hd(fake_ring(), fake_workspace(schedule=HD, stage=None)) == -1               # no send buffers
    assert hd(fake_ring(), fake_workspace(schedule=HD, partial=None)) == -1             # p > 2 needs partial sums
    ws = fake_workspace(schedule=HD)
    ws._keepalive[0][1] = None
    assert hd(fake_ring(), ws) == -1                                                    # one send buffer missing
    assert hd(fake_ring(), fake_workspace(schedule=HD, stage=0x40004)) == -2
    assert hd(fake_ring(), fake_workspace(schedule=HD, partial=0x50008)) == -2
    assert hd(fake_ring(mode=B.QUANT8), fake_workspace(mode=B.QUANT8, schedule=HD, stage_sc=None)) == -1
    assert hd(fake_ring(mode=9), fake_workspace(schedule=HD)) == -3
    assert hd(fake_ring(n=0, g=0, pay=0, sc=0), None) == 0                              # empty vector: nothing to do
    direct = lambda ring, ws: L.pipesgd_allreduce_direct(C.byref(ring), C.byref(ws) if ws is not None else None, None)
    assert direct(fake_ring(), None) == -1
    assert direct(fake_ring(), fake_workspace(schedule=DI, stage=0x40004)) == -2
    assert direct(fake_ring(mode=B.QUANT8), fake_workspace(mode=B.QUANT8, schedule=DI, stage_sc=None)) == -1
    assert direct(fake_ring(n=0, g=0, pay=0, sc=0), None) == 0


@pytest.mark.parametrize("mode", [B.NONE, B.TRUNC16, B.QUANT8])
def test_undersized_workspace_is_refused_on_the_host(mode):
    # an under-allocated staging buffer would be overrun by the kernels: the sizes the caller states are
    # compared with pipesgd_workspace_bytes before anything is launched
    L = B.lib()
    n, p = 4096 * 5 + 7, 4
    ring = fake_ring(p=p, mode=mode, n=n)
    calls = {
        B.WS_DIRECT: lambda ws: L.pipesgd_allreduce_direct(C.byref(ring), C.byref(ws), None),
        B.WS_HALVING_DOUBLING: lambda ws: L.pipesgd_allreduce_halving_doubling(C.byref(ring), C.byref(ws), None),
        B.WS_PIPELINED: lambda ws: L.pipesgd_allreduce_pipelined(C.byref(ring), C.byref(ws), 2, 0, 0.0, 0x1234, None, None),
    }
    for sched, call in calls.items():
        need = B.workspace_bytes(sched, mode, n, p)
        assert call(fake_workspace(p, mode, n, sched, shrink=(1, 0, 0))) == -4, sched
        if need[1]:
            assert call(fake_workspace(p, mode, n, sched, shrink=(0, 1, 0))) == -4, sched
        if need[2]:
            assert call(fake_workspace(p, mode, n, sched, shrink=(0, 0, 4))) == -4, sched
    assert "workspace" in B.strerror(-4)


def test_scales_are_only_looked_at_when_quantising():
    # ring->scales[] is documented as QUANT8-only: garbage there must not fail the other modes
    L = B.lib()
    for mode in (B.NONE, B.TRUNC16):
        ring = fake_ring(mode=mode, sc=0x30004)             # misaligned, and never read
        assert L.pipesgd_ring_reduce_scatter_step(C.byref(ring), 5, None) == -1    # reaches the step check
        ring = fake_ring(mode=mode, sc=0)
        assert L.pipesgd_ring_reduce_scatter_step(C.byref(ring), 5, None) == -1
    assert L.pipesgd_ring_reduce_scatter_step(C.byref(fake_ring(mode=B.QUANT8, sc=0x30004)), 0, None) == -2


def test_pipelined_schedule_validates_before_launching():
    L = B.lib()
    n, p = 4096 * 64, 4
    ring = fake_ring(p=p, mode=B.TRUNC16, n=n)
    ws = fake_workspace(p, B.TRUNC16, n, B.WS_PIPELINED)
    call = lambda segments, wg=0, link=0.0, ov=0x1234, w=ws: L.pipesgd_allreduce_pipelined(
        C.byref(ring), C.byref(w) if w is not None else None, segments, wg, C.c_float(link), ov, None, None)
    assert call(0) == -1 and call(-3) == -1
    assert call(65) == -4                                   # more sub-blocks than the library keeps events for
    assert call(2, wg=-1) == -1
    assert call(2, link=-1.0) == -1 and call(2, link=float("nan")) == -1
    assert call(2, ov=None) == -1
    assert call(2, w=None) == -1
    # a link so slow that one ring block would be under way for more than a second: refused up front
    # (16 tiles of 8 KiB per ring block = 0.125 MiB; 1e7 us per MiB -> 1.25 s)
    assert call(2, link=1.0e7) == -1


@pytest.mark.parametrize("mode", [B.NONE, B.TRUNC16, B.QUANT8])
@pytest.mark.parametrize("n", [0, 5, 4096, 4097, 60965224])
def test_workspace_bytes(mode, n):
    cb = {B.NONE: 4, B.TRUNC16: 2, B.QUANT8: 1}[mode]
    ns = -(-n // 4096) if mode == B.QUANT8 else 0
    for p in (1, 2, 4, 16):
        assert B.workspace_bytes(B.WS_RING, mode, n, p) == (0, 0, 0)
        for sched in (B.WS_PIPELINED, B.WS_DIRECT, B.WS_HALVING_DOUBLING):
            want = (0, 0, 0) if p == 1 else (cb * n, 4 * ns, 4 * n if sched == B.WS_HALVING_DOUBLING and p > 2 else 0)
            assert B.workspace_bytes(sched, mode, n, p) == want
    L = B.lib()
    out = (C.c_uint64 * 3)()
    assert L.pipesgd_workspace_bytes(9, mode, n, 4, out) == -3
    assert L.pipesgd_workspace_bytes(B.WS_DIRECT, 7, n, 4, out) == -3
    assert L.pipesgd_workspace_bytes(B.WS_DIRECT, mode, n, 0, out) == -1
    assert L.pipesgd_workspace_bytes(B.WS_DIRECT, mode, n, 4, None) == -1


def test_placement_offsets_separate_the_streams_of_a_workgroup():
    off = B.placement_offset
    for p in range(1, 17):
        for r in range(p):
            for slot in (B.BUF_SLOT_A, B.BUF_SLOT_B):
                # a ring hop of worker r: its gradient, its slot, the neighbour's slot
                hop = {off(B.BUF_GRADIENT, r, p), off(slot, r, p)}
                if p > 1:
                    hop.add(off(slot, (r - 1) % p, p))
                assert len(hop) == (3 if p > 1 else 2), (p, r, slot)
                # the update of replica r: slot, w, v
                assert len({off(slot, r, p), off(B.BUF_W, r, p), off(B.BUF_V, r, p)}) == 3, (p, r, slot)
                # the one-exchange and halving-doubling schedules: gradient, send buffer, partial sums, slot
                assert len({off(B.BUF_GRADIENT, r, p), off(B.BUF_STAGE, r, p), off(B.BUF_PARTIAL, r, p),
                            off(slot, r, p)}) == 4
            for kind in range(10):
                assert off(kind, r, p) % 256 == 0 and 0 <= off(kind, r, p) < 4096
    assert off(-1, 0, 4) == 0 and off(10, 0, 4) == 0 and off(0, -1, 4) == 0 and off(0, 4, 4) == 0 and off(0, 0, 0) == 0


def test_plumbing_places_buffers_where_the_library_advises():
    import torch
    from paper_1811_03619_amd.pipeline import staggered_zeros
    for kind in (B.BUF_GRADIENT, B.BUF_V, B.BUF_SLOT_B, B.BUF_PARTIAL):
        for r, p in ((0, 4), (3, 4), (4, 5), (7, 8)):
            for dtype in (torch.float32, torch.int16, torch.int8):
                t = staggered_zeros(1000, dtype, "cpu", kind, r, p)
                assert t.numel() == 1000 and t.dtype == dtype and int(t.abs().sum()) == 0
                assert t.data_ptr() % 4096 == B.placement_offset(kind, r, p)
                assert staggered_zeros(1000, dtype, "cpu", kind, r, p, stagger=False).data_ptr() % 4096 == 0
    assert staggered_zeros(0, torch.float32, "cpu", 0, 0, 1).numel() == 0


def test_codec_and_update_validation_errors():
    L = B.lib()
    assert L.pipesgd_compress(5, 0x1000, 10, 0x2000, None, None) == -3
    assert L.pipesgd_compress(0, None, 10, 0x2000, None, None) == -1
    assert L.pipesgd_compress(2, 0x1000, 10, 0x2000, None, None) == -1        # QUANT8 needs scales
    assert L.pipesgd_compress(1, 0x1004, 10, 0x2000, None, None) == -2
    assert L.pipesgd_compress(1, None, 0, None, None, None) == 0               # n = 0: no-op
    assert L.pipesgd_decompress(1, 0x2000, None, 10, None, None) == -1
    assert L.pipesgd_decompress(2, 0x2000, 0x3004, 10, 0x1000, None) == -2
    f = C.c_float
    assert L.pipesgd_apply_update(0, 0x1000, None, 10, None, None, f(.1), f(0), f(1), None) == -1
    assert L.pipesgd_apply_update(0, 0x1000, None, 10, 0x2000, None, f(.1), f(.9), f(1), None) == -1   # momentum needs v
    assert L.pipesgd_apply_update(0, 0x1000, None, 10, 0x2008, None, f(.1), f(0), f(1), None) == -2
    assert L.pipesgd_apply_update(3, 0x1000, None, 10, 0x2000, None, f(.1), f(0), f(1), None) == -3
    assert L.pipesgd_apply_update(0, 0x1000, None, 0, 0x2000, None, f(.1), f(0), f(1), None) == 0
    ptrs = (C.c_void_p * 17)(*([0x1000] * 17))
    assert L.pipesgd_apply_update_multi(0, 17, ptrs, None, 10, ptrs, None, f(.1), f(0), f(1), None) == -4
    assert L.pipesgd_apply_update_multi(0, 0, ptrs, None, 10, ptrs, None, f(.1), f(0), f(1), None) == -1
    assert L.pipesgd_pack(None, 3, 3, None) == -1
    assert L.pipesgd_pack(None, 0, 0, None) == 0


def test_static_scratch_capacity_is_checked_on_the_host():
    # needs no device memory: the addresses are never dereferenced
    L = B.lib()
    cap = B.STATIC_SCRATCH_BYTES
    ring_of = lambda mode, n, p: B.make_ring(mode, n, [0x10000] * p, [0x20000] * p, [0x30000] * p)
    call = lambda ring: L.pipesgd_allreduce_direct_static(C.byref(ring), None)
    assert call(ring_of(B.NONE, cap // 4 // 4 + 4096, 4)) == -4
    assert call(ring_of(B.TRUNC16, cap // 2 // 4 + 4096, 4)) == -4
    assert call(ring_of(B.QUANT8, cap // 4, 4)) == -4                 # the payloads alone fill it: no room for scales
    assert call(ring_of(B.NONE, cap, 1)) == -4
    assert call(ring_of(B.TRUNC16, 0, 4)) == 0                        # empty vector: nothing to do
    assert L.pipesgd_allreduce_direct_static(None, None) == -1
    assert call(ring_of(7, 4096, 4)) == -3


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1811_03619_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), fn
                assert "pipesgd_oracle" not in text, fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", fn)).read()
            assert "paper_1811_03619_amd" not in text and "pipesgd.h" not in text, fn


def test_timing_models_follow_the_papers_equations():
    # Eq. 2-4
    assert B.model_sync_time(100, 1.0, 5.0, 3.0) == 900.0
    assert B.model_pipe_ideal_time(100, 2, 1.0, 5.0, 3.0) == 450.0
    assert B.model_pipe_ideal_time(100, 1, 1.0, 5.0, 3.0) == B.model_sync_time(100, 1.0, 5.0, 3.0)
    assert B.model_pipe_time(100, 1.0, 5.0, 3.0) == 600.0          # compute bound
    assert B.model_pipe_time(100, 1.0, 1.0, 3.0) == 300.0          # communication bound
    assert B.model_pipe_time(7, 0.3, 0.4, 0.2) <= B.model_sync_time(7, 0.3, 0.4, 0.2)
    # Eq. 5: AlexNet-sized fp32 gradient over 10 Gb/s Ethernet, p = 4: the bandwidth term alone is
    # 2 * (3/4) * 243,860,896 B / 1.25e9 B/s = 0.29263 s (half of it with 16-bit truncation)
    n_bytes = 60_965_224 * 4
    t = B.model_ring_comm_time(4, n_bytes, 0.0, 1 / 1.25e9, 0.0)
    assert abs(t - 0.292633) < 1e-6
    assert abs(B.model_ring_comm_time(4, n_bytes / 2, 0.0, 1 / 1.25e9, 0.0) - t / 2) < 1e-12
    # all four terms: 2(p-1) alpha + 2((p-1)/p) n beta + ((p-1)/p) n gamma + S
    assert abs(B.model_ring_comm_time(4, 1000.0, 1e-3, 1e-6, 2e-6, 5e-3) - (6e-3 + 1.5e-3 + 1.5e-3 + 5e-3)) < 1e-15
    # Eq. 6 with L segments pays the latency and the synchronisation L times; L = 1 is Eq. 5
    e5 = B.model_ring_comm_time(8, 1e6, 1e-4, 1e-9, 1e-10, 1e-4, 1)
    e6 = B.model_ring_comm_time(8, 1e6, 1e-4, 1e-9, 1e-10, 1e-4, 4)
    assert abs((e6 - e5) - (3 * (2 * 7 * 1e-4 + 1e-4))) < 1e-15
    # Eq. 7
    assert B.model_scaling_efficiency(1.0, 5.0, 3.0) == 1.0
    assert B.model_scaling_efficiency(1.0, 1.0, 4.0) == 0.5


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 and a C program must link and run
    import subprocess
    src = tmp_path / "abi.c"
    src.write_text(r'''
#include <stdio.h>
#include "pipesgd.h"
int main(void) {
    pipesgd_ring ring;
    pipesgd_bucket b[4];
    uint64_t numels[3] = {10, 5000, 3}, offs[3], n_packed = 0;
    int nb = pipesgd_bucket_plan(numels, 3, 4096, b, 4, offs, &n_packed);
    ring.workers = 4;
    printf("%d %llu %llu %llu %s %d\n", nb, (unsigned long long)n_packed,
           (unsigned long long)pipesgd_chunk_elems(60965224ull, ring.workers),
           (unsigned long long)pipesgd_payload_bytes(PIPESGD_TRUNC16, 10), pipesgd_strerror(PIPESGD_ERR_MODE),
           pipesgd_ring_first_send(0, 0));
    return 0;
}
''')
    exe = tmp_path / "abi"
    inc = os.path.join(ROOT, "include")
    libdir = os.path.join(ROOT, "paper_1811_03619_amd")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, str(src),
                           "-L", libdir, "-lpipesgd", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)])
    out = subprocess.check_output([str(exe)], text=True).split()
    # buckets {10}, {5000} (oversized, alone), {3}: starts 0, 4096, 12288 -> packed length 16384
    assert out[:4] == ["3", "16384", "15245312", "20"] and out[-1] == "-1"
