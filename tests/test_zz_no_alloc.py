"""The allocation-free entry point, pipesgd_allreduce_direct_static, against the
entry point it is a variant of (pipesgd_allreduce_direct, whose send buffers the
caller allocates) and against the oracle's one-exchange branch: bit for bit,
through the C ABI, on two calls in a row -- the second on a smaller vector, so
that what the first call left in the shared device array must not matter."""
import numpy as np
import pytest

from paper_1811_03619_amd import binding as B
from paper_1811_03619_amd import workloads as W

pytestmark = pytest.mark.gpu

MODES = [B.NONE, B.TRUNC16, B.QUANT8]


def run_both(orc, mode, p, n, seed, buckets=None):
    from gpu_util import assert_bits_equal, dev_zeros, down, pay_buf, sync, up
    grads = [W.gaussian(n, 1e-3, seed, (mode, r, 0, 0)) for r in range(p)]
    if buckets:                                   # padding between buckets is zero by contract
        keep = np.zeros(n, bool)
        for st, nb in buckets:
            keep[st:st + nb] = True
        for g in grads:
            g[~keep] = 0.0
    ns = B.num_scales(mode, n)
    g_dev = [up(g) for g in grads]
    q8 = mode == B.QUANT8

    def fresh():
        return [pay_buf(mode, n, poison=not buckets) for _ in range(p)], [dev_zeros(ns, fill=None if buckets else -1.0) for _ in range(p)]

    slots_a, scs_a = fresh()
    B.allreduce_direct_static(B.make_ring(mode, n, g_dev, slots_a, scs_a if q8 else None, buckets))
    sync()
    slots_b, scs_b = fresh()
    stage = [pay_buf(mode, n) for _ in range(p)]
    stage_sc = [dev_zeros(ns, fill=-2.0) for _ in range(p)]
    B.allreduce_direct(B.make_ring(mode, n, g_dev, slots_b, scs_b if q8 else None, buckets),
                       B.make_workspace(stage, stage_sc if q8 else None))
    sync()
    for r in range(p):
        assert_bits_equal(down(slots_a[r], mode), down(slots_b[r], mode), f"static vs caller-allocated, payload r={r}")
        if q8:
            assert_bits_equal(down(scs_a[r]), down(scs_b[r]), f"static vs caller-allocated, scales r={r}")
    if not buckets:
        want = orc.allreduce_direct(mode, grads)
        for r in range(p):
            assert_bits_equal(down(slots_a[r], mode), want[r][0], f"static vs oracle, payload r={r}")
            if q8:
                assert_bits_equal(down(scs_a[r]), want[r][1], f"static vs oracle, scales r={r}")
    for g_d, g_h in zip(g_dev, grads):            # gradients are inputs: untouched
        assert_bits_equal(down(g_d), g_h, "gradient")


@pytest.mark.parametrize("mode", MODES)
def test_static_scratch_allreduce_two_calls_in_a_row(orc, mode):
    # 37 tiles and a ragged tail, then a smaller vector whose send buffers start elsewhere in the array
    run_both(orc, mode, 4, 4096 * 37 + 1111, seed=51)
    run_both(orc, mode, 4, 4096 * 5 + 3, seed=52)
    run_both(orc, mode, 3, 4097, seed=53)
    run_both(orc, mode, 1, 9000, seed=54)         # one worker: no send buffers at all


def test_static_scratch_allreduce_with_buckets(orc):
    specs = W.scaled_config(5, 16)
    buckets, offs, N = B.bucket_plan([s.numel for s in specs], 1 << 14)
    assert len(buckets) > 2
    run_both(orc, B.QUANT8, 4, N, seed=55, buckets=buckets)
    run_both(orc, B.TRUNC16, 4, N, seed=56, buckets=buckets)


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_static_scratch_allreduce_replays_from_a_hip_graph(orc, mode):
    # the callers this entry point is for: code under graph capture cannot allocate.  The call is captured
    # together with the update that consumes its result; every replay -- with eager work and synchronisation
    # in between -- is checked against the oracle's width-1 run (AllReduce, then update with that result).
    import torch
    from gpu_util import assert_bits_equal, assert_fp32_close_then_exact, dev_zeros, down, pay_buf, sync, up
    p, n, lr, m = 4, 4096 * 9 + 77, 0.01, 0.9
    grads = [W.gaussian(n, 1e-3, 61, (mode, r, 0, 0)) for r in range(p)]
    w0 = W.gaussian(n, 0.05, 62)
    g_dev = [up(g) for g in grads]
    slots = [pay_buf(mode, n) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, n), fill=-1.0) for _ in range(p)]
    w = [up(w0) for _ in range(p)]
    v = [dev_zeros(n, fill=0.0) for _ in range(p)]
    q8 = mode == B.QUANT8
    ring = B.make_ring(mode, n, g_dev, slots, scs if q8 else None)
    ua = B.UpdateArgs(slots, scs if q8 else None, w, v)
    B.allreduce_direct_static(ring)                  # first call on the device, outside capture: looks the array up
    sync()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        B.allreduce_direct_static(ring)
        B.apply_update_multi(mode, ua, n, lr, m, 1.0)
    sync()
    want = orc.allreduce_direct(mode, grads)
    w_ref, v_ref = w0.copy(), np.zeros(n, np.float32)
    other = torch.zeros(1 << 18, device="cuda:0")
    for rep in range(3):
        for t in slots:                              # the replay must rewrite the result, not find it there
            t.fill_(0x11)
        graph.replay()
        other.add_(1.0)
        sync()
        orc.sgd_update(mode, want[0][0], want[0][1], w_ref, v_ref, lr, m, 1.0)
        for r in range(p):
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r} replay {rep}")
            assert_fp32_close_then_exact(down(w[r]), w_ref, f"w r={r} replay {rep}")
            assert_fp32_close_then_exact(down(v[r]), v_ref, f"v r={r} replay {rep}")
    assert float(other[0]) == 3.0

