"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
element by element on the same seeded inputs.  Sizes span several 4096-element
tiles and a ragged tail; edge cases: empty, one element, fewer elements than
workers, empty ring blocks, 16 workers, special floating-point values.
"""
import os

import numpy as np
import pytest
import torch

from paper_1811_03619_amd import binding as B
from paper_1811_03619_amd import workloads as W
from paper_1811_03619_amd.pipeline import PipeSgdSim

from gpu_util import (DEV, assert_bits_equal, assert_fp32_close_then_exact, dev_zeros, down, pay_buf, sync, up)

pytestmark = pytest.mark.gpu

MODES = [B.NONE, B.TRUNC16, B.QUANT8]
SIZES = [1, 3, 4095, 4096, 4097, 4096 * 5 + 17, 4096 * 64, 1_000_003]


def special_values(n, seed):
    """Gaussian values with zeros, signed zeros, denormals, huge and tiny
    magnitudes and exact rounding ties sprinkled in."""
    x = W.gaussian(n, 0.02, seed)
    rng = np.random.Generator(np.random.Philox(key=seed + 1000))
    specials = np.array([0.0, -0.0, 1e-40, -1e-40, 1.17549435e-38, 1.0e37, -1.0e37, 1e-30, 0.5, 1.5, 2.5, -2.5,
                         127.0, -127.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7], dtype=np.float32)
    k = min(n, max(1, n // 50))
    idx = rng.choice(n, size=k, replace=False)
    x[idx] = specials[rng.integers(0, specials.size, size=k)]
    return x


# ------------------------------------------------------------------ codecs --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("n", SIZES)
def test_compress_decompress(orc, mode, n):
    x = special_values(n, 100 + n % 97) if n > 3 else W.gaussian(n, 1.0, 5)
    want_pay, want_sc = orc.compress(mode, x)
    pay = pay_buf(mode, n)
    ns = B.num_scales(mode, n)
    sc = dev_zeros(ns, fill=-1.0)
    B.compress(mode, up(x), n, pay, sc if mode == B.QUANT8 else None)
    sync()
    assert_bits_equal(down(pay, mode), want_pay, "payload")
    if mode == B.QUANT8:
        assert_bits_equal(down(sc), want_sc, "scales")
    out = dev_zeros(n, fill=float("nan"))
    B.decompress(mode, up(want_pay), up(want_sc) if mode == B.QUANT8 else None, n, out)
    sync()
    assert_bits_equal(down(out), orc.decompress(mode, want_pay, want_sc), "decompressed")


def test_quant8_ties_and_tiny_scales(orc):
    # exact ties (scale 127 -> inverse 1) and a block whose 127/scale overflows
    blk0 = np.zeros(4096, np.float32)
    blk0[:11] = [127.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 125.5, 126.5, -126.5]
    blk1 = np.zeros(4096, np.float32)
    blk1[:4] = [1e-40, 0.0, -5e-41, 1e-38]
    blk2 = np.zeros(4096, np.float32)                         # all-zero block
    x = np.concatenate([blk0, blk1, blk2, np.array([-3.0], np.float32)])
    want_pay, want_sc = orc.compress(B.QUANT8, x)
    pay, sc = pay_buf(B.QUANT8, x.size), dev_zeros(4, fill=-1.0)
    B.compress(B.QUANT8, up(x), x.size, pay, sc)
    sync()
    got = down(pay)
    assert got[:11].tolist() == [127, 0, 2, 2, 4, 0, -2, -2, 126, 126, -126]
    assert got[4096:4100].tolist() == [0, 0, 0, 3]
    assert_bits_equal(got, want_pay, "payload")
    assert_bits_equal(down(sc), want_sc, "scales")


# -------------------------------------------------------------------- ring --

def ring_buffers(mode, grads, poison=True):
    p, n = len(grads), grads[0].size
    g_dev = [up(g) for g in grads]
    slots = [pay_buf(mode, n, poison) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, n), fill=-1.0) for _ in range(p)]
    return g_dev, slots, scs


def make_grads(p, n, seed, sigma=1e-3):
    return [W.gaussian(n, sigma, seed, (11, r, 0, 0)) for r in range(p)]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("p,n", [(4, 4096 * 8 + 1234), (3, 4096 * 3 + 1), (2, 5000), (4, 4097)])
def test_ring_stepwise_against_oracle_states(orc, mode, p, n):
    grads = make_grads(p, n, 7 + p)
    g_dev, slots, scs = ring_buffers(mode, grads)
    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    R = orc.Ring(mode, grads)
    ce = R.ce
    assert ce == B.chunk_elems(n, p)

    def check_chunk(r, c, want_vals, what):
        lo, hi = min(n, c * ce), min(n, (c + 1) * ce)
        wp, ws = orc.compress(mode, want_vals[lo:hi])
        assert_bits_equal(down(slots[r], mode)[lo:hi], wp, what)
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r])[lo // 4096: lo // 4096 + ws.size], ws, what + " scales")

    B.ring_first_send(ring)
    sync()
    if mode != B.NONE:
        for r in range(p):
            check_chunk(r, r, grads[r], f"first send r={r}")
    for s in range(p - 1):
        B.ring_reduce_scatter_step(ring, s)
        R.reduce_scatter_step(s)
        sync()
        for r in range(p):
            check_chunk(r, (r - s - 1) % p, R.work(r), f"reduce-scatter round {s} r={r}")
    R.seal()
    for s in range(p - 1):
        B.ring_allgather_step(ring, s)
        R.allgather_step(s)
        sync()
        for r in range(p):
            c = (r - s) % p
            lo, hi = min(n, c * ce), min(n, (c + 1) * ce)
            assert_bits_equal(down(slots[r], mode)[lo:hi], R.result(r)[0][lo:hi], f"all-gather round {s} r={r}")
    for r in range(p):
        wp, ws = R.result(r)
        assert_bits_equal(down(slots[r], mode), wp, f"result r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), ws, f"result scales r={r}")
    R.close()


@pytest.mark.parametrize("schedule", [B.STEPWISE, B.FUSED])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("p,n", [(1, 9000), (2, 4096 * 4), (3, 50001), (4, 1), (4, 3), (4, 4096 * 21 + 77),
                                 (5, 12289), (8, 300007), (16, 70001)])
def test_allreduce_sim_equals_oracle(orc, schedule, mode, p, n):
    grads = [special_values(n, 31 * p + r) if n > 100 else W.gaussian(n, 1.0, 3, (0, r, 0, 0)) for r in range(p)]
    want = orc.allreduce(mode, grads)
    g_dev, slots, scs = ring_buffers(mode, grads)
    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_sim(ring, schedule)
    sync()
    for r in range(p):
        if mode == B.NONE:
            assert_fp32_close_then_exact(down(slots[r]), want[r][0], f"sum r={r}")
        else:
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
    for r in range(p):
        assert_bits_equal(down(g_dev[r]), grads[r], "gradients must not be modified")


@pytest.mark.parametrize("mode", MODES)
def test_empty_vector_is_a_no_op(orc, mode):
    p = 4
    g_dev = [dev_zeros(0) for _ in range(p)]
    slots = [pay_buf(mode, 0) for _ in range(p)]
    scs = [dev_zeros(0) for _ in range(p)]
    ring = B.make_ring(mode, 0, g_dev, slots, scs)
    B.allreduce_sim(ring, B.STEPWISE)
    B.allreduce_sim(ring, B.FUSED)
    B.apply_update(mode, slots[0], scs[0], 0, dev_zeros(0), dev_zeros(0), 0.1, 0.9)
    sync()


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_hand_worked_hop_cases(orc, mode):
    # the two-worker cases of the oracle's pins, through the HIP path: the
    # sender's operand is compressed, the receiver's is full precision
    ce = 4096
    g0, g1 = np.zeros(2 * ce, np.float32), np.zeros(2 * ce, np.float32)
    if mode == B.TRUNC16:
        g0[0] = g0[ce] = 1.0
        g1[0] = g1[ce] = -(2.0 ** -8 + 2.0 ** -16)
    else:
        for base in (0, ce):
            g0[base], g0[base + 1] = 127.0, 10.4
            g1[base], g1[base + 1] = 0.0, 20.4
    for schedule in (B.STEPWISE, B.FUSED):
        g_dev, slots, scs = ring_buffers(mode, [g0, g1])
        ring = B.make_ring(mode, 2 * ce, g_dev, slots, scs if mode == B.QUANT8 else None)
        B.allreduce_sim(ring, schedule)
        sync()
        for r in range(2):
            got = down(slots[r], mode)
            if mode == B.TRUNC16:
                assert (got[0], got[ce]) == (0x3F7E, 0x3F7F)
            else:
                assert (got[0], got[1], got[ce], got[ce + 1]) == (127, 30, 127, 31)
                assert down(scs[r]).tolist() == [127.0, 127.0]


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_precompressed_locals_variant(orc, mode):
    # Alg. 1 compresses the whole local gradient before the AllReduce; with the
    # exported codec calls a caller gets that variant by round-tripping each
    # local gradient first.
    p, n = 4, 4096 * 6 + 99
    grads = make_grads(p, n, 77)
    rt = [orc.decompress(mode, *orc.compress(mode, g)) for g in grads]
    want = orc.allreduce(mode, rt)
    g_dev, slots, scs = ring_buffers(mode, grads)
    tmp_pay, tmp_sc = pay_buf(mode, n), dev_zeros(B.num_scales(mode, n))
    rt_dev = [dev_zeros(n) for _ in range(p)]
    for r in range(p):
        B.compress(mode, g_dev[r], n, tmp_pay, tmp_sc if mode == B.QUANT8 else None)
        B.decompress(mode, tmp_pay, tmp_sc if mode == B.QUANT8 else None, n, rt_dev[r])
    ring = B.make_ring(mode, n, rt_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_sim(ring, B.STEPWISE)
    sync()
    for r in range(p):
        assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")


# --------------------------------------------------------------- bucketing --

@pytest.mark.parametrize("schedule", [B.STEPWISE, B.FUSED])
@pytest.mark.parametrize("mode", MODES)
def test_bucketed_allreduce(orc, schedule, mode):
    # ResNet-50's tensor list at 1/8 of each large dimension: 161 tensors, many
    # tiny ones, buckets of 64K elements
    p = 4
    specs = W.scaled_config(5, 8)
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 16)
    ob, oo, oN = orc.bucket_plan(numels, 1 << 16)
    assert (buckets, offs, N) == (ob, oo, oN) and 4 < len(buckets) <= B.MAX_BUCKETS
    packed = [orc.pack(W.gradient_tensors_for(specs, 5, r, seed=3), offs, N) for r in range(p)]
    want = orc.allreduce_bucketed(mode, packed, buckets)
    g_dev = [up(g) for g in packed]
    slots = [pay_buf(mode, N, poison=False) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    ring = B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
    B.allreduce_sim(ring, schedule)
    sync()
    for r in range(p):
        assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")


def test_pack_and_unpack(orc):
    specs = W.scaled_config(5, 8)[:60] + [W.TensorSpec("odd", (4097,), 1), W.TensorSpec("one", (1,), 1),
                                          W.TensorSpec("big", (4096 * 9,), 1)]
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 15)
    p = 2
    tens = [W.gradient_tensors_for(specs, 6, r, seed=9) for r in range(p)]
    # all tensors of a worker live in one allocation at odd (4-byte aligned) offsets
    starts = np.cumsum([0] + [ne + 1 for ne in numels])
    arena = [dev_zeros(int(starts[-1]) + 4) for _ in range(p)]
    for r in range(p):
        host = np.zeros(int(starts[-1]) + 4, np.float32)
        for ti, t in enumerate(tens[r]):
            host[starts[ti]:starts[ti] + t.size] = t
        arena[r].copy_(torch.from_numpy(host))
    packed = [dev_zeros(N) for _ in range(p)]
    tptr, pptr, ne = [], [], []
    for r in range(p):
        for ti, n_i in enumerate(numels):
            tptr.append(arena[r].data_ptr() + 4 * int(starts[ti]))
            pptr.append(packed[r].data_ptr() + 4 * offs[ti])
            ne.append(n_i)
    tab, total = B.segments_prepare(tptr, pptr, ne)
    tab_dev = torch.frombuffer(bytearray(bytes(tab)), dtype=torch.uint8).to(DEV)
    B.pack(tab_dev, len(ne), total)
    sync()
    for r in range(p):
        assert_bits_equal(down(packed[r]), orc.pack(tens[r], offs, N), f"packed r={r}")
    # scatter back into a cleared arena
    for r in range(p):
        arena[r].zero_()
    B.unpack(tab_dev, len(ne), total)
    sync()
    for r in range(p):
        host = down(arena[r])
        for ti, t in enumerate(tens[r]):
            assert_bits_equal(host[starts[ti]:starts[ti] + t.size], t, f"unpacked r={r} t={ti}")
            assert host[starts[ti] + t.size] == 0.0            # the gap after each tensor stays untouched


# ------------------------------------------------------------------ update --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("momentum,grad_scale", [(0.0, 1.0), (0.9, 1.0), (0.9, 0.25), (0.0, 0.25)])
@pytest.mark.parametrize("n", [1, 4096, 4096 * 7 + 321])
def test_apply_update(orc, mode, momentum, grad_scale, n):
    g = W.gaussian(n, 3e-4, 41)
    pay, sc = orc.compress(mode, g)
    w0, v0 = W.gaussian(n, 1.0, 43), W.gaussian(n, 0.1, 45)
    w_ref, v_ref = w0.copy(), v0.copy()
    orc.sgd_update(mode, pay, sc, w_ref, v_ref if momentum else None, 0.01, momentum, grad_scale)
    w, v = up(w0), up(v0)
    B.apply_update(mode, up(pay), up(sc) if mode == B.QUANT8 else None, n, w, v if momentum else None,
                   0.01, momentum, grad_scale)
    sync()
    assert_fp32_close_then_exact(down(w), w_ref, "w")
    assert_fp32_close_then_exact(down(v), v_ref, "v")          # untouched when momentum == 0


def test_apply_update_single_rounding_cases(orc):
    # the fused-multiply-add pins of the oracle, on the GPU
    g, w = up(np.array([1 + 2.0 ** -12], np.float32)), up(np.array([1 + 2.0 ** -11], np.float32))
    B.apply_update(B.NONE, g, None, 1, w, None, 1 + 2.0 ** -12)
    sync()
    assert down(w)[0] == np.float32(-2.0 ** -24)
    v = up(np.array([1 + 2.0 ** -12], np.float32))
    g = up(np.array([-(1 + 2.0 ** -11)], np.float32))
    w = up(np.array([0.0], np.float32))
    B.apply_update(B.NONE, g, None, 1, w, v, 2.0, 1 + 2.0 ** -12)
    sync()
    assert down(v)[0] == np.float32(2.0 ** -24) and down(w)[0] == np.float32(-2.0 ** -23)


@pytest.mark.parametrize("mode", MODES)
def test_apply_update_multi_all_replicas(orc, mode):
    p, n = 4, 4096 * 3 + 5
    pays = [orc.compress(mode, W.gaussian(n, 1e-3, 60 + r)) for r in range(p)]
    w0 = [W.gaussian(n, 1.0, 70 + r) for r in range(p)]
    v0 = [W.gaussian(n, 0.1, 80 + r) for r in range(p)]
    w, v = [up(x) for x in w0], [up(x) for x in v0]
    pd = [up(x[0]) for x in pays]
    sd = [up(x[1]) for x in pays] if mode == B.QUANT8 else None
    B.apply_update_multi(mode, B.UpdateArgs(pd, sd, w, v), n, 0.02, 0.9, 1.0)
    sync()
    for r in range(p):
        orc.sgd_update(mode, pays[r][0], pays[r][1], w0[r], v0[r], 0.02, 0.9, 1.0)
        assert_fp32_close_then_exact(down(w[r]), w0[r], f"w r={r}")
        assert_fp32_close_then_exact(down(v[r]), v0[r], f"v r={r}")


# ------------------------------------------------------- pipelined driver --

def run_both(orc, mode, grad_fn, w0, p, iters, lr, momentum, width, buckets=None, schedule=B.STEPWISE):
    n = w0.size
    sim = PipeSgdSim(mode, p, n, lr, momentum, 1.0, width, buckets, schedule)
    sim.set_model(w0)
    for t in range(1, iters + 1):
        ws = [sim.model(r) for r in range(p)]
        sim.set_gradients([grad_fn(r, ws[r], t) for r in range(p)])
        sim.iteration()
    sync()
    ws_ref, vs_ref = orc.pipe_sgd_run(mode, grad_fn, w0, p, iters, lr, momentum, 1.0, width, buckets)
    return sim, ws_ref, vs_ref


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("width", [3, 4])
def test_wider_pipelines_follow_algorithm_1(orc, mode, width):
    # Alg. 1 with iteration dependency K = width > 2: the update of iteration t applies the
    # aggregated gradient of iteration t-(K-1); the first K-1 updates are no-ops.  The gradient
    # depends on the model, so a wrong staleness changes every later iterate.
    p, n = 4, 4096 * 5 + 19
    wstar = W.gaussian(n, 1.0, 31, (mode, 0, 0, 0))
    grad_fn = lambda r, w, t: ((w - wstar) * np.float32(0.25 + 0.1 * r)).astype(np.float32)
    w0 = np.zeros(n, np.float32)
    sim, ws_ref, vs_ref = run_both(orc, mode, grad_fn, w0, p, 8, 0.05, 0.5, width)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs_ref[r], f"v r={r}")
    assert not np.array_equal(ws_ref[0], w0)


def test_config1_quadratic_ten_iterations(orc):
    # K = 4 workers, 1,048,576 parameters, lr 0.01, no momentum, no compression,
    # loss 0.5*||w - w*||^2: closed form s_10 = 0.6825982976 for staleness 1
    p, n = 4, 1 << 20
    wstar = W.gaussian(n, 1.0, 1, (1, 9, 0, 0))
    grad_fn = lambda r, w, t: (w - wstar).astype(np.float32)
    sim, ws_ref, _ = run_both(orc, B.NONE, grad_fn, np.zeros(n, np.float32), p, 10, 0.01, 0.0, 2)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
    ratio = (sim.model(0).astype(np.float64) - wstar) / (0.0 - wstar.astype(np.float64))
    assert abs(float(np.median(ratio)) - 0.6825982976) < 1e-6
    # part A of the same config: one AllReduce of N(0, 1e-3) vectors
    grads = [W.flat_gradient(1, r, seed=1) for r in range(p)]
    want = orc.allreduce(B.NONE, grads)
    sim.set_gradients(grads)
    slot = sim.allreduce()
    sync()
    for r in range(p):
        assert_fp32_close_then_exact(sim.result(r, slot)[0], want[r][0], f"sum r={r}")


def test_config2_mlp_momentum(orc):
    p = 4
    specs = W.config_tensors(2)
    n = sum(s.numel for s in specs)
    assert n == 648010
    grad_fn = lambda r, w, t: W.flat_gradient(2, r, seed=2, iteration=t)
    w0 = W.gaussian(n, 0.05, 2, (2, 99, 0, 0))
    sim, ws_ref, vs_ref = run_both(orc, B.NONE, grad_fn, w0, p, 4, 0.01, 0.9, 2)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs_ref[r], f"v r={r}")


@pytest.mark.parametrize("mode,cfg,shrink", [(B.TRUNC16, 3, 6), (B.QUANT8, 4, 8)])
@pytest.mark.parametrize("width", [1, 2])
def test_scaled_alexnet_and_vgg_pipelines(orc, mode, cfg, shrink, width):
    p = 4
    specs = W.scaled_config(cfg, shrink)
    n = sum(s.numel for s in specs)
    grad_fn = lambda r, w, t: np.concatenate(W.gradient_tensors_for(specs, cfg, r, seed=4, iteration=t))
    w0 = W.gaussian(n, 0.05, 4, (cfg, 99, 0, 0))
    sim, ws_ref, vs_ref = run_both(orc, mode, grad_fn, w0, p, 3, 0.01, 0.9, width)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs_ref[r], f"v r={r}")


@pytest.mark.parametrize("mode", [B.NONE, B.TRUNC16])
@pytest.mark.parametrize("schedule", [B.STEPWISE, B.FUSED])
def test_scaled_resnet_bucketed_pipeline(orc, mode, schedule):
    p = 4
    specs = W.scaled_config(5, 4)
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 17)
    grad_fn = lambda r, w, t: orc.pack(W.gradient_tensors_for(specs, 5, r, seed=5, iteration=t), offs, N)
    w0 = orc.pack(W.gradient_tensors_for(specs, 55, 0, seed=5), offs, N)
    sim, ws_ref, vs_ref = run_both(orc, mode, grad_fn, w0, p, 3, 0.01, 0.9, 2, buckets, schedule)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs_ref[r], f"v r={r}")


# ------------------------------------------------- every launch geometry --

GEOS = [(64, 4), (128, 2), (128, 4), (256, 1), (256, 2), (256, 4), (512, 1), (512, 2), (1024, 1)]
KINDS = [B.K_FIRST_SEND, B.K_REDUCE_SCATTER, B.K_ALLGATHER, B.K_FUSED, B.K_UPDATE, B.K_COMPRESS, B.K_DECOMPRESS,
         B.K_DIRECT_REDUCE]


@pytest.fixture
def restore_launch_configs():
    saved = {(k, m): B.get_launch_config(k, m) for k in KINDS for m in MODES}
    yield
    for (k, m), c in saved.items():
        B.set_launch_config(k, m, *c)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("geo", GEOS)
@pytest.mark.parametrize("lds", [0, 48 * 1024, 159 * 1024])
def test_every_launch_geometry_gives_the_same_bits(orc, restore_launch_configs, mode, geo, lds):
    # results must not depend on the tuning table: run the whole path with one
    # geometry for every kernel family (where that family supports it) on a
    # ragged, bucketed input and compare with the oracle
    used = []
    for kind in KINDS:
        rc = B.lib().pipesgd_set_launch_config(kind, mode, geo[0], geo[1], lds)
        assert rc in (0, -1)
        used.append(rc == 0)
    if not any(used):
        pytest.skip("geometry not applicable to this mode")
    p = 3
    numels = [5000, 4096, 12289, 77, 1, 30000]
    buckets, offs, N = B.bucket_plan(numels, 20000)
    tens = [[special_values(ne, 7 * r + ti + 1) if ne > 100 else W.gaussian(ne, 1.0, r, (0, ti, 0, 0))
             for ti, ne in enumerate(numels)] for r in range(p)]
    packed = [orc.pack(t, offs, N) for t in tens]
    want = orc.allreduce_bucketed(mode, packed, buckets)
    for schedule in (B.STEPWISE, B.FUSED):
        g_dev, slots, scs = ring_buffers(mode, packed, poison=False)
        ring = B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
        B.allreduce_sim(ring, schedule)
        sync()
        for r in range(p):
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r} schedule={schedule}")
            if mode == B.QUANT8:
                assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
    # the one-exchange schedule (its owner-side kernel has a geometry entry of its own), per bucket as the ring
    want_d = [np.zeros(N, dtype=orc.payload_dtype(mode)) for _ in range(p)]
    for (st, nb) in buckets:
        res = orc.allreduce_direct(mode, [g[st:st + nb] for g in packed])
        for r in range(p):
            want_d[r][st:st + nb] = res[r][0]
    g_dev, slots, scs = ring_buffers(mode, packed, poison=False)
    stage = [pay_buf(mode, N) for _ in range(p)]
    stage_sc = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    B.allreduce_direct(B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets),
                       B.make_workspace(stage, stage_sc if mode == B.QUANT8 else None))
    sync()
    for r in range(p):
        assert_bits_equal(down(slots[r], mode), want_d[r], f"one-exchange payload r={r}")
    # codec + update on a flat ragged vector
    n = 4096 * 3 + 1234
    x = special_values(n, 99)
    wp, ws = orc.compress(mode, x)
    pay, sc = pay_buf(mode, n), dev_zeros(B.num_scales(mode, n), fill=-1.0)
    B.compress(mode, up(x), n, pay, sc if mode == B.QUANT8 else None)
    out = dev_zeros(n, fill=float("nan"))
    B.decompress(mode, pay, sc if mode == B.QUANT8 else None, n, out)
    w0, v0 = W.gaussian(n, 1.0, 43), W.gaussian(n, 0.1, 45)
    w, v = up(w0), up(v0)
    B.apply_update(mode, pay, sc if mode == B.QUANT8 else None, n, w, v, 0.01, 0.9, 1.0)
    sync()
    assert_bits_equal(down(pay, mode), wp, "payload")
    if mode == B.QUANT8:
        assert_bits_equal(down(sc), ws, "scales")
    assert_bits_equal(down(out), orc.decompress(mode, wp, ws), "decompressed")
    orc.sgd_update(mode, wp, ws, w0, v0, 0.01, 0.9, 1.0)
    assert_fp32_close_then_exact(down(w), w0, "w")
    assert_fp32_close_then_exact(down(v), v0, "v")


def test_two_host_threads_launch_while_a_third_retunes(orc, restore_launch_configs):
    # The library keeps one piece of shared state, the launch-geometry table, one atomic word per entry: two
    # host threads driving independent rings on their own streams while a third thread keeps changing
    # geometries must each get the oracle's bits (results never depend on the geometry, and no launch may see
    # half of an old and half of a new entry).
    import threading
    mode, p, n, iters = B.TRUNC16, 4, 4096 * 23 + 321, 25
    jobs = []
    for j in range(2):
        grads = [W.gaussian(n, 1e-3, 90 + j, (j, r, 0, 0)) for r in range(p)]
        g_dev, slots, scs = ring_buffers(mode, grads)
        w0 = W.gaussian(n, 0.05, 95 + j)
        w, v = [up(w0) for _ in range(p)], [dev_zeros(n, fill=0.0) for _ in range(p)]
        jobs.append(dict(grads=grads, ring=B.make_ring(mode, n, g_dev, slots, None), slots=slots, w0=w0, w=w, v=v,
                         ua=B.UpdateArgs(slots, None, w, v), stream=torch.cuda.Stream(), keep=g_dev))
    sync()
    stop, errors = threading.Event(), []

    def retune():
        geos = [(64, 4), (128, 2), (128, 4), (256, 1), (256, 2), (256, 4), (512, 1), (512, 2), (1024, 1)]
        i = 0
        while not stop.is_set():
            t, q = geos[i % len(geos)]
            for kind in (B.K_FIRST_SEND, B.K_REDUCE_SCATTER, B.K_UPDATE, B.K_ALLGATHER):
                try:
                    B.set_launch_config(kind, mode, t, q, (i % 3) * 32768)
                except B.PipeSgdError:
                    pass                                  # a geometry this kind does not take: table unchanged
            i += 1

    def drive(job):
        try:
            for _ in range(iters):
                B.allreduce_sim(job["ring"], B.STEPWISE, job["stream"])
                B.apply_update_multi(mode, job["ua"], n, 0.01, 0.9, 1.0, job["stream"])
            job["stream"].synchronize()
        except Exception as e:                            # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=retune)] + [threading.Thread(target=drive, args=(job,)) for job in jobs]
    for t in threads:
        t.start()
    for t in threads[1:]:
        t.join()
    stop.set()
    threads[0].join()
    sync()
    assert not errors, errors
    for job in jobs:
        want = orc.allreduce(mode, job["grads"])
        w_ref, v_ref = job["w0"].copy(), np.zeros(n, np.float32)
        for _ in range(iters):
            orc.sgd_update(mode, want[0][0], None, w_ref, v_ref, 0.01, 0.9, 1.0)
        for r in range(p):
            assert_bits_equal(down(job["slots"][r], mode), want[r][0], f"payload r={r}")
            assert_fp32_close_then_exact(down(job["w"][r]), w_ref, f"w r={r}")
            assert_fp32_close_then_exact(down(job["v"][r]), v_ref, f"v r={r}")


def test_launch_config_validation():
    L = B.lib()
    assert L.pipesgd_set_launch_config(99, 0, 256, 4, 0) == -1
    assert L.pipesgd_set_launch_config(B.K_UPDATE, 5, 256, 4, 0) == -3
    assert L.pipesgd_set_launch_config(B.K_UPDATE, 0, 100, 4, 0) == -1           # unknown geometry
    assert L.pipesgd_set_launch_config(B.K_UPDATE, 0, 256, 4, 200 * 1024) == -1  # more LDS than a CU has
    assert L.pipesgd_set_launch_config(B.K_REDUCE_SCATTER, B.QUANT8, 256, 1, 0) == -1   # range needs a whole block
    assert L.pipesgd_set_launch_config(B.K_ALLGATHER, B.QUANT8, 256, 4, 0) == -1        # 16 KiB > a tile's 4 KiB payload
    t, q, l = B.get_launch_config(B.K_UPDATE, 0)
    assert (t * q) in (256, 512, 1024) and l >= 0


# -------------------------------------- pipelining within the AllReduce --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("p,n,segments", [(4, 4096 * 37 + 555, 4), (4, 4096 * 37 + 555, 1), (3, 50001, 3),
                                          (2, 4096 * 8, 64), (1, 9000, 2), (5, 12289, 2), (8, 300007, 5)])
@pytest.mark.parametrize("two_streams", [True, False])
def test_allreduce_pipelined_equals_oracle(orc, mode, p, n, segments, two_streams):
    grads = [special_values(n, 17 * p + r) for r in range(p)]
    want = orc.allreduce(mode, grads)
    g_dev, slots, scs = ring_buffers(mode, grads)
    recv = [pay_buf(mode, n) for _ in range(p)]
    recv_sc = [dev_zeros(B.num_scales(mode, n), fill=-2.0) for _ in range(p)]
    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    ov = B.Overlap()
    wire = torch.cuda.Stream() if two_streams else None
    for rep in range(2):                       # the second call reuses the events
        if rep == 1:
            for t in slots:
                t.fill_(0x33 if mode != B.NONE else 7.0)
        B.allreduce_pipelined(ring, B.make_workspace(recv, recv_sc if mode == B.QUANT8 else None), segments, ov,
                              None, wire if two_streams else None, wire_workgroups=(0 if rep == 0 else 3),
                              link_us_per_mib=(0.0 if rep == 0 else 20.0))
        sync()
        for r in range(p):
            if mode == B.NONE:
                assert_fp32_close_then_exact(down(slots[r]), want[r][0], f"sum r={r} rep={rep}")
            else:
                assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r} rep={rep}")
            if mode == B.QUANT8:
                assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r} rep={rep}")
    ov.close()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("segments", [1, 3, 7])
def test_allreduce_pipelined_with_buckets(orc, mode, segments):
    # sub-blocks are tile ranges counted across buckets: some sub-blocks span a bucket boundary
    p = 4
    specs = W.scaled_config(5, 8)
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 16)
    assert len(buckets) > 3
    packed = [orc.pack(W.gradient_tensors_for(specs, 5, r, seed=6), offs, N) for r in range(p)]
    want = orc.allreduce_bucketed(mode, packed, buckets)
    g_dev = [up(g) for g in packed]
    slots = [pay_buf(mode, N, poison=False) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    recv = [pay_buf(mode, N) for _ in range(p)]
    recv_sc = [dev_zeros(B.num_scales(mode, N), fill=-2.0) for _ in range(p)]
    ring = B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
    ov, rt = B.Overlap(), B.Runtime()
    B.allreduce_pipelined(ring, B.make_workspace(recv, recv_sc if mode == B.QUANT8 else None), segments, ov, rt.stream(0), rt.stream(1),
                          link_us_per_mib=10.0)
    rt.sync()
    sync()
    for r in range(p):
        if mode == B.NONE:
            assert_fp32_close_then_exact(down(slots[r]), want[r][0], f"sum r={r}")
        else:
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")
    ov.close()
    rt.close()


def test_allreduce_pipelined_rejects_bad_arguments():
    n = 4096 * 4
    g = [dev_zeros(n) for _ in range(2)]
    slots = [pay_buf(B.TRUNC16, n) for _ in range(2)]
    recv = [pay_buf(B.TRUNC16, n) for _ in range(2)]
    ov = B.Overlap()
    ring = B.make_ring(B.TRUNC16, n, g, slots, None)
    with pytest.raises(B.PipeSgdError):
        B.allreduce_pipelined(ring, B.make_workspace(recv), 0, ov)
    with pytest.raises(B.PipeSgdError):
        B.allreduce_pipelined(ring, B.make_workspace([recv[0], None]), 2, ov)
    sync()


# ------------------------------------------ Algorithm 1's two-thread runtime --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("width,schedule", [(1, B.STEPWISE), (2, B.STEPWISE), (3, B.STEPWISE), (5, B.STEPWISE),
                                            (1, B.FUSED), (2, B.FUSED)])
def test_two_stream_runtime_matches_oracle(orc, mode, width, schedule):
    p, n, lr, m, iters = 4, 4096 * 11 + 77, 0.01, 0.9, 5 if width <= 2 else 9
    grad_fn = lambda r, w, t: W.gaussian(n, 1e-3, 21, (mode, r, t, 0))
    w0 = W.gaussian(n, 0.05, 23)
    K = max(width, 2)
    sim = PipeSgdSim(mode, p, n, lr, m, 1.0, K)          # K slot sets (two also for the synchronous case)
    sim.set_model(w0)
    sync()
    rt = B.Runtime()
    for t in range(1, iters + 1):
        rt.sync()                                        # gradients change: the previous AllReduce must be done
        sim.set_gradients([grad_fn(r, None, t) for r in range(p)])
        sync()
        cur = t % K
        rt.iteration(sim.rings[cur], sim.updates[(cur + 1) % K], sim.updates[cur], schedule, width, lr, m, 1.0,
                     compute_us=150.0, compute_workgroups=8, time_update=(t % 2 == 1))
    rt.sync()
    total_ms, timed = rt.update_time()                   # every other update launch was bracketed by timing events
    assert timed == (iters + 1) // 2 and 0.0 < total_ms < 50.0 * timed
    assert rt.update_time() == (0.0, 0)                  # read out and started anew
    ws, vs = orc.pipe_sgd_run(mode, grad_fn, w0, p, iters, lr, m, 1.0, width)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs[r], f"v r={r}")
    rt.close()


@pytest.mark.parametrize("compute_us,wire_us", [(0.0, 0.0), (0.0, 400.0), (400.0, 0.0), (60.0, 500.0), (500.0, 60.0)])
@pytest.mark.parametrize("width", [2, 3])
def test_two_stream_runtime_is_insensitive_to_timing(orc, compute_us, wire_us, width):
    # whichever stream runs ahead, the ready marks must order every read after the write it needs:
    # the result never depends on how long the compute stand-in or the network stand-in takes.
    # The gradients are double-buffered here so that the host never has to wait between iterations.
    mode, p, n, lr, m, iters = B.TRUNC16, 4, 4096 * 7 + 99, 0.02, 0.9, 10
    grad_fn = lambda r, w, t: W.gaussian(n, 1e-3, 27, (width, r, t, 0))
    w0 = W.gaussian(n, 0.05, 29)
    K = max(width, 2)
    sim = PipeSgdSim(mode, p, n, lr, m, 1.0, K)
    sim.set_model(w0)
    g_sets = [[up(grad_fn(r, None, t)) for r in range(p)] for t in range(1, iters + 1)]   # one set per iteration
    rings = [[B.make_ring(mode, n, g_sets[t], sim.slots[i], None) for i in range(K)] for t in range(iters)]
    sync()
    rt = B.Runtime()
    for t in range(1, iters + 1):
        cur = t % K
        rt.iteration(rings[t - 1][cur], sim.updates[(cur + 1) % K], sim.updates[cur], B.STEPWISE, width, lr, m, 1.0,
                     compute_us=compute_us, compute_workgroups=4, wire_us=wire_us)
    rt.sync()
    ws, vs = orc.pipe_sgd_run(mode, grad_fn, w0, p, iters, lr, m, 1.0, width)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs[r], f"v r={r}")
    rt.close()


def test_runtime_rejects_widths_it_has_no_events_for():
    sim = PipeSgdSim(B.NONE, 2, 4096 * 2, 0.01, 0.0, 1.0, 2)
    rt = B.Runtime()
    for width in (0, -1, 8, 100):
        with pytest.raises(B.PipeSgdError):
            rt.iteration(sim.rings[0], sim.updates[1], sim.updates[0], B.STEPWISE, width, 0.01, 0.0)
    rt.sync()
    rt.close()


@pytest.mark.parametrize("width", [1, 2])
def test_runtime_rejected_call_enqueues_nothing_and_the_runtime_goes_on(orc, width):
    # Every field of the iteration is checked before the first launch or event record: a call with one bad
    # field returns its error with nothing in flight (the slots the AllReduce would write keep their poison),
    # the iteration count is not advanced, and the same iteration issued correctly afterwards gives the oracle's bits.
    import ctypes as C
    mode, p, n, lr, m, iters = B.TRUNC16, 4, 4096 * 6 + 33, 0.01, 0.9, 5
    grad_fn = lambda r, w, t: W.gaussian(n, 1e-3, 31, (width, r, t, 0))
    w0 = W.gaussian(n, 0.05, 33)
    sim = PipeSgdSim(mode, p, n, lr, m, 1.0, 2)
    sim.set_model(w0)
    sync()
    rt = B.Runtime()
    L = B.lib()

    def make_iter(ring, stale, fresh):
        it = B.RuntimeIter()
        it.ring = C.pointer(ring)
        it.schedule, it.width, it.replicas, it.compute_workgroups = B.STEPWISE, width, p, 2
        it.compute_us, it.wire_us, it.lr, it.momentum, it.grad_scale, it.flags = 20.0, 10.0, lr, m, 1.0, 0
        it.stale_g_sum_c = C.cast(stale.g_sum_c, C.c_void_p)
        it.fresh_g_sum_c = C.cast(fresh.g_sum_c, C.c_void_p)
        it.w, it.v = C.cast(stale.w, C.c_void_p), C.cast(stale.v, C.c_void_p)
        return it

    used = "fresh_g_sum_c" if width == 1 else "stale_g_sum_c"
    bad_w = (C.c_void_p * p)(*[sim.w[r].data_ptr() + (4 if r == 2 else 0) for r in range(p)])
    mutations = [
        (lambda it: setattr(it, "w", None), -1),
        (lambda it: setattr(it, "v", None), -1),                       # momentum without v
        (lambda it: setattr(it, used, None), -1),
        (lambda it: setattr(it, "w", C.cast(bad_w, C.c_void_p)), -2),
        (lambda it: setattr(it, "replicas", 0), -1),
        (lambda it: setattr(it, "replicas", 17), -4),
        (lambda it: setattr(it, "compute_us", -1.0), -1),
        (lambda it: setattr(it, "compute_us", 2.0e6), -1),
        (lambda it: setattr(it, "wire_us", float("nan")), -1),
        (lambda it: setattr(it, "compute_workgroups", 70000), -1),
        (lambda it: setattr(it, "schedule", 7), -3),
        (lambda it: setattr(it, "flags", 2), -1),
    ]
    if width >= 2:      # the stale slot set may not be the one the AllReduce writes: the two streams would race
        mutations.append((lambda it: setattr(it, "stale_g_sum_c", it.fresh_g_sum_c), -1))
    for t in range(1, iters + 1):
        rt.sync()
        sim.set_gradients([grad_fn(r, None, t) for r in range(p)])
        cur = t % 2
        if t == 3:
            for r in range(p):
                sim.slots[cur][r].fill_(0x5A5A)
            sync()
            for mutate, want_rc in mutations:
                it = make_iter(sim.rings[cur], sim.updates[1 - cur], sim.updates[cur])
                mutate(it)
                assert L.pipesgd_runtime_iteration(rt.handle, C.byref(it)) == want_rc, want_rc
            rt.sync()
            sync()
            for r in range(p):                                         # the AllReduce was never enqueued
                assert bool((sim.slots[cur][r] == 0x5A5A).all()), r
        sync()
        it = make_iter(sim.rings[cur], sim.updates[1 - cur], sim.updates[cur])
        assert L.pipesgd_runtime_iteration(rt.handle, C.byref(it)) == 0
    rt.sync()
    ws, vs = orc.pipe_sgd_run(mode, grad_fn, w0, p, iters, lr, m, 1.0, width)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs[r], f"v r={r}")
    rt.close()


def test_synthetic_compute_takes_about_the_requested_time():
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.synthetic_compute(50.0, 4)
    sync()
    for us in (200.0, 1000.0):
        a.record()
        B.synthetic_compute(us, 4)
        b.record()
        sync()
        ms = a.elapsed_time(b)
        assert us * 1e-3 * 0.9 <= ms <= us * 1e-3 * 1.5 + 0.05, (us, ms)
    with pytest.raises(B.PipeSgdError):
        B.synthetic_compute(-1.0, 4)
    with pytest.raises(B.PipeSgdError):
        B.synthetic_compute(10.0, 0)


# ------------------------------------------------------- measurement probes --

@pytest.mark.parametrize("mode", MODES)
def test_stream_probes_touch_exactly_what_they_say(mode):
    # pipesgd_probe_stream is measurement code, but it writes the caller's buffers: whole units only, nothing
    # past them, and exactly the documented data movement.
    p, n = 3, 4096 * 5 + 1500                        # the ragged tail must be left alone by every kind
    rng = np.random.Generator(np.random.Philox(key=77))
    w_h = [rng.standard_normal(n).astype(np.float32) for _ in range(p)]
    v_h = [rng.standard_normal(n).astype(np.float32) for _ in range(p)]
    slots = [pay_buf(mode, n) for _ in range(p)]
    for (t, q, lds) in [(64, 4, 53248), (256, 1, 0), (256, 4, 0), (1024, 1, 65536)]:
        whole = n // (t * q * 4) * (t * q * 4)
        for kind in (B.PROBE_READ, B.PROBE_COPY, B.PROBE_MIXED, B.PROBE_WRITE):
            w = [up(x) for x in w_h]
            v = [up(x) for x in v_h]
            ua = B.UpdateArgs(slots, None, w, v)
            B.probe_stream(kind, mode, ua, n, t, q, lds)
            sync()
            for r in range(p):
                gw, gv = down(w[r]), down(v[r])
                assert_bits_equal(gw[whole:], w_h[r][whole:], f"w tail kind {kind}")
                assert_bits_equal(gv[whole:], v_h[r][whole:], f"v tail kind {kind}")
                if kind == B.PROBE_READ:
                    assert_bits_equal(gw, w_h[r], "the read probe must not write w")
                    assert_bits_equal(gv, v_h[r], "the read probe must not write v")
                elif kind == B.PROBE_COPY:
                    assert_bits_equal(gw, w_h[r], "copy keeps w")
                    assert_bits_equal(gv[:whole], w_h[r][:whole], "copy: v <- w")
                elif kind == B.PROBE_MIXED:
                    assert_bits_equal(gw[:whole], v_h[r][:whole], "mixed: w <- v")
                    assert_bits_equal(gv[:whole], w_h[r][:whole], "mixed: v <- w")
                else:
                    assert np.isfinite(gw).all() and np.isfinite(gv).all()
                    assert (np.abs(gw[:whole]) < 1e-2).all() and (gv[:whole] < 0).all()
    ua = B.UpdateArgs(slots, None, [up(x) for x in w_h], [up(x) for x in v_h])
    for bad in [dict(kind=9), dict(t=100), dict(q=3), dict(lds=-1), dict(mode=5)]:
        a = dict(kind=B.PROBE_COPY, mode=mode, t=256, q=1, lds=0); a.update(bad)
        with pytest.raises(B.PipeSgdError):
            B.probe_stream(a["kind"], a["mode"], ua, n, a["t"], a["q"], a["lds"])
    sync()


# ---------------------------------------------------------------- HIP graph --

@pytest.mark.parametrize("mode,bucketed", [(B.NONE, False), (B.TRUNC16, True), (B.QUANT8, False)])
def test_graph_replay_equals_eager(orc, mode, bucketed):
    # two iterations captured into one graph; several replays, with eager work
    # and synchronisations in between, each checked against the oracle
    p, lr, m = 4, 0.01, 0.9
    if bucketed:
        specs = W.scaled_config(5, 8)
        numels = [s.numel for s in specs]
        buckets, offs, n = B.bucket_plan(numels, 1 << 16)
        grads = [orc.pack(W.gradient_tensors_for(specs, 5, r, seed=11), offs, n) for r in range(p)]
    else:
        buckets, n = None, 4096 * 13 + 99
        grads = [W.gaussian(n, 1e-3, 11, (mode, r, 0, 0)) for r in range(p)]
    w0 = W.gaussian(n, 0.05, 13)
    sim = PipeSgdSim(mode, p, n, lr, m, 1.0, 2, buckets)
    sim.set_gradients(grads)
    sim.set_model(w0)
    sim.iteration(); sim.iteration()                 # warm-up, eager: t = 2
    sync()
    graph = sim.capture_pair()
    scratch = torch.zeros(1 << 20, device="cuda:0")
    total = 2
    for rep in range(3):
        graph.replay()
        total += 2
        scratch.add_(1.0)                            # unrelated eager work between replays
        sync()
        ws, vs = orc.pipe_sgd_run(mode, lambda r, w, t: grads[r], w0, p, total, lr, m, 1.0, 2, buckets)
        for r in range(p):
            assert_fp32_close_then_exact(sim.model(r), ws[r], f"w r={r} after replay {rep}")
            assert_fp32_close_then_exact(sim.velocity(r), vs[r], f"v r={r} after replay {rep}")
    assert float(scratch[0]) == 3.0


# ------------------------------------------------ one launch per iteration --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("momentum", [0.0, 0.9])
@pytest.mark.parametrize("bucketed", [False, True])
def test_one_launch_iteration_equals_oracle(orc, mode, momentum, bucketed):
    p, lr, iters = 4, 0.01, 4
    if bucketed:
        specs = W.scaled_config(5, 8)
        numels = [s.numel for s in specs]
        buckets, offs, n = B.bucket_plan(numels, 1 << 16)
        grad_fn = lambda r, w, t: orc.pack(W.gradient_tensors_for(specs, 5, r, seed=31, iteration=t), offs, n)
    else:
        buckets, n = None, 4096 * 6 + 1001
        grad_fn = lambda r, w, t: W.gaussian(n, 1e-3, 31, (mode, r, t, 0))
    w0 = W.gaussian(n, 0.05, 33)
    sim, ws_ref, vs_ref = run_both(orc, mode, grad_fn, w0, p, iters, lr, momentum, 2, buckets, B.ONE_LAUNCH)
    for r in range(p):
        assert_fp32_close_then_exact(sim.model(r), ws_ref[r], f"w r={r}")
        assert_fp32_close_then_exact(sim.velocity(r), vs_ref[r], f"v r={r}")
    last = [grad_fn(r, None, iters) for r in range(p)]
    want = orc.allreduce_bucketed(mode, last, buckets) if buckets else orc.allreduce(mode, last)
    for r in range(p):
        pay, sc = sim.result(r)
        assert_bits_equal(pay, want[r][0], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(sc, want[r][1], f"scales r={r}")


def test_one_launch_iteration_rejects_aliased_slots():
    n = 4096 * 2
    sim = PipeSgdSim(B.TRUNC16, 2, n, 0.01, 0.9)
    with pytest.raises(B.PipeSgdError):
        B.iteration_fused(sim.rings[0], sim.updates[0], 0.01, 0.9)
    sync()


# ------------------------------------------------ the one-exchange schedule --

@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("p,n", [(1, 9000), (2, 4096 * 4), (3, 50001), (4, 3), (4, 4096 * 21 + 77), (5, 12289),
                                 (8, 300007), (16, 70001)])
def test_allreduce_direct_equals_oracle(orc, mode, p, n):
    grads = [special_values(n, 41 * p + r) if n > 100 else W.gaussian(n, 1.0, 3, (0, r, 0, 0)) for r in range(p)]
    want = orc.allreduce_direct(mode, grads)
    g_dev, slots, scs = ring_buffers(mode, grads)
    stage = [pay_buf(mode, n) for _ in range(p)]
    stage_sc = [dev_zeros(B.num_scales(mode, n), fill=-2.0) for _ in range(p)]
    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_direct(ring, B.make_workspace(stage, stage_sc if mode == B.QUANT8 else None))
    sync()
    for r in range(p):
        if mode == B.NONE:
            assert_fp32_close_then_exact(down(slots[r]), want[r][0], f"sum r={r}")
        else:
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
    if mode == B.NONE and p > 1:          # same order, no codec: the ring gives the same bits
        ring_res = orc.allreduce(mode, grads)
        assert_bits_equal(down(slots[0]), ring_res[0][0], "direct vs ring")


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_allreduce_direct_bucketed_and_hand_cases(orc, mode):
    p = 4
    specs = W.scaled_config(5, 8)
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 16)
    packed = [orc.pack(W.gradient_tensors_for(specs, 5, r, seed=3), offs, N) for r in range(p)]
    pays = [np.zeros(N, dtype=orc.payload_dtype(mode)) for _ in range(p)]
    scs_ref = [np.zeros(orc.num_scales(mode, N), np.float32) for _ in range(p)]
    for (st, nb) in buckets:                      # the oracle per bucket, as for the ring
        res = orc.allreduce_direct(mode, [g[st:st + nb] for g in packed])
        for r in range(p):
            pays[r][st:st + nb] = res[r][0]
            if mode == B.QUANT8:
                scs_ref[r][st // 4096: st // 4096 + res[r][1].size] = res[r][1]
    g_dev = [up(g) for g in packed]
    slots = [pay_buf(mode, N, poison=False) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    stage = [pay_buf(mode, N) for _ in range(p)]
    stage_sc = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    ring = B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
    B.allreduce_direct(ring, B.make_workspace(stage, stage_sc if mode == B.QUANT8 else None))
    sync()
    for r in range(p):
        assert_bits_equal(down(slots[r], mode), pays[r], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), scs_ref[r], f"scales r={r}")
    # the hand-worked two-worker cases of the oracle's pins
    ce = 4096
    g0, g1 = np.zeros(2 * ce, np.float32), np.zeros(2 * ce, np.float32)
    if mode == B.TRUNC16:
        g0[0] = g0[ce] = 1.0
        g1[0] = g1[ce] = -(2.0 ** -8 + 2.0 ** -16)
    else:
        for base in (0, ce):
            g0[base], g0[base + 1] = 127.0, 10.4
            g1[base], g1[base + 1] = 0.0, 20.4
    g_dev, slots, scs = ring_buffers(mode, [g0, g1])
    stage = [pay_buf(mode, 2 * ce) for _ in range(2)]
    stage_sc = [dev_zeros(2) for _ in range(2)]
    ring = B.make_ring(mode, 2 * ce, g_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_direct(ring, B.make_workspace(stage, stage_sc if mode == B.QUANT8 else None))
    sync()
    got = down(slots[1], mode)
    if mode == B.TRUNC16:
        assert (got[0], got[ce]) == (0x3F7F, 0x3F7E)
    else:
        assert (got[0], got[1], got[ce], got[ce + 1]) == (127, 31, 127, 30)


# ------------------------------------------- recursive halving and doubling --

def hd_buffers(mode, n, p, poison=True):
    stage = [pay_buf(mode, n, poison=poison) for _ in range(p)]
    stage_sc = [dev_zeros(B.num_scales(mode, n), fill=-2.0) for _ in range(p)]
    partial = [dev_zeros(n, fill=float("nan") if poison else None) for _ in range(p)] if p > 2 else None
    return stage, (stage_sc if mode == B.QUANT8 else None), partial


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("p,n", [(1, 9000), (2, 4096 * 4), (2, 50001), (4, 3), (4, 4096 * 21 + 77), (4, 4096 * 2 + 5),
                                 (8, 300007), (8, 4096 * 5), (16, 70001), (16, 4096 * 40 + 1)])
def test_allreduce_halving_doubling_equals_oracle(orc, mode, p, n):
    grads = [special_values(n, 43 * p + r) if n > 100 else W.gaussian(n, 1.0, 5, (0, r, 0, 0)) for r in range(p)]
    want = orc.allreduce_hd(mode, grads)
    g_dev, slots, scs = ring_buffers(mode, grads)
    stage, stage_sc, partial = hd_buffers(mode, n, p)
    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    for _ in range(2):                 # a second call on used scratch buffers gives the same result
        B.allreduce_halving_doubling(ring, B.make_workspace(stage, stage_sc, partial))
        sync()
        for r in range(p):
            if mode == B.NONE:
                assert_fp32_close_then_exact(down(slots[r]), want[r][0], f"sum r={r}")
            else:
                assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r}")
            if mode == B.QUANT8:
                assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
    for r in range(p):                 # the inputs are never modified
        assert_bits_equal(down(g_dev[r]), grads[r], f"gradient r={r}")


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_allreduce_halving_doubling_bucketed_and_hand_cases(orc, mode):
    p = 4
    specs = W.scaled_config(5, 8)
    numels = [s.numel for s in specs]
    buckets, offs, N = B.bucket_plan(numels, 1 << 16)
    packed = [orc.pack(W.gradient_tensors_for(specs, 5, r, seed=4), offs, N) for r in range(p)]
    pays = [np.zeros(N, dtype=orc.payload_dtype(mode)) for _ in range(p)]
    scs_ref = [np.zeros(orc.num_scales(mode, N), np.float32) for _ in range(p)]
    for (st, nb) in buckets:                      # the oracle per bucket, as for the ring
        res = orc.allreduce_hd(mode, [g[st:st + nb] for g in packed])
        for r in range(p):
            pays[r][st:st + nb] = res[r][0]
            if mode == B.QUANT8:
                scs_ref[r][st // 4096: st // 4096 + res[r][1].size] = res[r][1]
    g_dev = [up(g) for g in packed]
    slots = [pay_buf(mode, N, poison=False) for _ in range(p)]
    scs = [dev_zeros(B.num_scales(mode, N)) for _ in range(p)]
    stage, stage_sc, partial = hd_buffers(mode, N, p, poison=False)
    ring = B.make_ring(mode, N, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
    B.allreduce_halving_doubling(ring, B.make_workspace(stage, stage_sc, partial))
    sync()
    for r in range(p):
        assert_bits_equal(down(slots[r], mode), pays[r], f"payload r={r}")
        if mode == B.QUANT8:
            assert_bits_equal(down(scs[r]), scs_ref[r], f"scales r={r}")
    # the hand-worked four-worker cases of the oracle's pins: roles (c, c^2, c^1, c^3) in chunk c
    ce = 4096
    g = [np.zeros(p * ce, np.float32) for _ in range(p)]
    if mode == B.TRUNC16:
        vals = {0: 1 + 2.0 ** -8, 2: 0.0, 1: 1 + 2.0 ** -7, 3: 2.0 ** -8}
        for c in range(p):
            for d, x in vals.items():
                g[c ^ d][c * ce:(c + 1) * ce] = x
    else:
        vals = {0: 10.3, 2: 20.4, 1: 5.3, 3: 7.4}
        for c in range(p):
            for r in range(p):
                g[r][c * ce + r] = 127.0
            for d, x in vals.items():
                g[c ^ d][c * ce + 8] = x
    g_dev, slots, scs = ring_buffers(mode, g)
    stage, stage_sc, partial = hd_buffers(mode, p * ce, p)
    ring = B.make_ring(mode, p * ce, g_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_halving_doubling(ring, B.make_workspace(stage, stage_sc, partial))
    sync()
    for r in range(p):
        got = down(slots[r], mode)
        if mode == B.TRUNC16:
            assert np.all(got == 0x4000)
        else:
            assert [int(got[c * ce + 8]) for c in range(p)] == [42] * p
            assert down(scs[r]).tolist() == [127.0] * p


def test_allreduce_halving_doubling_rejects_bad_arguments():
    n = 4096 * 3
    for p in (3, 6):
        sim = PipeSgdSim(B.TRUNC16, p, n, 0.01, 0.9)
        stage, stage_sc, partial = hd_buffers(B.TRUNC16, n, p)
        partial = partial or [dev_zeros(n) for _ in range(p)]
        with pytest.raises(B.PipeSgdError):
            B.allreduce_halving_doubling(sim.rings[0], B.make_workspace(stage, None, partial))
    sim = PipeSgdSim(B.QUANT8, 4, n, 0.01, 0.9)
    stage, stage_sc, partial = hd_buffers(B.QUANT8, n, 4)
    with pytest.raises(B.PipeSgdError):
        B.allreduce_halving_doubling(sim.rings[0], B.make_workspace(stage, None, partial))          # scales of the send buffers missing
    with pytest.raises(B.PipeSgdError):
        B.allreduce_halving_doubling(sim.rings[0], B.make_workspace(stage, stage_sc, None))         # partial sums missing at p > 2
    with pytest.raises(B.PipeSgdError):
        B.allreduce_halving_doubling(sim.rings[0], B.make_workspace(None, stage_sc, partial))
    sync()


@pytest.mark.parametrize("mode", MODES)
def test_pipe_sgd_run_with_halving_doubling(orc, mode):
    # five pipelined iterations (width 2) with the halving-doubling AllReduce against
    # the oracle's schedule-specific AllReduce followed by the oracle's update
    p, n, lr, m, iters = 4, 4096 * 9 + 321, 0.05, 0.9, 5
    sim = PipeSgdSim(mode, p, n, lr, m, schedule=B.HALVING_DOUBLING)
    w0 = W.gaussian(n, 1.0, 21, (0, 0, 0, 0))
    sim.set_model(w0)
    w_ref, v_ref = w0.copy(), np.zeros(n, np.float32)
    stale = None
    for t in range(1, iters + 1):
        grads = [W.gaussian(n, 1e-2, 23, (mode, r, t, 0)) for r in range(p)]
        sim.set_gradients(grads)
        sim.iteration()
        sync()
        fresh = orc.allreduce_hd(mode, grads)
        if stale is not None:
            orc.sgd_update(mode, stale[0][0], stale[0][1], w_ref, v_ref, lr, m, 1.0)
        stale = fresh
        for r in range(p):
            assert_fp32_close_then_exact(sim.model(r), w_ref, f"w t={t} r={r}")
            assert_fp32_close_then_exact(sim.velocity(r), v_ref, f"v t={t} r={r}")


# ------------------------------------------------------------ random cases --

# PIPESGD_RANDOM_CASES=N widens the sweep for an occasional longer run
@pytest.mark.parametrize("case", range(int(os.environ.get("PIPESGD_RANDOM_CASES", "24"))))
def test_random_shapes_all_schedules(orc, case):
    # seeded random worker counts, lengths, bucket layouts and modes; every
    # AllReduce schedule and the update against the oracle
    rng = np.random.Generator(np.random.Philox(key=9000 + case))
    mode = int(rng.integers(0, 3))
    p = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 11, 16]))
    if rng.random() < 0.5:
        numels = [int(x) for x in rng.choice([1, 2, 7, 64, 100, 4095, 4096, 4097, 9000, 33000, 70000],
                                             size=int(rng.integers(1, 12)))]
        buckets, offs, n = B.bucket_plan(numels, int(rng.choice([4096, 20000, 65536])))
        if len(buckets) > B.MAX_BUCKETS:
            pytest.skip("more buckets than the library takes")
        tens = [[W.gaussian(ne, 1e-2, 100 + case, (r, ti, 0, 0)) for ti, ne in enumerate(numels)] for r in range(p)]
        grads = [orc.pack(t, offs, n) for t in tens]
    else:
        buckets, n = None, int(rng.integers(1, 200000))
        grads = [special_values(n, 1000 * case + r) if n > 100 else W.gaussian(n, 1.0, case, (0, r, 0, 0))
                 for r in range(p)]
    want = orc.allreduce_bucketed(mode, grads, buckets) if buckets else orc.allreduce(mode, grads)
    for schedule in (B.STEPWISE, B.FUSED):
        g_dev, slots, scs = ring_buffers(mode, grads, poison=not buckets)
        ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
        B.allreduce_sim(ring, schedule)
        sync()
        for r in range(p):
            assert_bits_equal(down(slots[r], mode), want[r][0], f"payload r={r} schedule={schedule}")
            if mode == B.QUANT8 and not buckets:
                assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
    if p & (p - 1) == 0:
        if buckets:
            want_hd = [[np.zeros(n, dtype=orc.payload_dtype(mode)), None] for _ in range(p)]
            for (st, nb) in buckets:
                res = orc.allreduce_hd(mode, [g[st:st + nb] for g in grads])
                for r in range(p):
                    want_hd[r][0][st:st + nb] = res[r][0]
        else:
            want_hd = orc.allreduce_hd(mode, grads)
        g_dev2, slots2, scs2 = ring_buffers(mode, grads, poison=not buckets)
        stage, stage_sc, partial = hd_buffers(mode, n, p, poison=not buckets)
        ring2 = B.make_ring(mode, n, g_dev2, slots2, scs2 if mode == B.QUANT8 else None, buckets)
        B.allreduce_halving_doubling(ring2, B.make_workspace(stage, stage_sc, partial))
        sync()
        for r in range(p):
            assert_bits_equal(down(slots2[r], mode), want_hd[r][0], f"payload r={r} halving-doubling")
            if mode == B.QUANT8 and not buckets:
                assert_bits_equal(down(scs2[r]), want_hd[r][1], f"scales r={r} halving-doubling")
    # the one-exchange schedule through both of its entry points (the second keeps its send buffers in the
    # library's static device array), each bucket against the oracle's one-exchange branch
    if buckets:
        want_d = [[np.zeros(n, dtype=orc.payload_dtype(mode)), None] for _ in range(p)]
        for (st, nb) in buckets:
            res = orc.allreduce_direct(mode, [g[st:st + nb] for g in grads])
            for r in range(p):
                want_d[r][0][st:st + nb] = res[r][0]
    else:
        want_d = orc.allreduce_direct(mode, grads)
    for static in (False, True):
        g_dev3, slots3, scs3 = ring_buffers(mode, grads, poison=not buckets)
        ring3 = B.make_ring(mode, n, g_dev3, slots3, scs3 if mode == B.QUANT8 else None, buckets)
        if static:
            B.allreduce_direct_static(ring3)
        else:
            stage3 = [pay_buf(mode, n) for _ in range(p)]
            stage_sc3 = [dev_zeros(B.num_scales(mode, n), fill=-2.0) for _ in range(p)]
            B.allreduce_direct(ring3, B.make_workspace(stage3, stage_sc3 if mode == B.QUANT8 else None))
        sync()
        for r in range(p):
            assert_bits_equal(down(slots3[r], mode), want_d[r][0], f"payload r={r} one-exchange static={static}")
            if mode == B.QUANT8 and not buckets:
                assert_bits_equal(down(scs3[r]), want_d[r][1], f"scales r={r} one-exchange static={static}")
    # the pipelined schedule (a random number of sub-blocks, two streams) gives the ring's bits
    g_dev4, slots4, scs4 = ring_buffers(mode, grads, poison=not buckets)
    recv4 = [pay_buf(mode, n) for _ in range(p)]
    recv_sc4 = [dev_zeros(B.num_scales(mode, n), fill=-2.0) for _ in range(p)]
    ov, rt4 = B.Overlap(), B.Runtime()
    B.allreduce_pipelined(B.make_ring(mode, n, g_dev4, slots4, scs4 if mode == B.QUANT8 else None, buckets),
                          B.make_workspace(recv4, recv_sc4 if mode == B.QUANT8 else None), int(rng.integers(1, 9)), ov,
                          rt4.stream(0), rt4.stream(1))
    rt4.sync()
    sync()
    for r in range(p):
        assert_bits_equal(down(slots4[r], mode), want[r][0], f"payload r={r} pipelined")
    ov.close()
    rt4.close()
    # update of all replicas from the result
    lr, m = float(rng.choice([0.01, 0.1])), float(rng.choice([0.0, 0.9]))
    w0 = [W.gaussian(n, 1.0, 7 + case, (r, 1, 0, 0)) for r in range(p)]
    v0 = [W.gaussian(n, 0.1, 7 + case, (r, 2, 0, 0)) for r in range(p)]
    w, v = [up(x) for x in w0], [up(x) for x in v0]
    args = B.UpdateArgs(slots, scs if mode == B.QUANT8 else None, w, v if m else None)
    B.apply_update_multi(mode, args, n, lr, m, 1.0)
    sync()
    for r in range(p):
        orc.sgd_update(mode, want[r][0], want[r][1], w0[r], v0[r] if m else None, lr, m, 1.0)
        assert_fp32_close_then_exact(down(w[r]), w0[r], f"w r={r}")
        assert_fp32_close_then_exact(down(v[r]), v0[r], f"v r={r}")


# ------------------------------------------------------- capacity and zeros --

@pytest.mark.parametrize("mode", MODES)
def test_sixty_four_buckets_and_all_zero_gradients(orc, mode):
    p = 4
    numels = [4096 + 17 * i for i in range(64)]                    # one tensor per bucket: the library's maximum
    buckets, offs, n = B.bucket_plan(numels, 4096)
    assert len(buckets) == 64
    grads = [orc.pack([W.gaussian(ne, 1e-3, 3, (r, ti, 0, 0)) for ti, ne in enumerate(numels)], offs, n)
             for r in range(p)]
    for ti in (0, 5, 63):                                          # some buckets are all zero on every worker
        for g in grads:
            g[offs[ti]:offs[ti] + numels[ti]] = 0.0
    want = orc.allreduce_bucketed(mode, grads, buckets)
    for schedule in (B.STEPWISE, B.FUSED):
        g_dev, slots, scs = ring_buffers(mode, grads, poison=False)
        ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None, buckets)
        B.allreduce_sim(ring, schedule)
        sync()
        for r in range(p):
            got = down(slots[r], mode)
            assert_bits_equal(got, want[r][0], f"payload r={r}")
            assert not got[offs[5]:offs[5] + numels[5]].any()       # zeros in, zero payload out
            if mode == B.QUANT8:
                assert_bits_equal(down(scs[r]), want[r][1], f"scales r={r}")
                assert down(scs[r])[offs[5] // 4096] == 0.0
    with pytest.raises(B.PipeSgdError):                             # 65 buckets: refused, nothing launched
        B.bucket_plan([4096] * 65, 4096)
    # an all-zero slot leaves the model untouched bit for bit
    w0 = W.gaussian(n, 1.0, 5)
    w = up(w0)
    zero_slot = pay_buf(mode, n, poison=False)
    zero_sc = dev_zeros(B.num_scales(mode, n))
    B.apply_update(mode, zero_slot, zero_sc if mode == B.QUANT8 else None, n, w, None, 0.1)
    sync()
    assert_bits_equal(down(w), w0, "w after a zero slot")
