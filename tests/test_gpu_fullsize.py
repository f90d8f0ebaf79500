"""GPU parity at the full sizes of the workload list, in the launch
configurations bench.py times (p = 4, all replicas updated in one launch, width
2; stepwise schedule on one stream, and for the bucketed workload through the
two-stream runtime, which is what bench.py runs it on by default), plus every
other schedule bench.py can quote a figure for.  The scalar oracle finishes one full-size iteration in a
second or two, so every output element is compared, not a sample.
"""
import time

import numpy as np
import pytest
import torch

from paper_1811_03619_amd import binding as B
from paper_1811_03619_amd import workloads as W
from paper_1811_03619_amd.pipeline import PipeSgdSim

from gpu_util import assert_bits_equal, assert_fp32_close_then_exact, sync

pytestmark = pytest.mark.gpu


def full_config_inputs(cfg, p, seed):
    specs = W.config_tensors(cfg)
    numels = [s.numel for s in specs]
    if cfg == 5:
        buckets, offs, n = B.bucket_plan(numels, 1 << 20)
    else:
        buckets, offs, n = None, list(np.cumsum([0] + numels[:-1])), int(sum(numels))
    grads = []
    for r in range(p):
        flat = np.zeros(n, dtype=np.float32)
        for t, o in zip(W.gradient_tensors(cfg, r, seed), offs):
            flat[o:o + t.size] = t
        grads.append(flat)
    return buckets, n, grads


def oracle_allreduce(orc, schedule, mode, grads, buckets):
    fn = {B.DIRECT: orc.allreduce_direct, B.HALVING_DOUBLING: orc.allreduce_hd}.get(schedule)
    if fn is None:                                  # the ring: stepwise and fused give the same bits
        return orc.allreduce_bucketed(mode, grads, buckets) if buckets else orc.allreduce(mode, grads)
    if not buckets:
        return fn(mode, grads)
    n, p = grads[0].size, len(grads)               # every bucket is reduced as a vector of its own
    out = [(np.zeros(n, dtype=orc.payload_dtype(mode)),
            np.zeros(orc.num_scales(mode, n), np.float32) if mode == B.QUANT8 else None) for _ in range(p)]
    for (st, nb) in buckets:
        res = fn(mode, [g[st:st + nb] for g in grads])
        for r in range(p):
            out[r][0][st:st + nb] = res[r][0]
            if mode == B.QUANT8:
                out[r][1][st // 4096: st // 4096 + res[r][1].size] = res[r][1]
    return out


@pytest.mark.parametrize("cfg,mode,schedule,streams", [
    (3, B.TRUNC16, B.STEPWISE, 2),     # the headline configuration as bench.py times it: the two-stream runtime
    (3, B.TRUNC16, B.STEPWISE, 1),     # and back to back on one stream
    (3, B.TRUNC16, B.FUSED, 1),
    (3, B.TRUNC16, B.FUSED, 2),        # bench.py --schedule fused also defaults to the two-stream runtime
    (4, B.QUANT8, B.STEPWISE, 2),
    (4, B.QUANT8, B.STEPWISE, 1),
    (4, B.QUANT8, B.FUSED, 1),
    (5, B.NONE, B.STEPWISE, 1),
    (5, B.NONE, B.FUSED, 1),
    (5, B.TRUNC16, B.STEPWISE, 1),
    (5, B.TRUNC16, B.STEPWISE, 2),
    (5, B.NONE, B.STEPWISE, 2),
    (5, B.TRUNC16, B.FUSED, 1),
    (5, B.TRUNC16, B.ONE_LAUNCH, 1),   # AllReduce and update of an iteration in one launch
    (3, B.TRUNC16, B.DIRECT, 1),       # the other schedules, each against its own oracle branch
    (3, B.TRUNC16, B.HALVING_DOUBLING, 1),
    (5, B.TRUNC16, B.HALVING_DOUBLING, 1),
    (5, B.TRUNC16, B.DIRECT, 1),
    (4, B.QUANT8, B.DIRECT, 1),
])
def test_full_size_two_iterations(orc, cfg, mode, schedule, streams):
    p, lr, m = 4, 0.01, 0.9
    t0 = time.time()
    buckets, n, grads = full_config_inputs(cfg, p, seed=1)
    w0 = W.gaussian(n, 0.05, 1, (cfg, 99, 0, 0))
    print(f"[cfg{cfg} mode{mode} sched{schedule}] n={n} inputs in {time.time() - t0:.1f}s", flush=True)

    sim = PipeSgdSim(mode, p, n, lr, m, 1.0, 2, buckets, schedule)
    sim.set_gradients(grads)
    sim.set_model(w0)
    if streams == 1:
        sim.iteration()        # t=1: AllReduce -> slot 1, update from the zero slot
        sim.iteration()        # t=2: AllReduce -> slot 0, update from slot 1
    else:
        sync()
        rt = B.Runtime()
        for t in (1, 2):       # the same two iterations, AllReduce on one stream and update on the other
            cur = t % 2
            rt.iteration(sim.rings[cur], sim.updates[1 - cur], sim.updates[cur], schedule, 2, lr, m, 1.0,
                         time_update=True)
        rt.sync()
        assert rt.update_time()[1] == 2
        rt.close()
    sync()

    t0 = time.time()
    A = oracle_allreduce(orc, schedule, mode, grads, buckets)
    w_ref, v_ref = w0.copy(), np.zeros(n, np.float32)
    orc.sgd_update(mode, A[0][0], A[0][1], w_ref, v_ref, lr, m, 1.0)     # the t=2 update (t=1's is a no-op)
    print(f"[cfg{cfg}] oracle in {time.time() - t0:.1f}s", flush=True)

    for slot in (0, 1):
        pay, sc = sim.result(0, slot)
        if mode == B.NONE:
            assert_fp32_close_then_exact(pay, A[0][0], f"sum slot {slot}")
        else:
            assert_bits_equal(pay, A[0][0], f"payload slot {slot}")
        if mode == B.QUANT8:
            assert_bits_equal(sc, A[0][1], f"scales slot {slot}")
        for r in range(1, p):                                   # replicas: identical bytes (compared on the device)
            assert torch.equal(sim.slots[slot][r], sim.slots[slot][0]), (slot, r)
            if mode == B.QUANT8:
                assert torch.equal(sim.slot_scales[slot][r], sim.slot_scales[slot][0]), (slot, r)
    # the oracle's replicas are identical by its own pins; compare every GPU replica to the one reference
    assert_fp32_close_then_exact(sim.model(0), w_ref, "w")
    assert_fp32_close_then_exact(sim.velocity(0), v_ref, "v")
    for r in range(1, p):
        assert torch.equal(sim.w[r], sim.w[0]) and torch.equal(sim.v[r], sim.v[0]), r
    for r in range(p):
        assert torch.equal(sim.g_local[r].cpu(), torch.from_numpy(grads[r])), "gradients must not be modified"


@pytest.mark.parametrize("mode", [B.TRUNC16, B.QUANT8])
def test_buffers_beyond_4_gib_sampled_tiles(orc, mode):
    """Largest size exercised: n > 2^31 elements per worker, so fp32 byte offsets pass 2^33 and 16-bit payload
    offsets pass 2^32.  The oracle would need minutes for the whole vector; chunks and quantisation blocks
    never interact, so a sampled tile's result depends only on the p workers' values in that tile and on the
    chunk it lies in -- the oracle computes it from a p-tile vector holding the tile at that chunk position."""
    p, lr, m = 2, 0.01, 0.9
    n = (1 << 31) + 4096 * 3 + 100
    ce = B.chunk_elems(n, p)
    dev = "cuda:0"

    def pattern(seed, length, sigma):
        return W.gaussian(length, sigma, seed, (77, 0, 0, 0))

    def tiled(pat):                                       # value at global index i is pat[i % len(pat)]
        t = torch.from_numpy(pat).to(dev)
        reps = -(-n // pat.size)
        return t.repeat(reps)[:n]

    def sample(pat, e0, ln):
        idx = (e0 + np.arange(ln, dtype=np.int64)) % pat.size
        return pat[idx]

    g_pat = [pattern(900 + r, 1000003 + 2 * r, 0.01) for r in range(p)]
    w_pat, v_pat = pattern(910, 999983, 0.05), pattern(911, 1000033, 0.001)
    g_dev = [tiled(x) for x in g_pat]
    w = [tiled(w_pat) for _ in range(p)]
    v = [tiled(v_pat) for _ in range(p)]
    slots = [torch.zeros(n, dtype={B.TRUNC16: torch.int16, B.QUANT8: torch.int8}[mode], device=dev) for _ in range(p)]
    ns = B.num_scales(mode, n)
    scs = [torch.zeros(max(ns, 1), dtype=torch.float32, device=dev)[:ns] for _ in range(p)]
    print(f"[beyond 4 GiB, mode {mode}] n={n} chunk={ce} buffers ready", flush=True)

    ring = B.make_ring(mode, n, g_dev, slots, scs if mode == B.QUANT8 else None)
    B.allreduce_sim(ring, B.STEPWISE)
    B.apply_update_multi(mode, B.UpdateArgs(slots, scs if mode == B.QUANT8 else None, w, v), n, lr, m, 1.0)
    sync()
    print("[beyond 4 GiB] device work done", flush=True)

    last_tile = (n - 1) // 4096
    tiles = sorted({0, 1, (1 << 30) // 4096 - 1, (1 << 30) // 4096, ce // 4096 - 1, ce // 4096, ce // 4096 + 1,
                    (1 << 31) // 4096 - 1, (1 << 31) // 4096, last_tile - 1, last_tile,
                    (3 << 29) // 4096, 123457, 400001})
    for T in tiles:
        e0 = T * 4096
        ln = min(4096, n - e0)
        c = e0 // ce
        assert (e0 - c * ce) % 4096 == 0
        small = []
        for r in range(p):                                # the tile at the start of chunk c of a p-tile vector
            x = np.zeros(c * 4096 + ln if c == p - 1 else p * 4096, dtype=np.float32)
            x[c * 4096:c * 4096 + ln] = sample(g_pat[r], e0, ln)
            small.append(x)
        assert B.chunk_elems(small[0].size, p) == 4096
        res = orc.allreduce(mode, small)
        want_pay = res[0][0][c * 4096:c * 4096 + ln]
        w_ref, v_ref = sample(w_pat, e0, ln).copy(), sample(v_pat, e0, ln).copy()
        orc.sgd_update(mode, want_pay, res[0][1][c:c + 1] if mode == B.QUANT8 else None, w_ref, v_ref, lr, m, 1.0)
        for r in range(p):
            got = slots[r][e0:e0 + ln].cpu().numpy()
            assert_bits_equal(got.view(np.uint16) if mode == B.TRUNC16 else got, want_pay, f"payload tile {T} r={r}")
            if mode == B.QUANT8:
                assert_bits_equal(scs[r][T:T + 1].cpu().numpy(), res[0][1][c:c + 1], f"scale tile {T} r={r}")
            assert_fp32_close_then_exact(w[r][e0:e0 + ln].cpu().numpy(), w_ref, f"w tile {T} r={r}")
            assert_fp32_close_then_exact(v[r][e0:e0 + ln].cpu().numpy(), v_ref, f"v tile {T} r={r}")
    # properties that hold at any size: replicas identical, gradients untouched, nothing written past the end
    assert torch.equal(slots[0], slots[1]) and torch.equal(w[0], w[1]) and torch.equal(v[0], v[1])
    for r in range(p):
        assert torch.equal(g_dev[r][-5000:].cpu(), torch.from_numpy(sample(g_pat[r], n - 5000, 5000)))
    del g_dev, w, v, slots, scs
    torch.cuda.empty_cache()
