"""Byte accounting of the path and the four side studies that `bench.py --study` prints:
pipelining within the AllReduce (Sec. 3.2, Fig. 3), Algorithm 1's two threads against
Eq. 2 and Eq. 4, Eq. 5 as a calculator, and the size sweep.  Measurement code: it only
calls the library through the binding and times it.
"""
from __future__ import annotations

import time


def payload_bytes_per_elem(mode: int) -> float:
    return {0: 4.0, 1: 2.0, 2: 1.0 + 4.0 / 4096.0}[mode]


def bytes_model(mode: int, n: int, p: int, momentum: bool, fused: bool = False, direct: bool = False,
                halving_doubling: bool = False):
    """Algorithmic bytes of one iteration, by phase.  Stepwise schedule: every
    hop's payload is written once and read once.  Fused schedule: each gradient
    is read once and each worker's result written once (hop payloads never
    reach memory), so it is priced with its own, smaller byte count."""
    cb = payload_bytes_per_elem(mode)
    upd = p * n * (cb + (16.0 if momentum else 8.0))
    if direct:
        # exchange 1: every worker reads (p-1)/p of its gradient and writes it compressed; owner: reads its
        # block and p-1 payloads, writes the result into p slots
        scatter = (p - 1) * (4.0 + cb) * n
        reduce_bcast = (4.0 + (p - 1) * cb + p * cb) * n
        return {"direct_scatter": scatter, "direct_reduce_broadcast": reduce_bcast, "update": upd,
                "total": scatter + reduce_bcast + upd}
    if halving_doubling:
        # first message: read the half given away, write it compressed.  Halving round h (= chunks kept per
        # worker): read own fp32 + the partner's payload over h chunks, write fp32 for the h/2 chunks kept
        # next and payload for the h/2 sent next (the last round writes one chunk of payload).  Doubling
        # round d: copy d chunks of payload.  All of it for p workers; a chunk is n/p elements.
        ce = n / p
        first = 0.0 if mode == 0 else p * (p // 2) * ce * (4.0 + cb)
        halving, h = 0.0, p // 2
        while h >= 1:
            out = cb if h == 1 else (4.0 + cb) / 2.0
            halving += p * h * ce * (4.0 + cb + out)
            h //= 2
        doubling = (p - 1) * n * 2.0 * cb
        return {"first_message": first, "halving": halving, "doubling": doubling, "update": upd,
                "total": first + halving + doubling + upd}
    if fused:
        ar = (4.0 * p + cb * p) * n
        return {"allreduce_fused": ar, "update": upd, "total": ar + upd}
    first = 0.0 if mode == 0 else (4.0 + cb) * n
    rs = (p - 1) * n * (cb + 4.0 + cb)
    ag = (p - 1) * n * 2.0 * cb
    return {"first_send": first, "reduce_scatter": rs, "allgather": ag, "update": upd,
            "total": first + rs + ag + upd}


def within_allreduce(sim, mode, n, p, reps: int = 15):
    """Pipelining within the AllReduce (Sec. 3.2, Fig. 3(b)): stage 1 moves each
    hop's compressed payload into the receiver's staging buffer (the stand-in for
    the wire) on one stream, stage 2 (decompress, sum, compress) runs on another
    on what has arrived.  Reports how much of the shorter stage the overlap hides."""
    import numpy as np
    import torch

    from paper_1811_03619_amd import binding as B

    from paper_1811_03619_amd.pipeline import payload_empty
    dev = sim.device
    ns = B.num_scales(mode, n)
    recv = [payload_empty(mode, n, dev) for _ in range(p)]
    recv_sc = [torch.zeros(max(ns, 1), dtype=torch.float32, device=dev)[:ns] for _ in range(p)] if mode == B.QUANT8 else None
    ring = sim.rings[0]
    ov = B.Overlap()
    # the library's two non-blocking streams: they run concurrently (two streams drawn from torch's pool may share
    # a hardware queue and then serialise), and nothing on them orders itself against the default stream
    rt = B.Runtime()
    comp, wire = rt.stream(0), rt.stream(1)

    def timed(fn):
        for _ in range(3):
            fn()
        rt.sync()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            rt.sync()
            ts.append((time.perf_counter() - t0) / reps * 1e3)
        return float(np.median(ts))

    ws = B.make_workspace(recv, recv_sc)

    def pipelined(seg, two_streams, **kw):
        return timed(lambda: B.allreduce_pipelined(ring, ws, seg, ov, comp, wire if two_streams else comp, **kw))

    res = {"study": "within-allreduce", "unit": "ms", "timing": "wall clock over back-to-back calls"}
    res["in_place_stepwise"] = round(timed(lambda: B.allreduce_sim(ring, B.STEPWISE, comp)), 5)
    res["reduce_rounds_in_place"] = round(
        timed(lambda: [B.ring_reduce_scatter_step(ring, s, comp) for s in range(p - 1)]), 5)
    res["transfer_rounds_only"] = round(timed(lambda: [B.ring_allgather_step(ring, s, comp) for s in range(p - 1)]), 5)
    res["sequential_transfer_then_reduce"] = round(pipelined(1, False), 5)
    res["pipelined_full_speed_transfer"] = {str(seg): round(pipelined(seg, True), 5) for seg in (1, 2, 4, 8)}
    # a link that is a resource of its own: after each transfer the wire stream idles for the time the bytes
    # would take on a network of the given speed (per worker); stage 2 overlaps that idle time
    res["network_link"] = []
    chunk_mib = B.payload_bytes(mode, B.chunk_elems(n, p)) / 2.0 ** 20
    for gbps in (200.0, 50.0, 12.5):
        us_per_mib = 2.0 ** 20 / (gbps * 1e3)              # GB/s -> us per MiB
        seq = pipelined(1, False, link_us_per_mib=us_per_mib)
        row = {"link_GBps_per_worker": gbps, "link_ms_per_round": round(chunk_mib * us_per_mib * 1e-3, 4),
               "sequential": round(seq, 5),
               "pipelined": {str(seg): round(pipelined(seg, True, link_us_per_mib=us_per_mib), 5)
                             for seg in (2, 4, 8)}}
        row["hidden_ms"] = round(seq - min(row["pipelined"].values()), 5)
        res["network_link"].append(row)
    # a link made of a few workgroups inside the same HBM (latency-bound, so it slows down under load)
    res["limited_link_in_hbm"] = []
    for k in (16,):
        row = {"wire_workgroups_per_worker": k, "sequential": round(pipelined(1, False, wire_workgroups=k), 5),
               "pipelined": {str(seg): round(pipelined(seg, True, wire_workgroups=k), 5) for seg in (2, 4)}}
        res["limited_link_in_hbm"].append(row)
    rt.close()
    ov.close()
    return res


def size_sweep(mode, p, momentum, seed, reps: int = 20, stagger: bool = True):
    """Whole iteration and update launch against the gradient length: where the
    path leaves the launch-bound regime and where the memory-side cache stops
    helping."""
    import numpy as np
    import torch

    from paper_1811_03619_amd import binding as B

    from paper_1811_03619_amd.pipeline import PipeSgdSim
    rows = []
    for m in (1 << 16, 1 << 18, 1 << 20, 1 << 22, 1 << 24, 1 << 25, 1 << 26, 1 << 27, 1 << 28):
        sim = PipeSgdSim(mode, p, m, 0.01, momentum, stagger=stagger)
        for r in range(p):
            sim.g_local[r].normal_(0.0, 1e-3, generator=torch.Generator(device=sim.device).manual_seed(seed + r))
        for _ in range(4):
            sim.iteration()
        torch.cuda.synchronize()
        it_ms, up_ms = [], []
        for _ in range(reps):
            a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            a.record()
            cur = sim.allreduce()
            b.record()
            sim.update_from(1 - cur)
            c.record()
            sim.t += 1
            torch.cuda.synchronize()
            it_ms.append(a.elapsed_time(c)); up_ms.append(b.elapsed_time(c))
        model = bytes_model(mode, m, p, momentum != 0.0)
        it, up = float(np.median(it_ms)), float(np.median(up_ms))
        rows.append({"elements_per_worker": m, "bytes_per_iter": int(model["total"]), "iteration_ms": round(it, 5),
                     "iteration_GBps": round(model["total"] / it / 1e6, 1), "update_ms": round(up, 5),
                     "update_GBps": round(model["update"] / up / 1e6, 1)})
        del sim
        torch.cuda.empty_cache()
    return {"study": "size-sweep", "workers": p, "mode": mode, "staggered_buffers": stagger, "rows": rows}


def ring_cost_model(mode, n, p, seed, reps: int = 30):
    """Eq. 5 as a calculator: alpha (per-round latency) is measured on a vector of
    one tile per chunk, beta (per byte sent) on the send-back rounds and gamma
    (per byte reduced) on the transmit-and-reduce rounds of the workload's size;
    the 2(p-1) rounds of other sizes are then predicted and measured."""
    import numpy as np
    import torch

    from paper_1811_03619_amd import binding as B

    from paper_1811_03619_amd.pipeline import PipeSgdSim

    def rounds_ms(m):
        sim = PipeSgdSim(mode, p, m, 0.01, 0.9)
        for r in range(p):
            sim.g_local[r].normal_(0.0, 1e-3, generator=torch.Generator(device=sim.device).manual_seed(seed + r))
        ring = sim.rings[0]
        B.ring_first_send(ring)

        def timed(fn):
            for _ in range(3):
                fn()
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(); fn(); b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return float(np.median(ts))

        rs = timed(lambda: [B.ring_reduce_scatter_step(ring, k) for k in range(p - 1)]) / (p - 1)
        ag = timed(lambda: [B.ring_allgather_step(ring, k) for k in range(p - 1)]) / (p - 1)
        both = timed(lambda: ([B.ring_reduce_scatter_step(ring, k) for k in range(p - 1)],
                              [B.ring_allgather_step(ring, k) for k in range(p - 1)]))
        del sim
        torch.cuda.empty_cache()
        return rs, ag, both

    cb = payload_bytes_per_elem(mode)
    rs0, ag0, _ = rounds_ms(p * 4096)                      # one tile per chunk: latency only
    alpha = 0.5 * (rs0 + ag0)
    rs1, ag1, both1 = rounds_ms(n)
    wire_bytes = cb * n                                    # Eq. 5's n: bytes of one worker's (compressed) gradient
    beta = (ag1 - alpha) / (wire_bytes / p)                # ms per byte sent by one worker in one round
    gamma = (rs1 - alpha) / (wire_bytes / p) - beta        # ms per byte reduced
    res = {"study": "ring-cost-model", "unit": "ms", "alpha_ms_per_round": round(alpha, 5),
           "beta_ms_per_MB": round(beta * 1e6, 6), "gamma_ms_per_MB": round(gamma * 1e6, 6),
           "fitted_on_elements": n, "measured_fit_size": round(both1, 5),
           "eq5_fit_size": round(B.model_ring_comm_time(p, wire_bytes, alpha, beta, gamma), 5), "predictions": []}
    for m in (n // 64, n // 16, n // 4, n // 2, 2 * n):
        m = max(p * 4096, m // 4096 * 4096)
        _, _, meas = rounds_ms(m)
        pred = B.model_ring_comm_time(p, cb * m, alpha, beta, gamma)
        res["predictions"].append({"elements": m, "eq5": round(pred, 5), "measured": round(meas, 5),
                                   "measured_over_eq5": round(meas / pred, 4)})
    return res


def two_thread_runtime(sim, schedule, iters: int = 30):
    """Algorithm 1's two threads as two streams: time per iteration against the
    duration of the compute stand-in, for width 2 (pipelined) and width 1
    (synchronous), next to Eq. 4 and Eq. 2 evaluated on the separately measured
    l_up and l_comm."""
    import numpy as np
    import torch

    from paper_1811_03619_amd import binding as B

    rt = B.Runtime()
    p = sim.p

    def alone(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    l_up = alone(lambda: sim.update_from(1))
    l_comm = alone(lambda: B.allreduce_sim(sim.rings[0], schedule))

    # a third result-slot set for the width-3 leg (Alg. 1 keeps K of them)
    from paper_1811_03619_amd.pipeline import payload_empty
    ns = B.num_scales(sim.mode, sim.n)
    slots3 = [payload_empty(sim.mode, sim.n, sim.device) for _ in range(p)]
    scales3 = [torch.zeros(max(ns, 1), dtype=torch.float32, device=sim.device)[:ns] for _ in range(p)]
    q8 = sim.mode == B.QUANT8
    rings = list(sim.rings) + [B.make_ring(sim.mode, sim.n, sim.g_local, slots3, scales3 if q8 else None, sim.buckets)]
    updates = list(sim.updates) + [B.UpdateArgs(slots3, scales3 if q8 else None, sim.w,
                                                sim.v if sim.momentum != 0.0 else None)]

    def per_iter(width, compute_us, wire_us):
        K = max(width, 2)

        def run(k):
            for i in range(k):
                cur = i % K
                rt.iteration(rings[cur], updates[(cur + 1) % K], updates[cur], schedule, width,
                             sim.lr, sim.momentum, sim.grad_scale, compute_us=compute_us, compute_workgroups=16,
                             wire_us=wire_us)
        run(4)
        rt.sync()
        t0 = time.perf_counter()
        run(iters)
        rt.sync()
        return (time.perf_counter() - t0) / iters * 1e3

    tables = []
    for wire in (0.0, 1.0):                   # ms the payloads spend "on the network"
        rows = []
        for l_comp in (0.0, 0.2, 0.4, 0.6, 0.8, 1.0, 1.4, 1.8):
            w2, w1 = per_iter(2, l_comp * 1e3, wire * 1e3), per_iter(1, l_comp * 1e3, wire * 1e3)
            w3 = per_iter(3, l_comp * 1e3, wire * 1e3)
            lc = l_comm + wire
            rows.append({"l_comp": l_comp, "pipelined": round(w2, 4), "pipelined_width_3": round(w3, 4),
                         "synchronous": round(w1, 4),
                         "eq4": round(B.model_pipe_time(1, l_up, l_comp, lc), 4),
                         "eq4_one_gpu": round(max(l_up + l_comm + l_comp, lc), 4),
                         "eq2": round(B.model_sync_time(1, l_up, l_comp, lc), 4),
                         "eq7_scaling_efficiency": round(B.model_scaling_efficiency(l_up, l_comp, lc), 4)})
        tables.append({"wire_ms": wire, "l_comm": round(l_comm + wire, 4), "rows": rows})
    rt.close()
    return {"study": "two-thread-runtime", "unit": "ms", "l_up": round(l_up, 4), "l_comm": round(l_comm, 4),
            "note": "eq4 = max(l_up + l_comp, l_comm) assumes the two threads use separate resources.  On one GPU the "
                    "AllReduce kernels and the update share HBM bandwidth, so the kernels' time lands on the compute "
                    "side as well: eq4_one_gpu = max(l_up + l_allreduce_kernels + l_comp, l_allreduce_kernels + wire); "
                    "the wire delay and the compute stand-in use no bandwidth",
            "tables": tables}


