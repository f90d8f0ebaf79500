#!/usr/bin/env python3
"""Benchmark of the Pipe-SGD aggregation + update path on one MI355X.

One "step" = one iteration of the whole hot path over one batch of synthetic
gradients already resident in HBM: the ring AllReduce of p = 4 simulated
workers (first send, p-1 transmit-and-reduce rounds with decompress-sum-
compress, p-1 send-back rounds, every hop's payload written to memory) and the
staleness-1 momentum-SGD update of all p model replicas.

The iterations run the way Algorithm 1 runs them: the AllReduce on the
communication stream, the update on the computation stream (the library's
two-stream runtime), so the AllReduce of iteration t overlaps the update that
applies iteration t-1's result.  One further block of iterations runs on one
stream so that the update kernel, the dominant one, is also timed alone.

Prints ONE JSON line.  `value` is algorithmic GB/s: the bytes the method moves
per iteration (every hop's payload written once and read once, every replica's
slot/w/v read and w/v written once) divided by the measured time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

MODE_OF_CONFIG = {1: 0, 2: 0, 3: 1, 4: 2, 5: 1}


from bench_studies import bytes_model, payload_bytes_per_elem  # noqa: E402  (the byte accounting)


INFINITY_CACHE_BYTES = 256 * 2 ** 20   # MI355X memory-side cache


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=5,
                    help="the block of --steps iterations is timed this many times; ms_per_step is the median block")
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = AlexNet-shaped, 61M, the headline)")
    ap.add_argument("--mode", type=int, default=None, help="override compression mode 0/1/2")
    ap.add_argument("--schedule", choices=["stepwise", "fused", "one-launch", "direct", "halving-doubling"],
                    default="stepwise",
                    help="stepwise: one launch per ring round, every hop payload in memory (the headline); fused: the "
                         "AllReduce in one launch; one-launch: AllReduce and update of an iteration in one launch")
    ap.add_argument("--workers", type=int, default=4)
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--momentum", type=float, default=None)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--cpu-seconds", type=float, default=8.0,
                    help="budget of each of the two oracle timings, one thread and all cores (0 = skip)")
    ap.add_argument("--phases", action="store_true",
                    help="also time each phase separately and run the memory-stream probes the update is measured against")
    ap.add_argument("--graph", action="store_true",
                    help="replay the iterations from a captured HIP graph (two iterations per replay); "
                         "the update kernel is then not bracketed by events, so roofline.achieved is null")
    ap.add_argument("--streams", choices=["auto", "1", "2"], default="auto",
                    help="2: through the library's two-stream runtime (Algorithm 1's two threads: the AllReduce on the "
                         "communication stream, the update on the computation stream, ordered by events), which is how "
                         "the method runs; one more block of --steps iterations then runs on one stream to time the "
                         "update kernel alone.  1: AllReduce and update back to back on one stream.  auto: 2 for the "
                         "ring schedules (stepwise, fused) on vectors of 4M elements or more, 1 for launch-bound "
                         "sizes, the other schedules and --graph")
    ap.add_argument("--two-streams", action="store_true", help="same as --streams 2")
    ap.add_argument("--no-stagger", action="store_true",
                    help="place every buffer at the start of a 4 KiB page instead of staggering them by multiples of "
                         "256 bytes (for comparison)")
    ap.add_argument("--study", choices=["within-allreduce", "two-thread-runtime", "ring-cost-model", "size-sweep"], default=None,
                    help="extra measurement printed as its own JSON line after the main one")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="after the timed region, launch this many plain copies of one worker's gradient "
                         "(pipesgd_compress in mode NONE: reads 4n, writes 4n bytes) so that a rocprofv3 --pmc "
                         "run of this command holds a kernel of known traffic to scale its counters by")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs the K simulated workers on ONE GPU; --gpus must be 1 "
              "(no multi-GPU path exists in this repository)", file=sys.stderr)
        return 2
    if args.repeats < 1 or args.steps < 1:
        print("bench.py: --steps and --repeats must be at least 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1811_03619_amd import binding as B
    from paper_1811_03619_amd import workloads as W
    from paper_1811_03619_amd.pipeline import PipeSgdSim

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3

    cfg, p = args.config, args.workers
    mode = MODE_OF_CONFIG[cfg] if args.mode is None else args.mode
    momentum = (0.0 if cfg == 1 else 0.9) if args.momentum is None else args.momentum
    schedule = {"stepwise": B.STEPWISE, "fused": B.FUSED, "one-launch": B.ONE_LAUNCH, "direct": B.DIRECT,
                "halving-doubling": B.HALVING_DOUBLING}[args.schedule]

    specs = W.config_tensors(cfg)
    numels = [s.numel for s in specs]
    buckets = None
    if cfg == 5:
        buckets, offs, n = B.bucket_plan(numels, 1 << 20)
    else:
        offs, n = list(np.cumsum([0] + numels[:-1])), int(sum(numels))

    streams = args.streams
    if args.two_streams:
        streams = "2"
    if streams == "auto":
        # launch-bound sizes (configs 1 and 2: a few MB per worker) lose on two streams: the event hand-offs
        # cost more than the overlap gains
        streams = "2" if (schedule in (B.STEPWISE, B.FUSED) and not args.graph and n >= (1 << 22)) else "1"
    two_streams = streams == "2"

    def host_gradient(r: int) -> np.ndarray:
        flat = np.zeros(n, dtype=np.float32)
        for t, o in zip(W.gradient_tensors(cfg, r, args.seed), offs):
            flat[o:o + t.size] = t
        return flat

    t0 = time.time()
    grads = [host_gradient(r) for r in range(p)]
    w0 = W.gaussian(n, 0.05, args.seed, (cfg, 99, 0, 0))
    gen_s = time.time() - t0

    sim = PipeSgdSim(mode, p, n, args.lr, momentum, 1.0, 2, buckets, schedule, stagger=not args.no_stagger)
    sim.set_gradients(grads)
    sim.set_model(w0)
    torch.cuda.synchronize()

    # ---- one timed block = exactly `steps` iterations; returns wall seconds and the durations (ms) of the
    # update launches in it, each bracketed by HIP events on the stream it is launched on
    rt = None
    graph = None
    if two_streams:
        if schedule not in (B.STEPWISE, B.FUSED) or args.graph:
            print("bench.py: --streams 2 takes the stepwise or fused schedule, without --graph", file=sys.stderr)
            return 2
        rt = B.Runtime()

        def block(k, timed=True):
            for _ in range(k):
                cur = (sim.t + 1) % 2
                rt.iteration(sim.rings[cur], sim.updates[1 - cur], sim.updates[cur], schedule, 2, sim.lr, sim.momentum,
                             sim.grad_scale, time_update=timed)
                sim.t += 1

        timed_blocks = [0]

        def run_block(k):
            # the timing events cost a few microseconds per iteration on this path, so only the first block
            # carries them; ms_per_step, the median block, is then a block without them
            first = timed_blocks[0] == 0
            timed_blocks[0] += 1
            rt.update_time()                                   # forget what was recorded before
            t_begin = time.perf_counter()
            block(k, timed=first)
            rt.sync()
            wall = time.perf_counter() - t_begin
            total_ms, launches = rt.update_time()
            return wall, ([total_ms / launches] * launches if launches else [])
    elif args.graph:
        if args.steps % 2 or args.warmup % 2:
            print("bench.py: --graph replays pairs of iterations: use even --steps and --warmup", file=sys.stderr)
            return 2

        def block(k, timed=True):
            if graph is None:
                for _ in range(k):
                    sim.iteration()
            else:
                for _ in range(k // 2):
                    graph.replay()

        def run_block(k):
            torch.cuda.synchronize()
            t_begin = time.perf_counter()
            block(k)
            torch.cuda.synchronize()
            return time.perf_counter() - t_begin, []
    else:
        def block(k, timed=True):
            for _ in range(k):
                sim.iteration()

    def run_block_one_stream(k):
        """k iterations back to back on torch's current stream, every update launch bracketed by events on it."""
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(k)]
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        if schedule == B.ONE_LAUNCH:
            for _ in range(k):
                sim.iteration()
        else:
            for i in range(k):
                cur = sim.allreduce()
                ev[i][0].record()
                sim.update_from(1 - cur)
                ev[i][1].record()
                sim.t += 1
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_begin
        return wall, ([a.elapsed_time(b) for a, b in ev] if schedule != B.ONE_LAUNCH else [])

    if not two_streams and not args.graph:
        run_block = run_block_one_stream

    block(args.warmup, timed=False)
    (rt.sync() if rt else torch.cuda.synchronize())
    if args.graph:
        graph = sim.capture_pair()
        graph.replay()
        torch.cuda.synchronize()

    block_ms, upd_all = [], []
    for _ in range(args.repeats):
        wall_s, upd = run_block(args.steps)
        block_ms.append(wall_s * 1e3 / args.steps)
        upd_all += upd
    ms_per_step = float(np.median(block_ms))
    upd_ms = float(np.mean(upd_all)) if upd_all else None
    alone = None
    if rt is not None:
        # Beside the AllReduce launches of the other stream the update shares the memory bandwidth, so its
        # duration there says nothing about the kernel.  One more block of `steps` iterations, on one stream,
        # times it alone (the roofline figure); that block does not enter ms_per_step.
        rt.sync()
        for _ in range(2):
            sim.iteration()
        wall_s, upd_alone = run_block_one_stream(args.steps)
        alone = {"ms_per_step": wall_s * 1e3 / args.steps, "launch_ms": float(np.mean(upd_alone)), "launches": len(upd_alone)}
        overlapped_ms, upd_ms, upd_all = upd_ms, alone["launch_ms"], upd_alone
        rt.close()

    n_true = int(sum(numels))          # bucket padding is processed but is not part of the model
    model = bytes_model(mode, n_true, p, momentum != 0.0, fused=(schedule in (B.FUSED, B.ONE_LAUNCH)), direct=(schedule == B.DIRECT),
                        halving_doubling=(schedule == B.HALVING_DOUBLING))
    value = model["total"] / (ms_per_step * 1e-3) / 1e9
    upd_gbs = model["update"] / (upd_ms * 1e-3) / 1e9 if upd_ms else None

    mode_name = ["none", "trunc16", "quant8"][mode]
    traffic, traffic_note = committed_traffic(cfg, mode_name, B.get_launch_config(B.K_UPDATE, mode))

    cb = payload_bytes_per_elem(mode)
    working_set = p * n * (4 + 2 * cb + 8)              # gradients, two slot sets, w and v of every worker
    round_payload = n * cb                               # what one ring round writes (p blocks of n/p) and the next reads
    cache = {
        "infinity_cache_bytes": INFINITY_CACHE_BYTES, "working_set_bytes": int(working_set),
        "ring_round_payload_bytes": int(round_payload),
        "whole_iteration": bool(working_set <= INFINITY_CACHE_BYTES),
        "allreduce_rounds": bool(round_payload <= INFINITY_CACHE_BYTES),
        "note": ("the whole working set fits the memory-side cache: the figures are not HBM figures"
                 if working_set <= INFINITY_CACHE_BYTES else
                 "a ring round's payloads fit the memory-side cache, so the next round may read them from there: "
                 "the AllReduce part of `value` is cache-assisted; the update streams its operands once and is not"
                 if round_payload <= INFINITY_CACHE_BYTES else "nothing on this path fits the memory-side cache"),
    }

    out = {
        "metric": "aggregation+update GB/s (fraction of HBM peak) and iters/s at K=4, 61M params",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"config{cfg}:{W.CONFIG_NAMES[cfg]}", "workers": p, "elements_per_worker": n_true,
            "packed_elements_per_worker": n,
            "tensors": len(specs), "buckets": len(buckets) if buckets else 1,
            "compression": mode_name, "momentum": momentum, "lr": args.lr,
            "pipeline_width": 2, "schedule": args.schedule, "hip_graph": bool(args.graph),
            "streams": 2 if two_streams else 1, "staggered_buffers": not args.no_stagger, "seed": args.seed,
        },
        "repeats": args.repeats,
        "ms_per_step_min": round(min(block_ms), 5),
        "ms_per_step_max": round(max(block_ms), 5),
        "timing": f"wall clock around each of {args.repeats} blocks of {args.steps} iterations (synchronised on both "
                  f"sides); ms_per_step is the median block, min and max are the fastest and slowest block",
        "iters_per_s": round(1e3 / ms_per_step, 2),
        "hbm_peak_fraction": round(value / HBM_PEAK_GBS, 4),
        "cache_assisted": cache,
        "bytes_per_iter": {k: int(v) for k, v in model.items()},
        "roofline": {
            "kernel": "update_kernel (decompress + momentum-SGD, all replicas, one launch)",
            "bound": "hbm", "achieved": round(upd_gbs, 2) if upd_gbs else None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(upd_gbs / HBM_PEAK_GBS, 4) if upd_gbs else None, "traffic": traffic,
            "traffic_note": traffic_note,
            "launch_ms": round(upd_ms, 5) if upd_ms else None, "launches_timed": len(upd_all),
            "algorithmic_bytes_per_launch": int(model["update"]),
            "launch_geometry": dict(zip(("threads", "quads", "lds_bytes"), B.get_launch_config(B.K_UPDATE, mode))),
        },
        "kernel_sources_sha256": kernel_sources_sha256(),
        "input_generation_s": round(gen_s, 2),
    }
    if alone is not None:
        out["roofline"]["measured_in"] = (
            f"one more block of {args.steps} iterations run back to back on one stream after the {args.repeats} "
            f"two-stream blocks, where the kernel has the memory to itself (that block: "
            f"{round(alone['ms_per_step'], 5)} ms per iteration; `bench.py --streams 1` runs everything that way)")
        out["roofline"]["beside_the_allreduce"] = {
            "launch_ms": round(overlapped_ms, 5) if overlapped_ms else None,
            "note": "duration of the same launch in the two-stream blocks, where the AllReduce kernels of the other "
                    "stream run beside it and share the bandwidth: not a figure of the kernel",
        }
        out["one_stream_ms_per_step"] = round(alone["ms_per_step"], 5)
    else:
        out["roofline"]["measured_in"] = "every timed iteration (one stream: the kernel runs alone)"

    if args.phases:
        out["phases_ms"] = time_phases(sim, B, torch, np)
    if buckets:
        out["bucketing"] = time_packing(sim, B, torch, np, numels, offs, n, model["total"], with_iteration=args.phases)
    if args.phases:
        out["ceiling"] = stream_ceiling(sim, B, torch, np)         # last: the probes overwrite w and v

    if args.calib_copy > 0:
        dst = torch.empty_like(sim.g_local[0])
        for _ in range(args.calib_copy):
            B.compress(B.NONE, sim.g_local[0], n, dst, None)
        torch.cuda.synchronize()
        out["calib_copy"] = {"kernel": "compress_kernel<0>", "launches": args.calib_copy,
                             "read_bytes_per_launch": 4 * n, "write_bytes_per_launch": 4 * n}

    study = None
    if args.study is not None:
        import bench_studies as studies
        if args.study == "within-allreduce":
            study = studies.within_allreduce(sim, mode, n, p)
        elif args.study == "two-thread-runtime":
            study = studies.two_thread_runtime(sim, schedule)
        elif args.study == "size-sweep":
            study = studies.size_sweep(mode, p, momentum, args.seed, stagger=not args.no_stagger)
        else:
            study = studies.ring_cost_model(mode, n, p, args.seed)

    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(mode, grads, w0, p, args.lr, momentum, buckets, model["total"],
                                           args.cpu_seconds)
    print(json.dumps(out), flush=True)
    if study is not None:
        print(json.dumps(study), flush=True)
    return 0


def time_packing(sim, B, torch, np, numels, offs, n, iter_bytes, with_iteration: bool, reps: int = 20):
    """Step a0, timed on its own (it is NOT part of the timed iteration, whose
    gradients already sit in the packed buffers): gather every worker's
    per-layer gradient tensors into its packed buffer, one launch for all
    tensors of all workers, and the scatter back.  With --phases also the
    iteration with one gather launch put in front of every AllReduce."""
    p, dev = sim.p, sim.device
    starts = np.cumsum([0] + [ne + (-ne) % 4 for ne in numels])        # 16-byte aligned tensors in one arena
    arenas = [torch.randn(int(starts[-1]), device=dev) * 1e-3 for _ in range(p)]
    tptr, pptr, ne = [], [], []
    for r in range(p):
        for ti, n_i in enumerate(numels):
            tptr.append(arenas[r].data_ptr() + 4 * int(starts[ti]))
            pptr.append(sim.g_local[r].data_ptr() + 4 * offs[ti])
            ne.append(n_i)
    tab, total = B.segments_prepare(tptr, pptr, ne)
    tab_dev = torch.frombuffer(bytearray(bytes(tab)), dtype=torch.uint8).to(dev)

    def timed(fn):
        ts = []
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.median(ts))

    pack_ms = timed(lambda: B.pack(tab_dev, len(ne), total))
    unpack_ms = timed(lambda: B.unpack(tab_dev, len(ne), total))
    moved = 8.0 * p * float(sum(numels))

    # the whole iteration with the gather in it: gather on the communication stream in front of the AllReduce,
    # the update beside both on the other stream
    res = {"tensors": len(numels), "workers": p, "launches": 1, "pack_ms": round(pack_ms, 5),
           "unpack_ms": round(unpack_ms, 5), "pack_GBps": round(moved / pack_ms / 1e6, 1),
           "unpack_GBps": round(moved / unpack_ms / 1e6, 1), "included_in_value": False}
    if with_iteration and sim.schedule in (B.STEPWISE, B.FUSED):
        rt = B.Runtime()
        comm = rt.stream(1)

        def run(k):
            for _ in range(k):
                cur = (sim.t + 1) % 2
                B.pack(tab_dev, len(ne), total, stream=comm)
                rt.iteration(sim.rings[cur], sim.updates[1 - cur], sim.updates[cur], sim.schedule, 2, sim.lr,
                             sim.momentum, sim.grad_scale)
                sim.t += 1
        run(6)
        rt.sync()
        blocks = []
        for _ in range(5):
            t0 = time.perf_counter()
            run(100)
            rt.sync()
            blocks.append((time.perf_counter() - t0) * 10.0)           # ms per iteration
        rt.close()
        ms = float(np.median(blocks))
        res["iteration_with_pack_ms"] = round(ms, 5)
        res["iteration_with_pack_GBps"] = round((iter_bytes + moved) / ms / 1e6, 1)
    return res


def kernel_sources_sha256() -> str:
    """Hash of the kernel sources: a counter summary under profiles/ holds for the code it was taken with."""
    import hashlib
    from paper_1811_03619_amd import buildlib
    h = hashlib.sha256()
    for name in ("pipesgd_kernels.hip", "pipesgd_device.hpp"):
        h.update(open(os.path.join(buildlib.CSRC, name), "rb").read())
    return h.hexdigest()


def committed_traffic(cfg: int, mode_name: str, update_geometry):
    """HBM-side bytes per update launch from the committed rocprofv3 --pmc
    summary of this workload (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy
    kernel of known size) -- only if that summary was taken with the kernel
    sources and the update launch geometry of this run; otherwise None and the
    reason."""
    import glob
    import re
    paths = sorted(glob.glob(os.path.join(ROOT, "profiles", f"pmc_traffic_config{cfg}_*{mode_name}*.txt")))
    if not paths:
        return None, "no counter summary under profiles/ for this workload"
    text = open(paths[0]).read()
    m = re.search(r"^update_kernel traffic_bytes_per_launch = (\d+)", text, flags=re.M)
    g = re.search(r"^update_kernel launch_config = threads (\d+) quads (\d+) lds_bytes (\d+)", text, flags=re.M)
    h = re.search(r"^kernel_sources_sha256 = ([0-9a-f]{64})", text, flags=re.M)
    name = os.path.basename(paths[0])
    if not (m and g and h):
        return None, f"{name} does not say which sources and launch geometry it was taken with"
    if tuple(int(x) for x in g.groups()) != tuple(update_geometry):
        return None, f"{name} was taken with update geometry {g.groups()}, this run uses {tuple(update_geometry)}"
    if h.group(1) != kernel_sources_sha256():
        return None, f"{name} was taken with other kernel sources than this tree's"
    return int(m.group(1)), f"from {name} (same kernel sources, same launch geometry)"


def time_phases(sim, B, torch, np, reps: int = 20):
    """Per-launch durations of each phase (separate pass, after the timed region)."""
    ring = sim.rings[0]
    p = sim.p
    res = {}

    def timed(fn):
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return round(float(np.median(ts)), 5)

    res["first_send"] = timed(lambda: B.ring_first_send(ring))
    res["reduce_scatter_step"] = [timed(lambda s=s: B.ring_reduce_scatter_step(ring, s)) for s in range(p - 1)]
    res["allgather_step"] = [timed(lambda s=s: B.ring_allgather_step(ring, s)) for s in range(p - 1)]
    res["allreduce_stepwise"] = timed(lambda: B.allreduce_sim(ring, B.STEPWISE))
    res["allreduce_fused"] = timed(lambda: B.allreduce_sim(ring, B.FUSED))
    if sim.schedule in (B.DIRECT, B.HALVING_DOUBLING):
        res["allreduce_selected_schedule"] = timed(lambda: sim.allreduce())
    # the stand-alone codecs on one worker's gradient (pipesgd_compress / pipesgd_decompress)
    from paper_1811_03619_amd.pipeline import payload_empty
    ns = B.num_scales(sim.mode, sim.n)
    pay = payload_empty(sim.mode, sim.n, sim.device)
    sc = torch.zeros(max(ns, 1), dtype=torch.float32, device=sim.device)[:ns] if sim.mode == B.QUANT8 else None
    back = torch.empty_like(sim.g_local[0])
    res["compress_one_worker"] = timed(lambda: B.compress(sim.mode, sim.g_local[0], sim.n, pay, sc))
    res["decompress_one_worker"] = timed(lambda: B.decompress(sim.mode, pay, sc, sim.n, back))
    # ceiling probe with the library's own plain copy (NONE "compression"): 4n bytes in, 4n out, Gaussian data
    res["plain_copy_one_gradient"] = timed(lambda: B.compress(B.NONE, sim.g_local[0], sim.n, back, None))
    res["plain_copy_GBps"] = round(8.0 * sim.n / res["plain_copy_one_gradient"] / 1e6, 1)
    res["update_all_replicas"] = timed(lambda: sim.update_from(1))
    one = B.UpdateArgs(sim.slots[1][:1], sim.slot_scales[1][:1] if sim.mode == B.QUANT8 else None, sim.w[:1],
                       sim.v[:1] if sim.momentum != 0.0 else None)
    res["update_one_replica"] = timed(lambda: B.apply_update_multi(sim.mode, one, sim.n, sim.lr, sim.momentum,
                                                                   sim.grad_scale))
    return res


def stream_ceiling(sim, B, torch, np, reps: int = 15):
    """What the memory system sustains for the update's access mix: the library's
    stream probes (the update's loads and stores over the update's own buffers,
    grid and cache policy, no arithmetic) in a handful of launch geometries, best
    of each.  Overwrites w and v, so it runs last."""
    ua = sim.updates[1]
    p, n, mode = sim.p, sim.n, sim.mode
    cb = payload_bytes_per_elem(mode)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.median(ts))

    geos = [(64, 4, 53248), (64, 4, 65536), (128, 2, 65536), (256, 1, 53248), (256, 1, 65536), (256, 1, 0),
            (256, 4, 0), (512, 2, 0), (256, 2, 53248)]
    kinds = {"read_only": (B.PROBE_READ, p * n * (cb + 8.0)), "write_only": (B.PROBE_WRITE, p * n * 8.0),
             "mixed_in_place": (B.PROBE_MIXED, p * n * (cb + 16.0)), "copy": (B.PROBE_COPY, p * n * 8.0)}
    res = {"what": "pipesgd_probe_stream over the update's buffers (all replicas), best launch geometry of each kind",
           "unit": "GB/s"}
    for name, (kind, nbytes) in kinds.items():
        best = None
        for (t, q, lds) in geos:
            ms = timed(lambda: B.probe_stream(kind, mode, ua, n, t, q, lds))
            if best is None or ms < best[0]:
                best = (ms, (t, q, lds))
        res[name] = {"GBps": round(nbytes / best[0] / 1e6, 1), "ms": round(best[0], 5), "bytes": int(nbytes),
                     "geometry": list(best[1])}
    upd_bytes = p * n * (cb + 16.0)
    t, q, lds = B.get_launch_config(B.K_UPDATE, mode)
    upd_ms = timed(lambda: sim.update_from(1))
    res["update_kernel"] = {"GBps": round(upd_bytes / upd_ms / 1e6, 1), "ms": round(upd_ms, 5), "geometry": [t, q, lds]}
    res["update_over_mixed_probe"] = round(res["update_kernel"]["GBps"] / res["mixed_in_place"]["GBps"], 4)
    # reads and writes take turns on the memory bus: the time of a mix is at least the sum of its parts' times
    rd, wr = res["read_only"]["GBps"], res["write_only"]["GBps"]
    res["no_interference_bound_GBps"] = round((cb + 16.0) / ((cb + 8.0) / rd + 8.0 / wr), 1)
    return res


def cpu_baseline(mode, grads, w0, p, lr, momentum, buckets, bytes_total, budget_s):
    """The oracle as it stands, same inputs, same iteration (AllReduce of p
    workers + update of p replicas).  `value` is the oracle on ONE host thread
    (it is single-threaded as written).  `all_cores` runs the same oracle calls
    on every host core at once: the vector is cut into as many 4096-aligned slabs
    as there are threads and each thread runs the oracle's AllReduce and update on
    its slab (the calls release the interpreter lock).  Same arithmetic per element
    and the same bytes; only the assignment of elements to ring blocks differs from
    the single call, which timing does not care about."""
    import concurrent.futures as cf

    import numpy as np

    import oracle
    n = w0.size

    def one_iteration(lo, hi, ws, vs, slot):
        g = [x[lo:hi] for x in grads]
        if buckets:
            bl = [(max(st, lo) - lo, min(st + nb, hi) - max(st, lo)) for st, nb in buckets if st < hi and st + nb > lo]
            A = oracle.allreduce_bucketed(mode, g, bl)
        else:
            A = oracle.allreduce(mode, g)
        use = A if slot is None else slot            # same work either way; the first pass has no earlier slot
        for r in range(p):
            oracle.sgd_update(mode, use[r][0], use[r][1], ws[r], vs[r] if momentum else None, lr, momentum, 1.0)
        return A

    def run(threads):
        if buckets and threads > 1:
            # whole buckets per thread: a new slab starts at the first bucket past each equal share of the elements
            cuts = [0]
            for st, nb in buckets:
                if st > 0 and st >= n * len(cuts) / threads and len(cuts) < threads:
                    cuts.append(st)
            cuts.append(n)
        else:
            step = -(-n // threads // 4096) * 4096 if threads > 1 else n
            cuts = list(range(0, n, max(step, 4096))) + [n]
        slabs = [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
        state = []
        for lo, hi in slabs:
            state.append([[w0[lo:hi].copy() for _ in range(p)], [np.zeros(hi - lo, np.float32) for _ in range(p)], None])
        iters, t0 = 0, time.perf_counter()
        with cf.ThreadPoolExecutor(max_workers=len(slabs)) as pool:
            while True:
                futs = [pool.submit(one_iteration, lo, hi, st[0], st[1], st[2]) for (lo, hi), st in zip(slabs, state)]
                for st, f in zip(state, futs):
                    st[2] = f.result()
                iters += 1
                el = time.perf_counter() - t0
                if el >= budget_s or el * (iters + 1) / iters > 2.5 * budget_s:
                    break
        return el / iters, iters, len(slabs)

    s1, it1, _ = run(1)
    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16") or 16)))
    sN, itN, used = run(cores) if cores > 1 else (s1, it1, 1)
    return {"value": round(bytes_total / s1 / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{it1} full iteration(s) of the same workload (all {p} workers, all {n} elements)",
            "s_per_iter": round(s1, 4), "iters_per_s": round(1.0 / s1, 4),
            "all_cores": {"value": round(bytes_total / sN / 1e9, 3), "unit": "GB/s", "cores": used, "kind": "oracle",
                          "sample": f"{itN} full iteration(s); the vector cut into {used} slabs, one oracle call "
                                    f"sequence per slab and thread",
                          "s_per_iter": round(sN, 4), "iters_per_s": round(1.0 / sN, 4),
                          "host_cpus_visible": os.cpu_count()}}


if __name__ == "__main__":
    sys.exit(main())
