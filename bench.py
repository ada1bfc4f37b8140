"""Throughput of the fused gossip + Adam (+ accumulate) step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A "step" is one iteration t of the decentralized accumulated Adam algorithm over the whole
workload: one call of dadam_gossip_step (all rows, all elements) followed by the exchange of the
ping-pong parameter buffers.  Inputs (parameters, a small pool of pre-generated gradient sets,
zero moments) are resident in HBM before the timed region starts.  Prints ONE JSON line.

The headline workload is the benchmark's configuration 2 (16 replicas, static exponential graph,
GPT-2-small tensor shapes, float32, s = 4); --config selects 1..5.  Without --config the same line
also carries, under "per_config", the same measurement of configurations 3, 4 and 5 (each with its
own step count, buffers freed in between) and, under "packed_frac", configuration 2 again with one
ordinary allocation per buffer instead of the placed arena.

Other measurements share the set-up (none of them is the benchmark's value): --path selects another
call sequence (unfused, mix, mix_consensus, accumulate, buckets), --bucket-streams and
--standin-backward shape the bucket sequence, --graph replays a recorded HIP graph, --layout selects
where the buffers sit in HBM, --prealloc-gib allocates that much first (a job's weights and
activations), --mode forces a kernel.  See --help.
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

HBM_PEAK_BYTES_PER_S = 8.0e12   # MI355X HBM3E, published peak

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, each in a run of its
# own, each scaled by what the same counter reads for a plain 1 GiB device copy) cannot be measured
# inside this script.  paper_2410_11998_amd/rocprof_summary.py writes them, per workload, kernel and
# phase, into profiles/hbm_traffic.txt from the profiler's own CSV files; the line quotes them only
# for the very kernel shape that was profiled and says where they come from.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic():
    """{(workload, kernel): {phase: (bytes, source)}} from profiles/hbm_traffic.txt; empty if absent."""
    table = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("#") or not line.strip():
                    continue
                workload, kernel, phase, nbytes, source = line.split()
                table.setdefault((workload, kernel), {})[phase] = (float(nbytes), source)
    except OSError:
        pass
    return table


def phase_of(t: int, s: int) -> str:
    if s == 1:
        return "alg1"
    if t % s == 0:
        return "fold"
    if (t - 1) % s == 0:
        return "loopstart"
    return "plain"


def algorithmic_bytes_per_replica_param(wl, phase: str) -> float:
    """Every distinct input read once, every output written once (per updated element)."""
    px = 2 if wl.param_dtype == "bf16" else 4
    pg = 2 if wl.grad_dtype == "bf16" else 4
    src = px * wl.n_cols / wl.n_rows      # each source buffer is one datum however many rows read it
    common = src + px + pg + 4 + 4        # x read, x written, g, m_hat, v_hat read
    if phase == "alg1":
        return common + 8                 # moments written back, no accumulator
    if phase == "plain":
        return common + 4 + 4             # b read, b written
    if phase == "loopstart":
        return common + 4                 # b written only
    if phase == "fold":
        return common + 4 + 4 + 8         # b read, b written (zero), moments written
    raise ValueError(phase)


def path_bytes_per_replica_param(wl, phase: str, path: str) -> float:
    """Bytes the kernels of a non-default --path have to move per updated element (for the fused and
    the bucketed path this is the algorithmic figure)."""
    px = 2 if wl.param_dtype == "bf16" else 4
    pg = 2 if wl.grad_dtype == "bf16" else 4
    src = px * wl.n_cols / wl.n_rows
    if path in ("fused", "buckets"):
        return algorithmic_bytes_per_replica_param(wl, phase)
    acc = {"alg1": pg + 8 + 8, "plain": pg + 4 + 4, "loopstart": pg + 4, "fold": pg + 4 + 4 + 8 + 8}[phase]
    if path == "accumulate":
        return acc
    if path in ("mix", "mix_consensus"):
        return src + px
    return (src + px + pg + 8) + acc          # unfused: update-only pass, then the accumulate pass


def cpu_baseline(wl, x0_sample, grad_samples, csrs, iters: int, threads: int = 1):
    """The CPU oracle as it stands, timed on this host on a bounded sample of the workload.

    threads > 1: the sample's coordinates are cut into that many slices and each thread runs the same
    oracle on its slice (coordinates never interact, so the slices are independent runs)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import dadam_oracle as O
    hp = O.Hyper(float(np.float32(wl.lr)), float(np.float32(wl.beta1)), float(np.float32(wl.beta2)),
                 float(np.float32(wl.eps)), wl.s)
    n = x0_sample[0].shape[0]
    ocsr = [O.Csr(np.asarray(rp), np.asarray(col), np.asarray(w, dtype=np.float64)) for rp, col, w in csrs]
    cuts = [n * k // threads for k in range(threads + 1)]

    def run_slice(k: int):
        lo, hi = cuts[k], cuts[k + 1]
        z = lambda: [np.zeros(hi - lo) for _ in range(wl.n_rows)]
        st = O.State([x[lo:hi].copy() for x in x0_sample], z(), z(), z())
        for t in range(1, iters + 1):
            g = [gi[lo:hi] for gi in grad_samples[(t - 1) % len(grad_samples)]]
            xn = O.dadam_step(st, g, ocsr[wl.slot_of_step(t)], t, hp, "O32m", wl.param_dtype)
            for i in range(wl.n_rows):
                st.x_src[i] = xn[i]

    t0 = time.perf_counter()
    if threads == 1:
        run_slice(0)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(run_slice, range(threads)))
    dt = time.perf_counter() - t0
    return wl.n_rows * n * iters / dt, dt


def host_cpu():
    """(model name, logical CPUs this process may run on) of the machine the baseline is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return model, n


def kernel_name(info, tile_mode: bool, wl, path: str, shared: bool = False) -> str:
    """Name of the kernel shape a launch uses, as the profile summaries spell it (a direct kernel whose rows
    share sources streams everything but the sources: "shared")."""
    dt = {"f32": "TF32", "bf16": "TBF16"}
    nt = "true" if info.streaming else "false"
    if not tile_mode and shared and info.streaming:
        nt = "shared"
    if path in ("mix", "mix_consensus"):
        return f"k_tile<{dt[wl.param_dtype]},{dt[wl.grad_dtype]},{info.mix_waves},{info.mix_vectors},{nt}>" if tile_mode else \
               f"k_direct<{dt[wl.param_dtype]},{dt[wl.grad_dtype]},{nt}>"
    if tile_mode:
        return f"k_tile<{dt[wl.param_dtype]},{dt[wl.grad_dtype]},{info.tile_waves},{info.tile_vectors},{nt}>"
    return f"k_direct<{dt[wl.param_dtype]},{dt[wl.grad_dtype]},{nt}>"


def measure(args, want_cpu_sample: bool):
    """Set up one workload, time it, free everything.  Returns (result dict, cpu sample or None)."""
    import numpy as np
    import torch
    from paper_2410_11998_amd import binding as B
    from paper_2410_11998_amd import workloads as WL

    dev = torch.device("cuda:0")
    wl = WL.workload(args.config, scale_div=args.scale_div)
    K = args.steps if args.steps is not None else wl.steps
    W = args.warmup
    layout = wl.layout()
    d, R, C = layout.d, wl.n_rows, wl.n_cols
    TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
    ADT = {"f32": B.DADAM_F32, "bf16": B.DADAM_BF16}
    pdt, gdt = TDT[wl.param_dtype], TDT[wl.grad_dtype]
    inplace = args.inplace or R != C

    # ---- resident inputs ----------------------------------------------------------------
    prealloc = torch.empty(args.prealloc_gib << 30, dtype=torch.uint8, device=dev) if args.prealloc_gib else None
    # Buffers in layout order: sources (own replicas, then receive buffers), outputs (unless in
    # place), m_hat, v_hat, b, then the gradient pool.
    n_pool = max(1, args.pool)
    kinds = [("x_src", pdt)] * C + ([] if inplace else [("x_dst", pdt)] * R) + [("m", torch.float32)] * R + \
            [("v", torch.float32)] * R + ([("b", torch.float32)] * R if wl.s > 1 else []) + [("g", gdt)] * (R * n_pool)
    esize = {torch.float32: 4, torch.bfloat16: 2}
    arena = None
    placement_advice = None
    if args.layout in ("spread", "rule", "whole"):
        from paper_2410_11998_amd.arena import SpreadArena
        arena = SpreadArena([d * esize[dt] for _, dt in kinds], dev, two_regions=(args.layout != "whole"),
                            calibrate=(args.layout == "spread"))
        bufs = arena.views([dt for _, dt in kinds])
        hbm_layout = arena.describe()
        placement_advice = {B.DADAM_PLACE_TWO_REGIONS: "two regions", B.DADAM_PLACE_ARENA_ELSEWHERE: "arena elsewhere",
                            B.DADAM_PLACE_TOO_LARGE: "too large"}.get(arena.advice, "none")
    else:
        bufs = [torch.empty(d, dtype=dt, device=dev) for _, dt in kinds]
        hbm_layout = "packed: one ordinary allocation per buffer"
    if args.prealloc_gib:
        hbm_layout += f"; {args.prealloc_gib} GiB allocated first"
    take = lambda name: [b for (k, _), b in zip(kinds, bufs) if k == name]
    x_src = take("x_src")
    x_dst = x_src[:R] if inplace else take("x_dst")
    m_hat, v_hat = take("m"), take("v")
    acc = take("b") if wl.s > 1 else None
    gflat = take("g")
    pool = [gflat[p * R:(p + 1) * R] for p in range(n_pool)]
    x0 = WL.normal_torch(WL.seed_for(wl.cfg, 0), (d,), wl.param_std, dev, pdt)     # one draw shared by all replicas
    for i in range(R):
        x_src[i].copy_(x0)
    for c in range(R, C):                                                          # neighbours' receive buffers
        x_src[c].copy_(WL.normal_torch(WL.seed_for(wl.cfg, 1) + c, (d,), wl.param_std, dev, pdt))
    del x0
    for t_ in ([] if inplace else x_dst) + m_hat + v_hat + (acc or []):
        t_.zero_()
    gen = torch.Generator(device=dev)
    tmp = torch.empty(d, dtype=torch.float32, device=dev)
    for p in range(n_pool):
        gen.manual_seed(WL.seed_for(wl.cfg, 2 + p))
        for i in range(R):
            tmp.normal_(0.0, wl.grad_std, generator=gen)
            pool[p][i].copy_(tmp)
    del tmp

    csrs = [wl.csr(k) for k in range(wl.n_slots())]
    h = B.dadam_init(R, C, d, layout.offsets, layout.numels, ADT[wl.param_dtype], ADT[wl.grad_dtype], wl.lr, wl.beta1,
                     wl.beta2, wl.eps, wl.s, -1.0, device=0)
    for k, (rp, col, w) in enumerate(csrs):
        B.dadam_set_topology(h, k, rp, col, w)
    B.dadam_bind(h, x_src, x_dst, m_hat, v_hat, acc)
    flags = B.DADAM_FUSE_ACCUM | {"auto": 0, "tile": B.DADAM_FORCE_TILE, "direct": B.DADAM_FORCE_DIRECT}[args.mode]
    tile_mode = (args.mode == "tile") or (args.mode == "auto" and B.dadam_slot_uses_tile_mode(h, 0))
    info = B.dadam_get_plan_info(h)
    if args.path == "mix_consensus" and args.mode != "direct" and info.tile_mode_possible:
        tile_mode = True                                  # the consensus error is a by-product of the staged tile
    tables = [B.grad_table(h, g) for g in pool]          # pointer tables marshalled once, as a training loop would

    # sample for the CPU baseline, taken before anything is updated
    # about 1e9 replica-param updates of CPU work: 2^26 / R coordinates per row
    sample = None
    if want_cpu_sample:
        ns = min(args.cpu_sample if args.cpu_sample else (1 << 26) // R, d)
        sample = (wl, ns, [x[:ns].to(torch.float64).cpu().numpy() for x in x_src],
                  [[g[:ns].to(torch.float64).cpu().numpy() for g in gs] for gs in pool], csrs)

    # tensor ranges of about --bucket-mb of parameters each, in layout order (the granularity at which
    # the paper's implementation updates and communicates)
    buckets = []
    if args.path == "buckets":
        per = int(args.bucket_mb * 1e6 / (2 if wl.param_dtype == "bf16" else 4))
        start, cur = 0, 0
        for k, n_k in enumerate(layout.numels):
            cur += int(n_k)
            if cur >= per or k == len(layout.numels) - 1:
                buckets.append((start, k + 1))
                start, cur = k + 1, 0
    mode_flags = flags & ~B.DADAM_FUSE_ACCUM
    consensus_out = torch.zeros(1, dtype=torch.float64, device=dev)
    side = [torch.cuda.Stream(device=dev) for _ in range(args.bucket_streams)] if args.bucket_streams > 1 else []
    standin = standin_out = None
    if args.standin_backward > 0 and args.path == "buckets":
        standin = torch.randn(args.standin_backward, args.standin_backward, device=dev, dtype=torch.bfloat16)
        standin_out = torch.empty_like(standin)
    launches_per_step = len(buckets) if args.path == "buckets" else 2 if args.path == "unfused" else 1

    def one_step(t: int):
        stream = B.current_stream()      # read at call time: a graph capture changes torch's current stream
        g = tables[t % len(tables)]
        slot = wl.slot_of_step(t)
        if args.path == "fused":
            B.dadam_gossip_step(h, slot, g, t, flags, stream)
        elif args.path == "unfused":
            B.dadam_gossip_step(h, slot, g, t, mode_flags, stream)
            B.dadam_accumulate(h, g, t, stream)
        elif args.path == "mix":
            B.dadam_mix(h, slot, mode_flags, stream)
        elif args.path == "mix_consensus":
            B.dadam_mix_consensus(h, slot, consensus_out, mode_flags, stream)
        elif args.path == "accumulate":
            B.dadam_accumulate(h, g, t, stream)
        elif standin is not None:
            # the single-GPU analogue of the paper's schedule: a stand-in "backward" of bucket k on the step's
            # stream, the bucket's update behind it - on the same stream, or on a side stream so that it runs
            # beside the stand-in of bucket k + 1
            main = torch.cuda.current_stream()
            for k, (tb, te) in enumerate(buckets):
                torch.matmul(standin, standin, out=standin_out)
                if args.standin_only:
                    continue
                if side:
                    st = side[k % len(side)]
                    ev = torch.cuda.Event()
                    ev.record(main)
                    st.wait_event(ev)
                    B.dadam_gossip_step_range(h, slot, g, t, flags, tb, te, st.cuda_stream)
                else:
                    B.dadam_gossip_step_range(h, slot, g, t, flags, tb, te, stream)
            for st in side:
                main.wait_stream(st)
        elif len(side) <= 1:
            for tb, te in buckets:
                B.dadam_gossip_step_range(h, slot, g, t, flags, tb, te, stream)
        else:
            # buckets dealt over side streams (default priority) so that one bucket's drain overlaps the next
            # one's ramp; the step's stream forks to them and joins them again
            main = torch.cuda.current_stream()
            fork = torch.cuda.Event()
            fork.record(main)
            for st in side:
                st.wait_event(fork)
            for k, (tb, te) in enumerate(buckets):
                B.dadam_gossip_step_range(h, slot, g, t, flags, tb, te, side[k % len(side)].cuda_stream)
            for st in side:
                join = torch.cuda.Event()
                join.record(st)
                main.wait_event(join)
        if not inplace and args.path != "accumulate":
            B.dadam_swap_x(h)

    t = 0
    for _ in range(W):
        t += 1
        one_step(t)
    torch.cuda.synchronize()

    graph, L = None, 1
    if args.graph:
        # One replayable graph of L consecutive iterations: a whole number of accumulation loops, of
        # the topology schedule's periods and of buffer exchanges, so that a replay leaves the handle as
        # it found it.  The iteration numbers (hence the bias corrections) are those of the capture.
        L = wl.s
        while (not inplace and L % 2) or L % wl.n_slots():
            L += wl.s
        K = max(L, K // L * L)
        t_graph = t
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for j in range(L):
                one_step(t_graph + 1 + j)
        graph.replay()                      # one untimed replay
        torch.cuda.synchronize()

    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    phases = []
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    if graph is None:
        for k in range(K):
            t += 1
            phases.append(phase_of(t, wl.s))
            ev0[k].record()
            one_step(t)
            ev1[k].record()
    else:
        for r in range(K // L):
            phases += [phase_of(t_graph + 1 + j, wl.s) for j in range(L)]
            ev0[r].record()
            graph.replay()
            ev1[r].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin

    region_ms = [elapsed / K * 1e3]
    for _ in range(max(0, args.repeats - 1)):
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        if graph is None:
            for k in range(K):
                t += 1
                one_step(t)
        else:
            for r in range(K // L):
                graph.replay()
        torch.cuda.synchronize()
        region_ms.append((time.perf_counter() - r0) / K * 1e3)

    # Host time of one library call through the Python binding: short bursts of at most 64 launches into an
    # idle queue (a longer run of launches fills the queue and then proceeds at the GPU's pace), nothing
    # waited for inside the burst; the fastest of five bursts.
    host_us = None
    if graph is None:
        burst = max(1, 64 // launches_per_step)
        best = float("inf")
        for _ in range(5):
            torch.cuda.synchronize()
            r0 = time.perf_counter()
            for k in range(burst):
                t += 1
                one_step(t)
            best = min(best, time.perf_counter() - r0)
        torch.cuda.synchronize()
        host_us = best / (burst * launches_per_step) * 1e6

    if graph is None:
        kernel_ms = [ev0[k].elapsed_time(ev1[k]) for k in range(K)]
    else:
        # inside a graph single launches cannot be bracketed: every iteration of a replay gets the replay's average
        kernel_ms = [ev0[r].elapsed_time(ev1[r]) / L for r in range(K // L) for _ in range(L)]
    avg_kernel_s = sum(kernel_ms) / K / 1e3
    replica_params = R * d
    value = replica_params * K / elapsed
    bytes_per_launch = replica_params * sum(path_bytes_per_replica_param(wl, p, args.path) for p in phases) / K
    achieved = bytes_per_launch / avg_kernel_s
    by_phase = {}
    for p, ms in zip(phases, kernel_ms):
        by_phase.setdefault(p, []).append(ms)

    # counter-measured HBM bytes, only for the kernel shape that was profiled
    import numpy as np
    kname = kernel_name(info, tile_mode, wl, args.path, shared=bool(np.bincount(csrs[0][1], minlength=C).max() > 1))
    traffic, traffic_source = None, None
    table = measured_traffic().get((wl.name, kname))
    if table is not None and args.path == "fused" and all(p in table for p in phases):
        traffic = sum(table[p][0] for p in phases) / K
        traffic_source = f"{sorted({table[p][1] for p in phases})[0]} ({kname}; rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not this run)"

    out = {
        "metric": "replica-params updated/sec for fused gossip+Adam step",
        "value": value,
        "unit": "replica-params/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": elapsed / K * 1e3,
        "ms_per_step_regions": {"n": len(region_ms), "median": sorted(region_ms)[len(region_ms) // 2], "min": min(region_ms),
                                "max": max(region_ms)},
        # host time of one library call through the Python binding, nothing waited for (None under --graph)
        "host_us_per_call": host_us,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",     # the arithmetic type; parameters and gradients are stored as config.param_dtype / grad_dtype
        "data": "synthetic",
        "config": {
            "workload": wl.name, "param_dtype": wl.param_dtype, "grad_dtype": wl.grad_dtype, "state_dtype": "f32", "n_rows": R, "n_sources": C, "d": d, "tensors": len(layout.names), "topology": wl.topology,
            "accum_s": wl.s, "kernel": kname, "lds_bytes_per_workgroup": int(info.lds_bytes_tile) if tile_mode else 0,
            "device_lds_limit": int(info.lds_limit_bytes), "device_xcds": int(info.n_xcds), "path": args.path,
            "launches_per_step": launches_per_step, "x_buffers": "in-place" if inplace else "ping-pong",
            "hbm_layout": hbm_layout, "placement_advice": placement_advice,
            "placement_probe_launches": arena.probe_launches if arena is not None else 0,
            "grad_pool": len(pool),
            "issue": "eager" if graph is None else f"graph of {L} iterations, replayed",
            "bucket_streams": max(1, len(side)) if args.path == "buckets" else None,
            "standin_backward": (f"{args.standin_backward}^3 bf16 matmul per bucket" + (" only" if args.standin_only else "")) if standin is not None else None,
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved / 1e9, "peak": HBM_PEAK_BYTES_PER_S / 1e9, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_BYTES_PER_S, "traffic": traffic, "traffic_source": traffic_source,
            "algorithmic_bytes_per_launch": bytes_per_launch, "avg_launch_ms": avg_kernel_s * 1e3,
            "ms_by_phase": {p: sum(v) / len(v) for p, v in by_phase.items()},
        },
    }

    torch.cuda.synchronize()
    B.dadam_destroy(h)
    if args.copy_calibration:
        n_cal = (1 << 30) // 4
        src = torch.empty(n_cal, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    return out, sample


def measure_and_release(args, want_cpu_sample: bool):
    """measure(), then make sure its device memory is back with the driver: the next measurement places
    its buffers by what is in use at that moment."""
    import gc
    import torch
    res = measure(args, want_cpu_sample)
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return res


def brief(res: dict) -> dict:
    """What "per_config" keeps of a measurement."""
    return {"workload": res["config"]["workload"], "kernel": res["config"]["kernel"], "steps": res["steps"],
            "value": res["value"], "ms_per_step": res["ms_per_step"], "ms_per_step_regions": res["ms_per_step_regions"],
            "avg_launch_ms": res["roofline"]["avg_launch_ms"], "ms_by_phase": res["roofline"]["ms_by_phase"],
            "algorithmic_bytes_per_launch": res["roofline"]["algorithmic_bytes_per_launch"],
            "achieved_GBps": res["roofline"]["achieved"], "frac": res["roofline"]["frac"],
            "host_us_per_call": res["host_us_per_call"], "hbm_layout": res["config"]["hbm_layout"]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None,
                    help="1..5; default: 2 as the headline plus configurations 3, 4, 5 and the packed layout on the side")
    ap.add_argument("--mode", choices=["auto", "tile", "direct"], default="auto")
    ap.add_argument("--inplace", action="store_true", help="update parameters in place instead of ping-pong")
    ap.add_argument("--pool", type=int, default=2, help="number of pre-generated gradient sets cycled through")
    ap.add_argument("--path", choices=["fused", "unfused", "mix", "mix_consensus", "accumulate", "buckets"], default="fused",
                    help="fused: one dadam_gossip_step per iteration (the benchmark); unfused: dadam_gossip_step without "
                         "accumulation followed by dadam_accumulate; mix: dadam_mix only; accumulate: dadam_accumulate only; "
                         "buckets: the fused step issued tensor range by tensor range (--bucket-mb)")
    ap.add_argument("--bucket-mb", type=float, default=25.0, help="target bucket size for --path buckets")
    ap.add_argument("--bucket-streams", type=int, default=1,
                    help="--path buckets: deal the buckets of a step over that many streams (1: the step's own stream)")
    ap.add_argument("--standin-backward", type=int, default=0,
                    help="--path buckets: before each bucket's update run an N x N bfloat16 matmul on the step's stream as a "
                         "stand-in for that bucket's backward pass; with --bucket-streams >= 2 the updates go to side "
                         "streams and overlap the next stand-in (the value then is not the benchmark's metric)")
    ap.add_argument("--standin-only", action="store_true", help="with --standin-backward: skip the updates (the stand-in alone)")
    ap.add_argument("--layout", choices=["spread", "rule", "whole", "packed"], default="spread",
                    help="spread: one arena over most of the free HBM, buffers dealt alternately over two stretches of it "
                         "that a timing probe finds to lie in different thirds of the memory (see "
                         "paper_2410_11998_amd/arena.py); rule: no probe, the two regions either side of the arena's 96 GiB "
                         "mark when the arena covers the device, equal distances otherwise; whole: the same arena, always "
                         "equal distances; packed: one ordinary allocation per buffer")
    ap.add_argument("--prealloc-gib", type=int, default=0,
                    help="allocate that much device memory first and keep it (stands for a job's weights and activations)")
    ap.add_argument("--scale-div", type=int, default=1, help="divide tensor dimensions (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-configs", action="store_true", help="headline only: skip per_config and packed_frac")
    ap.add_argument("--graph", action="store_true",
                    help="record a whole number of accumulation loops in a HIP graph once and time its replays "
                         "(launch gaps of --path buckets); per-launch times then are replay averages")
    ap.add_argument("--repeats", type=int, default=30,
                    help="after the timed region, time that many minus one further regions of the same length and "
                         "report their median, minimum and maximum next to the first, which stays the reported value")
    ap.add_argument("--cpu-sample", type=int, default=None, help="coordinates per row given to the CPU oracle")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of a known size (1 GiB read + 1 GiB written each), so that "
                         "profiler byte counters can be scaled by what they read for a known transfer")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; all replicas of the simulated run (or one node's share) live in "
              "one HBM and there is no multi-GPU path to time. Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(torch.device("cuda:0"))

    side_configs = args.config is None and not args.no_side_configs and args.path == "fused" and not args.graph
    if args.config is None:
        args.config = 2
    out, sample = measure_and_release(args, want_cpu_sample=not args.no_cpu_baseline)

    if side_configs:
        # the other configurations of the benchmark, each over its own step count, and configuration 2 again
        # with ordinary allocations; shorter runs of regions (the headline's regions carry the statistics)
        import copy
        per = {}
        for cfg in (3, 4, 5):
            a = copy.copy(args)
            a.config, a.steps, a.repeats, a.copy_calibration = cfg, None, min(args.repeats, 5), False
            res, _ = measure_and_release(a, want_cpu_sample=False)
            per[f"cfg{cfg}"] = brief(res)
        out["per_config"] = per
        a = copy.copy(args)
        a.layout, a.repeats, a.copy_calibration = "packed", min(args.repeats, 5), False
        res, _ = measure_and_release(a, want_cpu_sample=False)
        out["packed_frac"] = res["roofline"]["frac"]
        out["packed"] = brief(res)

    if sample is not None:
        wl, ns, x0_sample, g_samples, csrs = sample
        R = wl.n_rows
        iters = min(wl.steps, max(wl.s + 1, int(1.2e9 // (R * ns))))
        v, dt = cpu_baseline(wl, x0_sample, g_samples, csrs, iters)
        model, logical = host_cpu()
        # worker pools on this machine are sized to its share of the host: 16 threads at most
        threads = max(1, min(16, logical, int(os.environ.get("OMP_NUM_THREADS", "16") or 16)))
        vp, dtp = cpu_baseline(wl, x0_sample, g_samples, csrs, iters, threads=threads)
        out["cpu_baseline"] = {
            "value": v, "unit": "replica-params/s", "cores": 1, "kind": "oracle",
            "sample": f"first {ns} coordinates of all {R} rows, {iters} iterations of the same workload "
                      f"({dt:.1f} s of single-threaded NumPy float64)",
            "all_cores": {"value": vp, "unit": "replica-params/s", "cores": threads,
                          "how": f"the same sample cut into {threads} coordinate slices, one thread each ({dtp:.1f} s)"},
            "host_cpu": model, "host_logical_cpus": logical,
        }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
