#!/usr/bin/env python3
"""Benchmark of the NetMax iteration on one MI355X.

A step is one pass of the whole hot path over all M workers: peer sampling, local gradient
(synthetic for the flat workloads, grouped-GEMM perceptron gradient otherwise) and the fused
momentum apply + mix.  Prints ONE JSON line: whole-job worker-iterations/s, the HBM roofline of the
dominant kernel (mix) measured live with events on the launch stream, and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# Algorithmic HBM bytes per (worker, parameter) of the mix kernel with momentum: read x, v, g; write x', v'.
# The peer's row is a second read of a row of x that some workgroup of the same column chunk also reads as
# its own, so the minimum HBM traffic counts x once: 5 * 4 = 20 B.  (Counting the peer read too gives 24 B.)
MIX_BYTES_MIN, MIX_BYTES_NAIVE = 20, 24

# HBM bytes per mix launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs (profiles/mix_kernel_cfg3.md, mix_kernel_cfg4.md,
# iteration_cfg5.md), each
# counter scaled by what it reads for a plain device copy of known size.  Valid only for the kernel sources they
# were taken with: keyed by the sha256 prefix of k_mix.hip + layout.h + vec.h, reported as null otherwise.
_MIX_SOURCES = "c8b2061f1db7daaa.3f97687d5424e9a2.e54cf75f51c45279"
MEASURED_TRAFFIC = {"cfg3": {"sources": _MIX_SOURCES, "bytes": 14338993040},
                    "cfg4": {"sources": _MIX_SOURCES, "bytes": 12802386208},
                    "cfg5": {"sources": _MIX_SOURCES, "bytes": 10777505263}}


def mix_sources_digest() -> str:
    import hashlib
    d = os.path.join(ROOT, "paper_2009_05766_amd", "csrc")
    return ".".join(hashlib.sha256(open(os.path.join(d, f), "rb").read()).hexdigest()[:16]
                    for f in ("k_mix.hip", "layout.h", "vec.h"))


def describe(w) -> str:
    if w.model == "flat":
        return (f"{w.name}: M={w.M} workers, flat fp32 parameter vector D={w.D}, synthetic N(0,1e-3) gradients, "
                f"momentum {w.momentum} + consensus mix, links {w.links}")
    return (f"{w.name}: M={w.M} workers, MLP {'-'.join(map(str, w.dims))}, batch {w.batch}, {w.gemm_in} GEMM operands, "
            f"momentum {w.momentum} + consensus mix, links {w.links}")


def cpu_baseline(w, inp, budget_s: float = 12.0):
    """The oracle as it stands, on a bounded sample of the workload, single-threaded."""
    import numpy as np
    import oracle
    from netmax_inputs import hyperparameters
    h = hyperparameters(w, inp["rho"])
    oracle.set_threads(1)
    if w.model == "flat":
        cols = min(w.ld, 1 << 19)
        X0 = np.ascontiguousarray(inp["X0"][:, :cols])
        o = oracle.Oracle(M=w.M, ld=cols, D=cols, dims=(), batch=0, seed=w.seed, P=inp["P"], X0=X0, **h)
        scale = w.ld / cols
        sample = f"all {w.M} workers, first {cols} of {w.ld} columns"
    else:
        # per-worker cost: 6 flops per weight and batch row at about 1 GFLOP/s; keep one iteration near one second
        est = 6.0 * w.D * w.batch / 1e9
        m = int(max(2, min(w.M, round(1.0 / max(est, 1e-9)))))
        Pm = np.ascontiguousarray(inp["P"][:m, :m])
        Pm = Pm / Pm.sum(axis=1, keepdims=True)
        so = inp["shard_off"][:m + 1]
        o = oracle.Oracle(M=m, ld=w.ld, D=w.D, dims=w.dims, batch=w.batch, seed=w.seed, P=Pm,
                          X0=np.ascontiguousarray(inp["X0"][:m]), feats=inp["feats"][:so[-1]], labels=inp["labels"][:so[-1]],
                          shard_off=np.ascontiguousarray(so), **h)
        scale = w.M / m
        sample = f"the first {m} of {w.M} workers, full layer shapes" if m < w.M else f"all {w.M} workers, full shape"
    t0 = time.perf_counter()
    o.step(0)
    t1 = time.perf_counter() - t0
    iters = max(1, min(int(budget_s / max(t1, 1e-9)), 50))
    t0 = time.perf_counter()
    for it in range(1, 1 + iters):
        o.step(it)
    dt = (time.perf_counter() - t0) / iters
    # the same oracle with its loop over workers spread over the host's threads (same results: every worker reads
    # the previous iteration's copies only), reported beside the single-thread figure
    threads = max(1, min(16, os.cpu_count() or 1, o.M))          # one worker per thread at most
    oracle.set_threads(threads)
    iters_mt = max(1, min(int(0.5 * budget_s / max(dt, 1e-9)), 50))
    t0 = time.perf_counter()
    for it in range(1 + iters, 1 + iters + iters_mt):
        o.step(it)
    dt_mt = (time.perf_counter() - t0) / iters_mt
    oracle.set_threads(1)
    return {"value": w.M / (dt * scale), "unit": "worker-iterations/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample}, {iters} iterations timed, scaled to the whole workload",
            "all_threads": {"value": w.M / (dt_mt * scale), "cores": threads, "iterations": iters_mt}}


def measure(w, steps, warmup, mode, fuse, copy_probe, with_fused_variant=False):
    """One workload: inputs to HBM, warm-up, then `steps` timed iterations.  -> (result dict, inputs).
    with_fused_variant: where the library has one (flat models, perceptrons on the matrix-core kernels), also time
    the same number of iterations through netmax_run with netmax_set_fusion on (reported beside the result)."""
    import numpy as np
    import torch
    import paper_2009_05766_amd as nm
    from netmax_inputs import policy_for, make_shards, init_params, hyperparameters as hyper

    if fuse and mode == "calls":
        print("bench.py: --fuse needs --mode run or --mode graph (the three separate entry points are never fused)", file=sys.stderr)
        return None, None
    t_in = time.perf_counter()
    P, rho = policy_for(w)
    feats, labels, shard_off = make_shards(w)
    X0 = init_params(w)
    inp = dict(P=P, rho=rho, feats=feats, labels=labels, shard_off=shard_off, X0=X0)
    print(f"[bench] inputs of {w.name} generated in {time.perf_counter() - t_in:.1f} s", file=sys.stderr, flush=True)

    side = torch.cuda.Stream()          # default priority; a real stream, so that iterations can be captured
    torch.cuda.set_stream(side)
    gpu = nm.NetMax(M=w.M, D=w.D, ld=w.ld, model=nm.NETMAX_FLAT if w.model == "flat" else nm.NETMAX_MLP, dims=w.dims,
                    batch=w.batch, gemm_in=nm.NETMAX_BF16 if w.gemm_in == "bf16" else nm.NETMAX_F32, seed=w.seed, P=P,
                    X0=X0, feats=feats, labels=labels, shard_off=shard_off, **hyper(w, rho))
    torch.cuda.synchronize()
    cd0 = gpu.consensus_dist()

    for it in range(warmup):
        gpu.step(it)
    torch.cuda.synchronize()

    for _ in range(copy_probe):
        gpu.x_b.copy_(gpu.x_a) if gpu.params() is gpu.x_a else gpu.x_a.copy_(gpu.x_b)
    torch.cuda.synchronize()

    K = steps
    K_ev = K if mode == "calls" else min(K, 50)      # phase timing: events around every entry point
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K_ev)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K_ev):
        it = warmup + k
        e = ev[k]
        e[0].record()
        nm.netmax_sample_peers(gpu.ctx, it, gpu.peers)
        e[1].record()
        nm.netmax_local_step(gpu.ctx, it)
        e[2].record()
        nm.netmax_mix(gpu.ctx, it, gpu.peers)
        e[3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if mode != "calls":
        if fuse:
            nm.netmax_set_fusion(gpu.ctx, True)
        first = warmup + K_ev
        gpu.run(first, 4, use_graph=mode == "graph")          # captures both directions outside the timed region
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gpu.run(first + 4, K, use_graph=mode == "graph")
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    fused_variant = None
    if with_fused_variant and not fuse and (w.model == "flat" or w.gemm_in == "bf16"):
        try:
            nm.netmax_set_fusion(gpu.ctx, True)
        except nm.NetmaxError:
            pass                                   # a perceptron none of whose layers runs on the matrix-core kernels
        else:
            first = warmup + K_ev + 4 + K
            gpu.run(first, 4)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            gpu.run(first + 4, K)
            torch.cuda.synchronize()
            wall_fused = time.perf_counter() - t1
            nm.netmax_set_fusion(gpu.ctx, False)
            fused_variant = {"value": w.M * K / wall_fused, "ms_per_step": wall_fused * 1e3 / K, "launch": "run+fused"}

    ms = np.array([[e[j].elapsed_time(e[j + 1]) for j in range(3)] for e in ev])   # sample, grad, mix
    ms_sample, ms_grad, ms_mix = ms.mean(axis=0)
    cd1 = gpu.consensus_dist()
    ms_per_step = wall * 1e3 / K
    value = w.M * K / wall

    elems = w.M * w.ld
    mix_s = ms_mix * 1e-3
    achieved = MIX_BYTES_MIN * elems / mix_s / 1e9
    rec = MEASURED_TRAFFIC.get(w.name)
    traffic = rec["bytes"] if rec and rec["sources"] == mix_sources_digest() else None
    roofline = {"bound": "hbm", "kernel": "mix_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "bytes_per_worker_param": MIX_BYTES_MIN, "avg_launch_ms": float(ms_mix),
                "achieved_counting_peer_read": MIX_BYTES_NAIVE * elems / mix_s / 1e9}

    out = {"metric": "worker-iterations/sec (sample+grad+mix)", "value": value, "unit": "worker-iterations/s",
           "n_gpus": 1, "steps": K, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.gemm_in == "bf16" else "f32",
           "data": "synthetic", "config": {"workload": describe(w), "M": w.M, "D": w.D, "iterations": K,
                                           "launch": mode + ("+fused" if fuse else "")},
           "phase_ms": {"sample_peers": float(ms_sample), "local_step": float(ms_grad), "mix": float(ms_mix)},
           "consensus_distance": {"before": cd0, "after": cd1},
           "roofline": roofline}
    if fused_variant:
        out["fused_variant"] = fused_variant
    gpu.close()
    del gpu
    torch.cuda.set_stream(torch.cuda.default_stream())
    torch.cuda.empty_cache()
    return out, inp


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", help="cfg1..cfg5 (default: cfg3, the HBM-bound ResNet18-sized mix)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short measurements of the other four workloads (key per_config)")
    ap.add_argument("--mode", choices=("calls", "run", "graph"), default="calls",
                    help="calls: the three entry points per step, events around each phase (default); run: one "
                         "netmax_run call for all steps; graph: netmax_run replaying captured HIP graphs")
    ap.add_argument("--fuse", action="store_true",
                    help="with --mode run or graph, perceptron workloads on the matrix-core kernels: apply the update "
                         "inside the weight-gradient kernels (netmax_set_fusion)")
    ap.add_argument("--copy-probe", type=int, default=0,
                    help="before the timed region, run this many plain device copies of the parameter matrix "
                         "(a kernel of known traffic, used to scale profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, nothing sharded); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from netmax_inputs import workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    w = workload(args.workload)
    out, inp = measure(w, args.steps, args.warmup, args.mode, args.fuse, args.copy_probe, with_fused_variant=not args.no_per_config)
    if out is None:
        return 2
    if not args.no_per_config:
        # the other four workloads in the same process: fewer steps, all steps enqueued by one netmax_run call (the
        # phase split from a separate pass with events around each entry point); no CPU baseline for them
        per = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            if name == w.name:
                continue
            small = name in ("cfg1", "cfg2")
            o, _ = measure(workload(name), 400 if small else 40, 20 if small else 5, "run", False, 0, with_fused_variant=True)
            per[name] = {"workload": o["config"]["workload"], "value": o["value"], "unit": o["unit"], "steps": o["steps"],
                         "us_per_step": o["ms_per_step"] * 1e3,
                         "phase_us": {k: v * 1e3 for k, v in o["phase_ms"].items()},
                         "mix_roofline_frac": o["roofline"]["frac"], "mix_achieved_GBs": o["roofline"]["achieved"],
                         "dtype": o["dtype"], "launch": o["config"]["launch"]}
            if "fused_variant" in o:
                per[name]["fused_variant"] = o["fused_variant"]
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
