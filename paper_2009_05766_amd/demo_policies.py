"""A synthetic rerun of the paper's headline comparison in shape (Section V-B/V-C): the same decentralized
training under a uniform peer-selection policy and under the policy Algorithm 3 generates for the network's
iteration times, on a heterogeneous network, compared at equal simulated time.

Both runs use the asynchronous schedule (one active worker per global step, drawn with the activity
probabilities of Eq. (d4)).  Global steps happen at rate sum_i 1 / tbar_i (every worker i finishes an
iteration every tbar_i = sum_m t_im p_im time units on average, Eq. (d3)), so a budget of simulated time buys
each policy a different number of global steps.  Reported: steps done, mean training loss of the workers' last
batches, consensus distance.  Nothing here is timed on a network; the iteration times are the synthetic
link model of the workload (`netmax_inputs.iteration_times`).

    python -m paper_2009_05766_amd.demo_policies [--workload cfg1] [--time 400] [--links four_group_12]
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def run_policy(w, inp, P, rho, t, budget, chunk=200):
    import torch
    from . import binding as nm
    from netmax_inputs import hyperparameters
    h = hyperparameters(w, rho)
    gpu = nm.NetMax(M=w.M, D=w.D, ld=w.ld, model=nm.NETMAX_FLAT if w.model == "flat" else nm.NETMAX_MLP, dims=w.dims,
                    batch=w.batch, gemm_in=nm.NETMAX_BF16 if w.gemm_in == "bf16" else nm.NETMAX_F32, seed=w.seed, P=P,
                    X0=inp["X0"], feats=inp["feats"], labels=inp["labels"], shard_off=inp["shard_off"], **h)
    p_act = nm.netmax_activity(t, P)
    nm.netmax_set_activity(gpu.ctx, p_act)
    tbar, rate = nm.netmax_mean_times(t, P)                # Eq. (d3); global steps per unit of simulated time
    steps = int(budget * rate)
    active = torch.zeros(chunk, dtype=torch.int32, device=gpu.device)
    peers = torch.zeros(chunk, dtype=torch.int32, device=gpu.device)
    done = 0
    while done < steps:
        n = min(chunk, steps - done)
        nm.netmax_async_run(gpu.ctx, done, n, active, peers)
        done += n
    losses = gpu.losses()
    out = dict(steps=steps, steps_per_time=rate, mean_iteration_time=float(tbar.mean()),
               loss=None if losses is None else float(losses.mean().item()), consensus_dist=gpu.consensus_dist(), rho=rho)
    gpu.close()
    return out


def run_dynamic(w, inp, P, rho, networks, segment_time, adaptive, K, R, periods=4, beta=0.5, chunk=200):
    """A network whose slow link moves from segment to segment (Section V-A).  adaptive: Algorithm 1's loop, the
    workers smooth the iteration times they see (Algorithm 2) and the monitor regenerates the policy `periods` times
    per segment; otherwise the policy stays as given.  How often each worker is active always follows the true
    iteration times of the segment (Eq. (d3), (d4))."""
    import torch
    from . import binding as nm
    from .monitor import Monitor
    from netmax_inputs import hyperparameters
    h = hyperparameters(w, rho)
    gpu = nm.NetMax(M=w.M, D=w.D, ld=w.ld, model=nm.NETMAX_FLAT if w.model == "flat" else nm.NETMAX_MLP, dims=w.dims,
                    batch=w.batch, gemm_in=nm.NETMAX_BF16 if w.gemm_in == "bf16" else nm.NETMAX_F32, seed=w.seed, P=P,
                    X0=inp["X0"], feats=inp["feats"], labels=inp["labels"], shard_off=inp["shard_off"], **h)
    mon = Monitor(gpu, alpha=h["lr"], K=K, R=R, beta=beta, initial_times=networks[0])
    active = torch.zeros(chunk, dtype=torch.int32, device=gpu.device)
    peers = torch.zeros(chunk, dtype=torch.int32, device=gpu.device)
    done, policies = 0, 0
    for t in networks:
        mon.set_network(t)
        for _ in range(periods):                                         # the monitor's schedule period T_s
            nm.netmax_set_activity(gpu.ctx, nm.netmax_activity(t, P))
            _, rate = nm.netmax_mean_times(t, P)
            left = int(segment_time / periods * rate)
            while left > 0:
                n = min(chunk, left)
                nm.netmax_async_run(gpu.ctx, done, n, active, peers)
                if adaptive:
                    mon.observe_async(active, peers, n)
                done += n
                left -= n
            if adaptive:
                pol = mon.reschedule()
                if pol is not None:
                    P, policies = pol["P"], policies + 1
    losses = gpu.losses()
    out = dict(steps=done, policies_generated=policies, loss=None if losses is None else float(losses.mean().item()),
               consensus_dist=gpu.consensus_dist())
    gpu.close()
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--links", default=None, help="link recipe (default: the workload's)")
    ap.add_argument("--time", type=float, default=400.0, help="budget of simulated time (fastest link = 1)")
    ap.add_argument("--dynamic", type=int, default=0, metavar="SEGMENTS",
                    help="a network whose slow link (2x to 100x) moves: this many segments of --time each; compares a "
                         "fixed uniform policy with the monitor loop that regenerates the policy --periods times per segment")
    ap.add_argument("--periods", type=int, default=4, help="with --dynamic: policy regenerations per segment")
    ap.add_argument("--K", type=int, default=40)
    ap.add_argument("--R", type=int, default=6)
    args = ap.parse_args(argv)
    from . import binding as nm
    from netmax_inputs import workload, make_shards, init_params, iteration_times, default_rho
    w = workload(args.workload)
    links = args.links or w.links
    feats, labels, shard_off = make_shards(w)
    inp = dict(feats=feats, labels=labels, shard_off=shard_off, X0=init_params(w))
    t = iteration_times(links, w.M)
    alpha = float(np.float32(w.lr))
    uniform = (np.ones((w.M, w.M)) - np.eye(w.M)) / (w.M - 1)
    if args.dynamic > 0:
        from netmax_inputs import dynamic_times
        nets = dynamic_times(links, w.M, args.dynamic)
        rho_u = default_rho(uniform, w.lr)
        rows = {"uniform policy, fixed": run_dynamic(w, inp, uniform, rho_u, nets, args.time, False, args.K, args.R, args.periods),
                "monitor loop (Algorithms 1-3)": run_dynamic(w, inp, uniform, rho_u, nets, args.time, True, args.K, args.R, args.periods)}
        print(json.dumps({"workload": w.name, "links": links, "segments": args.dynamic, "time_per_segment": args.time,
                          "runs": rows}, indent=1))
        return 0
    pol = nm.netmax_generate_policy(t, alpha, args.K, args.R)
    rows = {"uniform policy": run_policy(w, inp, uniform, default_rho(uniform, w.lr), t, args.time),
            "generated policy (Algorithm 3)": run_policy(w, inp, pol["P"], float(np.float32(pol["rho"])), t, args.time)}
    print(json.dumps({"workload": w.name, "links": links, "simulated_time": args.time, "runs": rows}, indent=1))
    return 0


if __name__ == "__main__":
    sys.exit(main())
