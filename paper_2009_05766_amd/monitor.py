"""The control loop around the iteration on a simulated network (Algorithm 1 together with the time
bookkeeping of Algorithm 2): the workers record smoothed iteration times, the monitor collects them every
scheduling period, generates a policy (Algorithm 3) and hands it back to the workers.

Everything numeric happens in the library: netmax_update_times keeps the moving averages and the workers'
clocks on the device, netmax_generate_policy computes (P, rho), netmax_set_policy rebuilds the sampling
thresholds and mix weights.  This module only sequences those calls.

The moving averages start from a caller-given estimate of the iteration times instead of Algorithm 2's zeros:
with zeros the first policies would be generated from times that no worker has measured yet.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np

from . import binding as B


class Monitor:
    def __init__(self, run: "B.NetMax", *, alpha: float, K: int, R: int, beta: float, initial_times: np.ndarray,
                 adj: Optional[np.ndarray] = None, eps: float = 1e-3):
        import torch
        self.run, self.alpha, self.K, self.R, self.beta, self.adj, self.eps = run, alpha, K, R, beta, adj, eps
        M = run.M
        assert initial_times.shape == (M, M)
        self.ema = torch.from_numpy(np.ascontiguousarray(initial_times, dtype=np.float32)).to(run.device)
        self.clock = torch.zeros(M, dtype=torch.float32, device=run.device)
        self.times = None

    def set_network(self, t: np.ndarray):
        """The simulated network's true iteration times t_im from now on."""
        import torch
        self.times = torch.from_numpy(np.ascontiguousarray(t, dtype=np.float32)).to(self.run.device)

    def observe(self, peers=None):
        """Algorithm 2's UpdateTimeVector for the peers drawn in this iteration."""
        B.netmax_update_times(self.run.ctx, self.run.peers if peers is None else peers, self.times, self.beta,
                              self.ema, self.clock)

    def observe_async(self, active, peers, n_steps: int):
        """The same bookkeeping for a run of global steps of the asynchronous schedule (netmax_async_run's output)."""
        B.netmax_update_times_async(self.run.ctx, active, peers, n_steps, self.times, self.beta, self.ema, self.clock)

    def collect(self) -> np.ndarray:
        """The matrix of smoothed iteration times the monitor gathers from the workers (Algorithm 1)."""
        import torch
        torch.cuda.current_stream(self.run.device).synchronize()
        return self.ema.cpu().numpy().astype(np.float64)

    def install(self, P: np.ndarray, rho: float):
        B.netmax_set_policy(self.run.ctx, P, rho)

    def reschedule(self):
        """One pass of Algorithm 1's loop body.  Returns the generated policy (dict) or None if no grid point was
        feasible, in which case the workers keep their current policy."""
        try:
            pol = B.netmax_generate_policy(self.collect(), self.alpha, self.K, self.R, adj=self.adj, eps=self.eps)
        except B.NetmaxError as e:
            if e.code != B.NETMAX_EINFEASIBLE:
                raise
            return None
        self.install(pol["P"], pol["rho"])
        return pol


def replay(run: "B.NetMax", monitor: Optional[Monitor], networks: Sequence[np.ndarray], iters_per_segment: int,
           first_iter: int = 0, reschedule_every: Optional[int] = None):
    """Runs the iteration through a sequence of network states (one time matrix per segment).  With a monitor the
    policy is regenerated every `reschedule_every` iterations (default: once per segment, at its end).  Returns one
    record per segment: iteration reached, simulated time (slowest worker's clock), consensus distance and the
    consensus weight in force."""
    period = iters_per_segment if reschedule_every is None else reschedule_every
    it = first_iter
    history = []
    rho = None
    for t in networks:
        if monitor is not None:
            monitor.set_network(t)
        for _ in range(iters_per_segment):
            run.sample_peers(it)
            if monitor is not None:
                monitor.observe()
            run.local_step(it)
            run.mix(it)
            it += 1
            if monitor is not None and (it - first_iter) % period == 0:
                pol = monitor.reschedule()
                if pol is not None:
                    rho = pol["rho"]
        rec = dict(iteration=it, consensus_dist=run.consensus_dist(), rho=rho)
        if monitor is not None:
            rec["sim_time"] = float(monitor.clock.max().item())
        history.append(rec)
    return history
