"""Builds the GPU run and the oracle run of one workload from the same seeded inputs."""
from __future__ import annotations

import numpy as np

from netmax_inputs import Workload, policy_for, make_shards, init_params, hyperparameters


def inputs_of(w: Workload):
    P, rho = policy_for(w)
    feats, labels, shard_off = make_shards(w)
    X0 = init_params(w)
    return dict(P=P, rho=rho, feats=feats, labels=labels, shard_off=shard_off, X0=X0)


def hyper(w: Workload, rho: float):
    return hyperparameters(w, rho)


def make_gpu(w: Workload, inp, fixed_weight=None, **over):
    """fixed_weight: use the same second-step weight for every drawn pair (gossip / AD-PSGD averaging)."""
    import paper_2009_05766_amd as nm
    h = hyper(w, inp["rho"])
    h.update(over)
    if fixed_weight is not None:
        h.update(mix_mode=nm.NETMAX_MIX_FIXED, fixed_weight=fixed_weight)
    return nm.NetMax(M=w.M, D=w.D, ld=w.ld, model=nm.NETMAX_FLAT if w.model == "flat" else nm.NETMAX_MLP,
                     dims=w.dims, batch=w.batch, gemm_in=nm.NETMAX_BF16 if w.gemm_in == "bf16" else nm.NETMAX_F32,
                     seed=w.seed, P=inp["P"], X0=inp["X0"], feats=inp["feats"], labels=inp["labels"],
                     shard_off=inp["shard_off"], **h)


def make_oracle(w: Workload, inp, operands_bf16=False, fixed_weight=None, **over):
    """operands_bf16: the oracle rounds the operands of every matrix product to bfloat16, as the bf16
    workload prescribes; False gives exact arithmetic."""
    import oracle
    h = hyper(w, inp["rho"])
    h.update(over)
    return oracle.Oracle(operands_bf16=operands_bf16, fixed_weight=fixed_weight, M=w.M, ld=w.ld, D=w.D, dims=w.dims, batch=w.batch, seed=w.seed, P=inp["P"],
                         X0=inp["X0"], feats=inp["feats"], labels=inp["labels"], shard_off=inp["shard_off"], **h)


def rel_err_rows(a: np.ndarray, b: np.ndarray) -> float:
    """max over workers of ||a_i - b_i||_2 / ||b_i||_2 (b = oracle)."""
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    num = np.sqrt(((a - b) ** 2).sum(axis=1))
    den = np.maximum(np.sqrt((b ** 2).sum(axis=1)), 1e-30)
    return float((num / den).max())


def max_abs_err(a: np.ndarray, b: np.ndarray) -> float:
    """Largest element-wise difference |a - b| (computed in double)."""
    return float(np.abs(a.astype(np.float64) - b.astype(np.float64)).max()) if a.size else 0.0


def compare_on_device(got_dev, want_host: np.ndarray, slab: int = 1 << 20):
    """Element-by-element comparison of a device matrix [M, n] with the oracle's host matrix, done with torch on
    the device in double, slab by slab (test arithmetic only).  -> (max over rows of ||got_i - want_i|| / ||want_i||,
    max |got - want|, max |want|)."""
    import torch
    want = torch.from_numpy(want_host).to(got_dev.device)
    assert want.shape == got_dev.shape
    M, n = want.shape
    num = torch.zeros(M, dtype=torch.float64, device=want.device)
    den = torch.zeros_like(num)
    worst = ref = 0.0
    for c in range(0, n, slab):
        a, b = got_dev[:, c:c + slab].double(), want[:, c:c + slab].double()
        d = a - b
        num += (d * d).sum(1)
        den += (b * b).sum(1)
        worst = max(worst, float(d.abs().max()))
        ref = max(ref, float(b.abs().max()))
    rel = float((num.sqrt() / den.sqrt().clamp_min(1e-30)).max())
    return rel, worst, ref
