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
