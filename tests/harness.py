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


def compare_on_device(got_dev, want_host: np.ndarray, slab: int = 1 << 20, per_row: bool = False):
    """Element-by-element comparison of a device matrix [M, n] with the oracle's host matrix, done with torch on
    the device in double, slab by slab (test arithmetic only).  -> (max over rows of ||got_i - want_i|| / ||want_i||,
    max |got - want|, max |want|); per_row=True gives the per-row ratios as an array instead of their maximum."""
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
    rel = num.sqrt() / den.sqrt().clamp_min(1e-30)
    return (rel.cpu().numpy() if per_row else float(rel.max())), worst, ref


def relu_disagreements(gpu, Z):
    """Hidden units whose ReLU decision in the library's last local step (stored activation positive) differs from
    the sign of the oracle's pre-activation.  Z: list over hidden layers of [M, B, width] (oracle.local_hidden).
    -> (list over hidden layers of (worker, sample, unit) index arrays, largest |z| among the disputed units
    relative to its layer's root mean square)."""
    where, closest = [], 0.0
    for l, z in enumerate(Z):
        differ = (gpu.hidden(l + 1).cpu().numpy() > 0) != (z > 0)
        where.append(np.argwhere(differ))
        if differ.any():
            closest = max(closest, float(np.abs(z[differ]).max() / np.sqrt((z * z).mean())))
    return where, closest


def columns_touched_by(dims, ld, disputed):
    """Boolean mask over a parameter row: the columns whose gradient a disputed ReLU decision changes.  A decision
    of unit k of hidden layer h (h = 1 ..) switches the back-propagated error of that unit on or off: it changes
    column k of W_{h-1} and b_{h-1}[k] directly and, through the error handed further down, every parameter of the
    layers below.  Parameter layout per layer: W row-major [in][out], then b [out]."""
    mask = np.zeros(ld, dtype=bool)
    off = [0]
    for l in range(len(dims) - 1):
        off.append(off[-1] + dims[l] * dims[l + 1] + dims[l + 1])
    for h, units in disputed.items():              # h: hidden layer (1-based), units: set of unit indices
        if not units:
            continue
        l = h - 1
        din, dout = dims[l], dims[l + 1]
        ks = np.fromiter(units, dtype=np.int64)
        mask[(off[l] + np.arange(din)[:, None] * dout + ks[None, :]).ravel()] = True
        mask[off[l] + din * dout + ks] = True
        mask[:off[l]] = True
    return mask
