"""Seeded data shards and initial parameters (inputs only, no method arithmetic).

The shards stand in for the paper's image datasets (MNIST / CIFAR, Section V-A):
same shapes (32x32x3 inputs flattened to 3072 features, 10 classes), synthetic
values.  Labels come from seeded Gaussian clusters or from a seeded random
"teacher" network, evaluated once here on the host.
"""
from __future__ import annotations

import numpy as np

from .configs import BASE_SEED, Workload


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _teacher(dims, rng):
    return [(rng.standard_normal((dims[l], dims[l + 1])) / np.sqrt(dims[l])).astype(np.float32)
            for l in range(len(dims) - 1)]


def _teacher_labels(x: np.ndarray, Ws) -> np.ndarray:
    a = x
    for l, W in enumerate(Ws):
        a = a @ W
        if l + 1 < len(Ws):
            a = np.maximum(a, 0.0)
    return np.argmax(a, axis=1).astype(np.int32)


def make_shards(w: Workload):
    """Return (feats, labels, shard_off).

    feats: [n_total, dims[0]] float32, or uint16 bfloat16 bit patterns when
    w.gemm_in == "bf16"; labels: int32 [n_total]; shard_off: int64 [M+1], worker i
    owns rows shard_off[i] .. shard_off[i+1]-1.  Flat workloads return (None, None, None).
    """
    if w.model == "flat":
        return None, None, None
    n, d_in, n_cls = w.n_per_worker, w.dims[0], w.dims[-1]
    shard_off = (np.arange(w.M + 1, dtype=np.int64) * n)
    labels = np.empty(w.M * n, dtype=np.int32)
    feats = np.empty((w.M * n, d_in), dtype=np.uint16 if w.gemm_in == "bf16" else np.float32)
    rng_shared = np.random.default_rng(BASE_SEED + 2)
    if w.data == "clusters":
        means = 2.0 * rng_shared.standard_normal((n_cls, d_in))      # means ~ N(0, 4 I)
    else:
        Ws = _teacher(w.dims, rng_shared)
    for i in range(w.M):
        rng = np.random.default_rng([BASE_SEED + 1, i])
        if w.data == "clusters":
            y = rng.integers(0, n_cls, size=n).astype(np.int32)
            x = (means[y] + rng.standard_normal((n, d_in))).astype(np.float32)
        elif w.data == "teacher_normal":
            x = rng.standard_normal((n, d_in), dtype=np.float32)
            y = _teacher_labels(x, Ws)
        elif w.data == "teacher_uniform":
            x = rng.random((n, d_in), dtype=np.float32)
            if w.gemm_in == "bf16":
                x = bf16_bits_to_f32(f32_to_bf16_bits(x))
            # centre the inputs for the teacher only, so that its classes are balanced
            y = _teacher_labels(x - np.float32(0.5), Ws)
        else:
            raise ValueError(w.data)
        labels[i * n:(i + 1) * n] = y
        feats[i * n:(i + 1) * n] = f32_to_bf16_bits(x) if w.gemm_in == "bf16" else x
    return feats, labels, shard_off


def init_params(w: Workload, spread: float = 0.1) -> np.ndarray:
    """x^0 as float32 [M, ld]: a shared seeded initialisation plus a per-worker
    perturbation of relative size `spread`, so the initial consensus distance is
    positive.  MLP layout per layer: W row-major [in][out], then b [out] (zeros).
    Padding columns D..ld-1 are zero."""
    X = np.zeros((w.M, w.ld), dtype=np.float32)
    rng0 = np.random.default_rng(BASE_SEED + 3)
    if w.model == "flat":
        scale = np.full(w.D, 0.1, dtype=np.float32)
    else:
        scale = np.zeros(w.D, dtype=np.float32)
        o = 0
        for l in range(w.n_layers):
            fan_in, fan_out = w.dims[l], w.dims[l + 1]
            scale[o:o + fan_in * fan_out] = 1.0 / np.sqrt(fan_in)
            o += fan_in * fan_out + fan_out
    base = rng0.standard_normal(w.D, dtype=np.float32) * scale
    for i in range(w.M):
        rng = np.random.default_rng([BASE_SEED + 3, i + 1])
        X[i, :w.D] = base + np.float32(spread) * scale * rng.standard_normal(w.D, dtype=np.float32)
    return X
