"""The five synthetic workloads, shaped like the paper's experiments.

The paper trains image classifiers (MobileNet ~4.2M, ResNet18 ~11.7M, VGG19
parameters; 32x32x3 CIFAR images; batch 128, momentum 0.9, learning rate 0.1:
Section V-A "Datasets and models" / "Configurations") on clusters whose links
differ in speed by 2x to 100x (Section V-A "Network").  Neither its datasets nor
its networks are available, so every workload here is seeded and synthetic with
those shapes and ratios.  Values the workload list leaves open are frozen here:
the learning rate of the two perceptron workloads cfg2 and cfg5 is 0.01 (the
paper's setting for its MNIST runs, Section V-F / Appendix E), that of the flat
workloads cfg3 and cfg4 is 0.1 (its CIFAR10 setting, Section V-A); cfg5's shards
hold 4096 images per worker.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

BASE_SEED = 20090576  # per-purpose seeds are offsets from this
PAD = 2048            # rows are padded with zeros to a multiple of this many columns


def _round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                  # 1..5
    M: int                      # workers
    model: str                  # "flat" | "mlp"  (softmax regression = 1-layer mlp)
    dims: Tuple[int, ...]       # layer widths, () for flat
    D: int                      # parameters per worker
    ld: int                     # padded row length (multiple of PAD = 2048)
    batch: int                  # 0 for flat
    n_per_worker: int           # samples in each worker's shard, 0 for flat
    lr: float
    momentum: float
    weight_decay: float
    grad_sigma: float           # std of the synthetic gradient (flat only)
    gemm_in: str                # "f32" | "bf16": storage type of the features and GEMM operands
    T: int                      # iterations of the full run
    links: str                  # link-matrix recipe, see policy.link_speeds
    data: str                   # data recipe, see data.make_shards
    floor_policy: bool          # floor P at 1/(4M) and renormalise (lognormal recipes)

    @property
    def seed(self) -> int:
        """Seed of the counter-based generator inside the method (peer, batch, gradient draws)."""
        return BASE_SEED + 100 + self.index

    @property
    def n_layers(self) -> int:
        return max(len(self.dims) - 1, 0)


def mlp_param_count(dims: Tuple[int, ...]) -> int:
    return sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))


def _mk(name, index, M, model, dims, D, batch, n, lr, mu, sigma, gemm_in, T, links, data, floor):
    if model == "mlp":
        D = mlp_param_count(dims)
    return Workload(name=name, index=index, M=M, model=model, dims=tuple(dims), D=D,
                    ld=_round_up(D, PAD), batch=batch, n_per_worker=n, lr=lr, momentum=mu,
                    weight_decay=0.0, grad_sigma=sigma, gemm_in=gemm_in, T=T, links=links,
                    data=data, floor_policy=floor)


_SIGMA = 1e-3 ** 0.5  # N(0, 1e-3) is read as variance 1e-3

_WORKLOADS = {
    # M=8, softmax regression 256 -> 10, two groups of four, intra links 10x faster
    "cfg1": _mk("cfg1", 1, 8, "mlp", (256, 10), 0, 32, 1024, 0.05, 0.0, 0.0, "f32", 100,
                "two_tier_10", "clusters", False),
    # M=16, MLP 784-512-10, four groups, intra/inter ratio 12
    "cfg2": _mk("cfg2", 2, 16, "mlp", (784, 512, 10), 0, 64, 4096, 0.01, 0.9, 0.0, "f32", 1000,
                "four_group_12", "teacher_normal", False),
    # M=64, flat ResNet18-sized vector, lognormal(0,1) rack-to-rack speeds, 8 racks
    "cfg3": _mk("cfg3", 3, 64, "flat", (), 11_200_000, 0, 0, 0.1, 0.9, _SIGMA, "f32", 200,
                "racks8_lognormal", "none", True),
    # M=32, flat VGG19(CIFAR)-sized vector, machine 100x / rack 10x / cross-rack 1x
    "cfg4": _mk("cfg4", 4, 32, "flat", (), 20_000_000, 0, 0, 0.1, 0.9, _SIGMA, "f32", 200,
                "three_tier_100_10_1", "none", False),
    # M=128, MLP 3072-1024-1024-10 on 32x32x3 images, bf16 operands, lognormal(0,1.5) links
    "cfg5": _mk("cfg5", 5, 128, "mlp", (3072, 1024, 1024, 10), 0, 128, 4096, 0.01, 0.9, 0.0,
                "bf16", 500, "lognormal_1p5", "teacher_uniform", True),
}

WORKLOAD_NAMES = tuple(_WORKLOADS)


def workload(name: str, *, M: Optional[int] = None, D: Optional[int] = None,
             n_per_worker: Optional[int] = None, T: Optional[int] = None,
             dims: Optional[Tuple[int, ...]] = None, batch: Optional[int] = None) -> Workload:
    """Return a workload, optionally shrunk (same recipes, smaller shape) for tests."""
    w = _WORKLOADS[name]
    kw = {}
    if M is not None:
        kw["M"] = M
    if T is not None:
        kw["T"] = T
    if n_per_worker is not None:
        kw["n_per_worker"] = n_per_worker
    if batch is not None:
        kw["batch"] = batch
    if dims is not None:
        assert w.model == "mlp"
        kw["dims"] = tuple(dims)
        kw["D"] = mlp_param_count(tuple(dims))
        kw["ld"] = _round_up(kw["D"], PAD)
    if D is not None:
        assert w.model == "flat"
        kw["D"] = D
        kw["ld"] = _round_up(D, PAD)
    return replace(w, **kw) if kw else w


def hyperparameters(w: Workload, rho: float) -> dict:
    """The scalar hyper-parameters as the single-precision values both implementations receive."""
    import numpy as np
    f = lambda v: float(np.float32(v))
    return dict(lr=f(w.lr), momentum=f(w.momentum), weight_decay=f(w.weight_decay), rho=f(rho),
                grad_sigma=f(w.grad_sigma))
