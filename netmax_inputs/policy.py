"""Policy matrices P built from synthetic, seeded link-speed matrices.

The paper derives P from measured iteration times (Section III-C); here P is an
*input* of the iteration, obtained by normalising a symmetric link-speed matrix
row by row, so that fast links are chosen more often (Section II-B
"Probability").  The speed ratios follow the paper's heterogeneity range (links
slowed 2x to 100x, Section V-A; up to 12x across WAN regions, Section I).
"""
from __future__ import annotations

import numpy as np

from .configs import BASE_SEED, Workload


def link_speeds(recipe: str, M: int, seed: int = BASE_SEED) -> np.ndarray:
    """Symmetric M x M matrix of link speeds with a zero diagonal."""
    rng = np.random.default_rng(seed)
    i = np.arange(M)
    if recipe == "two_tier_10":
        g = i // max(M // 2, 1)
        s = np.where(g[:, None] == g[None, :], 10.0, 1.0)
    elif recipe == "four_group_12":
        g = i // max(M // 4, 1)
        s = np.where(g[:, None] == g[None, :], 12.0, 1.0)
    elif recipe == "racks8_lognormal":
        n_racks = 8 if M >= 8 else M
        r = np.minimum(i // max(M // n_racks, 1), n_racks - 1)
        R = rng.lognormal(0.0, 1.0, size=(n_racks, n_racks))
        R = np.triu(R) + np.triu(R, 1).T
        R[np.diag_indices(n_racks)] *= 10.0
        s = R[r[:, None], r[None, :]]
    elif recipe == "three_tier_100_10_1":
        machine = i // max(M // 8, 1)
        rack = i // max(M // 2, 1)
        s = np.where(machine[:, None] == machine[None, :], 100.0,
                     np.where(rack[:, None] == rack[None, :], 10.0, 1.0))
    elif recipe == "lognormal_1p5":
        z = rng.standard_normal((M, M))
        z = np.triu(z, 1)
        z = z + z.T
        s = np.exp(1.5 * z)
    elif recipe == "uniform":
        s = np.ones((M, M))
    else:
        raise ValueError(f"unknown link recipe {recipe!r}")
    s = np.array(s, dtype=np.float64)
    np.fill_diagonal(s, 0.0)
    return s


def policy_from_speeds(s: np.ndarray) -> np.ndarray:
    """p_im = s_im / sum_m s_im ("rows normalised")."""
    s = np.asarray(s, dtype=np.float64)
    return s / s.sum(axis=1, keepdims=True)


def floor_and_renormalise(P: np.ndarray, floor: float) -> np.ndarray:
    """Raise every off-diagonal entry to at least `floor`, then renormalise rows.

    Mirrors the lower bound that constraint (o3) of the paper's optimisation
    problem puts on every neighbour probability."""
    P = np.array(P, dtype=np.float64)
    off = ~np.eye(P.shape[0], dtype=bool)
    P[off] = np.maximum(P[off], floor)
    return P / P.sum(axis=1, keepdims=True)


def default_rho(P: np.ndarray, lr: float) -> float:
    """rho = p_min+ / (4 lr): the largest mix weight lr*rho/p_im is then 1/4, inside (o3)."""
    pos = P[P > 0]
    return float(pos.min() / (4.0 * float(np.float32(lr))))


def policy_for(w: Workload):
    """(P, rho) of a workload: float64 M x M row-stochastic matrix and the consensus weight."""
    s = link_speeds(w.links, w.M, BASE_SEED + 0)
    P = policy_from_speeds(s)
    if w.floor_policy:
        P = floor_and_renormalise(P, 1.0 / (4.0 * w.M))
    rho = float(np.float32(default_rho(P, w.lr)))
    return P, rho


def iteration_times(recipe: str, M: int, seed: int = BASE_SEED, compute: float = 0.05) -> np.ndarray:
    """Synthetic iteration-time matrix for policy generation: t_im = max(C, N_im) with the communication time
    N_im inversely proportional to the link speed (fastest link = 1 time unit) and a common compute time C
    (Section II-B "Iteration time"); the diagonal holds C, the duration of an iteration without a pull."""
    s = link_speeds(recipe, M, seed)
    with np.errstate(divide="ignore"):
        n = np.where(s > 0, s.max() / s, 0.0)
    t = np.maximum(n, compute)
    np.fill_diagonal(t, compute)
    return t


def dynamic_times(recipe: str, M: int, n_segments: int, seed: int = BASE_SEED, compute: float = 0.05):
    """Iteration-time matrices of a network that changes: in every segment one randomly chosen link of the
    base network is slowed down by a factor between 2 and 100 (log-uniform), and the slow link moves from
    segment to segment (Section V-A "Network": one link slowed by 2x to 100x, changed every few minutes).
    Returns a list of n_segments float64 M x M matrices."""
    rng = np.random.default_rng(seed + 7)
    base = iteration_times(recipe, M, seed, compute)
    out = []
    for _ in range(n_segments):
        i = int(rng.integers(0, M))
        j = int((i + 1 + rng.integers(0, M - 1)) % M)
        f = float(np.exp(rng.uniform(np.log(2.0), np.log(100.0))))
        t = base.copy()
        t[i, j] *= f
        t[j, i] *= f
        out.append(t)
    return out
