"""ctypes front end of the CPU oracle (oracle/netmax_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it.  All
arguments are numpy arrays on the host; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "netmax_oracle.c")
_LIB = os.path.join(_DIR, "libnetmax_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (generic x86-64 code, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        L.ora_set_threads.restype = C.c_int
        L.ora_thresholds.restype = C.c_int
        L.ora_peer_of_word.restype = C.c_int32
        L.ora_grad_mlp.restype = C.c_double
        L.ora_round_bf16.restype = C.c_double
        L.ora_consensus_dist.restype = C.c_double
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype, *shape_opts) -> np.ndarray:
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a


def set_threads(n: int) -> int:
    return int(lib().ora_set_threads(C.c_int(n)))


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().ora_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def thresholds(P: np.ndarray):
    """-> (T uint32 [M,M], last int32 [M]); raises ValueError on an invalid row."""
    P = np.ascontiguousarray(P, dtype=np.float64)
    M = P.shape[0]
    T = np.empty((M, M), dtype=np.uint32)
    last = np.empty(M, dtype=np.int32)
    if lib().ora_thresholds(C.c_int(M), _p(P), _p(T), _p(last)) != 0:
        raise ValueError("invalid policy matrix")
    return T, last


def peer_of_word(Trow: np.ndarray, last: int, u: int) -> int:
    Trow = _chk(Trow, np.uint32)
    return int(lib().ora_peer_of_word(C.c_int(Trow.shape[0]), _p(Trow), C.c_int32(last), C.c_uint32(u)))


def sample_peers(T: np.ndarray, last: np.ndarray, seed: int, it: int) -> np.ndarray:
    M = T.shape[0]
    peer = np.empty(M, dtype=np.int32)
    lib().ora_sample_peers(C.c_int(M), _p(_chk(T, np.uint32)), _p(_chk(last, np.int32)),
                           C.c_uint64(seed), C.c_uint64(it), _p(peer))
    return peer


def mix_weights(P: np.ndarray, adj: Optional[np.ndarray], alpha: float, rho: float) -> np.ndarray:
    P = np.ascontiguousarray(P, dtype=np.float64)
    M = P.shape[0]
    if adj is not None:
        adj = np.ascontiguousarray(adj, dtype=np.uint8)
    w = np.empty((M, M), dtype=np.float64)
    lib().ora_mix_weights(C.c_int(M), _p(P), _p(adj), C.c_double(alpha), C.c_double(rho), _p(w))
    return w


def mix_weights_fixed(P: np.ndarray, weight: float) -> np.ndarray:
    P = np.ascontiguousarray(P, dtype=np.float64)
    M = P.shape[0]
    w = np.empty((M, M), dtype=np.float64)
    lib().ora_mix_weights_fixed(C.c_int(M), _p(P), C.c_double(weight), _p(w))
    return w


def sample_batch(M: int, B: int, shard_off: np.ndarray, seed: int, it: int) -> np.ndarray:
    idx = np.empty((M, B), dtype=np.int32)
    lib().ora_sample_batch(C.c_int(M), C.c_int(B), _p(_chk(shard_off, np.int64)),
                           C.c_uint64(seed), C.c_uint64(it), _p(idx))
    return idx


def synth_grad(M: int, D: int, ld: int, sigma: float, seed: int, it: int,
               out: Optional[np.ndarray] = None, col0: int = 0) -> np.ndarray:
    """G [M, ld] = columns col0 .. col0+ld-1 of the full gradient matrix; the first D of them are valid."""
    assert col0 % 4 == 0
    G = np.empty((M, ld), dtype=np.float32) if out is None else _chk(out, np.float32)
    lib().ora_synth_grad(C.c_int(M), C.c_int64(D), C.c_int64(ld), C.c_int64(col0), C.c_double(sigma),
                         C.c_uint64(seed), C.c_uint64(it), _p(G))
    return G


def round_bf16(x: float) -> float:
    return float(lib().ora_round_bf16(C.c_double(x)))


def grad_mlp(dims: Sequence[int], params: np.ndarray, feats: np.ndarray, labels: np.ndarray,
             idx: np.ndarray, operands_bf16: bool = False):
    """One worker. feats: float32 or uint16 (bfloat16 bits) [n, dims[0]]. -> (grad float32 [D], loss).
    operands_bf16: round both operands of every matrix product to bfloat16 (the bf16 workload's arithmetic)."""
    d = np.asarray(dims, dtype=np.int64)
    nl = len(dims) - 1
    Dp = int(sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(nl)))
    assert params.shape[0] >= Dp
    bf16 = feats.dtype == np.uint16
    assert bf16 or feats.dtype == np.float32
    assert feats.flags.c_contiguous and feats.shape[1] == dims[0]
    idx = _chk(idx, np.int32)
    assert idx.min() >= 0 and idx.max() < feats.shape[0]
    grad = np.empty(Dp, dtype=np.float32)
    loss = lib().ora_grad_mlp(C.c_int(nl), _p(d), _p(_chk(params, np.float32)), _p(feats), C.c_int(int(bf16)),
                              C.c_int(int(operands_bf16)), _p(_chk(labels, np.int32)), _p(idx), C.c_int(idx.shape[0]),
                              _p(grad))
    return grad, float(loss)


def local_grad(dims: Sequence[int], X: np.ndarray, feats: np.ndarray, labels: np.ndarray,
               shard_off: np.ndarray, idx: np.ndarray, out: Optional[np.ndarray] = None,
               operands_bf16: bool = False):
    """All workers. X, G: float32 [M, ld]; idx int32 [M, B] shard-local. -> (G, loss float64 [M])."""
    d = np.asarray(dims, dtype=np.int64)
    M, ld = X.shape
    bf16 = feats.dtype == np.uint16
    assert bf16 or feats.dtype == np.float32
    assert feats.flags.c_contiguous and feats.shape[1] == dims[0]
    G = np.empty_like(X) if out is None else _chk(out, np.float32)
    loss = np.empty(M, dtype=np.float64)
    lib().ora_local_grad(C.c_int(M), C.c_int64(ld), C.c_int(len(dims) - 1), _p(d), _p(_chk(X, np.float32)),
                         _p(feats), C.c_int(int(bf16)), C.c_int(int(operands_bf16)), _p(_chk(labels, np.int32)),
                         _p(_chk(shard_off, np.int64)),
                         _p(_chk(idx, np.int32)), C.c_int(idx.shape[1]), _p(G), _p(loss))
    return G, loss


def hidden_mlp(dims: Sequence[int], params: np.ndarray, feats: np.ndarray, idx: np.ndarray,
               operands_bf16: bool = False):
    """One worker: the pre-activations of the hidden layers on the batch, as a list of float64 [B, dims[l+1]]."""
    d = np.asarray(dims, dtype=np.int64)
    nl = len(dims) - 1
    bf16 = feats.dtype == np.uint16
    assert bf16 or feats.dtype == np.float32
    assert feats.flags.c_contiguous and feats.shape[1] == dims[0]
    idx = _chk(idx, np.int32)
    B = idx.shape[0]
    z = np.empty(B * int(sum(dims[1:nl])), dtype=np.float64)
    lib().ora_hidden_mlp(C.c_int(nl), _p(d), _p(_chk(params, np.float32)), _p(feats), C.c_int(int(bf16)),
                         C.c_int(int(operands_bf16)), _p(idx), C.c_int(B), _p(z))
    out, o = [], 0
    for l in range(1, nl):
        out.append(z[o:o + B * dims[l]].reshape(B, dims[l]))
        o += B * dims[l]
    return out


def local_hidden(dims: Sequence[int], X: np.ndarray, feats: np.ndarray, shard_off: np.ndarray, idx: np.ndarray,
                 operands_bf16: bool = False):
    """All workers: list over hidden layers of float64 [M, B, dims[l+1]] pre-activations."""
    d = np.asarray(dims, dtype=np.int64)
    nl = len(dims) - 1
    M, ld = X.shape
    B = idx.shape[1]
    bf16 = feats.dtype == np.uint16
    assert bf16 or feats.dtype == np.float32
    assert feats.flags.c_contiguous and feats.shape[1] == dims[0]
    per = B * int(sum(dims[1:nl]))
    Z = np.empty((M, per), dtype=np.float64)
    lib().ora_local_hidden(C.c_int(M), C.c_int64(ld), C.c_int(nl), _p(d), _p(_chk(X, np.float32)), _p(feats),
                           C.c_int(int(bf16)), C.c_int(int(operands_bf16)), _p(_chk(shard_off, np.int64)),
                           _p(_chk(idx, np.int32)), C.c_int(B), _p(Z))
    out, o = [], 0
    for l in range(1, nl):
        out.append(Z[:, o:o + B * dims[l]].reshape(M, B, dims[l]))
        o += B * dims[l]
    return out


def mix(Xcur: np.ndarray, G: np.ndarray, V: np.ndarray, peer: np.ndarray, w: np.ndarray,
        alpha: float, mu: float, wd: float = 0.0, out: Optional[np.ndarray] = None,
        convex_form: bool = False) -> np.ndarray:
    """Momentum apply + mix for all workers; V is updated in place; returns x^{t+1}."""
    M, ld = Xcur.shape
    Xn = np.empty_like(Xcur) if out is None else _chk(out, np.float32)
    assert peer.min() >= 0 and peer.max() < M
    f = lib().ora_mix_convex if convex_form else lib().ora_mix
    f(C.c_int(M), C.c_int64(ld), _p(_chk(Xcur, np.float32)), _p(_chk(G, np.float32)), _p(_chk(V, np.float32)),
      _p(Xn), _p(_chk(peer, np.int32)), _p(_chk(w, np.float64)), C.c_double(alpha), C.c_double(mu), C.c_double(wd))
    return Xn


def activity(t: np.ndarray, P: np.ndarray, adj: Optional[np.ndarray] = None) -> np.ndarray:
    """p_i of Eq. (d4) from the mean iteration times of Eq. (d3)."""
    t = np.ascontiguousarray(t, dtype=np.float64)
    P = np.ascontiguousarray(P, dtype=np.float64)
    M = P.shape[0]
    if adj is not None:
        adj = np.ascontiguousarray(adj, dtype=np.uint8)
    out = np.empty(M, dtype=np.float64)
    lib().ora_activity(C.c_int(M), _p(t), _p(P), _p(adj), _p(out))
    return out


def async_draw(Tact: np.ndarray, last_act: int, T: np.ndarray, last: np.ndarray, seed: int, k: int):
    """(i_k, m_k) of global step k of the asynchronous schedule."""
    M = T.shape[0]
    i, m = C.c_int32(0), C.c_int32(0)
    lib().ora_async_draw(C.c_int(M), _p(_chk(Tact, np.uint32)), C.c_int32(last_act), _p(_chk(T, np.uint32)),
                         _p(_chk(last, np.int32)), C.c_uint64(seed), C.c_uint64(k), C.byref(i), C.byref(m))
    return int(i.value), int(m.value)


def async_apply(X: np.ndarray, V: np.ndarray, g: np.ndarray, i: int, m: int, w: float, alpha: float, mu: float,
                wd: float = 0.0):
    """In-place update of the active worker's row of X and V."""
    M, ld = X.shape
    lib().ora_async_apply(C.c_int(M), C.c_int64(ld), _p(_chk(X, np.float32)), _p(_chk(V, np.float32)),
                          _p(_chk(g, np.float32)), C.c_int(i), C.c_int(m), C.c_double(w), C.c_double(alpha),
                          C.c_double(mu), C.c_double(wd))


def update_times(peer: np.ndarray, t: np.ndarray, beta: float, ema: np.ndarray, clock: Optional[np.ndarray] = None):
    """Algorithm 2's UpdateTimeVector on a simulated network; ema [M, M] and clock [M] (float32) change in place."""
    M = peer.shape[0]
    lib().ora_update_times(C.c_int(M), _p(_chk(peer, np.int32)), _p(_chk(t, np.float32)), C.c_double(beta),
                           _p(_chk(ema, np.float32)), _p(None if clock is None else _chk(clock, np.float32)))


def update_times_async(active: np.ndarray, peers: np.ndarray, t: np.ndarray, beta: float, ema: np.ndarray,
                       clock: Optional[np.ndarray] = None):
    """UpdateTimeVector for a run of global steps of the asynchronous schedule (in order)."""
    M = t.shape[0]
    lib().ora_update_times_async(C.c_int(M), C.c_int64(active.shape[0]), _p(_chk(active, np.int32)), _p(_chk(peers, np.int32)),
                                 _p(_chk(t, np.float32)), C.c_double(beta), _p(_chk(ema, np.float32)),
                                 _p(None if clock is None else _chk(clock, np.float32)))


def consensus_dist(X: np.ndarray, D: Optional[int] = None) -> float:
    M, ld = X.shape
    return float(lib().ora_consensus_dist(C.c_int(M), C.c_int64(ld if D is None else D), C.c_int64(ld),
                                          _p(_chk(X, np.float32))))


class Oracle:
    """State machine over the functions above: one instance = M workers of one workload."""

    def __init__(self, *, M, ld, D, dims, batch, lr, momentum, weight_decay, rho, grad_sigma, seed, P,
                 adj=None, X0, feats=None, labels=None, shard_off=None, col0=0, operands_bf16=False, fixed_weight=None):
        self.operands_bf16 = operands_bf16
        self.fixed_weight = fixed_weight     # None: Algorithm 2's weights; a number: the same weight for every pair
        self.col0 = col0   # flat model: the state is a window of columns of a larger problem
        self.M, self.ld, self.D, self.dims, self.batch = M, ld, D, tuple(dims), batch
        self.lr, self.mu, self.wd, self.sigma, self.seed = float(lr), float(momentum), float(weight_decay), float(grad_sigma), int(seed)
        self.adj = adj
        self.set_policy(P, rho)
        self.X = np.array(X0, dtype=np.float32, copy=True)
        self.Xn = np.empty_like(self.X)
        self.V = np.zeros_like(self.X)
        self.G = np.zeros_like(self.X)
        self.feats, self.labels, self.shard_off = feats, labels, shard_off
        self.loss = None

    def set_policy(self, P, rho):
        self.P, self.rho = np.ascontiguousarray(P, dtype=np.float64), float(rho)
        self.T, self.last = thresholds(self.P)
        self.w = (mix_weights(self.P, self.adj, self.lr, self.rho) if self.fixed_weight is None
                  else mix_weights_fixed(self.P, self.fixed_weight))

    def sample_peers(self, it):
        return sample_peers(self.T, self.last, self.seed, it)

    # ---- asynchronous schedule (one active worker per global step) ----
    def set_activity(self, p_act):
        """p_i of Eq. (d4); thresholds as for a policy row."""
        p_act = np.ascontiguousarray(p_act, dtype=np.float64)
        Tm, lastm = thresholds(np.tile(p_act, (self.M, 1)))
        self.Tact, self.last_act = np.ascontiguousarray(Tm[0]), int(lastm[0])

    def async_step(self, k):
        """Global step k: draw (i_k, m_k), worker i_k's gradient at counter k, update of its row in place."""
        i, m = async_draw(self.Tact, self.last_act, self.T, self.last, self.seed, k)
        self.local_step(k)                       # all rows; only row i is used (same counters as the row alone)
        async_apply(self.X, self.V, np.ascontiguousarray(self.G[i]), i, m, float(self.w[i, m]), self.lr, self.mu, self.wd)
        return i, m

    def local_step(self, it):
        if len(self.dims) == 0:
            synth_grad(self.M, self.D, self.ld, self.sigma, self.seed, it, out=self.G, col0=self.col0)
        else:
            idx = sample_batch(self.M, self.batch, self.shard_off, self.seed, it)
            _, self.loss = local_grad(self.dims, self.X, self.feats, self.labels, self.shard_off, idx, out=self.G,
                                      operands_bf16=self.operands_bf16)
        return self.G

    def mix(self, peer):
        mix(self.X, self.G, self.V, peer, self.w, self.lr, self.mu, self.wd, out=self.Xn)
        self.X, self.Xn = self.Xn, self.X
        return self.X

    def step(self, it):
        peer = self.sample_peers(it)
        self.local_step(it)
        self.mix(peer)
        return peer

    def consensus_dist(self):
        return consensus_dist(self.X, self.D)
