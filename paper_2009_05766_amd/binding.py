"""ctypes binding of libnetmax.so: the same entry points as include/netmax.h, argument
marshalling only.  Device memory comes from PyTorch tensors (their data_ptr()); every step of
the iteration runs in the library's HIP kernels.  There is no CPU fallback: a missing library or
a failing call raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnetmax.so")

NETMAX_MAX_LAYERS = 7
NETMAX_TILE = 2048
NETMAX_STATIC_PARTIALS = 65536
NETMAX_STATIC_MAX_LD = NETMAX_STATIC_PARTIALS * 1024
NETMAX_OK, NETMAX_EINVAL, NETMAX_EINFEASIBLE, NETMAX_ESTATE, NETMAX_EDEVICE, NETMAX_ENOMEM = range(6)
NETMAX_FLAT, NETMAX_MLP = 0, 1
NETMAX_F32, NETMAX_BF16 = 0, 1
NETMAX_MIX_POLICY, NETMAX_MIX_FIXED = 0, 1

EXPORTS = (
    "netmax_init", "netmax_build_tables", "netmax_generate_policy", "netmax_set_policy", "netmax_set_lr", "netmax_bind_state",
    "netmax_bind_data", "netmax_pack", "netmax_unpack", "netmax_sample_peers", "netmax_sample_batch", "netmax_local_step", "netmax_mix", "netmax_run", "netmax_update_times", "netmax_update_times_async", "netmax_activity", "netmax_mean_times", "netmax_set_activity", "netmax_async_run", "netmax_set_fusion", "netmax_set_barrier_patience",
    "netmax_consensus_dist", "netmax_consensus_dist_static", "netmax_params", "netmax_losses", "netmax_read_losses", "netmax_read_hidden", "netmax_iteration", "netmax_get_tables",
    "netmax_last_error", "netmax_destroy",
)


class NetmaxError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"netmax status {code}: {text}")
        self.code = code


class netmax_config(C.Structure):
    _fields_ = [
        ("M", C.c_int32), ("D", C.c_int64), ("ld", C.c_int64),
        ("model", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int64 * (NETMAX_MAX_LAYERS + 1)),
        ("batch", C.c_int32), ("gemm_in", C.c_int32),
        ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float), ("rho", C.c_float),
        ("grad_sigma", C.c_float),
        ("seed", C.c_uint64), ("strict_o3", C.c_int32),
        ("P", C.c_void_p), ("adj", C.c_void_p), ("stream", C.c_void_p),
        ("mix_mode", C.c_int32), ("fixed_weight", C.c_float),
    ]


_lib = None


def load():
    """Loads the built library (building it first only if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build
        build()
    # torch first: its ROCm build carries its own HIP runtime, and the library must bind to that copy (the one the
    # device pointers and streams it is handed come from), not bring a second runtime into the process
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
    sig = {
        "netmax_init": (C.c_int, [C.POINTER(vp), C.POINTER(netmax_config)]),
        "netmax_build_tables": (C.c_int, [i32, vp, vp, f32, f32, i32, i32, f32, vp, vp, vp]),
        "netmax_generate_policy": (C.c_int, [i32, vp, vp, C.c_double, i32, i32, C.c_double, vp, vp, vp, vp, vp]),
        "netmax_set_policy": (C.c_int, [vp, vp, f32]),
        "netmax_set_lr": (C.c_int, [vp, f32]),
        "netmax_bind_state": (C.c_int, [vp, vp, vp, vp, vp]),
        "netmax_bind_data": (C.c_int, [vp, vp, vp, vp]),
        "netmax_pack": (C.c_int, [vp, vp, i64, vp]),
        "netmax_unpack": (C.c_int, [vp, vp, vp, i64]),
        "netmax_sample_peers": (C.c_int, [vp, u64, vp]),
        "netmax_sample_batch": (C.c_int, [vp, u64, vp]),
        "netmax_local_step": (C.c_int, [vp, u64]),
        "netmax_mix": (C.c_int, [vp, u64, vp]),
        "netmax_run": (C.c_int, [vp, u64, i32, vp, i32]),
        "netmax_update_times": (C.c_int, [vp, vp, vp, f32, vp, vp]),
        "netmax_update_times_async": (C.c_int, [vp, vp, vp, C.c_uint64, vp, f32, vp, vp]),
        "netmax_set_fusion": (C.c_int, [vp, i32]),
        "netmax_set_barrier_patience": (C.c_int, [vp, i64]),
        "netmax_activity": (C.c_int, [C.c_int32, vp, vp, vp, vp]),
        "netmax_mean_times": (C.c_int, [C.c_int32, vp, vp, vp, vp, C.POINTER(C.c_double)]),
        "netmax_set_activity": (C.c_int, [vp, vp]),
        "netmax_async_run": (C.c_int, [vp, C.c_uint64, C.c_uint64, vp, vp]),
        "netmax_consensus_dist": (C.c_int, [vp, C.POINTER(C.c_double)]),
        "netmax_consensus_dist_static": (C.c_int, [i32, i64, i64, vp, vp, vp]),
        "netmax_params": (vp, [vp]),
        "netmax_losses": (vp, [vp]),
        "netmax_read_losses": (C.c_int, [vp, vp]),
        "netmax_read_hidden": (C.c_int, [vp, i32, vp]),
        "netmax_iteration": (u64, [vp]),
        "netmax_get_tables": (C.c_int, [vp, vp, vp, vp]),
        "netmax_last_error": (C.c_char_p, [vp]),
        "netmax_destroy": (C.c_int, [vp]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def _err(ctx) -> str:
    t = load().netmax_last_error(ctx)
    return t.decode() if t else ""


def _check(rc: int, ctx=None):
    if rc != NETMAX_OK:
        raise NetmaxError(rc, _err(ctx))


def _host(a: Optional[np.ndarray], dtype) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dp(t, dtype=None):
    """Device pointer of a contiguous CUDA/HIP torch tensor."""
    import torch
    assert isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous(), "need a contiguous device tensor"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


# ---- the C entry points, one Python function each -------------------------------------------------

def netmax_build_tables(P: np.ndarray, adj: Optional[np.ndarray], lr: float, rho: float, strict_o3: bool = False,
                        mix_mode: int = NETMAX_MIX_POLICY, fixed_weight: float = 0.5):
    P = _host(P, np.float64)
    M = P.shape[0]
    adj = _host(adj, np.uint8)
    thr = np.empty((M, M), np.uint32)
    last = np.empty(M, np.int32)
    w = np.empty((M, M), np.float32)
    _check(load().netmax_build_tables(M, _hp(P), _hp(adj), lr, rho, int(strict_o3), mix_mode, fixed_weight, _hp(thr),
                                      _hp(last), _hp(w)))
    return thr, last, w


def netmax_generate_policy(t: np.ndarray, alpha: float, K: int, R: int, adj: Optional[np.ndarray] = None,
                           eps: float = 1e-3):
    """-> dict(P, rho, tbar, lambda2, t_conv); raises NetmaxError(NETMAX_EINFEASIBLE) if no grid point is feasible."""
    t = _host(t, np.float64)
    M = t.shape[0]
    adj = _host(adj, np.uint8)
    P = np.empty((M, M), np.float64)
    out = (C.c_double * 4)()
    ptr = lambda k: C.c_void_p(C.addressof(out) + 8 * k)
    rc = load().netmax_generate_policy(M, _hp(t), _hp(adj), alpha, K, R, eps, _hp(P), ptr(0), ptr(1), ptr(2), ptr(3))
    if rc != NETMAX_OK:
        raise NetmaxError(rc, "policy generation failed" if rc != NETMAX_EINFEASIBLE else "no feasible grid point")
    return dict(P=P, rho=out[0], tbar=out[1], lambda2=out[2], t_conv=out[3])


def netmax_init(*, M: int, D: int, ld: int, model: int, dims: Sequence[int] = (), batch: int = 0,
                gemm_in: int = NETMAX_F32, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                rho: float, grad_sigma: float = 0.0, seed: int, strict_o3: bool = False, P: np.ndarray,
                adj: Optional[np.ndarray] = None, stream: int = 0, mix_mode: int = NETMAX_MIX_POLICY,
                fixed_weight: float = 0.5):
    cfg = netmax_config()
    cfg.M, cfg.D, cfg.ld, cfg.model = M, D, ld, model
    cfg.n_layers = max(len(dims) - 1, 0)
    for k, d in enumerate(dims):
        cfg.dims[k] = d
    cfg.batch, cfg.gemm_in = batch, gemm_in
    cfg.lr, cfg.momentum, cfg.weight_decay, cfg.rho, cfg.grad_sigma = lr, momentum, weight_decay, rho, grad_sigma
    cfg.seed, cfg.strict_o3 = seed, int(strict_o3)
    P = _host(P, np.float64)
    assert P.shape == (M, M)
    adj = _host(adj, np.uint8)
    cfg.P, cfg.adj = P.ctypes.data, (adj.ctypes.data if adj is not None else None)
    cfg.stream = stream
    cfg.mix_mode, cfg.fixed_weight = mix_mode, fixed_weight
    ctx = C.c_void_p()
    _check(load().netmax_init(C.byref(ctx), C.byref(cfg)))
    return ctx


def netmax_set_policy(ctx, P: np.ndarray, rho: float):
    P = _host(P, np.float64)
    _check(load().netmax_set_policy(ctx, _hp(P), rho), ctx)


def netmax_set_lr(ctx, lr: float):
    _check(load().netmax_set_lr(ctx, lr), ctx)


def netmax_bind_state(ctx, x_a, x_b, v, g):
    import torch
    _check(load().netmax_bind_state(ctx, _dp(x_a, torch.float32), _dp(x_b, torch.float32), _dp(v, torch.float32),
                                    _dp(g, torch.float32)), ctx)


def netmax_bind_data(ctx, feats, labels, shard_off: np.ndarray):
    import torch
    so = _host(shard_off, np.int64)
    _check(load().netmax_bind_data(ctx, _dp(feats), _dp(labels, torch.int32), _hp(so)), ctx)


def netmax_pack(ctx, rows, row_ld: int, tiled):
    import torch
    _check(load().netmax_pack(ctx, _dp(rows, torch.float32), row_ld, _dp(tiled, torch.float32)), ctx)


def netmax_unpack(ctx, tiled, rows, row_ld: int):
    import torch
    _check(load().netmax_unpack(ctx, _dp(tiled, torch.float32), _dp(rows, torch.float32), row_ld), ctx)


def netmax_sample_peers(ctx, it: int, peers):
    import torch
    _check(load().netmax_sample_peers(ctx, it, _dp(peers, torch.int32)), ctx)


def netmax_sample_batch(ctx, it: int, idx):
    import torch
    _check(load().netmax_sample_batch(ctx, it, _dp(idx, torch.int32)), ctx)


def netmax_local_step(ctx, it: int):
    _check(load().netmax_local_step(ctx, it), ctx)


def netmax_mix(ctx, it: int, peers):
    import torch
    _check(load().netmax_mix(ctx, it, _dp(peers, torch.int32)), ctx)


def netmax_run(ctx, first_iter: int, n_iters: int, peers, use_graph: bool = False):
    import torch
    _check(load().netmax_run(ctx, first_iter, n_iters, _dp(peers, torch.int32), int(use_graph)), ctx)


def netmax_set_fusion(ctx, on: bool):
    _check(load().netmax_set_fusion(ctx, int(bool(on))), ctx)


def netmax_set_barrier_patience(ctx, polls: int):
    _check(load().netmax_set_barrier_patience(ctx, polls), ctx)


def netmax_activity(t: np.ndarray, P: np.ndarray, adj: Optional[np.ndarray] = None) -> np.ndarray:
    t, P, adj = _host(t, np.float64), _host(P, np.float64), _host(adj, np.uint8)
    M = P.shape[0]
    out = np.empty(M, np.float64)
    rc = load().netmax_activity(M, _hp(t), _hp(P), _hp(adj), _hp(out))
    if rc != NETMAX_OK:
        raise NetmaxError(rc, "a worker's mean iteration time is not positive")
    return out


def netmax_mean_times(t: np.ndarray, P: np.ndarray, adj: Optional[np.ndarray] = None):
    """-> (tbar float64 [M] of Eq. (d3), global steps per unit of time = sum_i 1 / tbar_i)."""
    t, P, adj = _host(t, np.float64), _host(P, np.float64), _host(adj, np.uint8)
    M = P.shape[0]
    tbar = np.empty(M, np.float64)
    rate = C.c_double()
    rc = load().netmax_mean_times(M, _hp(t), _hp(P), _hp(adj), _hp(tbar), C.byref(rate))
    if rc != NETMAX_OK:
        raise NetmaxError(rc, "a worker's mean iteration time is not positive")
    return tbar, rate.value


def netmax_set_activity(ctx, p_act: np.ndarray):
    p_act = _host(p_act, np.float64)
    _check(load().netmax_set_activity(ctx, _hp(p_act)), ctx)


def netmax_async_run(ctx, first_step: int, n_steps: int, active, peers):
    import torch
    assert active.numel() >= n_steps and peers.numel() >= n_steps
    _check(load().netmax_async_run(ctx, first_step, n_steps, _dp(active, torch.int32), _dp(peers, torch.int32)), ctx)


def netmax_update_times(ctx, peers, t, beta: float, ema, clock=None):
    import torch
    _check(load().netmax_update_times(ctx, _dp(peers, torch.int32), _dp(t, torch.float32), beta, _dp(ema, torch.float32),
                                      None if clock is None else _dp(clock, torch.float32)), ctx)


def netmax_update_times_async(ctx, active, peers, n_steps: int, t, beta: float, ema, clock=None):
    import torch
    _check(load().netmax_update_times_async(ctx, _dp(active, torch.int32), _dp(peers, torch.int32), n_steps,
                                            _dp(t, torch.float32), beta, _dp(ema, torch.float32),
                                            None if clock is None else _dp(clock, torch.float32)), ctx)


def netmax_consensus_dist(ctx) -> float:
    out = C.c_double()
    _check(load().netmax_consensus_dist(ctx, C.byref(out)), ctx)
    return out.value


def netmax_consensus_dist_static(M: int, D: int, ld: int, x, cd, stream: int = 0):
    """x: device float tensor (tile layout), cd: device float64 tensor [1]; enqueues on `stream`, allocates nothing."""
    import torch
    _check(load().netmax_consensus_dist_static(M, D, ld, _dp(x, torch.float32), _dp(cd, torch.float64), stream))


def netmax_params(ctx) -> int:
    return load().netmax_params(ctx) or 0


def netmax_losses(ctx) -> int:
    return load().netmax_losses(ctx) or 0


def netmax_read_losses(ctx, out):
    import torch
    _check(load().netmax_read_losses(ctx, _dp(out, torch.float32)), ctx)


def netmax_read_hidden(ctx, layer: int, out):
    import torch
    _check(load().netmax_read_hidden(ctx, layer, _dp(out, torch.float32)), ctx)


def netmax_iteration(ctx) -> int:
    return int(load().netmax_iteration(ctx))


def netmax_get_tables(ctx, M: int):
    thr = np.empty((M, M), np.uint32)
    last = np.empty(M, np.int32)
    w = np.empty((M, M), np.float32)
    _check(load().netmax_get_tables(ctx, _hp(thr), _hp(last), _hp(w)), ctx)
    return thr, last, w


def netmax_destroy(ctx):
    _check(load().netmax_destroy(ctx))


# ---- a holder for the device buffers of one run ---------------------------------------------------

class NetMax:
    """Owns the torch tensors (device memory) of one run and forwards every step to the library.

    x_a, x_b, v, g are flat device tensors of M * ld floats in the library's worker-interleaved tile
    layout; get()/set() convert from and to row-major [M, cols] through netmax_unpack / netmax_pack."""

    def __init__(self, *, M, D, ld, model, dims=(), batch=0, gemm_in=NETMAX_F32, lr, momentum=0.0,
                 weight_decay=0.0, rho, grad_sigma=0.0, seed, P, adj=None, strict_o3=False,
                 mix_mode=NETMAX_MIX_POLICY, fixed_weight=0.5, X0: Optional[np.ndarray] = None, feats=None, labels=None, shard_off=None, device="cuda:0"):
        import torch
        assert ld % NETMAX_TILE == 0, "ld must be a multiple of NETMAX_TILE"
        self.M, self.D, self.ld, self.batch, self.dims = M, D, ld, batch, tuple(dims)
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self._own = torch.cuda.current_stream(self.device)     # the stream every library call of this run uses
        self.stream = self._own.cuda_stream
        self.ctx = netmax_init(M=M, D=D, ld=ld, model=model, dims=dims, batch=batch, gemm_in=gemm_in, lr=lr,
                               momentum=momentum, weight_decay=weight_decay, rho=rho, grad_sigma=grad_sigma,
                               seed=seed, strict_o3=strict_o3, P=P, adj=adj, stream=self.stream, mix_mode=mix_mode,
                               fixed_weight=fixed_weight)
        kw = dict(dtype=torch.float32, device=self.device)
        self.x_a = torch.zeros(M * ld, **kw)
        self.x_b = torch.zeros(M * ld, **kw)
        self.v = torch.zeros(M * ld, **kw)
        self.g = torch.zeros(M * ld, **kw)
        self.peers = torch.zeros(M, dtype=torch.int32, device=self.device)
        netmax_bind_state(self.ctx, self.x_a, self.x_b, self.v, self.g)
        if X0 is not None:
            self.set("x", X0)
        self.feats = self.labels = None
        if feats is not None:
            if isinstance(feats, np.ndarray):
                if feats.dtype == np.uint16:   # bfloat16 bit patterns
                    feats = torch.from_numpy(feats.view(np.int16)).to(self.device).view(torch.bfloat16)
                else:
                    feats = torch.from_numpy(feats).to(self.device)
            if isinstance(labels, np.ndarray):
                labels = torch.from_numpy(labels).to(self.device)
            self.feats, self.labels = feats.contiguous(), labels.contiguous()
            netmax_bind_data(self.ctx, self.feats, self.labels, shard_off)

    # ---- state access --------------------------------------------------------------------------
    def _join(self):
        """Orders the caller's current stream with the run's stream (they differ when the run was created under
        another `torch.cuda.stream`): work queued on either is finished before the other goes on."""
        import torch
        cur = torch.cuda.current_stream(self.device)
        if cur.cuda_stream != self.stream:
            cur.synchronize()
            self._own.synchronize()

    def _buffer(self, name: str):
        if name == "x":
            return self.params()
        return {"v": self.v, "g": self.g}[name]

    def set(self, name: str, rows):
        """Loads row-major [M, >= D] values (numpy or device tensor) into x (current), v or g."""
        import torch
        if isinstance(rows, np.ndarray):
            rows = torch.from_numpy(np.ascontiguousarray(rows, dtype=np.float32)).to(self.device)
        rows = rows.contiguous()
        assert rows.shape[0] == self.M and rows.shape[1] >= self.D
        self._join()
        netmax_pack(self.ctx, rows, rows.shape[1], self._buffer(name))
        self._own.synchronize()                                # `rows` may be a temporary

    def get(self, name: str, cols: Optional[int] = None):
        """Row-major device tensor [M, cols] of x (current), v or g; cols defaults to ld (padding as zeros)."""
        import torch
        cols = self.ld if cols is None else cols
        out = torch.zeros((self.M, cols), dtype=torch.float32, device=self.device)
        self._join()
        netmax_unpack(self.ctx, self._buffer(name), out, cols)
        self._join()
        return out

    def get_window(self, name: str, col0: int, width: int):
        """Row-major [M, width] copy of columns col0 .. col0+width-1 (inside one tile) without a full unpack."""
        assert col0 // NETMAX_TILE == (col0 + width - 1) // NETMAX_TILE
        t, o = divmod(col0, NETMAX_TILE)
        self._join()
        buf = self._buffer(name).view(self.ld // NETMAX_TILE, self.M, NETMAX_TILE)
        return buf[t, :, o:o + width].contiguous()

    # ---- the iteration -------------------------------------------------------------------------
    def sample_peers(self, it: int):
        netmax_sample_peers(self.ctx, it, self.peers)
        return self.peers

    def local_step(self, it: int):
        netmax_local_step(self.ctx, it)

    def mix(self, it: int, peers=None):
        netmax_mix(self.ctx, it, self.peers if peers is None else peers)

    def step(self, it: int):
        netmax_sample_peers(self.ctx, it, self.peers)
        netmax_local_step(self.ctx, it)
        netmax_mix(self.ctx, it, self.peers)

    def run(self, first_iter: int, n_iters: int, use_graph: bool = False):
        netmax_run(self.ctx, first_iter, n_iters, self.peers, use_graph)

    def consensus_dist(self) -> float:
        return netmax_consensus_dist(self.ctx)

    def params(self):
        """The flat tile-layout tensor that currently holds x^t."""
        p = netmax_params(self.ctx)
        return self.x_a if p == self.x_a.data_ptr() else self.x_b

    def losses(self):
        """Mean batch loss per worker of the last local step (device tensor [M]), None for flat models."""
        import torch
        if not netmax_losses(self.ctx):
            return None
        out = torch.empty(self.M, dtype=torch.float32, device=self.device)
        self._join()
        netmax_read_losses(self.ctx, out)
        self._join()
        return out

    def hidden(self, layer: int):
        """Outputs of hidden layer `layer` of the last local step, device tensor [M, batch, dims[layer]]."""
        import torch
        out = torch.empty((self.M, self.batch, self.dims[layer]), dtype=torch.float32, device=self.device)
        self._join()
        netmax_read_hidden(self.ctx, layer, out)
        self._join()
        return out

    def close(self):
        if self.ctx is not None:
            netmax_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
