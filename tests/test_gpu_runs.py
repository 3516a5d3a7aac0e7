"""GPU parity over whole runs: the five workloads, per step from identical state and as T-step free runs."""
import numpy as np
import pytest
import torch

from netmax_inputs import workload
from harness import inputs_of, make_gpu, make_oracle, rel_err_rows, max_abs_err, relu_disagreements, columns_touched_by

pytestmark = pytest.mark.gpu

# tolerances on the parameters, relative L2 per worker
TOL_STEP, TOL_RUN = 1e-5, 1e-4


def _sync_gpu_from_oracle(gpu, o):
    """The GPU run takes over the oracle's state (never the other way round: what the oracle computes depends on
    nothing the library produced)."""
    gpu.set("x", o.X)
    gpu.set("v", o.V)


def _has_relu(w):
    return len(w.dims) > 2


class _Disputes:
    """Tracks, for ReLU networks, which hidden units had a ReLU decision on which the library and the oracle differ
    (counted from the oracle's pre-activations), so that the element-wise bound can leave out exactly the columns
    such a decision touches.  Nothing to track for flat models and softmax regression."""

    def __init__(self, w, inp, operands_bf16=False):
        self.w, self.inp, self.bf16 = w, inp, operands_bf16
        self.reset()

    def reset(self):
        self.units = {h: set() for h in range(1, len(self.w.dims) - 1)}

    def before_step(self, o, it):
        import oracle
        if _has_relu(self.w):
            idx = oracle.sample_batch(self.w.M, self.w.batch, self.inp["shard_off"], self.w.seed, it)
            self.Z = oracle.local_hidden(self.w.dims, o.X, self.inp["feats"], self.inp["shard_off"], idx,
                                         operands_bf16=self.bf16)

    def after_step(self, gpu):
        if _has_relu(self.w):
            where, _ = relu_disagreements(gpu, self.Z)
            for h, d in enumerate(where, start=1):
                self.units[h] |= set(d[:, 2].tolist())

    def check(self, X, o, tol, what):
        """Row norm, and the same tolerance in the maximum norm element by element (outside the columns a disputed
        ReLU decision touches).  -> the row-norm error."""
        rel = rel_err_rows(X, o.X)
        assert rel < tol, (what, rel)
        err = np.abs(X.astype(np.float64) - o.X).max(axis=0)
        if any(self.units.values()):
            err = err[~columns_touched_by(self.w.dims, self.w.ld, self.units)]
        if err.size:
            assert err.max() <= tol * np.abs(o.X).max(), (what, float(err.max()))
        return rel


def _free_run(w, T, ora_threads=8, cd_rel=1e-3):
    import oracle
    oracle.set_threads(ora_threads)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp), make_oracle(w, inp)
    cd0 = gpu.consensus_dist()
    assert cd0 == pytest.approx(o.consensus_dist(), rel=1e-6)
    for it in range(T):
        gpu.step(it)
        peer = o.step(it)
        assert np.array_equal(gpu.peers.cpu().numpy(), peer)
    X = gpu.get("x").cpu().numpy()
    err = rel_err_rows(X, o.X)
    if not _has_relu(w):                         # the T-step tolerance element by element, in the maximum norm
        assert max_abs_err(X, o.X) <= TOL_RUN * np.abs(o.X).max()
    cd = gpu.consensus_dist()
    assert cd == pytest.approx(o.consensus_dist(), rel=cd_rel)
    assert np.all(X[:, w.D:] == 0)
    oracle.set_threads(1)
    gpu.close()
    return err, cd0, cd


def _stepwise(w, T, tol, ora_threads=8):
    import oracle
    oracle.set_threads(ora_threads)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp), make_oracle(w, inp)
    disputes = _Disputes(w, inp)
    worst = 0.0
    for it in range(T):
        _sync_gpu_from_oracle(gpu, o)
        disputes.reset()
        disputes.before_step(o, it)
        gpu.step(it)
        peer = o.step(it)
        assert np.array_equal(gpu.peers.cpu().numpy(), peer)
        disputes.after_step(gpu)
        worst = max(worst, disputes.check(gpu.get("x").cpu().numpy(), o, tol, it))
    oracle.set_threads(1)
    gpu.close()
    return worst


def _windows(w, T, K, tol, ora_threads=8, operands_bf16=False):
    """The whole horizon T in windows of K steps: at the start of each window the GPU run takes over the
    oracle's state, then both run K steps freely.  Needed for ReLU networks: a hidden pre-activation within
    rounding distance of zero gets derivative 0 on one side and 1 on the other, a discontinuous change of
    the gradient (about 1/sqrt(batch * active units) of its norm) that no summation order can avoid and
    that the dynamics then amplify.  Returns the worst end-of-window error."""
    import oracle
    oracle.set_threads(ora_threads)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp), make_oracle(w, inp, operands_bf16=operands_bf16)
    disputes = _Disputes(w, inp, operands_bf16)
    worst = 0.0
    for it in range(T):
        if it % K == 0:
            _sync_gpu_from_oracle(gpu, o)
            disputes.reset()
        disputes.before_step(o, it)
        gpu.step(it)
        peer = o.step(it)
        assert np.array_equal(gpu.peers.cpu().numpy(), peer)
        disputes.after_step(gpu)
        if (it + 1) % K == 0 or it + 1 == T:
            worst = max(worst, disputes.check(gpu.get("x").cpu().numpy(), o, tol, it))
    oracle.set_threads(1)
    gpu.close()
    return worst


def test_cfg1_full_run():
    w = workload("cfg1")
    assert _stepwise(w, 20, TOL_STEP) < TOL_STEP
    err, cd0, cd = _free_run(w, w.T)
    assert err < TOL_RUN, err
    assert cd < cd0


def test_cfg2_full_shape_per_step():
    """Ten iterations, each from identical state (the whole horizon in windows: test_gpu_full_shape.py)."""
    w = workload("cfg2")
    assert _stepwise(w, 10, TOL_STEP) < TOL_STEP


def test_cfg2_reduced_shape_full_T():
    w = workload("cfg2", dims=(64, 48, 10), n_per_worker=512)
    assert _windows(w, w.T, 50, TOL_RUN) < TOL_RUN
    err, cd0, cd = _free_run(w, w.T, cd_rel=0.1)
    print(f"cfg2 reduced shape, free run of {w.T} steps: relative error {err:.3e}")
    assert err < 5e-2, err          # sanity only: ReLU kinks make long free runs drift apart (see _windows)


@pytest.mark.parametrize("name", ["cfg3", "cfg4"])
def test_flat_reduced_shape_full_T(name):
    w = workload(name, D=2**16)
    assert _stepwise(w, 5, TOL_STEP) < TOL_STEP
    err, cd0, cd = _free_run(w, w.T)
    assert err < TOL_RUN, err


TOL_BF16 = 2e-2
# bf16 operands against the oracle with the same operand rounding, over a window of several steps: an
# activation that fp32 and double accumulation place on different sides of a bf16 rounding boundary
# differs by one bf16 ulp (2^-8 of that element); with ~1e5 activations per step that happens every
# step, so windows drift faster than in the fp32 workloads while staying far below the bf16 tolerance.
TOL_RUN_BF16_SAME = 1e-3


def test_cfg5_reduced_shape():
    w = workload("cfg5", M=8, n_per_worker=512, dims=(3072, 256, 128, 10))
    # against the oracle with the same bf16 operands: fp32 tolerances per step and per window
    assert _windows(w, 10, 1, TOL_STEP, operands_bf16=True) < TOL_STEP
    assert _windows(w, 40, 10, TOL_RUN_BF16_SAME, operands_bf16=True) < TOL_RUN_BF16_SAME
    # against exact arithmetic: the bf16 tolerance, per step and over a free run
    assert _stepwise(w, 3, TOL_BF16) < TOL_BF16
    err, cd0, cd = _free_run(w, 40, cd_rel=0.1)
    assert err < TOL_BF16, err


def test_cfg5_all_workers_tiny_layers_full_T():
    w = workload("cfg5", n_per_worker=64, dims=(48, 32, 16, 10), batch=16)
    assert _windows(w, w.T, 5, TOL_RUN_BF16_SAME, operands_bf16=True) < TOL_RUN_BF16_SAME
    assert _windows(w, w.T, 25, TOL_BF16) < TOL_BF16             # against exact arithmetic
    err, cd0, cd = _free_run(w, w.T, cd_rel=0.2)
    print(f"cfg5 tiny layers, free run of {w.T} steps against exact arithmetic: relative error {err:.3e}")
    assert err < 0.1, err           # sanity only: operand rounding plus ReLU kinks over 500 free steps


@pytest.mark.parametrize("name", ["cfg3", "cfg4"])
def test_flat_full_shape_full_T_sampled_columns(name):
    """Full-size free run over the whole horizon T = 200 in the benchmark's launch configuration.  The update is
    separable by column, so the oracle follows windows of columns (start, tile and chunk boundaries, ragged end) of
    all workers for all 200 iterations; every element of x and v against the run tolerance.  (All columns for a
    short horizon: test_gpu_full_shape.py.)"""
    import oracle
    w = workload(name)
    T = w.T
    P, rho = __import__("netmax_inputs").policy_for(w)
    M, ld = w.M, w.ld
    import paper_2009_05766_amd as nm
    from harness import hyper
    gpu = nm.NetMax(M=M, D=w.D, ld=ld, model=nm.NETMAX_FLAT, seed=w.seed, P=P, **hyper(w, rho))
    # x^0 written on the device straight into the library's buffer (a seeded stand-in of init_params at this
    # size; which value lands in which column does not matter, the oracle reads the windows back)
    g = torch.Generator(device="cuda").manual_seed(7)
    gpu.x_a.normal_(0.0, 0.1, generator=g)
    pad = gpu.x_a.view(ld // nm.NETMAX_TILE, M, nm.NETMAX_TILE)[-1, :, w.D - (ld - nm.NETMAX_TILE):]
    pad.zero_()
    TILE = nm.NETMAX_TILE
    last_tile = (ld // TILE - 1) * TILE
    windows = [0, TILE - 256, TILE * 8 * 5, TILE * (8 * 64 + 3) + 512, (ld // 2) // TILE * TILE + 1024, last_tile - 256,
               last_tile, w.D - 256]
    width = 256
    oracles = []
    tiles_view = gpu.x_a.view(ld // TILE, M, TILE)          # the documented layout, read with torch alone
    for c0 in windows:
        cols = torch.arange(c0, c0 + width, device=gpu.x_a.device)
        x0 = tiles_view[cols // TILE, :, cols % TILE].T.contiguous().cpu().numpy()   # no library kernel touches the oracle's input
        assert np.array_equal(x0, gpu.get_window("x", c0, width).cpu().numpy())
        valid = min(width, w.D - c0)
        oracles.append(oracle.Oracle(M=M, ld=width, D=valid, dims=(), batch=0, seed=w.seed, P=P, X0=x0, col0=c0,
                                     **hyper(w, rho)))
    peers = torch.empty((T, M), dtype=torch.int32, device="cuda")
    for it in range(T):
        gpu.step(it)
        peers[it] = gpu.peers
    peers = peers.cpu().numpy()
    for it in range(T):
        for o in oracles:
            assert np.array_equal(o.step(it), peers[it])
    worst = 0.0
    for c0, o in zip(windows, oracles):
        for what, want in (("x", o.X), ("v", o.V)):
            got = gpu.get_window(what, c0, width).cpu().numpy()
            assert rel_err_rows(got, want) < TOL_RUN
            assert max_abs_err(got, want) <= TOL_RUN * np.abs(want).max()
            worst = max(worst, max_abs_err(got, want) / np.abs(want).max())
    print(f"{name} full shape, free run of {T} iterations, {len(windows)} windows of {width} columns: worst max|d|/max {worst:.2e}")
    gpu.close()


def test_checkpoint_resume_is_bit_exact():
    w = workload("cfg4", D=10000, T=20)
    inp = inputs_of(w)
    a = make_gpu(w, inp)
    for it in range(20):
        a.step(it)
    b = make_gpu(w, inp)
    for it in range(10):
        b.step(it)
    Xh, Vh = b.get("x").cpu().numpy().copy(), b.get("v").cpu().numpy().copy()
    b.close()
    c = make_gpu(w, dict(inp, X0=Xh))
    c.set("v", Vh)
    for it in range(10, 20):
        c.step(it)
    assert np.array_equal(a.get("x").cpu().numpy(), c.get("x").cpu().numpy())
    assert np.array_equal(a.get("v").cpu().numpy(), c.get("v").cpu().numpy())
    a.close(); c.close()


def test_generated_policy_installed_mid_run():
    """The monitor's product (Algorithm 3) arriving during training (Algorithm 2, "received new policy"):
    policy and rho generated from an iteration-time matrix, installed after 10 iterations.  The library's policy
    is checked against the oracle's; both runs then install the oracle's."""
    import paper_2009_05766_amd as nm
    from oracle import policy as opol
    from netmax_inputs import iteration_times
    w = workload("cfg4", M=16, D=30000, T=30)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp), make_oracle(w, inp)
    t = iteration_times("four_group_12", w.M)
    alpha = float(np.float32(w.lr))
    ref = opol.generate_policy(t, alpha, 40, 6)
    pol = nm.netmax_generate_policy(t, alpha, 40, 6)
    assert pol["rho"] == pytest.approx(ref["rho"], rel=1e-12) and np.abs(pol["P"] - ref["P"]).max() < 1e-8
    rho = float(np.float32(ref["rho"]))
    for it in range(w.T):
        if it == 10:
            nm.netmax_set_policy(gpu.ctx, ref["P"], rho)
            o.set_policy(ref["P"], rho)
        gpu.step(it)
        assert np.array_equal(gpu.peers.cpu().numpy(), o.step(it))
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    gpu.close()


def test_dynamic_network_replay_with_monitor():
    """Algorithm 1 + Algorithm 2's time bookkeeping on a network whose slow link moves (Section V-A): workers
    smooth the iteration times they see, every segment the monitor turns the collected matrix into a policy.
    GPU side: netmax_update_times / netmax_generate_policy through the Monitor; oracle side: ora_update_times and the
    oracle's Algorithm 3.  Moving averages, clocks and the generated policies are compared; both runs then install
    the oracle's policy, so that the trajectories stay comparable draw by draw."""
    import oracle
    from oracle import policy as opol
    from netmax_inputs import dynamic_times, iteration_times
    from paper_2009_05766_amd.monitor import Monitor
    w = workload("cfg3", M=12, D=20000, T=90)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp), make_oracle(w, inp)
    alpha, K, R, beta = float(np.float32(w.lr)), 40, 6, 0.7
    prior = 1.3 * iteration_times("two_tier_10", w.M)            # a biased first estimate, so that every average moves
    nets = dynamic_times("two_tier_10", w.M, 3)
    mon = Monitor(gpu, alpha=alpha, K=K, R=R, beta=beta, initial_times=prior)
    ema = prior.astype(np.float32)
    clock = np.zeros(w.M, np.float32)
    it = 0
    for t in nets:
        mon.set_network(t)
        t32 = t.astype(np.float32)
        for _ in range(30):
            peers = gpu.sample_peers(it)
            mon.observe()
            gpu.local_step(it)
            gpu.mix(it)
            po = o.step(it)
            oracle.update_times(po, t32, beta, ema, clock)
            assert np.array_equal(peers.cpu().numpy(), po)
            it += 1
        got = mon.collect()
        assert np.allclose(got, ema, rtol=1e-6, atol=0)
        assert np.allclose(mon.clock.cpu().numpy(), clock, rtol=1e-6)
        ref = opol.generate_policy(ema.astype(np.float64), alpha, K, R)
        mine = mon.reschedule()                                  # from the device's own averages
        assert (ref is None) == (mine is None)
        if ref is not None:
            assert mine["t_conv"] == pytest.approx(ref["t_conv"], rel=1e-4)
            if mine["rho"] == pytest.approx(ref["rho"], rel=1e-9) and mine["tbar"] == pytest.approx(ref["tbar"], rel=1e-5):
                assert np.abs(mine["P"] - ref["P"]).max() < 1e-5
            rho = float(np.float32(ref["rho"]))
            mon.install(ref["P"], rho)
            o.set_policy(ref["P"], rho)
    assert (ema != prior.astype(np.float32)).sum() > 8 * w.M    # the averages moved
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    assert gpu.consensus_dist() == pytest.approx(o.consensus_dist(), rel=1e-3)
    gpu.close()


def test_replay_driver_runs_segments():
    """The replay driver (sampling, time bookkeeping, local step, mix, periodic rescheduling) against the same
    sequence of library calls made by hand."""
    from netmax_inputs import dynamic_times, iteration_times
    from paper_2009_05766_amd.monitor import Monitor, replay
    w = workload("cfg1")
    inp = inputs_of(w)
    nets = dynamic_times("two_tier_10", w.M, 2)
    prior = iteration_times("two_tier_10", w.M)
    kw = dict(alpha=float(np.float32(w.lr)), K=20, R=6, beta=0.5, initial_times=prior)
    a, b = make_gpu(w, inp), make_gpu(w, inp)
    hist = replay(a, Monitor(a, **kw), nets, 20)
    mon = Monitor(b, **kw)
    it = 0
    for t in nets:
        mon.set_network(t)
        for _ in range(20):
            b.sample_peers(it)
            mon.observe()
            b.local_step(it)
            b.mix(it)
            it += 1
        mon.reschedule()
    assert torch.equal(a.get("x"), b.get("x"))
    assert len(hist) == 2 and hist[-1]["iteration"] == 40 and hist[-1]["sim_time"] == float(mon.clock.max().item())
    assert hist[-1]["sim_time"] > 0 and np.isfinite(hist[-1]["consensus_dist"])
    a.close(), b.close()


def test_fixed_weight_averaging_mode():
    """Gossip / AD-PSGD averaging (weight 1/2 for every pulled model) under the link-speed-tuned policy."""
    w = workload("cfg3", M=16, D=20000, T=40)
    inp = inputs_of(w)
    gpu, o = make_gpu(w, inp, fixed_weight=0.5), make_oracle(w, inp, fixed_weight=0.5)
    for it in range(w.T):
        gpu.step(it)
        assert np.array_equal(gpu.peers.cpu().numpy(), o.step(it))
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    assert gpu.consensus_dist() == pytest.approx(o.consensus_dist(), rel=1e-3)
    gpu.close()


@pytest.mark.parametrize("name,over", [("cfg1", dict()), ("cfg3", dict(M=16, D=50000)),
                                       ("cfg5", dict(M=4, n_per_worker=128, dims=(256, 128, 128, 10), batch=64)),
                                       ("cfg2", dict(M=4, n_per_worker=256, dims=(96, 64, 10)))])
def test_graph_replay_matches_the_individual_calls(name, over):
    """netmax_run with HIP graph replay: several replays of both ping-pong directions, with eager work of
    the same context and synchronisations in between; every replay is compared with the eager path bit for bit."""
    import paper_2009_05766_amd as nm
    w = workload(name, **over)
    inp = inputs_of(w)
    eager = make_gpu(w, inp)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = make_gpu(w, inp)
        it = 0
        for n in (3, 1, 4, 2, 5):
            graph.run(it, n, use_graph=True)
            side.synchronize()
            for k in range(n):
                eager.step(it + k)
            torch.cuda.synchronize()
            it += n
            assert nm.netmax_iteration(graph.ctx) == it
            assert np.array_equal(graph.peers.cpu().numpy(), eager.peers.cpu().numpy())
            assert np.array_equal(graph.get("x").cpu().numpy(), eager.get("x").cpu().numpy()), (it, n)
            assert np.array_equal(graph.get("v").cpu().numpy(), eager.get("v").cpu().numpy())
            assert graph.consensus_dist() == eager.consensus_dist()          # eager work between replays
        # the un-captured multi-iteration path gives the same again
        graph.run(it, 3, use_graph=False)
        for k in range(3):
            eager.step(it + k)
        side.synchronize()
        torch.cuda.synchronize()
        assert np.array_equal(graph.get("x").cpu().numpy(), eager.get("x").cpu().numpy())
        # a new learning rate drops the captured graphs; the next replay uses it
        lr2 = float(np.float32(w.lr * 0.5))
        nm.netmax_set_lr(graph.ctx, lr2)
        nm.netmax_set_lr(eager.ctx, lr2)
        graph.run(it + 3, 2, use_graph=True)
        for k in range(2):
            eager.step(it + 3 + k)
        side.synchronize()
        torch.cuda.synchronize()
        assert np.array_equal(graph.get("x").cpu().numpy(), eager.get("x").cpu().numpy())
        graph.close()
    # the null stream cannot be captured: a clear error instead
    with pytest.raises(nm.NetmaxError) as e:
        eager.run(100, 1, use_graph=True)
    assert e.value.code == nm.NETMAX_ESTATE
    eager.close()


def test_smoke_entry_point():
    import __graft_entry__
    __graft_entry__.smoke()


def _async_pair(w, inp, **over):
    import oracle
    import paper_2009_05766_amd as nm
    from netmax_inputs import iteration_times
    gpu, o = make_gpu(w, inp, **over), make_oracle(w, inp, **over)
    p_act = oracle.activity(iteration_times(w.links, w.M), inp["P"])
    assert np.allclose(nm.netmax_activity(iteration_times(w.links, w.M), inp["P"]), p_act, rtol=1e-13)
    nm.netmax_set_activity(gpu.ctx, p_act)
    o.set_activity(p_act)
    return gpu, o


def test_async_schedule_flat():
    """One active worker per global step (Eq. (c2)-(c4)): draws bit-exact, the active rows within the run tolerance,
    everybody else untouched; then a synchronous iteration on top of the asynchronously reached state."""
    import paper_2009_05766_amd as nm
    w = workload("cfg3", M=8, D=5000, T=10)
    inp = inputs_of(w)
    gpu, o = _async_pair(w, inp)
    n = 160
    active = torch.zeros(n, dtype=torch.int32, device="cuda")
    peers = torch.zeros(n, dtype=torch.int32, device="cuda")
    nm.netmax_async_run(gpu.ctx, 0, 100, active, peers)
    nm.netmax_async_run(gpu.ctx, 100, 60, active[100:], peers[100:])     # a run continues where the last one stopped
    want = np.array([o.async_step(k) for k in range(n)], dtype=np.int32)
    assert np.array_equal(active.cpu().numpy(), want[:, 0]) and np.array_equal(peers.cpu().numpy(), want[:, 1])
    assert len(set(want[:, 0])) == w.M
    assert nm.netmax_iteration(gpu.ctx) == n
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    assert rel_err_rows(gpu.get("v").cpu().numpy(), o.V) < TOL_RUN
    i_last = int(want[-1, 0])
    assert np.allclose(gpu.get("g").cpu().numpy()[i_last], o.G[i_last], rtol=0, atol=2e-6 * w.grad_sigma * 6)
    assert gpu.consensus_dist() == pytest.approx(o.consensus_dist(), rel=1e-3)
    gpu.step(n)
    assert np.array_equal(gpu.peers.cpu().numpy(), o.step(n))
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    gpu.close()


@pytest.mark.parametrize("name,over", [("cfg1", dict()), ("cfg5", dict(M=4, n_per_worker=128, dims=(256, 128, 128, 10), batch=64)),
                                       # more workers: several independent global steps per batch of launches
                                       ("cfg1", dict(M=40, n_per_worker=64, dims=(24, 10), batch=8)),
                                       ("cfg2", dict(M=16, n_per_worker=64, dims=(40, 24, 10), batch=16)),
                                       ("cfg5", dict(M=12, n_per_worker=128, dims=(256, 128, 128, 10), batch=64))])
def test_async_schedule_perceptron(name, over):
    import paper_2009_05766_amd as nm
    w = workload(name, **over)
    inp = inputs_of(w)
    bf = w.gemm_in == "bf16"
    gpu, o = _async_pair(w, inp)
    if bf:
        o.operands_bf16 = True
    n = 24
    active = torch.zeros(n, dtype=torch.int32, device="cuda")
    peers = torch.zeros(n, dtype=torch.int32, device="cuda")
    worst = 0.0
    for k0 in range(0, n, 6):                       # windows: re-synchronised so that ReLU flips do not accumulate
        _sync_gpu_from_oracle(gpu, o)
        nm.netmax_async_run(gpu.ctx, k0, 6, active[k0:], peers[k0:])
        want = np.array([o.async_step(k) for k in range(k0, k0 + 6)], dtype=np.int32)
        assert np.array_equal(active[k0:k0 + 6].cpu().numpy(), want[:, 0])
        assert np.array_equal(peers[k0:k0 + 6].cpu().numpy(), want[:, 1])
        worst = max(worst, rel_err_rows(gpu.get("x").cpu().numpy(), o.X))
    assert worst < (1e-3 if bf else TOL_RUN), worst
    gpu.close()


def test_async_schedule_flat_many_workers_in_batches():
    """With many workers most consecutive global steps touch different rows; the library runs such steps as one
    batch of launches.  Same draws, same rows as the oracle's strictly sequential steps, including the steps at which
    a batch has to end (a worker active twice, a pull from a row just written, a write to a row just pulled)."""
    import paper_2009_05766_amd as nm
    w = workload("cfg3", M=64, D=3000, T=10)
    inp = inputs_of(w)
    gpu, o = _async_pair(w, inp)
    n = 700
    active = torch.zeros(n, dtype=torch.int32, device="cuda")
    peers = torch.zeros(n, dtype=torch.int32, device="cuda")
    nm.netmax_async_run(gpu.ctx, 0, n, active, peers)
    want = np.array([o.async_step(k) for k in range(n)], dtype=np.int32)
    assert np.array_equal(active.cpu().numpy(), want[:, 0]) and np.array_equal(peers.cpu().numpy(), want[:, 1])
    # the run contains the conflicts that end a batch
    a, m = want[:, 0], want[:, 1]
    assert (a[1:] == a[:-1]).any() or (m[1:] == a[:-1]).any() or (a[1:] == m[:-1]).any()
    assert rel_err_rows(gpu.get("x").cpu().numpy(), o.X) < TOL_RUN
    assert rel_err_rows(gpu.get("v").cpu().numpy(), o.V) < TOL_RUN
    assert max_abs_err(gpu.get("x").cpu().numpy(), o.X) <= TOL_RUN * np.abs(o.X).max()
    gpu.close()


def test_async_time_bookkeeping_matches_oracle():
    import oracle
    import paper_2009_05766_amd as nm
    from netmax_inputs import iteration_times
    w = workload("cfg3", M=8, D=3000, T=5)
    inp = inputs_of(w)
    gpu, o = _async_pair(w, inp)
    n, beta = 300, 0.7
    t = iteration_times(w.links, w.M).astype(np.float32)
    active = torch.zeros(n, dtype=torch.int32, device="cuda")
    peers = torch.zeros(n, dtype=torch.int32, device="cuda")
    nm.netmax_async_run(gpu.ctx, 0, n, active, peers)
    ema = torch.zeros((w.M, w.M), dtype=torch.float32, device="cuda")
    clock = torch.zeros(w.M, dtype=torch.float32, device="cuda")
    nm.netmax_update_times_async(gpu.ctx, active, peers, n, torch.from_numpy(t).cuda(), beta, ema, clock)
    want = np.array([oracle.async_draw(o.Tact, o.last_act, o.T, o.last, o.seed, k) for k in range(n)], dtype=np.int32)
    ema_o, clock_o = np.zeros((w.M, w.M), np.float32), np.zeros(w.M, np.float32)
    oracle.update_times_async(np.ascontiguousarray(want[:, 0]), np.ascontiguousarray(want[:, 1]), t, beta, ema_o, clock_o)
    assert np.allclose(ema.cpu().numpy(), ema_o, rtol=1e-6, atol=0) and np.allclose(clock.cpu().numpy(), clock_o, rtol=1e-5)
    assert np.count_nonzero(ema_o) > w.M
    gpu.close()


def test_async_schedule_needs_activities():
    import paper_2009_05766_amd as nm
    w = workload("cfg3", M=4, D=3000, T=5)
    gpu = make_gpu(w, inputs_of(w))
    a = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(nm.NetmaxError) as e:
        nm.netmax_async_run(gpu.ctx, 0, 4, a, a.clone())
    assert e.value.code == nm.NETMAX_ESTATE
    with pytest.raises(nm.NetmaxError) as e:
        nm.netmax_set_activity(gpu.ctx, np.array([0.5, 0.5, 0.5, -0.5]))
    assert e.value.code == nm.NETMAX_EINVAL
    nm.netmax_set_activity(gpu.ctx, np.array([0.0, 1.0, 0.0, 0.0]))
    nm.netmax_async_run(gpu.ctx, 0, 4, a, a.clone())
    assert a.cpu().numpy().tolist() == [1, 1, 1, 1]          # a worker of probability 0 is never active
    gpu.close()


def test_policy_comparison_demo_runs(capsys):
    """The uniform-versus-generated-policy comparison at equal simulated time (a demonstration, not a claim):
    it runs, both policies get the steps their mean iteration times allow, and both keep training."""
    import json
    from paper_2009_05766_amd import demo_policies
    assert demo_policies.main(["--workload", "cfg1", "--time", "60", "--K", "20", "--R", "6"]) == 0
    out = json.loads(capsys.readouterr().out)
    runs = out["runs"]
    assert set(runs) == {"uniform policy", "generated policy (Algorithm 3)"}
    for r in runs.values():
        assert r["steps"] == int(60 * r["steps_per_time"]) and r["steps"] > 20
        assert np.isfinite(r["loss"]) and np.isfinite(r["consensus_dist"]) and r["loss"] < 2.4   # below ln 10 + margin


def test_dynamic_network_demo_runs(capsys):
    """The moving-slow-link demonstration: the monitor loop on the asynchronous schedule regenerates policies from
    the smoothed times the workers saw and installs them, the fixed uniform policy generates none, both train."""
    import json
    from paper_2009_05766_amd import demo_policies
    assert demo_policies.main(["--workload", "cfg1", "--dynamic", "3", "--time", "40", "--periods", "2",
                               "--K", "20", "--R", "6"]) == 0
    runs = json.loads(capsys.readouterr().out)["runs"]
    fixed, loop = runs["uniform policy, fixed"], runs["monitor loop (Algorithms 1-3)"]
    assert fixed["policies_generated"] == 0 and 1 <= loop["policies_generated"] <= 6
    for r in (fixed, loop):
        assert r["steps"] > 20 and np.isfinite(r["loss"]) and np.isfinite(r["consensus_dist"]) and r["loss"] < 2.4


@pytest.mark.parametrize("over", [dict(M=4, n_per_worker=128, dims=(256, 128, 128, 10), batch=64),
                                  dict(M=9, n_per_worker=150, dims=(256, 256, 128, 10), batch=96),
                                  dict(M=3, n_per_worker=100, dims=(200, 128, 128, 10), batch=64),
                                  dict(M=2, n_per_worker=300, dims=(3072, 1024, 1024, 10))])
def test_fused_weight_gradient_and_mix(over):
    """netmax_run with the second-step update applied inside the weight-gradient kernels against the separate
    kernels: the same x and v (the gradient and the update are computed by the same instructions in the same
    order), also when replayed as a graph, and back to the separate kernels afterwards."""
    import paper_2009_05766_amd as nm
    w = workload("cfg5", **over)
    inp = inputs_of(w)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plain, fused = make_gpu(w, inp), make_gpu(w, inp)
        nm.netmax_set_fusion(fused.ctx, True)
        it = 0
        for n, graph in ((3, False), (2, True), (3, True), (1, False)):
            plain.run(it, n, use_graph=False)
            fused.run(it, n, use_graph=graph)
            side.synchronize()
            it += n
            assert np.array_equal(plain.peers.cpu().numpy(), fused.peers.cpu().numpy())
            xa, xb = plain.get("x").cpu().numpy(), fused.get("x").cpu().numpy()
            va, vb = plain.get("v").cpu().numpy(), fused.get("v").cpu().numpy()
            assert np.array_equal(xa, xb), (it, float(np.abs(xa - xb).max()))
            assert np.array_equal(va, vb), (it, float(np.abs(va - vb).max()))
        if w.D < 1 << 18:                                   # and against the oracle directly, as for the separate kernels
            o = make_oracle(w, inp)
            for k in range(it):
                o.step(k)
            assert rel_err_rows(xb, o.X) < TOL_BF16
        nm.netmax_set_fusion(fused.ctx, False)
        plain.run(it, 2)
        fused.run(it, 2)
        side.synchronize()
        assert np.array_equal(plain.get("x").cpu().numpy(), fused.get("x").cpu().numpy())
        assert np.array_equal(plain.get("g").cpu().numpy(), fused.get("g").cpu().numpy())
        plain.close(), fused.close()


def test_fusion_needs_matrix_core_layers():
    import paper_2009_05766_amd as nm
    w = workload("cfg1")
    gpu = make_gpu(w, inputs_of(w))
    with pytest.raises(nm.NetmaxError) as e:
        nm.netmax_set_fusion(gpu.ctx, True)
    assert e.value.code == nm.NETMAX_ESTATE
    nm.netmax_set_fusion(gpu.ctx, False)
    gpu.close()


@pytest.mark.parametrize("name,over", [("cfg3", dict(M=16, D=50000)), ("cfg4", dict(M=5, D=9000))])
def test_fused_synthetic_gradient_and_mix(name, over):
    """Flat models: the gradient generated inside the update kernel.  g, x and v equal those of the two separate
    kernels bit for bit, eagerly and as a graph; the oracle agrees as for the separate kernels."""
    import paper_2009_05766_amd as nm
    w = workload(name, **over)
    inp = inputs_of(w)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plain, fused, o = make_gpu(w, inp), make_gpu(w, inp), make_oracle(w, inp)
        nm.netmax_set_fusion(fused.ctx, True)
        it = 0
        for n, graph in ((3, False), (4, True), (2, False)):
            plain.run(it, n)
            fused.run(it, n, use_graph=graph)
            side.synchronize()
            for k in range(n):
                o.step(it + k)
            it += n
            for name_ in ("x", "v", "g"):
                assert np.array_equal(plain.get(name_).cpu().numpy(), fused.get(name_).cpu().numpy()), (it, name_)
        assert rel_err_rows(fused.get("x").cpu().numpy(), o.X) < TOL_RUN
        assert np.all(fused.get("g").cpu().numpy()[:, w.D:] == 0)
        plain.close(), fused.close()


def test_fused_update_with_weight_decay_fixed_weight_and_policy_change():
    """The fused path reads the same tables and hyper-parameters as the separate kernels: weight decay, the
    fixed-weight mode, a new learning rate and a new policy between runs."""
    import paper_2009_05766_amd as nm
    from netmax_inputs import iteration_times
    from oracle import policy as opol
    w = workload("cfg5", M=6, n_per_worker=128, dims=(256, 128, 128, 10), batch=64)
    inp = inputs_of(w)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plain = make_gpu(w, inp, fixed_weight=0.5, weight_decay=float(np.float32(1e-3)))
        fused = make_gpu(w, inp, fixed_weight=0.5, weight_decay=float(np.float32(1e-3)))
        nm.netmax_set_fusion(fused.ctx, True)
        ref = opol.generate_policy(iteration_times("two_tier_10", w.M), float(np.float32(w.lr)), 20, 6)
        it = 0
        for stage in range(3):
            if stage == 1:
                for g in (plain, fused):
                    nm.netmax_set_lr(g.ctx, float(np.float32(w.lr * 0.5)))
            if stage == 2 and ref is not None:
                for g in (plain, fused):
                    nm.netmax_set_policy(g.ctx, ref["P"], float(np.float32(ref["rho"])))
            plain.run(it, 3)
            fused.run(it, 3, use_graph=(stage == 1))
            side.synchronize()
            it += 3
            assert np.array_equal(plain.peers.cpu().numpy(), fused.peers.cpu().numpy())
            assert np.array_equal(plain.get("x").cpu().numpy(), fused.get("x").cpu().numpy()), stage
            assert np.array_equal(plain.get("v").cpu().numpy(), fused.get("v").cpu().numpy()), stage
        plain.close(), fused.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_small_configurations_run_modes(seed):
    """The seeded random shapes of test_gpu_kernels through the other ways of running: netmax_run eagerly and as a
    replayed graph (bit-identical to the separate calls), the flat models' fused variant (bit-identical), then the
    asynchronous schedule from the state reached, against the oracle."""
    import paper_2009_05766_amd as nm
    from test_gpu_kernels import _random_case
    from netmax_inputs import iteration_times
    name, over, bf16 = _random_case(seed)
    w = workload(name, **over)
    inp = inputs_of(w)
    if w.model != "flat":
        inp["labels"] = np.minimum(inp["labels"], w.dims[-1] - 1).astype(np.int32)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        calls, eager, graph = make_gpu(w, inp), make_gpu(w, inp), make_gpu(w, inp)
        o = make_oracle(w, inp, operands_bf16=bf16)
        if w.model == "flat":
            nm.netmax_set_fusion(eager.ctx, True)
        for it in range(3):
            calls.step(it)
            assert np.array_equal(calls.peers.cpu().numpy(), o.step(it))
        eager.run(0, 3)
        graph.run(0, 2, use_graph=True)
        graph.run(2, 1, use_graph=True)
        side.synchronize()
        for other in (eager, graph):
            for what in ("x", "v"):
                assert np.array_equal(calls.get(what).cpu().numpy(), other.get(what).cpu().numpy()), (name, over, what)
        tol = 2e-3 if bf16 else 3e-5
        assert rel_err_rows(calls.get("x").cpu().numpy(), o.X) < tol
        # asynchronous schedule on top: the oracle's state goes to the GPU first, both then take the same global steps
        _sync_gpu_from_oracle(calls, o)
        t = iteration_times("two_tier_10", w.M)
        p_act = nm.netmax_activity(t, inp["P"])
        nm.netmax_set_activity(calls.ctx, p_act)
        o.set_activity(p_act)
        n = 5
        active = torch.zeros(n, dtype=torch.int32, device="cuda")
        peers = torch.zeros(n, dtype=torch.int32, device="cuda")
        nm.netmax_async_run(calls.ctx, 3, n, active, peers)
        side.synchronize()
        want = np.array([o.async_step(3 + k) for k in range(n)], dtype=np.int32)
        assert np.array_equal(active.cpu().numpy(), want[:, 0]) and np.array_equal(peers.cpu().numpy(), want[:, 1])
        assert rel_err_rows(calls.get("x").cpu().numpy(), o.X) < tol
        for g in (calls, eager, graph):
            g.close()


@pytest.mark.parametrize("over,T", [(dict(), 100),                                                  # cfg1 itself, its whole horizon
                                    (dict(M=2, dims=(7, 3), batch=1, n_per_worker=5), 12),
                                    (dict(M=5, dims=(33, 32), batch=37, n_per_worker=90), 12),    # 32 classes, odd widths
                                    (dict(M=64, dims=(256, 10), batch=32, n_per_worker=64), 30),
                                    (dict(M=200, dims=(100, 12), batch=20, n_per_worker=40), 9),
                                    (dict(M=300, dims=(64, 5), batch=8, n_per_worker=16), 6)])    # more workers than compute units
def test_small_model_iterations_in_one_kernel(over, T):
    """Softmax-regression models small enough for a workgroup's LDS run whole iterations inside one kernel: netmax_run
    launches it once for all T iterations (cooperatively, a grid barrier per iteration) where all workers' workgroups
    fit the device, else once per iteration.  Against the individual entry points (peer draw, local step with the same
    gradient code, the mix kernel with the same update function): bit-identical x, v, g, peers, losses; against
    the oracle: bit-exact peers, parameters within the run tolerance."""
    w = workload("cfg1", **over)
    inp = inputs_of(w)
    if over:
        inp["labels"] = np.minimum(inp["labels"], w.dims[-1] - 1).astype(np.int32)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        calls, one, graph, o = make_gpu(w, inp), make_gpu(w, inp), make_gpu(w, inp), make_oracle(w, inp)
        import oracle
        oracle.set_threads(8)
        for it in range(T):
            calls.step(it)
            assert np.array_equal(calls.peers.cpu().numpy(), o.step(it))
        one.run(0, T - 3)                      # one launch
        one.run(T - 3, 1)                      # a single iteration: the same kernel without a barrier
        one.run(T - 2, 2)
        graph.run(0, T, use_graph=True)        # replayed graph of the one-kernel iteration
        side.synchronize()
        for other in (one, graph):
            for what in ("x", "v", "g"):
                assert np.array_equal(calls.get(what).cpu().numpy(), other.get(what).cpu().numpy()), (over, what)
            assert np.array_equal(calls.peers.cpu().numpy(), other.peers.cpu().numpy())
            assert np.array_equal(calls.losses().cpu().numpy(), other.losses().cpu().numpy())
        X = calls.get("x").cpu().numpy()
        assert rel_err_rows(X, o.X) < TOL_RUN
        assert max_abs_err(X, o.X) <= TOL_RUN * np.abs(o.X).max()
        np.testing.assert_allclose(calls.losses().cpu().numpy(), o.loss, rtol=1e-4)
        assert one.consensus_dist() == pytest.approx(o.consensus_dist(), rel=1e-4)   # also reads the barrier's fault flag
        oracle.set_threads(1)
        for g in (calls, one, graph):
            g.close()


@pytest.mark.gpu
def test_barrier_that_gives_up_is_reported():
    """The failure path of the device-wide barrier, forced from the host: with a patience of zero polls every
    workgroup that is not the last to arrive gives up at once, raises the fault flag and goes on, so the launch ends
    by itself; the next consensus distance reports a device error instead of a number.  With the patience restored
    (which clears the flag) a fresh context's run matches the individual entry points again."""
    import paper_2009_05766_amd as nm
    w = workload("cfg1")
    inp = inputs_of(w)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        bad, good, calls = make_gpu(w, inp), make_gpu(w, inp), make_gpu(w, inp)
        nm.netmax_set_barrier_patience(bad.ctx, 0)
        bad.run(0, 40)
        side.synchronize()
        with pytest.raises(nm.NetmaxError) as e:
            bad.consensus_dist()
        assert e.value.code == nm.NETMAX_EDEVICE
        nm.netmax_set_barrier_patience(bad.ctx, 1 << 24)      # clears the flag; the parameters stay what they are
        assert np.isfinite(bad.consensus_dist())
        nm.netmax_set_barrier_patience(good.ctx, 1 << 24)
        good.run(0, 40)
        for it in range(40):
            calls.step(it)
        side.synchronize()
        assert np.array_equal(good.get("x").cpu().numpy(), calls.get("x").cpu().numpy())
        assert good.consensus_dist() == calls.consensus_dist()
        for g in (bad, good, calls):
            g.close()
