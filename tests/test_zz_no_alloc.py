"""The consensus distance through the entry point that allocates nothing (its partial sums live in a fixed device
array of the library) against the context-based entry point: same kernels, same summation order, so the same
double, on two calls in a row of which the second has the smaller input (the array still holds the first call's
partial sums)."""
import numpy as np
import pytest
import torch

import paper_2009_05766_amd as nm
from netmax_inputs import workload
from harness import inputs_of, make_gpu

pytestmark = pytest.mark.gpu


def _both(w, steps):
    inp = inputs_of(w)
    gpu = make_gpu(w, inp)
    for it in range(steps):
        gpu.step(it)
    want = gpu.consensus_dist()
    cd = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    nm.netmax_consensus_dist_static(w.M, w.D, w.ld, gpu.params(), cd, gpu.stream)
    got = float(cd.cpu()[0])
    import oracle
    ref = oracle.consensus_dist(gpu.get("x").cpu().numpy(), w.D)
    gpu.close()
    return got, want, ref


def test_consensus_dist_static_matches_the_context_entry_point():
    big = workload("cfg3", M=24, D=2048 * 300 + 777)        # 301 tiles: 602 partial sums
    small = workload("cfg4", M=5, D=3000)                    # 2 tiles: 4 partial sums, the rest of the array is stale
    for w in (big, small, big):
        got, want, ref = _both(w, 2)
        assert got == want, (w.M, w.D, got, want)
        assert got == pytest.approx(ref, rel=1e-9)


def test_consensus_dist_static_rejects_what_does_not_fit():
    x = torch.zeros(2 * nm.NETMAX_TILE, dtype=torch.float32, device="cuda")
    cd = torch.zeros(1, dtype=torch.float64, device="cuda")
    too_long = nm.NETMAX_STATIC_MAX_LD + nm.NETMAX_TILE
    for args in ((2, too_long, too_long), (1, 100, nm.NETMAX_TILE), (2, 100, 100), (2, nm.NETMAX_TILE + 1, nm.NETMAX_TILE)):
        with pytest.raises(nm.NetmaxError) as e:
            nm.netmax_consensus_dist_static(args[0], args[1], args[2], x, cd)
        assert e.value.code == nm.NETMAX_EINVAL
    assert "NETMAX_STATIC_MAX_LD" in str(pytest.raises(nm.NetmaxError, nm.netmax_consensus_dist_static, 2, too_long, too_long, x, cd).value)
    # the largest admissible problem is accepted as far as the argument checks go (not launched here: it would
    # need 2 x 256 MB of input); a small one right after an error still works
    nm.netmax_consensus_dist_static(2, nm.NETMAX_TILE, nm.NETMAX_TILE, x, cd)
    torch.cuda.synchronize()
    assert float(cd.cpu()[0]) == 0.0
