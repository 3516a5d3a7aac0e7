"""The seeded input generators: shapes, determinism, and that they carry no method state."""
import numpy as np
import pytest

from netmax_inputs import (workload, policy_for, make_shards, init_params, WORKLOAD_NAMES,
                           f32_to_bf16_bits, bf16_bits_to_f32)


def test_parameter_counts():
    assert workload("cfg1").D == 2570
    assert workload("cfg2").D == 407050
    assert workload("cfg3").D == 11_200_000 and workload("cfg3").ld == 11_200_512
    assert workload("cfg4").D == 20_000_000
    assert workload("cfg5").D == 4_206_602
    for n in WORKLOAD_NAMES:
        w = workload(n)
        assert w.ld % 2048 == 0 and w.ld - 2048 < w.D <= w.ld


@pytest.mark.parametrize("name", WORKLOAD_NAMES)
def test_policies_are_row_stochastic_and_deterministic(name):
    w = workload(name)
    P, rho = policy_for(w)
    P2, rho2 = policy_for(w)
    assert np.array_equal(P, P2) and rho == rho2 and rho > 0
    assert P.shape == (w.M, w.M) and np.all(P >= 0) and np.all(np.diag(P) == 0)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-12)


def test_cfg1_policy_values():
    P, _ = policy_for(workload("cfg1"))
    assert P[0, 1] == pytest.approx(10 / 34) and P[0, 4] == pytest.approx(1 / 34)
    P2, _ = policy_for(workload("cfg2"))
    assert P2[0, 1] == pytest.approx(12 / 48) and P2[0, 4] == pytest.approx(1 / 48)


def test_bf16_round_trip_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.140625, 0.0, 1.0 + 2**-8, 1.0 + 3 * 2**-8], np.float32)
    b = f32_to_bf16_bits(x)
    y = bf16_bits_to_f32(b)
    assert y[0] == 1.0 and y[4] == 0.0
    assert y[5] == 1.0                    # tie rounds to even mantissa
    assert y[6] == 1.0 + 2**-6            # tie rounds up to even
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0**-8)


def test_shards_and_init_small():
    w = workload("cfg5", M=4, n_per_worker=64, dims=(48, 32, 16, 10), batch=8)
    feats, labels, off = make_shards(w)
    assert feats.dtype == np.uint16 and feats.shape == (256, 48) and list(off) == [0, 64, 128, 192, 256]
    f = bf16_bits_to_f32(feats)
    assert f.min() >= 0 and f.max() <= 1 and labels.min() >= 0 and labels.max() < 10
    assert len(np.unique(labels)) > 3
    X = init_params(w)
    assert X.shape == (4, w.ld) and np.all(X[:, w.D:] == 0) and not np.array_equal(X[0], X[1])
    assert np.array_equal(X, init_params(w))
    w1 = workload("cfg1")
    f1, l1, _ = make_shards(w1)
    assert f1.shape == (8 * 1024, 256) and f1.dtype == np.float32 and set(np.unique(l1)) == set(range(10))
