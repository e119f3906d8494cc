"""Pins for the oracle's general aggregation weights, the mask-overlap count and
the SGD model update (CPU only).  None of the expected values below comes from
the oracle itself: they are closed forms, brute force over the index lists, or
high-precision arithmetic."""
from __future__ import annotations

import mpmath
import numpy as np
import pytest

from oracle import oracle
from paper_2501_05633_amd import workloads

f32 = np.float32


def _rounds(T, N, d, k, seed=None):
    cfg = workloads.scaled(workloads.CONFIGS["tiny"], d=d, N=N, k=k)
    wl = workloads.Workload(cfg, "cpu", seed=seed)
    return [wl.grads(t).numpy() for t in range(T)]


# ------------------------------------------------------------------ weights ----
def test_explicit_uniform_weights_change_nothing():
    rounds = _rounds(5, 4, 1500, 30)
    a, b = oracle.Oracle(4, 1500, 30, 1.0), oracle.Oracle(4, 1500, 30, 1.0)
    b.set_weights(np.full(4, f32(1.0) / f32(4.0), dtype=f32))
    ga = gb = None
    for g in rounds:
        ia, va, ga = a.step(g, ga)
        ib, vb, gb = b.step(g, gb)
        assert np.array_equal(ia, ib) and np.array_equal(va, vb) and np.array_equal(ga, gb)


def test_weighted_aggregate_is_the_weighted_sum_of_the_sent_lists():
    # g = sum_n omega_n ghat_n, rebuilt from the (index, value) lists in ascending worker order.
    N, d, k = 5, 3000, 60
    w = np.array([0.05, 0.4, 0.25, 0.2, 0.1], dtype=f32)
    o = oracle.Oracle(N, d, k, 0.7)
    o.set_weights(w)
    agg = None
    for g in _rounds(4, N, d, k):
        idx, val, agg = o.step(g, agg)
        ref32 = np.zeros(d, dtype=f32)
        ref64 = np.zeros(d)
        for n in range(N):
            ref32[idx[n]] = ref32[idx[n]] + w[n] * val[n]           # binary32, product rounded first
            ref64[idx[n]] += float(w[n]) * val[n].astype(np.float64)
        assert np.array_equal(agg, ref32)
        np.testing.assert_allclose(agg, ref64, rtol=2e-6, atol=1e-9)


def test_sole_sender_sees_no_distortion_under_any_weights():
    # If worker n alone sent entry j, the aggregate there is omega_n * a_n, so the
    # posterior distortion is 0 and the factor is tanh(1/mu) whatever omega_n is
    # -- provided the distortion uses the SAME omega_n as the aggregation.
    N, d, k, mu = 3, 64, 4, 0.8
    w = np.array([0.5, 0.3, 0.2], dtype=f32)
    # a power-of-two weight keeps w*a exact; for the others allow 1 ulp in |1+Delta|
    g0 = np.zeros((N, d), dtype=f32)
    for n in range(N):
        g0[n, 8 * n:8 * n + 4] = [9.0, -8.0, 7.0, -6.0]             # disjoint supports: sole senders
        g0[n, 40:60] = 1e-3 * (n + 1)
    o = oracle.Oracle(N, d, k, mu)
    o.set_weights(w)
    idx, val, agg = o.step(g0, None)
    for n in range(N):
        assert list(idx[n]) == list(range(8 * n, 8 * n + 4))
    g1 = np.zeros((N, d), dtype=f32)
    for n in range(N):
        g1[n, 8 * n:8 * n + 4] = [9.0, -8.0, 7.0, -6.0]             # same values again: a^t = a^{t-1} there
    o.step(g1, agg)
    t = oracle.tanh32(f32(1.0) / f32(mu))
    sc = o.score
    for n in range(N):
        for q, v in enumerate([9.0, 8.0, 7.0, 6.0]):
            got = sc[n, 8 * n + q]
            want = f32(v) * f32(t)
            assert abs(float(got) - float(want)) <= 4 * np.spacing(want), (n, q, got, want)
    # and a swapped pair of weights in the distortion would not give this: worker 0 with omega_1
    wrong = oracle.likelihood_sent(9.0, 9.0, float(w[0] * f32(9.0)), float(w[1]), mu)
    assert abs(wrong - t) > 1e-2


def test_zero_weight_worker_does_not_reach_the_aggregate():
    N, d, k = 3, 500, 25
    rounds = _rounds(3, N, d, k)
    o = oracle.Oracle(N, d, k, 0.0)
    o.set_weights(np.array([0.5, 0.0, 0.5], dtype=f32))
    o2 = oracle.Oracle(2, d, k, 0.0)                                 # the two other workers alone, omega = 1/2
    agg = agg2 = None
    for g in rounds:
        _, _, agg = o.step(g, agg)
        _, _, agg2 = o2.step(g[[0, 2]], agg2)
        assert np.array_equal(agg, agg2)


# ------------------------------------------------------------------ overlap ----
def test_mask_overlap_counts_against_the_index_lists():
    N, d, k = 6, 4000, 200
    o = oracle.Oracle(N, d, k, 1.0)
    agg = None
    for g in _rounds(4, N, d, k):
        idx, _, agg = o.step(g, agg)
        per_entry = np.bincount(idx.ravel(), minlength=d)            # how many workers chose j
        want = np.bincount(per_entry, minlength=N + 1)
        got = o.mask_overlap()
        assert got.dtype == np.int64 and got.shape == (N + 1,)
        assert np.array_equal(got, want)
        assert got.sum() == d and int((np.arange(N + 1) * got).sum()) == N * k


def test_mask_overlap_closed_cases():
    # identical workers agree on everything; k = d selects everything
    g = np.tile(np.random.default_rng(3).standard_normal(300).astype(f32), (4, 1))
    o = oracle.Oracle(4, 300, 30, 1.0)
    assert list(o.mask_overlap()) == [300, 0, 0, 0, 0]               # before any round: nothing selected
    o.step(g, None)
    assert list(o.mask_overlap()) == [270, 0, 0, 0, 30]
    o = oracle.Oracle(4, 300, 300, 1.0)
    o.step(g, None)
    assert list(o.mask_overlap()) == [0, 0, 0, 0, 300]
    # disjoint supports: every selected entry has exactly one owner
    g = np.zeros((3, 90), dtype=f32)
    for n in range(3):
        g[n, 30 * n:30 * n + 10] = 1.0 + np.arange(10)
    o = oracle.Oracle(3, 90, 10, 0.0)
    o.step(g, None)
    assert list(o.mask_overlap()) == [60, 30, 0, 0]


# --------------------------------------------------------------- SGD update ----
def test_sgd_update_matches_high_precision_arithmetic():
    rng = np.random.default_rng(11)
    theta = rng.standard_normal(2000).astype(f32)
    g = (rng.standard_normal(2000) * 10.0 ** rng.uniform(-4, 2, 2000)).astype(f32)
    eta = f32(1e-2)
    got = oracle.sgd_update(theta, g, eta)
    mpmath.mp.prec = 200
    for j in range(0, 2000, 7):
        exact = mpmath.mpf(float(theta[j])) - mpmath.mpf(float(eta)) * mpmath.mpf(float(g[j]))
        # two roundings: half an ulp of the product plus half an ulp of the result
        tol = 0.5 * float(np.spacing(np.abs(f32(eta) * g[j]))) + 0.5 * float(np.spacing(np.abs(got[j]))) + 1e-45
        assert abs(float(got[j]) - float(exact)) <= tol * 1.0000001, j


def test_sgd_update_exact_cases_and_rounding_order():
    th = np.array([1.0, -2.0, 0.5, 0.0], dtype=f32)
    g = np.array([2.0, 4.0, -1.0, 0.0], dtype=f32)
    assert np.array_equal(oracle.sgd_update(th, g, 0.25), np.array([0.5, -3.0, 0.75, 0.0], dtype=f32))
    assert np.array_equal(oracle.sgd_update(th, g, 0.0), th)
    # product rounded on its own (no fused multiply-add): eta*g = (1+2^-12)^2 rounds to
    # 1 + 2^-11, so theta - eta*g is exactly 0, whereas a fused update would give -2^-24
    x = f32(1.0 + 2.0 ** -12)
    out = oracle.sgd_update(np.array([1.0 + 2.0 ** -11], dtype=f32), np.array([x], dtype=f32), x)
    assert out[0] == f32(0.0)
    with pytest.raises(ValueError):
        oracle.sgd_update(np.zeros(3, dtype=f32), np.zeros(4, dtype=f32), 0.1)
