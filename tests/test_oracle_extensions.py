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


# ------------------------------------------------------------ score variants ----
def test_default_variant_is_algorithm_2():
    rounds = _rounds(5, 4, 1500, 30)
    a, b = oracle.Oracle(4, 1500, 30, 1.0), oracle.Oracle(4, 1500, 30, 1.0)
    b.set_score_variant(0, 0)
    ga = gb = None
    for g in rounds:
        ia, va, ga = a.step(g, ga)
        ib, vb, gb = b.step(g, gb)
        assert np.array_equal(ia, ib) and np.array_equal(va, vb) and np.array_equal(ga, gb)
    with pytest.raises(ValueError):
        b.set_score_variant(4, 0)
    with pytest.raises(ValueError):
        b.set_score_variant(0, 3)


def test_prior_is_the_correctly_rounded_root():
    # |a|^(1/2): the binary32 nearest to the exact root; |a|^(1/4), |a|^(1/8): that step repeated
    mpmath.mp.prec = 200
    rng = np.random.default_rng(21)
    xs = np.concatenate([np.abs(rng.standard_normal(300)) * 10.0 ** rng.uniform(-30, 30, 300),
                         [0.0, 1.0, 4.0, 2.0, 1e-45, 3.4e38]]).astype(f32)
    for x in xs:
        p = f32(oracle.prior(-x, 1))
        assert p == f32(oracle.prior(x, 1))                               # magnitude only
        exact = mpmath.sqrt(mpmath.mpf(float(x)))
        lo, hi = np.nextafter(p, f32(-np.inf)), np.nextafter(p, f32(np.inf))
        assert abs(mpmath.mpf(float(p)) - exact) <= abs(mpmath.mpf(float(lo)) - exact)
        assert abs(mpmath.mpf(float(p)) - exact) <= abs(mpmath.mpf(float(hi)) - exact)
        assert oracle.prior(x, 2) == oracle.prior(oracle.prior(x, 1), 1)
        assert oracle.prior(x, 3) == oracle.prior(oracle.prior(x, 2), 1)
        assert oracle.prior(x, 0) == float(x)
    assert oracle.prior(16.0, 1) == 4.0 and oracle.prior(16.0, 2) == 2.0 and oracle.prior(256.0, 3) == 2.0


def test_exponent_does_not_change_plain_topk():
    # Remark on sub-linear scaling: without the regulariser the exponent does not affect the sorting.
    rounds = _rounds(5, 3, 2500, 50)
    ref = oracle.Oracle(3, 2500, 50, 0.0)
    others = []
    for m in (1, 2, 3):
        o = oracle.Oracle(3, 2500, 50, 0.0)
        o.set_score_variant(m, 0)
        others.append(o)
    for g in rounds:
        i0, v0, a0 = ref.step(g, None)
        for o in others:
            i, v, a = o.step(g, None)
            assert np.array_equal(i, i0) and np.array_equal(v, v0) and np.array_equal(a, a0)


def test_exponent_scores_and_selection_invariant():
    N, d, k = 3, 3000, 60
    for m in (1, 2):
        o = oracle.Oracle(N, d, k, 1.0)
        o.set_score_variant(m, 0)
        agg = None
        for t, g in enumerate(_rounds(4, N, d, k)):
            prev_mask = o.mask if t else np.zeros((N, d), dtype=np.uint8)
            idx, val, agg = o.step(g, agg)
            sc, a, msk = o.score, o.a, o.mask
            root = np.abs(a)
            for _ in range(m):
                root = np.sqrt(root)                                  # numpy's binary32 sqrt is correctly rounded too
            assert sc.dtype == np.float32 and np.all(sc <= root)
            assert np.array_equal(sc[prev_mask == 0], root[prev_mask == 0])   # factor exactly 1 off the previous mask
            if t:
                assert np.any(sc[prev_mask == 1] < root[prev_mask == 1])
            for n in range(N):
                assert msk[n].sum() == k
                assert sc[n][msk[n] == 1].min() >= sc[n][msk[n] == 0].max()


def test_exponent_half_commutes_with_scaling_by_four():
    # sqrt(4^p x) = 2^p sqrt(x) exactly, so scaling every gradient (and the fed-back
    # aggregate) by a power of 4 leaves the masks of the y = 1/2 variant unchanged.
    N, d, k = 3, 2000, 40
    rounds = _rounds(4, N, d, k)
    base, scaled = oracle.Oracle(N, d, k, 0.8), oracle.Oracle(N, d, k, 0.8)
    base.set_score_variant(1, 0)
    scaled.set_score_variant(1, 0)
    ga = gb = None
    for g in rounds:
        ia, va, ga = base.step(g, ga)
        ib, vb, gb = scaled.step(g * f32(16.0), gb)
        assert np.array_equal(ia, ib)
        assert np.array_equal(va * f32(16.0), vb) and np.array_equal(ga * f32(16.0), gb)


def test_general_exponent_prior_is_the_correctly_rounded_power():
    # |a|^y for a general binary32 y in (0, 1): nearest binary32 to the exact power (200-bit reference);
    # for y = 1/2 it is the correctly rounded square root, i.e. the m = 1 variant, by another route
    mpmath.mp.prec = 200
    rng = np.random.default_rng(51)
    for y in (0.9, 0.75, 0.5, f32(1.0) / f32(3.0), 0.1, 0.999, 1e-3):
        y = f32(y)
        xs = np.concatenate([np.abs(rng.standard_normal(400)), 10.0 ** rng.uniform(-44.9, 38.5, 400)]).astype(f32)
        got = oracle.prior_pow_array(xs, y)
        for x, p in zip(xs, got):
            exact = mpmath.mpf(float(x)) ** mpmath.mpf(float(y))
            lo, hi = np.nextafter(p, f32(0)), np.nextafter(p, f32(np.inf))
            assert abs(mpmath.mpf(float(p)) - exact) <= abs(mpmath.mpf(float(lo)) - exact), (x, y)
            assert abs(mpmath.mpf(float(p)) - exact) <= abs(mpmath.mpf(float(hi)) - exact), (x, y)
    xs = np.concatenate([np.abs(rng.standard_normal(3000)), 10.0 ** rng.uniform(-44.9, 38.5, 3000)]).astype(f32)
    assert np.array_equal(oracle.prior_pow_array(xs, 0.5), np.array([oracle.prior(x, 1) for x in xs], dtype=f32))
    assert oracle.prior_pow(0.0, 0.3) == 0.0 and oracle.prior_pow(1.0, 0.3) == 1.0 and oracle.prior_pow(-8.0, f32(1.0) / f32(3.0)) == 2.0


def test_general_exponent_rounds():
    N, d, k, mu, y = 4, 3000, 60, 1.5, f32(0.7)
    rounds = _rounds(5, N, d, k)
    o = oracle.Oracle(N, d, k, mu)
    o.set_prior_exponent(y)
    agg = None
    for t, g in enumerate(rounds):
        prev_mask = o.mask if t else np.zeros((N, d), dtype=np.uint8)
        a_prev, agg_prev = o.a, agg
        idx, val, agg = o.step(g, agg)
        sc, a, msk, e = o.score, o.a, o.mask, o.e
        pr = oracle.prior_pow_array(a.ravel(), y).reshape(N, d)
        assert np.array_equal(sc[prev_mask == 0], pr[prev_mask == 0]) and np.all(sc <= pr)
        for n in range(N):
            assert msk[n].sum() == k and sc[n][msk[n] == 1].min() >= sc[n][msk[n] == 0].max()
            assert np.array_equal(a[n][idx[n]], val[n]) and np.all(e[n][idx[n]] == 0)
            for j in np.flatnonzero(prev_mask[n])[:5]:
                fct = oracle.likelihood_sent_kind(a[n, j], a_prev[n, j], agg_prev[j], f32(1.0) / f32(N), mu, 0)
                assert sc[n, j] == pr[n, j] * f32(fct)
    # with the regulariser off the exponent does not change what is selected (the remark's statement;
    # continuous data, no ties), y = 1 is Algorithm 2, and the argument is checked
    p0, p1, p2 = oracle.Oracle(N, d, k, 0.0), oracle.Oracle(N, d, k, 0.0), oracle.Oracle(N, d, k, mu)
    p1.set_prior_exponent(y)
    p2.set_prior_exponent(0.3)
    p2.set_prior_exponent(1.0)
    ref = oracle.Oracle(N, d, k, mu)
    g2 = gr = None
    for g in rounds:
        i0, v0, _ = p0.step(g, None)
        i1, v1, _ = p1.step(g, None)
        assert np.array_equal(i0, i1) and np.array_equal(v0, v1)
        i2, v2, g2 = p2.step(g, g2)
        ir, vr, gr = ref.step(g, gr)
        assert np.array_equal(i2, ir) and np.array_equal(g2, gr)
    for bad in (0.0, -0.5, 1.5, float("nan")):
        with pytest.raises(ValueError):
            o.set_prior_exponent(bad)


def test_clipped_linear_likelihood():
    # cumulative function of a uniform innovation: min(|1 + Delta| / mu, 1)
    mpmath.mp.prec = 200
    rng = np.random.default_rng(31)
    for _ in range(300):
        a_now, a_bef, g_bef = (f32(x) for x in rng.standard_normal(3))
        w, mu = f32(rng.uniform(0.02, 1.0)), f32(rng.uniform(0.05, 5.0))
        got = oracle.likelihood_sent_kind(a_now, a_bef, g_bef, w, mu, 1)
        m = mpmath.mpf
        den = m(float(w)) * m(float(a_now))
        num = m(float(g_bef)) - m(float(w)) * m(float(a_bef))
        x = abs(1 + num / den) / m(float(mu))
        want = min(x, m(1))
        # five roundings, conditioned by 1/|den| through the sum 1 + Delta
        cond = (abs(num / den) + 1) / max(abs(1 + num / den), m(2) ** -60)
        tol = float(want) * 2.0 ** -23 * (3 + 3 * float(cond)) + 1e-30
        assert abs(got - float(want)) <= tol, (a_now, a_bef, g_bef, w, mu, got, float(want))
        assert 0.0 <= got <= 1.0
    # closed cases: cancelled entry, sole sender, saturation, monotone in |1 + Delta|
    assert oracle.likelihood_sent_kind(2.0, 2.0, 0.0, 0.5, 1.0, 1) == 0.0
    assert oracle.likelihood_sent_kind(2.0, 2.0, 1.0, 0.5, 4.0, 1) == 0.25
    assert oracle.likelihood_sent_kind(2.0, 2.0, 1.0, 0.5, 0.5, 1) == 1.0
    assert oracle.likelihood_sent_kind(0.0, 2.0, 1.0, 0.5, 1.0, 1) == 1.0      # zero denominator: no information
    vals = [oracle.likelihood_sent_kind(1.0, 1.0, g, 1.0, 2.0, 1) for g in np.linspace(0.0, 3.0, 40)]
    assert all(b >= a for a, b in zip(vals, vals[1:])) and vals[0] == 0.0 and vals[-1] == 1.0
    # and the same kind argument with 0 is the tanh likelihood
    assert oracle.likelihood_sent_kind(1.3, 0.7, 0.2, 0.25, 0.9, 0) == oracle.likelihood_sent(1.3, 0.7, 0.2, 0.25, 0.9)


def test_clipped_linear_rounds_keep_the_invariants():
    N, d, k = 4, 3000, 60
    o = oracle.Oracle(N, d, k, 2.0)
    o.set_score_variant(0, 1)
    agg = None
    damped = 0
    for t, g in enumerate(_rounds(5, N, d, k)):
        prev_mask = o.mask if t else np.zeros((N, d), dtype=np.uint8)
        idx, val, agg = o.step(g, agg)
        sc, a, msk, e = o.score, o.a, o.mask, o.e
        assert np.all(sc <= np.abs(a)) and np.array_equal(sc[prev_mask == 0], np.abs(a)[prev_mask == 0])
        damped += int((sc[prev_mask == 1] < np.abs(a)[prev_mask == 1]).sum())
        for n in range(N):
            assert msk[n].sum() == k and sc[n][msk[n] == 1].min() >= sc[n][msk[n] == 0].max()
            assert np.array_equal(a[n][idx[n]], val[n]) and np.all(e[n][idx[n]] == 0)
    assert damped > 0


def test_erf_is_correctly_rounded_on_samples_and_specials():
    # the erf step of the Gaussian likelihood: nearest binary32 to the exact erf (200-bit reference)
    mpmath.mp.prec = 200
    rng = np.random.default_rng(41)
    xs = np.concatenate([rng.uniform(0, 4.2, 3000), 10.0 ** rng.uniform(-44, 0.6, 3000)]).astype(f32)
    got = oracle.erf32_array(xs)
    for x, y in zip(xs, got):
        exact = mpmath.erf(mpmath.mpf(float(x)))
        lo, hi = np.nextafter(y, f32(-1)), np.nextafter(y, f32(2))
        assert abs(mpmath.mpf(float(y)) - exact) <= abs(mpmath.mpf(float(lo)) - exact), x
        assert abs(mpmath.mpf(float(y)) - exact) <= abs(mpmath.mpf(float(hi)) - exact), x
    assert oracle.erf32(0.0) == 0.0 and oracle.erf32(3.9192) < 1.0 and oracle.erf32(3.92) == 1.0
    assert oracle.erf32(100.0) == 1.0 and oracle.erf32(float("inf")) == 1.0
    assert oracle.erf32(1e-45) == float(f32(1e-45))          # 2/sqrt(pi) * the smallest denormal rounds to it


def test_gaussian_likelihood():
    # cumulative function of a Gaussian innovation, constants dropped: erf(|1 + Delta| / mu)
    mpmath.mp.prec = 200
    rng = np.random.default_rng(43)
    for _ in range(300):
        a_now, a_bef, g_bef = (f32(x) for x in rng.standard_normal(3))
        w, mu = f32(rng.uniform(0.02, 1.0)), f32(rng.uniform(0.05, 5.0))
        got = oracle.likelihood_sent_kind(a_now, a_bef, g_bef, w, mu, 2)
        m = mpmath.mpf
        den = m(float(w)) * m(float(a_now))
        num = m(float(g_bef)) - m(float(w)) * m(float(a_bef))
        x = abs(1 + num / den) / m(float(mu))
        want = mpmath.erf(x)
        # five roundings of the argument, conditioned by 1/|den| through the sum 1 + Delta; erf'(x) x <= erf(x)
        cond = (abs(num / den) + 1) / max(abs(1 + num / den), m(2) ** -60)
        tol = float(want) * 2.0 ** -23 * (3 + 3 * float(cond)) + 1e-30
        assert abs(got - float(want)) <= tol, (a_now, a_bef, g_bef, w, mu, got, float(want))
        assert 0.0 <= got <= 1.0
    assert oracle.likelihood_sent_kind(2.0, 2.0, 0.0, 0.5, 1.0, 2) == 0.0                       # cancelled entry
    assert oracle.likelihood_sent_kind(2.0, 2.0, 1.0, 0.5, 4.0, 2) == oracle.erf32(0.25)        # sole sender: Delta = 0
    assert oracle.likelihood_sent_kind(2.0, 2.0, 1.0, 0.5, 0.125, 2) == 1.0                     # saturation
    assert oracle.likelihood_sent_kind(0.0, 2.0, 1.0, 0.5, 1.0, 2) == 1.0                       # zero denominator
    vals = [oracle.likelihood_sent_kind(1.0, 1.0, g, 1.0, 2.0, 2) for g in np.linspace(0.0, 9.0, 60)]
    assert all(b >= a for a, b in zip(vals, vals[1:])) and vals[0] == 0.0 and vals[-1] == 1.0
    # it is neither of the other two
    assert oracle.likelihood_sent_kind(1.3, 0.7, 0.2, 0.25, 0.9, 2) not in (
        oracle.likelihood_sent_kind(1.3, 0.7, 0.2, 0.25, 0.9, 0), oracle.likelihood_sent_kind(1.3, 0.7, 0.2, 0.25, 0.9, 1))


def test_gaussian_likelihood_rounds_keep_the_invariants_and_use_erf():
    N, d, k, mu = 4, 3000, 60, 2.0
    o = oracle.Oracle(N, d, k, mu)
    o.set_score_variant(0, 2)
    agg = None
    checked = 0
    for t, g in enumerate(_rounds(5, N, d, k)):
        prev_mask = o.mask if t else np.zeros((N, d), dtype=np.uint8)
        a_prev = o.a
        agg_prev = agg
        idx, val, agg = o.step(g, agg)
        sc, a, msk, e = o.score, o.a, o.mask, o.e
        assert np.all(sc <= np.abs(a)) and np.array_equal(sc[prev_mask == 0], np.abs(a)[prev_mask == 0])
        for n in range(N):
            assert msk[n].sum() == k and sc[n][msk[n] == 1].min() >= sc[n][msk[n] == 0].max()
            assert np.array_equal(a[n][idx[n]], val[n]) and np.all(e[n][idx[n]] == 0)
            for j in np.flatnonzero(prev_mask[n])[:5]:         # the round's score is |a| times the step's factor
                fct = oracle.likelihood_sent_kind(a[n, j], a_prev[n, j], agg_prev[j], f32(1.0) / f32(N), mu, 2)
                assert sc[n, j] == f32(abs(a[n, j])) * f32(fct)
                checked += 1
    assert checked > 0


# ------------------------------------------------------------ global Top-k ----
def test_global_topk_selects_the_largest_entries_of_the_unsparsified_aggregate():
    # "Statistical Global Top-k": the genie-aided workers apply Top-k to the aggregated accumulated
    # gradient.  Brute force in binary64 on data whose magnitudes are far apart compared to rounding.
    N, d, k = 5, 3000, 75
    w = np.array([0.3, 0.1, 0.2, 0.25, 0.15], dtype=f32)
    o = oracle.Oracle(N, d, k, 1.0)
    o.set_weights(w)
    e = np.zeros((N, d))
    for g in _rounds(5, N, d, k):
        idx, val, agg = o.step_global(g)
        a = e + g.astype(np.float64)
        abar = (w.astype(np.float64)[:, None] * a).sum(axis=0)
        order = np.lexsort((np.arange(d), -np.abs(abar)))
        gap = np.abs(abar)[order[k - 1]] - np.abs(abar)[order[k]]
        assert gap > 1e-5                                              # no near-tie at the threshold in this data
        want = np.sort(order[:k])
        for n in range(N):
            assert np.array_equal(idx[n], want)                        # one mask for all workers
            np.testing.assert_allclose(val[n], a[n, want], rtol=1e-5, atol=1e-6)
        ref = np.zeros(d)
        ref[want] = abar[want]
        np.testing.assert_allclose(agg, ref, rtol=1e-5, atol=1e-6)
        assert np.all(agg[np.setdiff1d(np.arange(d), want)] == 0)
        e = a.copy()
        e[:, want] = 0.0
        np.testing.assert_allclose(o.e, e, rtol=1e-5, atol=1e-6)
        assert list(o.mask_overlap()) == [d - k] + [0] * (N - 1) + [k]


def test_global_topk_exact_conservation_and_special_cases():
    N, d, k = 3, 1000, 40
    rounds = _rounds(3, N, d, k)
    o = oracle.Oracle(N, d, k, 0.0)
    for g in rounds:
        e_old = o.e
        idx, val, agg = o.step_global(g)
        a, e, m = o.a, o.e, o.mask
        assert np.array_equal(a, e_old + g)                            # single rounded add
        assert np.array_equal(np.where(m == 1, f32(0), a), e)          # eps = a off the mask, +0 on it
        for n in range(N):
            assert np.array_equal(a[n][idx[n]], val[n])
    # identical workers: the aggregate is each worker's own vector, so global Top-k is their Top-k
    g = np.tile(np.random.default_rng(4).standard_normal(500).astype(f32), (4, 1))
    a_, b_ = oracle.Oracle(4, 500, 25, 0.0), oracle.Oracle(4, 500, 25, 0.0)
    i1, v1, g1 = a_.step_global(g)
    i2, v2, g2 = b_.step(g, None)
    assert np.array_equal(i1, i2) and np.array_equal(v1, v2) and np.array_equal(g1, g2)
    # k = d: nothing is dropped
    o = oracle.Oracle(3, 200, 200, 1.0)
    gg = _rounds(1, 3, 200, 200)[0]
    _, _, agg = o.step_global(gg)
    np.testing.assert_allclose(agg, gg.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
    assert np.all(o.e == 0)
    # cancelling workers (the toy example's situation): the genie sees the cancellation at once
    g = np.array([[100.0, 1.0, 0.5], [-100.0, 1.0, 0.25]], dtype=f32)
    o = oracle.Oracle(2, 3, 1, 1.0)
    idx, val, agg = o.step_global(g)
    assert idx.ravel().tolist() == [1, 1] and agg.tolist() == [0.0, 1.0, 0.0]


def test_global_and_local_rounds_share_their_state():
    # a local RegTop-k round after a global one regularises with the global mask as previous mask
    N, d, k = 3, 1500, 30
    rounds = _rounds(4, N, d, k)
    o = oracle.Oracle(N, d, k, 1.0)
    _, _, agg = o.step_global(rounds[0])
    prev = o.mask
    idx, val, agg = o.step(rounds[1], agg)
    sc, a = o.score, o.a
    assert np.array_equal(sc[prev == 0], np.abs(a)[prev == 0])
    assert np.any(sc[prev == 1] < np.abs(a)[prev == 1])
    assert o.round == 2


# ------------------------------------------------------------- per-worker k ----
def _numpy_topk_sets(score, k):
    """Indices of the k largest scores, lower index first among equals, ascending (full sort)."""
    order = np.lexsort((np.arange(score.size), -score.astype(np.float64)))
    return np.sort(order[:k])


def test_equal_worker_k_is_the_scalar_k():
    rounds = _rounds(5, 4, 1500, 30)
    a, b = oracle.Oracle(4, 1500, 30, 1.0), oracle.Oracle(4, 1500, 30, 1.0)
    b.set_worker_k([30, 30, 30, 30])
    ga = gb = None
    for g in rounds:
        ia, va, ga = a.step(g, ga)
        ib, vb, gb = b.step(g, gb)
        assert np.array_equal(ia, ib) and np.array_equal(va, vb) and np.array_equal(ga, gb)
        assert np.array_equal(a.e, b.e)


def test_worker_k_without_regulariser_is_algorithm1_with_each_workers_own_k():
    # mu = 0: every worker runs Algorithm 1 on its own, with its own k_n -- rebuilt here with a full
    # sort; the unused rest of each output row is (-1, 0); the aggregate is the weighted sum of the lists.
    N, d, k = 4, 700, 50
    kn = [1, 17, 50, 33]
    o = oracle.Oracle(N, d, k, 0.0)
    o.set_worker_k(kn)
    e = np.zeros((N, d), dtype=f32)
    for g in _rounds(6, N, d, k):
        idx, val, agg = o.step(g, None)
        a = e + g
        ref = np.zeros(d, dtype=f32)
        for n in range(N):
            want = _numpy_topk_sets(np.abs(a[n]), kn[n])
            assert np.array_equal(idx[n, :kn[n]], want)
            assert np.array_equal(val[n, :kn[n]], a[n, want])
            assert np.all(idx[n, kn[n]:] == -1) and np.all(val[n, kn[n]:] == 0)
            e[n] = a[n]
            e[n, want] = 0
            ref[want] = ref[want] + f32(1.0) / f32(N) * a[n, want]
        assert np.array_equal(o.e, e)
        assert np.array_equal(agg, ref)


def test_worker_k_with_regulariser_selects_k_n_largest_scores_and_conserves():
    N, d, k = 5, 900, 90
    kn = [90, 1, 45, 10, 89]
    o = oracle.Oracle(N, d, k, 0.9)
    o.set_worker_k(kn)
    agg = None
    for g in _rounds(6, N, d, k):
        e_before = o.e
        idx, val, agg = o.step(g, agg)
        sc, a, mask = o.score, o.a, o.mask
        assert np.array_equal(a, e_before + g)
        for n in range(N):
            want = _numpy_topk_sets(sc[n], kn[n])           # brute force on the oracle's scores
            assert np.array_equal(idx[n, :kn[n]], want)
            assert int(mask[n].sum()) == kn[n]
            sent = np.zeros(d, dtype=f32)
            sent[want] = val[n, :kn[n]]
            assert np.array_equal((sent + o.e[n]).view(np.uint32), a[n].view(np.uint32))   # a = ghat + eps
    assert np.array_equal(o.mask_overlap(), np.bincount(o.mask.sum(0), minlength=N + 1))


def test_a_worker_that_keeps_everything_has_no_error_and_k_n_is_checked():
    N, d, k = 3, 120, 120
    o = oracle.Oracle(N, d, k, 1.0)
    o.set_worker_k([120, 5, 60])
    agg = None
    for g in _rounds(4, N, d, k):
        idx, val, agg = o.step(g, agg)
        assert np.array_equal(idx[0], np.arange(d)) and np.array_equal(val[0], g[0])   # eps_0 stays 0
        assert not o.e[0].any()
    for bad in ([0, 5, 5], [121, 5, 5], [5, 5]):
        with pytest.raises(ValueError):
            o.set_worker_k(bad)
