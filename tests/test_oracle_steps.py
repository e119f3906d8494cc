"""Pins for the single steps of the CPU oracle: tanh, the likelihood of a
previously sent entry (posterior distortion + tanh), and the Top_k selector.

Each check compares the oracle with something it does not compute itself:
arbitrary-precision arithmetic (mpmath), closed forms stated in the paper, or
brute force with a library sort.
"""
import numpy as np
import pytest
import mpmath as mp

from oracle import oracle

f32 = np.float32


def _round_f32(v) -> np.float32:
    """Round an mpmath real to the nearest binary32 (ties to even) exactly."""
    v = mp.mpf(v)
    if v == 0:
        return f32(0.0)
    m, e = mp.frexp(v)                      # v = m * 2**e, 0.5 <= |m| < 1
    e = int(e)
    emin = -149
    q = max(e - 24, emin)                   # exponent of one unit in the last place
    scaled = v / mp.mpf(2) ** q
    n = int(mp.nint(scaled))                # mp.nint rounds half to even
    return f32(float(mp.mpf(n) * mp.mpf(2) ** q))


# ---------------------------------------------------------------- tanh ----

def test_tanh_is_correctly_rounded_on_samples():
    mp.mp.prec = 200
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.uniform(0, 10, 3000), 10.0 ** rng.uniform(-40, 1, 3000),
        [0.0, 1e-45, 1.1754944e-38, 2.0 ** -12, 0.5, 1.0, 9.0, 9.0109, 9.02, 20.0, 1e30],
    ]).astype(np.float32)
    got = oracle.tanh32_array(xs)
    for x, y in zip(xs, got):
        want = _round_f32(mp.tanh(mp.mpf(float(x))))
        assert y == want, (x, y, want)


def test_tanh_special_values():
    assert oracle.tanh32(0.0) == 0.0
    assert oracle.tanh32(float("inf")) == 1.0
    assert oracle.tanh32(9.02) == 1.0
    assert oracle.tanh32(1e-30) == float(f32(1e-30))
    xs = np.linspace(0, 12, 20001, dtype=np.float32)
    ys = oracle.tanh32_array(xs)
    assert np.all(np.diff(ys) >= 0) and ys.max() == 1.0 and ys.min() == 0.0


# ---------------------------------------------------- likelihood factor ----

def test_cancelled_entry_is_damped_to_zero():
    # Limiting case (2) of the section "RegTop-k Algorithm": the entry cancelled
    # in the aggregate (g^{t-1} = 0) and a^t = a^{t-1} give Delta = -1, factor 0.
    rng = np.random.default_rng(2)
    for _ in range(200):
        a = f32(rng.standard_normal() * 10 ** rng.uniform(-6, 6))
        if a == 0:
            continue
        for N in (1, 2, 3, 8, 20):
            w = f32(1.0) / f32(N)
            for mu in (0.1, 1.0, 10.0):
                assert oracle.likelihood_sent(a, a, 0.0, w, mu) == 0.0


def test_sole_sender_has_zero_distortion():
    # If only worker n sent entry j, g^{t-1} = w a^{t-1}: Delta = 0 and the
    # factor is tanh(1/mu) whatever a^t is.
    for N in (1, 2, 4, 16):
        w = f32(1.0) / f32(N)
        for mu in (0.1, 0.5, 1.0, 4.0, 10.0):
            ap = f32(3.25)
            gprev = f32(w * ap)
            want = oracle.tanh32(float(f32(1.0) / f32(mu)))
            for a_now in (0.1, -7.0, 1e10):
                assert oracle.likelihood_sent(a_now, ap, gprev, w, mu) == want


def test_likelihood_matches_the_distortion_formula_in_high_precision():
    # tanh(|1 + (g - w a_prev)/(w a)| / mu) evaluated with 200-bit arithmetic.
    mp.mp.prec = 200
    rng = np.random.default_rng(3)
    worst = 0.0
    for _ in range(3000):
        N = int(rng.integers(1, 33))
        w = f32(1.0) / f32(N)
        mu = f32(10 ** rng.uniform(-1, 1))
        a, ap, gp = (f32(v) for v in rng.standard_normal(3) * 10 ** rng.uniform(-3, 3))
        if a == 0:
            continue
        got = oracle.likelihood_sent(a, ap, gp, w, mu)
        W, A, AP, GP, MU = (mp.mpf(float(v)) for v in (w, a, ap, gp, mu))
        D = (GP - W * AP) / (W * A)
        want = mp.tanh(abs(1 + D) / MU)
        # binary32 rounding of the four steps before tanh, amplified by the
        # cancellation in 1 + D; tanh' <= 1.
        tol = 4e-7 * float((abs(D) + 1 + abs(GP / (W * A)) + abs(AP / A)) / MU) + 1e-7
        err = abs(float(want) - got)
        worst = max(worst, err / tol)
        assert err <= tol, (N, mu, a, ap, gp, got, float(want))
    assert worst > 0  # the check is not vacuous


def test_factor_range_and_monotonicity():
    # The factor is a cumulative function of |1+Delta|: within [0,1], increasing
    # in |1+Delta| with its minimum at Delta = -1.
    w, mu, a = f32(0.25), 1.0, f32(2.0)
    ap = f32(2.0)
    # g_prev sweeps so that 1+Delta = g_prev/(w a) sweeps through [-4, 4]
    rs = np.linspace(-4, 4, 401)
    fs = [oracle.likelihood_sent(a, ap, float(f32(w * a * r + w * ap - w * a)), w, mu) for r in rs]
    fs = np.array(fs)
    assert fs.min() >= 0.0 and fs.max() <= 1.0
    mid = len(rs) // 2
    assert fs[mid] == 0.0
    assert np.all(np.diff(fs[mid:]) >= 0) and np.all(np.diff(fs[:mid + 1]) <= 0)


def test_degenerate_denominator_and_mu_limit():
    w = f32(0.5)
    assert oracle.likelihood_sent(0.0, 1.0, 1.0, w, 1.0) == 1.0       # w a = 0
    assert oracle.likelihood_sent(1e-45, 1.0, 1.0, w, 1.0) == 1.0     # w a underflows to 0
    # mu -> 0: the regulariser tends to 1 (first extreme case in the paper)
    assert oracle.likelihood_sent(1.0, 0.7, 0.2, w, 1e-30) == 1.0


# ------------------------------------------------------------ selector ----

def _brute_topk(score, k):
    score = np.asarray(score, dtype=np.float32)
    order = np.lexsort((np.arange(score.size), -score.astype(np.float64)))
    m = np.zeros(score.size, dtype=np.uint8)
    m[order[:k]] = 1
    return m


@pytest.mark.parametrize("d,k", [(1, 1), (7, 3), (64, 64), (257, 1), (1000, 10), (4096, 2048)])
def test_topk_mask_against_full_sort(d, k):
    rng = np.random.default_rng(d * 31 + k)
    for trial in range(8):
        if trial % 4 == 0:
            s = np.abs(rng.standard_normal(d))
        elif trial % 4 == 1:
            s = rng.integers(0, 4, d).astype(np.float64)      # heavy ties
        elif trial % 4 == 2:
            s = np.full(d, 2.5)                                # all equal
        else:
            s = np.zeros(d)                                    # all zero
        m = oracle.topk_mask(s, k)
        assert m.sum() == k
        assert np.array_equal(m, _brute_topk(s, k))


def test_topk_ties_take_the_lowest_indices():
    s = np.array([1, 5, 5, 5, 0, 5], dtype=np.float32)
    assert oracle.topk_mask(s, 2).tolist() == [0, 1, 1, 0, 0, 0]
    assert oracle.topk_mask(s, 4).tolist() == [0, 1, 1, 1, 0, 1]
    assert oracle.topk_mask(s, 5).tolist() == [1, 1, 1, 1, 0, 1]
