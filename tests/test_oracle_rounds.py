"""Pins for whole rounds of the CPU oracle (Algorithm 2 + aggregation):
reduction to plain Top-k, conservation, the paper's toy example, k = d, and
metamorphic relations.  The plain Top-k with error feedback used for comparison
(Algorithm 1) is written here with numpy's sort, not with the oracle.
"""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2501_05633_amd import workloads

f32 = np.float32
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _topk_ef_numpy(grads_per_round, k):
    """Algorithm 1 for every worker with a library sort; returns per-round index sets."""
    N, d = grads_per_round[0].shape
    e = np.zeros((N, d), dtype=np.float32)
    out = []
    for g in grads_per_round:
        a = e + g
        sets, agg = [], np.zeros(d, dtype=np.float64)
        for n in range(N):
            order = np.lexsort((np.arange(d), -np.abs(a[n]).astype(np.float64)))
            sel = np.sort(order[:k])
            sets.append(sel)
            e[n] = a[n]
            e[n, sel] = 0.0
            agg[sel] += a[n, sel].astype(np.float64) / N
        out.append((sets, a.copy(), agg))
    return out


def _tiny_rounds(T=6, N=4, d=2000, k=20, seed=None):
    cfg = workloads.scaled(workloads.CONFIGS["tiny"], d=d, N=N, k=k)
    wl = workloads.Workload(cfg, "cpu", seed=seed)
    return [wl.grads(t).numpy() for t in range(T)]


def _run(o, rounds):
    res, agg = [], None
    for g in rounds:
        idx, val, agg = o.step(g, agg)
        res.append((idx.copy(), val.copy(), agg.copy(), o.a, o.e, o.score, o.mask))
    return res


def test_round0_is_plain_topk():
    # "The algorithm starts with applying standard Top-k in the initial round."
    rounds = _tiny_rounds(T=1)
    ref = _topk_ef_numpy(rounds, 20)
    for mu in (0.1, 1.0, 10.0):
        idx, val, agg = oracle.Oracle(4, 2000, 20, mu).step(rounds[0], None)
        for n in range(4):
            assert np.array_equal(idx[n], ref[0][0][n])
        np.testing.assert_allclose(agg, ref[0][2], rtol=1e-6, atol=0)


def test_mu_zero_is_algorithm1_for_all_rounds():
    rounds = _tiny_rounds(T=6)
    ref = _topk_ef_numpy(rounds, 20)
    res = _run(oracle.Oracle(4, 2000, 20, 0.0), rounds)
    for t in range(6):
        for n in range(4):
            assert np.array_equal(res[t][0][n], ref[t][0][n]), (t, n)
        assert np.array_equal(res[t][3], ref[t][1])            # accumulated gradients
        np.testing.assert_allclose(res[t][2], ref[t][2], rtol=2e-6, atol=1e-30)


def test_tiny_positive_mu_equals_mu_zero_without_exact_cancellation():
    rounds = _tiny_rounds(T=5)
    r0 = _run(oracle.Oracle(4, 2000, 20, 0.0), rounds)
    r1 = _run(oracle.Oracle(4, 2000, 20, 2.0 ** -100), rounds)
    for t in range(5):
        assert np.array_equal(r0[t][0], r1[t][0])
        assert np.array_equal(r0[t][1], r1[t][1])


def test_conservation_and_mask_shape():
    # ghat = s . a and eps^{t+1} = a - ghat: a = ghat + eps exactly, eps in {0, a}.
    rounds = _tiny_rounds(T=6)
    o = oracle.Oracle(4, 2000, 20, 1.0)
    agg = None
    e_before = np.zeros((4, 2000), dtype=np.float32)
    for g in rounds:
        idx, val, agg = o.step(g, agg)
        a, e, m = o.a, o.e, o.mask
        assert np.array_equal(a, e_before + g)                 # one rounded add
        assert np.all(m.sum(axis=1) == 20)
        ghat = np.zeros_like(a)
        for n in range(4):
            assert np.all(np.diff(idx[n]) > 0)
            assert np.array_equal(np.flatnonzero(m[n]), idx[n])
            ghat[n, idx[n]] = val[n]
            assert np.array_equal(val[n], a[n, idx[n]])
        assert np.array_equal(ghat + e, a)
        assert np.all((e == 0) | (e == a))
        assert np.all(e[m == 1] == 0)
        # aggregation: brute-force dense sum in the same worker order
        acc = np.zeros(2000, dtype=np.float32)
        for n in range(4):
            acc = acc + f32(0.25) * ghat[n]
        assert np.array_equal(acc, agg)
        assert np.all(agg[m.sum(axis=0) == 0] == 0)
        e_before = e


def test_unsent_entries_keep_factor_one_and_scores_are_bounded():
    rounds = _tiny_rounds(T=4)
    o = oracle.Oracle(4, 2000, 20, 1.0)
    agg, prev_mask = None, np.zeros((4, 2000), dtype=np.uint8)
    changed = 0
    for g in rounds:
        idx, val, agg = o.step(g, agg)
        a, sc = o.a, o.score
        assert np.array_equal(sc[prev_mask == 0], np.abs(a)[prev_mask == 0])   # C = 1
        assert np.all(sc >= 0) and np.all(sc <= np.abs(a))
        changed += int((sc[prev_mask == 1] < np.abs(a)[prev_mask == 1]).sum())
        # a previously sent entry restarts from zero error: a = g there
        assert np.array_equal(a[prev_mask == 1], g[prev_mask == 1])
        prev_mask = o.mask
    assert changed > 0    # the regulariser did act


def test_selection_invariant_on_regularised_rounds():
    rounds = _tiny_rounds(T=5, d=5000, k=50)
    o = oracle.Oracle(4, 5000, 50, 1.0)
    agg = None
    for g in rounds:
        idx, val, agg = o.step(g, agg)
        sc, m = o.score, o.mask
        for n in range(4):
            lo = sc[n][m[n] == 1].min()
            hi = sc[n][m[n] == 0].max()
            assert lo >= hi
            if lo == hi:
                tie_in = np.flatnonzero((sc[n] == lo) & (m[n] == 1))
                tie_out = np.flatnonzero((sc[n] == lo) & (m[n] == 0))
                assert tie_in.max() < tie_out.min()


def test_k_equals_d_is_dense_averaging_for_any_mu():
    # S = 1: Top-k, RegTop-k and the unsparsified run coincide.
    rounds = _tiny_rounds(T=4, d=300, k=300)
    ref = None
    for mu in (0.0, 0.5, 4.0):
        res = _run(oracle.Oracle(4, 300, 300, mu), rounds)
        for t, g in enumerate(rounds):
            assert np.all(res[t][4] == 0)                       # no residual
            np.testing.assert_allclose(res[t][2], g.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
        aggs = [r[2] for r in res]
        if ref is not None:
            for x, y in zip(ref, aggs):
                assert np.array_equal(x, y)
        ref = aggs


def _read_gold(name):
    out = {}
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                out[k.strip()] = [float(x) for x in v.split()]
    return out


def _toy_grad(theta, xs):
    z = np.exp(-(xs @ theta))
    return (-(z / (1 + z))[:, None] * xs).astype(np.float32)


def test_toy_example_first_two_rounds():
    gold = _read_gold("toy_logistic.txt")
    xs = np.array([gold["x1"], gold["x2"]])
    theta = np.array(gold["theta0"])
    c = gold["c"][0]
    g = _toy_grad(theta, xs)
    np.testing.assert_allclose(g, -c * xs, rtol=1e-6)
    o = oracle.Oracle(2, 2, 1, 1.0)
    idx, val, agg = o.step(g, None)
    assert idx.ravel().tolist() == [0, 0]                       # both send the large entry
    assert agg.tolist() == [0.0, 0.0]                           # which cancels exactly
    np.testing.assert_allclose(o.e[:, 1], [-c, -c], rtol=1e-6)
    # theta does not move (zero aggregate), so the gradient repeats
    idx, val, agg = o.step(g, agg)
    assert np.all(o.score[:, 0] == 0.0)                         # Delta = -1: damped to zero
    assert idx.ravel().tolist() == [1, 1]
    np.testing.assert_allclose(agg, [0.0, -2 * c], rtol=1e-6)


def test_toy_example_closed_loop_stall():
    gold = _read_gold("toy_logistic.txt")
    xs = np.array([gold["x1"], gold["x2"]])
    eta = gold["eta"][0]

    def risk(theta):
        return float(np.mean(np.log1p(np.exp(-(xs @ theta)))))

    def run(mu, T):
        theta = np.array(gold["theta0"])
        o = oracle.Oracle(2, 2, 1, mu)
        agg, first_move = None, None
        for t in range(T):
            idx, val, agg = o.step(_toy_grad(theta, xs), agg)
            if first_move is None and np.any(agg != 0):
                first_move = t
            theta = theta - eta * agg.astype(np.float64)
        return first_move, risk(theta)

    stall = int(gold["stall_rounds_min"][0])
    move_topk, risk_topk = run(0.0, stall)
    assert move_topk is None
    move_topk, _ = run(0.0, 110)
    assert gold["stall_rounds_min"][0] <= move_topk <= gold["stall_rounds_max"][0]
    move_reg, risk_reg = run(1.0, stall)
    assert move_reg == 1
    r0 = risk(np.array(gold["theta0"]))
    assert abs(risk_topk - r0) < 1e-12          # no progress for about 100 iterations
    assert risk_reg < 0.5 * r0


def _table1_gradients():
    gold = _read_gold("table1_iteration1.txt")
    target, s1, s2 = (np.array(gold[key]) for key in ("target", "sent1", "sent2"))
    g = np.stack([s1, s2])
    g[0, 2] = 2 * target[2] - s2[2]          # the dropped entries follow from the aggregation target
    g[1, 3] = 2 * target[3] - s1[3]
    return gold, target, s1, s2, g


def test_first_row_of_the_papers_table_of_accumulated_gradients():
    # The printed numbers are consistent with Top_3 per worker and averaging with omega = 1/2,
    # and RegTop-k equals Top-k in the first iteration; the oracle reproduces the printed row.
    gold, target, s1, s2, g = _table1_gradients()
    np.testing.assert_allclose(g.mean(axis=0), target, atol=0.01)       # entries are printed with two decimals (rounded or cut)
    assert abs(g[0, 2]) < np.abs(s1[[0, 1, 3]]).min() and abs(g[1, 3]) < np.abs(s2[[0, 1, 2]]).min()
    for mu in (0.0, 1.0):
        o = oracle.Oracle(2, 4, 3, mu)
        idx, val, agg = o.step(g.astype(f32), None)
        assert idx.tolist() == [[0, 1, 3], [0, 1, 2]]
        ghat = np.zeros((2, 4))
        for n in range(2):
            ghat[n, idx[n]] = val[n]
        np.testing.assert_allclose(ghat[0], s1, atol=1e-6)
        np.testing.assert_allclose(ghat[1], s2, atol=1e-6)
        np.testing.assert_allclose(agg, (s1 + s2) / 2, rtol=1e-6)
        np.testing.assert_allclose(o.e, [[0, 0, g[0, 2], 0], [0, 0, 0, g[1, 3]]], rtol=1e-6)


def test_power_of_two_scaling_and_sign_flip_keep_the_masks():
    rounds = _tiny_rounds(T=5)
    base = _run(oracle.Oracle(4, 2000, 20, 1.0), rounds)
    for factor in (2.0 ** 7, 2.0 ** -9, -1.0):
        res = _run(oracle.Oracle(4, 2000, 20, 1.0), [g * f32(factor) for g in rounds])
        for t in range(5):
            assert np.array_equal(res[t][0], base[t][0])
            assert np.array_equal(res[t][1], base[t][1] * f32(factor))
            assert np.array_equal(res[t][2], base[t][2] * f32(factor))


def test_worker_permutation_permutes_rows():
    # N a power of two: w is exact, so the aggregate does not depend on the order
    rounds = _tiny_rounds(T=1)
    perm = [2, 0, 3, 1]
    a = oracle.Oracle(4, 2000, 20, 1.0).step(rounds[0], None)
    b = oracle.Oracle(4, 2000, 20, 1.0).step(rounds[0][perm], None)
    assert np.array_equal(a[0][perm], b[0]) and np.array_equal(a[1][perm], b[1])


def test_argument_checks():
    for bad in ((0, 10, 1, 1.0), (2, 0, 1, 1.0), (2, 10, 0, 1.0), (2, 10, 11, 1.0), (2, 10, 1, -1.0),
                (2, 10, 1, float("nan"))):
        with pytest.raises(ValueError):
            oracle.Oracle(*bad)


def test_masks_of_different_workers_coordinate_under_the_regulariser():
    # Appendix "Comparing Sparsification Masks": with RegTop-k the workers, who all
    # see the same previous aggregate, end up dropping the same entries, whereas
    # Top-k workers sparsify independently.  Setting of the paper's linear
    # regression (N = 20, J = 100, D_n = 500, eta = 1e-2, U = 0, sigma^2 = 5,
    # h^2 = 1, eps^2 = 0.5), S = 0.9, measured once the iterates are near the optimum.
    N, J, D, eta, k = 20, 100, 500, 1e-2, 90
    rng = np.random.default_rng(0)
    X = rng.standard_normal((N, D, J))
    u = rng.normal(0.0, np.sqrt(5.0), N)
    truth = u[:, None] + rng.standard_normal((N, J))
    y = np.einsum("ndj,nj->nd", X, truth) + np.sqrt(0.5) * rng.standard_normal((N, D))

    def unanimous(mu):
        o = oracle.Oracle(N, J, k, mu)
        theta, agg, acc = np.zeros(J), None, []
        for it in range(420):
            r = np.einsum("ndj,j->nd", X, theta) - y
            g = (2.0 / D) * np.einsum("ndj,nd->nj", X, r)
            _, _, agg = o.step(g.astype(np.float32), agg)
            theta = theta - eta * agg.astype(np.float64)
            if it >= 380:
                cnt = o.mask.sum(axis=0)
                acc.append(int(((cnt == 0) | (cnt == N)).sum()))     # entries all workers agree on
        return float(np.mean(acc))

    assert unanimous(1.0) > 70          # most of the 100 entries are kept or dropped by all workers
    assert unanimous(0.0) < 35          # plain Top-k: hardly any agreement


def _lowdim_log_gap(seed, k, mu, T=60):
    # the appendix's low-dimensional study: N = 2, J = 4, D_n = 20, U = 0, sigma^2 = h^2 = 1, eps^2 = 0.5,
    # eta = 1e-2; gradient X^T (X theta - y), the scaling under which the unsparsified run decays at the
    # rate of the curves plotted in the paper (about 0.8 per iteration at first, 0.86 later)
    wl = workloads.PaperLinReg("cpu", N=2, J=4, D=20, sigma2=1.0, normalised=False,
                               seed=workloads.BASE_SEED + 200 + seed)
    o = oracle.Oracle(2, 4, k, mu)
    theta, agg = np.zeros(4, dtype=f32), None
    for _ in range(T):
        g = wl.grads(torch.from_numpy(theta)).numpy()
        _, _, agg = o.step(g, agg)
        theta = oracle.sgd_update(theta, agg, wl.eta)
    return float(np.log(wl.gap(torch.from_numpy(theta))))


def test_low_dimensional_study_regtopk_tracks_the_unsparsified_run_where_topk_stalls():
    # Figure "Optimality gap ... in the low-dimensional case with J = 4" and the text of the appendix: for
    # S = 0.75 and S = 0.5 Top-k stays at a fixed distance from the optimum (log gap about -2.4 ... -3.4 after
    # 60 iterations in the plotted sample problem) while RegTop-k follows the unsparsified run (about -9.3);
    # for S = 0.25 neither converges.  One sample problem in full, then counts over ten problems.
    gold = _read_gold("lowdim_figure.txt")
    stall, track = -5.0, 1.0               # what "stalls" and "tracks" mean below; the plotted curves satisfy both
    for S in ("S075", "S050"):
        assert min(gold["topk_" + S]) > stall and max(gold["regtopk_" + S]) < min(gold["dense_" + S]) + track
    assert min(gold["topk_S025"]) > stall and min(gold["regtopk_S025"]) > stall
    first = gold["dense_S100_first"]
    assert abs((first[1] - first[0]) - np.log(0.8)) < 0.01             # the step scaling used by _lowdim_log_gap
    dense = _lowdim_log_gap(2, 4, 0.0)
    assert dense < -9.0
    for k in (3, 2):
        assert _lowdim_log_gap(2, k, 0.0) > stall                      # Top-k stalls
        for mu in (0.25, 0.5, 1.0):
            assert _lowdim_log_gap(2, k, mu) < dense + track           # RegTop-k tracks the unsparsified run
    assert _lowdim_log_gap(2, 1, 0.0) > stall and _lowdim_log_gap(2, 1, 1.0) > stall
    tracked_reg = tracked_top = 0
    for seed in range(10):
        d = _lowdim_log_gap(seed, 4, 0.0)
        tracked_top += _lowdim_log_gap(seed, 3, 0.0) < d + track
        tracked_reg += min(_lowdim_log_gap(seed, 3, mu) for mu in (0.25, 0.5, 1.0, 2.0, 5.0)) < d + track
    assert tracked_reg >= 8 and tracked_top <= 4                       # mu is tuned per problem, as in the paper


def test_linear_regression_n20_what_the_oracle_reproduces_of_the_papers_claims():
    # Section "Linear Regression Problem" (N = 20, J = 100, D_n = 500, eta = 1e-2, S = 0.6).
    # Reproduced, and pinned here: with identical ground truths and no label noise (figure
    # "Homogeneity vs heterogeneity", left) Top-k and RegTop-k both track the unsparsified run; with
    # heterogeneous workers (sigma^2 = 5) Top-k stays at a fixed distance from the optimum, orders of
    # magnitude above the unsparsified run.  NOT reproduced by this reading of Algorithm 2 for any mu
    # on a grid 1e-3 .. 1e2 (oracle/linreg_study.py; table in the design document): RegTop-k reaching
    # the unsparsified gap in the heterogeneous case -- that claim stays "parity unpinned".
    from oracle import linreg_study as ls
    T = 1500
    dense_h = ls.run(0, 1.0, 0.0, homogeneous=True, T=T)
    topk_h = ls.run(0, 0.6, 0.0, homogeneous=True, T=T)
    reg_h = ls.run(0, 0.6, 1.0, homogeneous=True, T=T)
    assert dense_h < 1e-3 and topk_h < 3 * dense_h and reg_h < 3 * dense_h, (dense_h, topk_h, reg_h)
    dense = ls.run(0, 1.0, 0.0, T=T)
    topk = ls.run(0, 0.6, 0.0, T=T)
    assert dense < 1e-3 and topk > 100 * dense, (dense, topk)
    # Top-k has stalled, not merely slowed down: 1000 more iterations change nothing
    assert abs(ls.run(0, 0.6, 0.0, T=T + 1000) - topk) < 0.3 * topk


def test_round_level_wiring_of_the_distortion_sole_sender_and_two_senders():
    # Which quantities the round hands to the distortion: g^{t-1} (the aggregate), a^{t-1} (what the
    # worker sent then) and a^t (its new accumulated gradient) -- with gradients that change between
    # the rounds, so that a^{t-1} != a^t on the sent entries.
    # (1) One worker: every sent entry had a sole sender, the aggregate there is omega * a^{t-1}
    #     exactly, the distortion is 0 and the score is |a^t| * tanh(1/mu); unsent entries score |a^t|.
    mu = 0.7
    rng = np.random.default_rng(5)
    g0 = rng.standard_normal((1, 12)).astype(np.float32)
    g1 = rng.standard_normal((1, 12)).astype(np.float32)
    o = oracle.Oracle(1, 12, 4, mu)
    idx0, val0, agg0 = o.step(g0, None)
    o.step(g1, agg0)
    a1, sc1 = o.a[0], o.score[0]
    f = np.float32(oracle.tanh32(np.float32(1.0) / np.float32(mu)))
    sent = np.zeros(12, dtype=bool)
    sent[idx0[0]] = True
    assert np.array_equal(a1[sent], g1[0][sent]) and np.array_equal(a1[~sent], (g0 + g1)[0][~sent])
    assert np.array_equal(sc1[sent], np.abs(a1[sent]) * f)
    assert np.array_equal(sc1[~sent], np.abs(a1[~sent]))
    # (2) Two workers that both sent entry 0 in round 0: Delta_1 = (g^0 - w v_1) / (w a_1^1) with
    #     g^0 = w v_1 + w v_2, evaluated here in 200-bit arithmetic from the binary32 inputs.
    import mpmath
    mpmath.mp.prec = 200
    g0 = np.array([[4.0, 0.1, 0.2], [3.0, 0.3, -0.1]], dtype=np.float32)
    g1 = np.array([[1.7, 0.05, 0.1], [-2.2, 0.2, 0.3]], dtype=np.float32)
    o = oracle.Oracle(2, 3, 1, mu)
    idx0, val0, agg0 = o.step(g0, None)
    assert idx0.tolist() == [[0], [0]]
    o.step(g1, agg0)
    w = mpmath.mpf(0.5)
    for n in range(2):
        a_now = mpmath.mpf(float(g1[n, 0]))                      # the error was cleared on the sent entry
        delta = (mpmath.mpf(float(agg0[0])) - w * mpmath.mpf(float(g0[n, 0]))) / (w * a_now)
        want = abs(a_now) * mpmath.tanh(abs(1 + delta) / mpmath.mpf(float(np.float32(mu))))
        assert abs(mpmath.mpf(float(o.score[n, 0])) - want) <= 4e-7 * want, (n, o.score[n, 0], want)
