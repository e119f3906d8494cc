"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element, on seeded synthetic gradients (sizes the oracle finishes in seconds,
several chunks of 4096 and ragged tails), plus the degenerate cases."""
import numpy as np
import pytest
import torch

from paper_2501_05633_amd import binding, workloads
from tests.parity import run_both

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl_fn(cfg):
    wl = workloads.Workload(cfg, DEV)
    return lambda t, agg: wl.grads(t)


def _used_dense(stats):
    return [[w["used_dense"] for w in st] for st in stats]


@pytest.mark.parametrize("mu", [1.0, 0.1, 10.0, 0.0])
def test_tiny_config_all_rounds(mu):
    cfg = workloads.CONFIGS["tiny"]
    print("case tiny mu=%g" % mu, flush=True)
    stats, tol = run_both(cfg.N, cfg.d, cfg.k, mu, _wl_fn(cfg), cfg.T, label="tiny mu=%g" % mu)
    assert tol == 0
    for st in stats:                                          # the speculation is either verified or replaced
        assert all(w["used_dense"] == 1 or w["n_valid"] >= cfg.k for w in st)


def test_linear_regression_closed_loop():
    cfg = workloads.CONFIGS["linreg"]
    print("case linreg", flush=True)
    wl = workloads.LinRegWorkload(cfg, DEV)
    theta = torch.zeros(cfg.d, device=DEV)

    def fn(t, agg):
        nonlocal theta
        if agg is not None:
            theta = theta - wl.eta * agg
        return wl.grads(theta)

    stats, tol = run_both(cfg.N, cfg.d, cfg.k, cfg.mu, fn, cfg.T, label="linreg", check_state_every=10)
    assert tol == 0


@pytest.mark.parametrize("name,d,N,k,T", [
    ("cnn", 300_001, 3, 300, 6),            # ragged tail, scalar-load path (d % 4 != 0)
    ("large_cnn", 1_000_000, 4, 10_000, 8),  # 245 chunks, several regions
    ("transformer", 400_000, 2, 400, 5),
])
def test_layered_workloads_scaled_down(name, d, N, k, T):
    cfg = workloads.scaled(workloads.CONFIGS[name], d=d, N=N, k=k)
    print("case %s d=%d N=%d k=%d" % (name, d, N, k), flush=True)
    stats, tol = run_both(N, d, k, 1.0, _wl_fn(cfg), T, label=name, check_state_every=3)
    assert tol == 0
    dense = _used_dense(stats)
    print("dense rounds per worker:", dense, flush=True)
    # the speculative single-sweep path must carry some of the later rounds
    assert any(all(x == 0 for x in row) for row in dense[1:])


def test_forced_dense_selection_matches_too():
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=200_000, N=3, k=2_000)
    print("case forced dense", flush=True)
    stats, tol = run_both(3, 200_000, 2_000, 1.0, _wl_fn(cfg), 5, label="dense", force_dense=True)
    assert tol == 0
    assert all(all(x == 1 for x in row) for row in _used_dense(stats))


@pytest.mark.parametrize("d,k", [(1, 1), (5, 2), (4096, 1), (4097, 4097), (12289, 12289), (10_000, 10_000),
                                 (8192, 8191), (20_000, 1)])
def test_extreme_k(d, k):
    print("case extreme d=%d k=%d" % (d, k), flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(d * 7 + k)
    base = torch.randn(3, d, generator=gen, device=DEV)

    def fn(t, agg):
        return (base + 0.3 * torch.randn(3, d, generator=gen, device=DEV)).contiguous()

    stats, tol = run_both(3, d, k, 1.0, fn, 4, label="d=%d k=%d" % (d, k))
    assert tol == 0


@pytest.mark.parametrize("kind", ["zeros", "equal", "few_values", "half_zero", "denormal", "huge_range"])
def test_tie_heavy_and_degenerate_inputs(kind):
    N, d, k = 3, 30_000, 700
    print("case degenerate %s" % kind, flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(17)

    def fn(t, agg):
        if kind == "zeros":
            return torch.zeros(N, d, device=DEV)
        if kind == "equal":
            return torch.full((N, d), 0.75, device=DEV)
        if kind == "few_values":      # many exact ties at the threshold
            return torch.randint(-3, 4, (N, d), generator=gen, device=DEV).float()
        if kind == "half_zero":
            x = torch.randint(-2, 3, (N, d), generator=gen, device=DEV).float()
            x[:, d // 2:] = 0
            return x
        if kind == "denormal":
            return torch.randn(N, d, generator=gen, device=DEV) * 1e-41
        u = torch.rand(N, d, generator=gen, device=DEV) * 60 - 30
        return torch.randn(N, d, generator=gen, device=DEV) * torch.pow(10.0, u)

    stats, tol = run_both(N, d, k, 1.0, fn, 5, label=kind)
    assert tol == 0


def test_cancelling_workers_are_damped():
    # Two workers with opposite large entries (the situation of the paper's toy
    # example, at scale): after the first aggregation those entries score 0.
    N, d, k = 2, 50_000, 500
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    small = torch.randn(d, generator=gen, device=DEV) * 0.01
    big = torch.zeros(d, device=DEV)
    big[::100] = 50.0
    g = torch.stack([small + big, small - big]).contiguous()
    stats, tol = run_both(N, d, k, 1.0, lambda t, agg: g, 4, label="cancel")
    assert tol == 0


def test_state_roundtrip_and_reset():
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=150_000, N=2, k=1_500)
    wl = workloads.Workload(cfg, DEV)
    a = binding.RegTopk(2, 150_000, 1_500, 1.0, device=DEV)
    b = binding.RegTopk(2, 150_000, 1_500, 1.0, device=DEV, own_arena=True)   # hipMalloc'ed arena
    agg = None
    for t in range(3):
        idx, val, agg = a.step(wl.grads(t), agg)
        agg = agg.clone()
    e, pidx, pval, tt = a.get_state()
    assert tt == 3
    b.set_state(e, pidx, pval, tt)
    g = wl.grads(3)
    ra = [x.clone() for x in a.step(g, agg)]
    rb = [x.clone() for x in b.step(g, agg)]
    torch.cuda.synchronize()
    for x, y in zip(ra, rb):
        assert torch.equal(x, y)
    assert all(w["used_window"] == 0 for w in b.stats())     # no history after set_state: sampled bound, no window
    a.reset()
    b.reset()
    g0 = wl.grads(0)
    ra = [x.clone() for x in a.step(g0, None)]
    rb = [x.clone() for x in b.step(g0, None)]
    for x, y in zip(ra, rb):
        assert torch.equal(x, y)
    a.close()
    b.close()


def test_same_input_twice_gives_identical_bits():
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=500_000, N=4, k=5_000)
    wl = workloads.Workload(cfg, DEV)
    outs = []
    for rep in range(2):
        r = binding.RegTopk(4, 500_000, 5_000, 1.0, device=DEV)
        agg, acc = None, []
        for t in range(4):
            idx, val, agg = r.step(wl.grads(t), agg)
            agg = agg.clone()
            acc.append((idx.clone(), val.clone(), agg))
        outs.append(acc)
        r.close()
    for x, y in zip(*outs):
        for p, q in zip(x, y):
            assert torch.equal(p, q)


def test_error_codes():
    lib = binding.load()
    with pytest.raises(binding.RegTopkError) as ei:
        binding.RegTopk(0, 10, 1, 1.0, device=DEV)
    assert ei.value.code == binding.INVALID_ARG
    with pytest.raises(binding.RegTopkError):
        binding.RegTopk(2, 10, 11, 1.0, device=DEV)
    with pytest.raises(binding.RegTopkError):
        binding.RegTopk(2, 10, 1, -1.0, device=DEV)
    r = binding.RegTopk(2, 1000, 10, 1.0, device=DEV)
    g = torch.randn(2, 1000, device=DEV)
    r.step(g, None)
    with pytest.raises(binding.RegTopkError):     # round 1 with mu > 0 needs g^{t-1}
        r.step(g, None)
    with pytest.raises(ValueError):
        r.step(g[:, :999].contiguous(), None)
    r.close()


def test_scale_shocks_force_both_kinds_of_failed_speculation():
    # The gradient scale collapses (bound too high: fewer than k valid candidates)
    # and later explodes (bound too low: the candidate buffer overflows): both
    # must end in the dense selection and still match the oracle exactly, and the
    # speculation must be back one round after a collapse or a single spike.
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=600_000, N=3, k=6_000)
    wl = workloads.Workload(cfg, DEV)
    scale = {4: 1e-3, 5: 1e-3, 6: 1e-3, 9: 1e4}

    def fn(t, agg):
        return (wl.grads(t) * scale.get(t, 1.0)).contiguous()

    stats, tol = run_both(3, 600_000, 6_000, 1.0, fn, 13, label="shock", check_state_every=4)
    assert tol == 0
    dense = _used_dense(stats)
    print("dense per round:", dense, "overflow:", [[w["overflow"] for w in st] for st in stats], flush=True)
    assert all(x == 1 for x in dense[4]) and not any(w["overflow"] for w in stats[4])   # collapse: too few valid candidates
    assert all(x == 0 for x in dense[5]) and all(x == 0 for x in dense[6])              # ... caught up one round later
    assert all(w["overflow"] == 1 for w in stats[9])                                     # spike: overflow
    assert all(x == 0 for x in dense[10])                                                # ... and back
    assert all(x == 0 for x in dense[-1])


def test_jitter_of_the_gradient_scale_per_worker_and_round():
    # Every worker's gradients are scaled by its own factor, drawn anew in every round: uniform in
    # [0.7, 1.3] for 16 rounds, then log-normal (sigma 0.5) for 10.  The k-th score then moves by
    # more than any margin of a steady run; whatever mix of kept and failed speculations results,
    # every round matches the oracle, and under the milder jitter the speculation mostly holds.
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=600_000, N=4, k=6_000)
    wl = workloads.Workload(cfg, DEV)
    gen = torch.Generator().manual_seed(77)
    T = 26
    uni = 0.7 + 0.6 * torch.rand(T, 4, generator=gen)
    logn = torch.exp(0.5 * torch.randn(T, 4, generator=gen))
    factors = torch.where(torch.arange(T)[:, None] < 16, uni, logn)

    def fn(t, agg):
        return (wl.grads(t) * factors[t].to(DEV)[:, None]).contiguous()

    stats, tol = run_both(4, 600_000, 6_000, 1.0, fn, T, label="jitter", check_state_every=5)
    assert tol == 0
    dense = _used_dense(stats)
    print("dense per round:", [sum(x) for x in dense], flush=True)
    assert sum(sum(x) for x in dense[6:16]) <= 8          # of 40 worker-rounds under the uniform jitter


def test_eighty_rounds_of_jitter_shocks_and_spikes():
    # a long run in which everything that can upset the speculation happens again and again:
    # log-normal jitter of every worker's scale, collapses and explosions of all workers'
    # gradients, spikes of single workers -- every round against the oracle
    N, d, k, T = 3, 300_000, 3_000, 80
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=d, N=N, k=k)
    wl = workloads.Workload(cfg, DEV)
    gen = torch.Generator().manual_seed(1)
    f = torch.exp(0.4 * torch.randn(T, N, generator=gen))
    for t in range(10, T, 17):
        f[t] *= [1e-3, 50.0, 0.05, 300.0][(t // 17) % 4]
    for t in range(5, T, 13):
        f[t, t % N] *= 20.0

    def fn(t, agg):
        return (wl.grads(t) * f[t].to(DEV)[:, None]).contiguous()

    stats, tol = run_both(N, d, k, 1.0, fn, T, label="soak", check_state_every=10)
    assert tol == 0
    dense = [sum(x) for x in _used_dense(stats)]
    print("dense selections per round:", dense, flush=True)
    assert 0 < sum(dense) < T * N // 3          # both paths are exercised, the speculation mostly holds


def test_more_than_32_workers_and_odd_sizes():
    # 33 workers (two batches in the aggregation), d a multiple of 4 but not of 4096
    N, d, k = 33, 70_004, 350
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    shared = torch.randn(d, generator=gen, device=DEV)

    def fn(t, agg):
        return (shared + torch.randn(N, d, generator=gen, device=DEV)).contiguous()

    stats, tol = run_both(N, d, k, 1.0, fn, 5, label="N=33")
    assert tol == 0


def test_maximum_number_of_workers():
    # N = 65535, the most the interface admits (grid dimension), on very short rows
    N, d, k = 65535, 8, 2
    print("case N=65535", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    shared = torch.randn(d, generator=gen, device=DEV)

    def fn(t, agg):
        return (shared + torch.randn(N, d, generator=gen, device=DEV)).contiguous()

    stats, tol = run_both(N, d, k, 1.0, fn, 3, label="N=65535", check_overlap=True)
    assert tol == 0


def test_windowed_selection_with_many_ties_at_the_threshold():
    # Values on a coarse grid that hardly change from round to round: the k-th
    # score is predictable (windowed selection) and massively tied.
    N, d, k = 2, 200_000, 3_000
    gen = torch.Generator(device=DEV)
    gen.manual_seed(3)
    base = torch.randint(-40, 41, (N, d), generator=gen, device=DEV).float() * 0.25

    def fn(t, agg):
        return base.clone()

    stats, tol = run_both(N, d, k, 1.0, fn, 8, label="grid ties")
    assert tol == 0
    print("window per round:", [[w["used_window"] for w in st] for st in stats],
          "ties:", [[(w["n_ties_taken"], w["n_ties_total"]) for w in st] for st in stats], flush=True)


def test_caller_owned_previous_aggregate_and_two_contexts_on_two_streams():
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=300_000, N=2, k=3_000)
    wl = workloads.Workload(cfg, DEV)
    ref = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    a = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    b = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    agg_ref = agg_a = agg_b = None
    for t in range(5):
        g = wl.grads(t)
        torch.cuda.synchronize()
        r0 = [x.clone() for x in ref.step(g, agg_ref)]
        agg_ref = r0[2]
        with torch.cuda.stream(sa):
            ra = a.step(g, agg_a)
            agg_a = ra[2].clone()          # a copy owned by the caller is handed back next round
        with torch.cuda.stream(sb):
            rb = b.step(g, agg_b)
            agg_b = rb[2].clone()
        torch.cuda.synchronize()
        for x, y, z in zip(r0, ra, rb):
            assert torch.equal(x, y) and torch.equal(x, z)
    ref.close(); a.close(); b.close()


def test_two_contexts_on_two_streams_with_the_dense_selection_forced():
    # the dense selection synchronises its blocks with grid barriers; launches of different contexts
    # on one device are kept apart by the library, so two streams that both take it in every round
    # must give what a single context gives
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=300_000, N=2, k=3_000)
    wl = workloads.Workload(cfg, DEV)
    ref = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    a = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    b = binding.RegTopk(2, 300_000, 3_000, 1.0, device=DEV)
    for r in (ref, a, b):
        r.set_option(binding.OPT_FORCE_DENSE, 1)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    agg_ref = agg_a = agg_b = None
    for t in range(4):
        print("  round %d" % t, flush=True)
        g = wl.grads(t)
        torch.cuda.synchronize()
        r0 = [x.clone() for x in ref.step(g, agg_ref)]
        agg_ref = r0[2]
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            ra = a.step(g, agg_a)
            agg_a = ra[2].clone()
        with torch.cuda.stream(sb):
            rb = b.step(g, agg_b)
            agg_b = rb[2].clone()
        torch.cuda.synchronize()
        for x, y, z in zip(r0, ra, rb):
            assert torch.equal(x, y) and torch.equal(x, z)
        for r in (a, b):
            assert all(w["used_dense"] == 1 for w in r.stats())
    ref.close(); a.close(); b.close()


def test_sixty_rounds_of_the_scaled_down_target_workload():
    # a long horizon: the controller's window narrows to its minimum and the speculative bound follows
    # the slowly drifting k-th score for dozens of rounds; every round is compared
    cfg = workloads.scaled(workloads.CONFIGS["large_cnn"], d=1_000_000, N=4, k=10_000)
    print("case 60 rounds", flush=True)
    stats, tol = run_both(4, 1_000_000, 10_000, 1.0, _wl_fn(cfg), 60, label="60 rounds", check_state_every=20)
    assert tol == 0
    dense = _used_dense(stats)
    window = [[w["used_window"] for w in st] for st in stats]
    assert sum(sum(r) for r in dense[10:]) == 0
    assert sum(sum(r) for r in window[10:]) >= 4 * 45          # the window holds the k-th score in nearly every round
