"""Parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times: every round of the HIP path against the CPU
oracle (bit-exact index sets, 1e-6 relative values, residuals and aggregate),
long enough for the speculative single-sweep path and the windowed selection
to carry the later rounds."""
import numpy as np
import pytest
import torch

from paper_2501_05633_amd import workloads
from tests.parity import run_both

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,T", [("large_cnn", 10), ("cnn", 5), ("transformer", 3)])
def test_full_size_rounds(name, T):
    cfg = workloads.CONFIGS[name]
    wl = workloads.Workload(cfg, DEV)
    print("case full size %s N=%d d=%d k=%d T=%d" % (name, cfg.N, cfg.d, cfg.k, T), flush=True)

    def fn(t, agg):
        print("  round %d" % t, flush=True)
        return wl.grads(t)

    stats, tol = run_both(cfg.N, cfg.d, cfg.k, cfg.mu, fn, T, label=name, check_state_every=T - 1)
    assert tol == 0
    dense = [[w["used_dense"] for w in st] for st in stats]
    window = [[w["used_window"] for w in st] for st in stats]
    print("dense per round:", [sum(r) for r in dense], "window per round:", [sum(r) for r in window], flush=True)
    if name == "large_cnn":
        assert any(sum(r) == 0 for r in dense[1:])            # speculative rounds happened
        assert any(sum(r) == cfg.N for r in window)           # and the windowed selection


@pytest.mark.parametrize("what", ["mu=0.1", "mu=10", "bf16", "roots=1,clipped", "weights"])
def test_full_size_variants_of_the_target_workload(what):
    # the other ways the target workload (N = 16, d = 25.6M, k = 256k) is run: the mu sweep of the
    # benchmark list, bfloat16 gradients, a score variant, general weights -- two or three rounds each
    cfg = workloads.CONFIGS["large_cnn"]
    wl = workloads.Workload(cfg, DEV)
    print("case full size large_cnn %s" % what, flush=True)
    kw = {}
    mu = cfg.mu
    if what.startswith("mu="):
        mu = float(what[3:])
    elif what == "bf16":
        kw["grad_dtype"] = torch.bfloat16
    elif what == "roots=1,clipped":
        kw.update(prior_roots=1, likelihood=1)
    elif what == "weights":
        kw["weights"] = np.random.default_rng(2).dirichlet(np.full(cfg.N, 4.0)).astype(np.float32)

    def fn(t, agg):
        print("  round %d" % t, flush=True)
        return wl.grads(t)

    T = 2 if what in ("mu=10", "weights") else 3
    stats, tol = run_both(cfg.N, cfg.d, cfg.k, mu, fn, T, label="large_cnn " + what, check_state_every=T - 1, **kw)
    assert tol == 0


def test_full_size_global_topk_rounds():
    from oracle import oracle as orc
    from paper_2501_05633_amd import binding
    cfg = workloads.CONFIGS["large_cnn"]
    wl = workloads.Workload(cfg, DEV)
    print("case full size large_cnn global Top-k", flush=True)
    o = orc.Oracle(cfg.N, cfg.d, cfg.k, cfg.mu)
    r = binding.RegTopk(cfg.N, cfg.d, cfg.k, cfg.mu, device=DEV)
    for t in range(2):
        print("  round %d" % t, flush=True)
        g = wl.grads(t)
        idx, val, agg = r.step_global(g)
        torch.cuda.synchronize()
        ic, vc, ac = o.step_global(g.cpu().numpy())
        assert np.array_equal(idx.cpu().numpy(), ic)
        assert np.array_equal(val.cpu().numpy().view(np.uint32), vc.view(np.uint32))
        np.testing.assert_allclose(agg.cpu().numpy(), ac, rtol=1e-6, atol=0)
    r.close()
