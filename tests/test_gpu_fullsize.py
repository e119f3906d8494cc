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
