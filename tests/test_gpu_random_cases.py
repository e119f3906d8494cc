"""Seeded random sweep of small configurations: sizes, k, mu, value patterns and
options drawn at random, every round compared with the CPU oracle bit for bit
(indices, values, aggregate, residual).  Meant to hit the corners no hand-written
case names: d around chunk and word borders, k = 1 and k = d, heavy ties, zeros,
mixed kinds of rounds."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2501_05633_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
f32 = np.float32


def _draw_case(rng):
    N = int(rng.choice([1, 2, 3, 5, 8, 17, 33]))
    d = int(rng.choice([1, 2, 3, 31, 32, 33, 100, 1000, 4095, 4096, 4097, 8192, 12289, 30000, 65537]))
    k = int(rng.choice([1, max(1, d // 100), max(1, d // 10), max(1, d // 2), d]))
    mu = float(rng.choice([0.0, 0.05, 1.0, 7.0]))
    pattern = str(rng.choice(["gauss", "grid", "sparse", "const", "wide"]))
    opts = {
        "weights": rng.dirichlet(np.ones(N)).astype(f32) if rng.random() < 0.3 else None,
        "roots": int(rng.choice([0, 0, 0, 1, 2])),
        "exponent": float(rng.choice([1.0, 1.0, 1.0, 0.8, 0.35])),
        "likelihood": int(rng.choice([0, 0, 1, 2])),
        "force_dense": bool(rng.random() < 0.2),
        "bf16": bool(rng.random() < 0.25),
        "kinds": "".join(rng.choice(list("LLLG"), size=4)),
    }
    return N, d, k, mu, pattern, opts


def _grads(rng, pattern, N, d, t):
    if pattern == "gauss":
        g = rng.standard_normal((N, d))
    elif pattern == "grid":                      # few distinct magnitudes: ties everywhere
        g = rng.integers(-3, 4, size=(N, d)) * 0.25
    elif pattern == "sparse":                    # mostly exact zeros
        g = rng.standard_normal((N, d)) * (rng.random((N, d)) < 0.05)
    elif pattern == "const":
        g = np.full((N, d), 0.5 if t % 2 == 0 else -0.5)
    else:                                        # magnitudes over many binades, incl. denormals
        g = rng.standard_normal((N, d)) * 10.0 ** rng.integers(-42, 30, size=(N, d)).astype(np.float64)
    return np.clip(g, -3e38, 3e38).astype(f32)


@pytest.mark.parametrize("block", range(6))
def test_random_small_configurations(block):
    rng = np.random.default_rng(20250105 + block)
    for case in range(12):
        N, d, k, mu, pattern, opts = _draw_case(rng)
        label = "block %d case %d: N=%d d=%d k=%d mu=%g %s %s" % (block, case, N, d, k, mu, pattern, {
            kk: (v if not isinstance(v, np.ndarray) else "set") for kk, v in opts.items()})
        print(label, flush=True)
        o = orc.Oracle(N, d, k, mu)
        r = binding.RegTopk(N, d, k, mu, device=DEV)
        o.set_score_variant(opts["roots"], opts["likelihood"])
        r.set_option(binding.OPT_PRIOR_ROOTS, opts["roots"])
        r.set_option(binding.OPT_LIKELIHOOD, opts["likelihood"])
        if opts["exponent"] != 1.0 and opts["roots"] == 0:
            o.set_prior_exponent(opts["exponent"])
            r.set_option(binding.OPT_PRIOR_EXPONENT, opts["exponent"])
        if opts["force_dense"]:
            r.set_option(binding.OPT_FORCE_DENSE, 1)
        if opts["weights"] is not None:
            o.set_weights(opts["weights"])
            r.set_weights([float(x) for x in opts["weights"]])
        agg_g = agg_c = None
        for t, kind in enumerate(opts["kinds"]):
            g = torch.from_numpy(_grads(rng, pattern, N, d, t)).to(DEV)
            if opts["bf16"] and kind == "L":
                g = g.to(torch.bfloat16)
            g_host = g.float().cpu().numpy()
            if kind == "G":
                res_g = r.step_global(g.float().contiguous())
                res_c = o.step_global(g_host)
            else:
                res_g = r.step(g.contiguous(), agg_g)
                res_c = o.step(g_host, agg_c)
            torch.cuda.synchronize()
            idx, val, agg = (x.cpu().numpy() for x in res_g)
            assert np.array_equal(idx, res_c[0]), label + " round %d (%s): indices" % (t, kind)
            assert np.array_equal(val.view(np.uint32), res_c[1].view(np.uint32)), label + " round %d: values" % t
            assert np.array_equal(agg.view(np.uint32), res_c[2].view(np.uint32)), label + " round %d: aggregate" % t
            assert np.array_equal(r.mask_overlap().cpu().numpy(), o.mask_overlap()), label + " round %d: overlap" % t
            agg_g, agg_c = res_g[2].clone(), res_c[2]
        e = r.get_state()[0].cpu().numpy()
        assert np.array_equal(e.view(np.uint32), o.e.view(np.uint32)), label + ": residual"
        r.stats()                                  # raises if a device-side consistency check failed
        r.close()
        o.close()


@pytest.mark.parametrize("block", range(2))
def test_random_configurations_with_per_worker_k(block):
    # the same sweep with every worker keeping its own k_n (drawn per case, redrawn once mid-run)
    rng = np.random.default_rng(20260105 + block)
    for case in range(12):
        N, d, k, mu, pattern, opts = _draw_case(rng)
        if N == 1:
            N = 4
        label = "worker-k block %d case %d: N=%d d=%d k=%d mu=%g %s dense=%s" % (
            block, case, N, d, k, mu, pattern, opts["force_dense"])
        print(label, flush=True)
        o = orc.Oracle(N, d, k, mu)
        r = binding.RegTopk(N, d, k, mu, device=DEV)
        if opts["force_dense"]:
            r.set_option(binding.OPT_FORCE_DENSE, 1)
        agg_g = agg_c = None
        for t in range(5):
            if t in (0, 3):
                kn = [int(x) for x in rng.integers(1, k + 1, size=N)]
                kn[int(rng.integers(N))] = k
                kn[int(rng.integers(N))] = 1
                o.set_worker_k(kn)
                r.set_worker_k(kn)
            g = torch.from_numpy(_grads(rng, pattern, N, d, t)).to(DEV)
            res_g = r.step(g.contiguous(), agg_g)
            res_c = o.step(g.cpu().numpy(), agg_c)
            torch.cuda.synchronize()
            idx, val, agg = (x.cpu().numpy() for x in res_g)
            assert np.array_equal(idx, res_c[0]), label + " round %d: indices" % t
            assert np.array_equal(val.view(np.uint32), res_c[1].view(np.uint32)), label + " round %d: values" % t
            assert np.array_equal(agg.view(np.uint32), res_c[2].view(np.uint32)), label + " round %d: aggregate" % t
            assert np.array_equal(r.mask_overlap().cpu().numpy(), o.mask_overlap()), label + " round %d: overlap" % t
            agg_g, agg_c = res_g[2].clone(), res_c[2]
        e = r.get_state()[0].cpu().numpy()
        assert np.array_equal(e.view(np.uint32), o.e.view(np.uint32)), label + ": residual"
        r.stats()
        r.close()
        o.close()
