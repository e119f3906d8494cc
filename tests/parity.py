"""Shared driver of the GPU parity tests: runs the HIP path and the CPU oracle
round by round on the same gradients and compares everything they return.

The HIP path is reached only through ``paper_2501_05633_amd.binding`` (the
C ABI); the oracle only through ``oracle.oracle``.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import oracle as orc
from paper_2501_05633_amd import binding

REL_TOL = 1e-6     # values, residuals, aggregates (binary32, same operation order on both sides)


def _rel_close(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    bound = REL_TOL * np.abs(want)
    bad = err > bound
    assert not bad.any(), "%s: %d entries beyond %.0e relative, worst %g vs %g" % (
        what, int(bad.sum()), REL_TOL, got[bad][0], want[bad][0])


def ulp_threshold_ties(o: orc.Oracle, n: int, idx_gpu: np.ndarray, idx_cpu: np.ndarray):
    """Index mismatches of one worker and how many of them are scores within one
    unit in the last place of the k-th largest score (the only tolerated kind)."""
    only_gpu = np.setdiff1d(idx_gpu, idx_cpu)
    only_cpu = np.setdiff1d(idx_cpu, idx_gpu)
    if only_gpu.size == 0 and only_cpu.size == 0:
        return 0, 0
    sc = o.score[n]
    tau = sc[idx_cpu].min()
    tb = np.float32(tau).view(np.uint32).astype(np.int64)
    near = 0
    for j in np.concatenate([only_gpu, only_cpu]):
        jb = np.float32(sc[j]).view(np.uint32).astype(np.int64)
        near += int(abs(jb - tb) <= 1)
    return int(only_gpu.size + only_cpu.size), near


def compare_round(o: orc.Oracle, res_gpu, res_cpu, label="", worker_k=None):
    """Bit-exact index sets; values/aggregate within REL_TOL.  Returns the number
    of tolerated 1-ulp threshold ties (reported by the callers)."""
    idx_g, val_g, agg_g = (x.cpu().numpy() for x in res_gpu)
    idx_c, val_c, agg_c = res_cpu
    tolerated = 0
    for n in range(idx_c.shape[0]):
        if not np.array_equal(idx_g[n], idx_c[n]):
            total, near = ulp_threshold_ties(o, n, idx_g[n], idx_c[n])
            assert total == near, "%s worker %d: %d index mismatches, only %d are 1-ulp threshold ties" % (
                label, n, total, near)
            tolerated += total
            print("REPORT %s worker %d: %d mismatching indices, all within 1 ulp of the threshold" % (label, n, total))
        else:
            _rel_close(val_g[n], val_c[n], "%s val[%d]" % (label, n))
        kn = idx_g.shape[1] if worker_k is None else int(worker_k[n])
        assert np.all(np.diff(idx_g[n, :kn].astype(np.int64)) > 0), "%s worker %d: indices not ascending" % (label, n)
        assert np.all(idx_g[n, kn:] == -1) and np.all(val_g[n, kn:] == 0), "%s worker %d: rest of the row" % (label, n)
    if tolerated == 0:
        _rel_close(agg_g, agg_c, label + " agg")
    return tolerated


def run_both(N, d, k, mu, grads_fn, T, device="cuda:0", force_dense=False, closed_loop=None,
             label="", check_state_every=1, cand_target=None, weights=None, check_overlap=False,
             on_round=None, grad_dtype=None, prior_roots=0, likelihood=0, worker_k=None, prior_exponent=None):
    """grads_fn(t, agg_prev_or_None) -> [N,d] float32 tensor on the GPU.

    Each side feeds its own aggregate back as g^{t-1}.  Returns per-round stats
    of the HIP path.  `weights`: aggregation weights omega_n for both sides;
    `check_overlap`: also compare the mask-overlap counts of every round;
    `on_round(t, res_gpu, res_cpu)`: hook after the comparison of round t;
    `worker_k`: entries kept per worker (a list, or a function t -> list applied
    before round t) for both sides;
    `grad_dtype`: torch.bfloat16 (or a function t -> dtype) rounds the generated
    gradients to bfloat16 first and hands the HIP path the 16-bit tensor, the
    oracle the same values widened to binary32.
    """
    dev = torch.device(device)
    o = orc.Oracle(N, d, k, mu)
    r = binding.RegTopk(N, d, k, mu, device=dev)
    if force_dense:
        r.set_option(binding.OPT_FORCE_DENSE, 1)
    if cand_target is not None:
        r.set_option(binding.OPT_CAND_TARGET, cand_target)
    if prior_roots or likelihood:
        o.set_score_variant(prior_roots, likelihood)
        r.set_option(binding.OPT_PRIOR_ROOTS, prior_roots)
        r.set_option(binding.OPT_LIKELIHOOD, likelihood)
    if prior_exponent is not None:
        o.set_prior_exponent(prior_exponent)
        r.set_option(binding.OPT_PRIOR_EXPONENT, float(np.float32(prior_exponent)))
    if weights is not None:
        o.set_weights(np.asarray(weights, dtype=np.float32))
        r.set_weights([float(np.float32(x)) for x in weights])
    agg_g = None
    agg_c = None
    stats = []
    tolerated = 0
    kn_now = None
    for t in range(T):
        kn_t = worker_k(t) if callable(worker_k) else (worker_k if t == 0 else None)
        if kn_t is not None:
            kn_now = [int(x) for x in kn_t]
            o.set_worker_k(kn_now)
            r.set_worker_k(kn_now)
        g = grads_fn(t, agg_g)
        assert g.is_cuda and g.dtype == torch.float32
        dt = grad_dtype(t) if callable(grad_dtype) else grad_dtype
        if dt is not None and dt != torch.float32:
            g = g.to(dt).contiguous()
        g_host = g.float().cpu().numpy()
        res_g = r.step(g, agg_g)
        torch.cuda.synchronize(dev)
        res_c = o.step(g_host, agg_c)
        st = r.stats()
        stats.append(st)
        tolerated += compare_round(o, res_g, res_c, "%s round %d" % (label, t), worker_k=kn_now)
        if check_overlap:
            ov_g = r.mask_overlap().cpu().numpy()
            assert np.array_equal(ov_g, o.mask_overlap()), "%s round %d: mask overlap %s vs %s" % (
                label, t, ov_g, o.mask_overlap())
        if on_round is not None:
            on_round(t, res_g, res_c)
        agg_g = res_g[2].clone()
        agg_c = res_c[2]
        if check_state_every and (t % check_state_every == 0 or t == T - 1) and tolerated == 0:
            e_g, pidx, pval, tt = r.get_state()
            torch.cuda.synchronize(dev)
            assert tt == t + 1
            e_c = o.e
            _rel_close(e_g.cpu().numpy(), e_c, "%s round %d eps" % (label, t))
            assert np.array_equal(pidx.cpu().numpy(), res_c[0])
    r.close()
    o.close()
    return stats, tolerated
