"""The tanh step of the HIP path against the oracle's, for EVERY binary32
argument from 0 up to beyond the saturation point (about 1.09e9 values), plus
arguments above it.  Both must be the correctly rounded binary32 tanh.  The
same for the erf step of the Gaussian likelihood (saturation at 3.9192)."""
import concurrent.futures as cf

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2501_05633_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _oracle_parallel(x: np.ndarray, threads=16, fn=None) -> np.ndarray:
    parts = np.array_split(x, threads)
    with cf.ThreadPoolExecutor(threads) as ex:      # ctypes releases the GIL
        outs = list(ex.map(fn or orc.tanh32_array, parts))
    return np.concatenate(outs)


def test_tanh_exhaustive_up_to_saturation():
    hi = int(np.float32(9.03).view(np.uint32))
    slab = 1 << 26
    mismatches = 0
    for lo in range(0, hi + 1, slab):
        n = min(slab, hi + 1 - lo)
        bits = torch.arange(lo, lo + n, dtype=torch.int64, device=DEV).to(torch.int32)
        x = bits.view(torch.float32)
        y = binding.tanh_f32(x).cpu().numpy()
        want = _oracle_parallel(x.cpu().numpy())
        bad = np.flatnonzero(y.view(np.uint32) != want.view(np.uint32))
        if bad.size:
            print("slab %#x: %d mismatches, first x=%r got=%r want=%r" % (
                lo, bad.size, x[int(bad[0])].item(), y[bad[0]], want[bad[0]]), flush=True)
        mismatches += bad.size
        print("slab %#x done" % lo, flush=True)
    assert mismatches == 0


def test_tanh_above_saturation_and_specials():
    x = torch.tensor([9.0109, 9.011, 9.02, 9.03, 10.0, 88.0, 1e10, 3.4e38, float("inf"), 0.0, 1e-45, 1e-38],
                     dtype=torch.float32, device=DEV)
    y = binding.tanh_f32(x).cpu().numpy()
    want = orc.tanh32_array(x.cpu().numpy())
    assert np.array_equal(y.view(np.uint32), want.view(np.uint32))
    assert y[4] == 1.0 and y[8] == 1.0 and y[9] == 0.0


def test_erf_exhaustive_up_to_saturation():
    hi = int(np.float32(3.93).view(np.uint32))
    slab = 1 << 26
    mismatches = 0
    for lo in range(0, hi + 1, slab):
        n = min(slab, hi + 1 - lo)
        bits = torch.arange(lo, lo + n, dtype=torch.int64, device=DEV).to(torch.int32)
        x = bits.view(torch.float32)
        y = binding.erf_f32(x).cpu().numpy()
        want = _oracle_parallel(x.cpu().numpy(), fn=orc.erf32_array)
        bad = np.flatnonzero(y.view(np.uint32) != want.view(np.uint32))
        if bad.size:
            print("erf slab %#x: %d mismatches, first x=%r got=%r want=%r" % (
                lo, bad.size, x[int(bad[0])].item(), y[bad[0]], want[bad[0]]), flush=True)
        mismatches += bad.size
        print("erf slab %#x done" % lo, flush=True)
    assert mismatches == 0


def test_erf_above_saturation_and_specials():
    x = torch.tensor([3.9192, 3.919206, 3.92, 3.93, 4.0, 10.0, 88.0, 1e10, 3.4e38, float("inf"), 0.0, 1e-45, 1e-38, 1e-20],
                     dtype=torch.float32, device=DEV)
    y = binding.erf_f32(x).cpu().numpy()
    want = orc.erf32_array(x.cpu().numpy())
    assert np.array_equal(y.view(np.uint32), want.view(np.uint32))
    assert y[0] < 1.0 and y[2] == 1.0 and y[9] == 1.0 and y[10] == 0.0


@pytest.mark.parametrize("y", [0.9, 0.75, 0.5, 1.0 / 3.0, 0.1, 0.999, 1e-3])
def test_power_on_a_dense_sample_of_all_positive_arguments(y):
    # the general-exponent prior |a|^y: every 37th binary32 bit pattern from 0 to the largest finite
    # value (57 million arguments per exponent, denormals included), plus the neighbourhood of 1
    y = float(np.float32(y))
    top = int(np.float32(3.4e38).view(np.uint32))
    slab = 1 << 30
    mismatches = 0
    for lo in range(0, top, slab):
        bits = torch.arange(lo, min(lo + slab, top), 37, dtype=torch.int64, device=DEV).to(torch.int32)
        x = bits.view(torch.float32)
        got = binding.pow_f32(x, y).cpu().numpy()
        xs = x.cpu().numpy()
        parts = np.array_split(xs, 16)
        with cf.ThreadPoolExecutor(16) as ex:
            want = np.concatenate(list(ex.map(lambda p: orc.prior_pow_array(p, y), parts)))
        bad = np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))
        if bad.size:
            print("y=%r slab %#x: %d mismatches, first x=%r got=%r want=%r" % (
                y, lo, bad.size, xs[bad[0]], got[bad[0]], want[bad[0]]), flush=True)
        mismatches += bad.size
        print("pow y=%r slab %#x done" % (y, lo), flush=True)
    one = int(np.float32(1.0).view(np.uint32))
    x = torch.arange(one - 200000, one + 200000, dtype=torch.int64, device=DEV).to(torch.int32).view(torch.float32)
    got = binding.pow_f32(x, y).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), orc.prior_pow_array(x.cpu().numpy(), y).view(np.uint32))
    assert mismatches == 0
