"""CPU-side checks of the boundary: the C-ABI library loads and exports every
symbol the header declares; size queries (host logic) behave.  No GPU calls."""
import os
import re

import pytest

from paper_2501_05633_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build_library(verbose=False)
    return binding.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "regtopk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(regtopk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert "regtopk_create" in names and "regtopk_step" in names and "regtopk_destroy" in names
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.SYMBOLS) == names


def test_workspace_bytes_host_logic(lib):
    assert binding.workspace_bytes(0, 10, 1) == 0
    assert binding.workspace_bytes(2, 10, 11) == 0
    assert binding.workspace_bytes(2, 2 ** 31, 5) == 0
    small = binding.workspace_bytes(4, 10_000, 100)
    assert small >= 4 * 10_000 * 4 and small % 256 == 0
    # the target workload: state + outputs + candidates stay within a few GB
    big = binding.workspace_bytes(16, 25_600_000, 256_000)
    assert 16 * 25_600_000 * 4 < big < 3 * 16 * 25_600_000 * 4


def test_workspace_bytes_grows_with_k_and_never_wraps(lib):
    # the candidate capacity is a 32-bit slot count inside the kernels: for every k up to d = 2^31 - 1
    # the layout must be computed without wrapping (it once was 4k + 25 % truncated to 32 bits)
    N, d = 1, 2 ** 31 - 1
    ks = [1, 1000, 10 ** 6, 10 ** 8, 5 * 10 ** 8, 8 * 10 ** 8, 858_993_459, 858_993_460, 9 * 10 ** 8,
          10 ** 9, 2 ** 30, 2 ** 30 + 1, 2 * 10 ** 9, d - 1, d]
    sizes = [binding.workspace_bytes(N, d, k) for k in ks]
    assert all(b > 0 for b in sizes)
    assert all(b1 >= b0 for b0, b1 in zip(sizes, sizes[1:])), list(zip(ks, sizes))
    for k, b in zip(ks, sizes):
        # state, double-buffered index/value lists, and four words per slot of a candidate list that
        # holds at least the min(2k, d) entries of the dense selection
        assert b >= 4 * N * d + 16 * N * k + 16 * N * min(2 * k, d), (k, b)
    # k = d: every entry can be a candidate once; the arena stays a small multiple of the state
    assert sizes[-1] <= 12 * 4 * N * d
    for N, d in ((3, 4096 * 7 + 5), (16, 25_600_000), (4, 124_000_000), (5, 1), (2, 4096)):
        prev = 0
        for k in sorted({1, 2, d // 1000 + 1, d // 100 + 1, d // 10 + 1, d // 4, d // 4 + 1, d // 2 + 1, d - 1, d} - {0}):
            if k > d:
                continue
            b = binding.workspace_bytes(N, d, k)
            assert b >= prev and b >= 4 * N * d + 16 * N * k, (N, d, k, b)
            assert b <= 12 * 4 * N * d + (1 << 22) * N, (N, d, k, b)
            prev = b


def test_product_path_refuses_to_run_without_gpu(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        binding.RegTopk(2, 100, 5, 1.0)


def test_product_sources_do_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2501_05633_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "workloads.py", (dirpath, f)


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 and as C++ on its own
    import subprocess
    hdr = os.path.join(ROOT, "include", "regtopk.h")
    src = tmp_path / "use.c"
    src.write_text('#include "%s"\nint main(void) { regtopk_result r; (void)r; return regtopk_last_error() == 0; }\n' % hdr)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", str(src)])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", str(src)])
