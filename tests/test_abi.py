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
