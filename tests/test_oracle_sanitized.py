"""The CPU oracle and the host-side size logic of the HIP library under
AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; nothing here needs or
touches a GPU)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["g++", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", *SAN,
                           os.path.join(ROOT, "oracle", "sanitize_driver.cpp"),
                           os.path.join(ROOT, "oracle", "regtopk_oracle.cpp"), "-o", str(exe)])
    out = subprocess.run([str(exe)], env=ENV, capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "scenarios ok" in out.stdout


def test_oracle_long_double_has_a_64_bit_significand():
    # the oracle's tanh is "tanhl rounded once to binary32": correct rounding needs the x87 format
    import numpy as np
    assert np.finfo(np.longdouble).nmant >= 63


HOST_DRIVER = r'''
#include "regtopk.h"
#include <stdio.h>
int main(void) {
  /* the size logic over the whole admitted range: never 0, never shrinking, never wrapping */
  long bad = 0;
  const long long ds[] = {1, 5, 4096, 4097, 1000003, 25600000, 2147483647LL};
  for (int i = 0; i < 7; ++i) {
    size_t prev = 0;
    for (long long k = 1; k <= ds[i]; k = k * 3 + 1) {
      size_t b = regtopk_workspace_bytes(3, ds[i], k);
      if (b < prev || b == 0) ++bad;
      prev = b;
    }
    if (regtopk_workspace_bytes(3, ds[i], ds[i]) < prev) ++bad;
    if (regtopk_workspace_bytes(3, ds[i], ds[i] + 1) != 0) ++bad;
    if (regtopk_global_workspace_bytes(ds[i], ds[i]) != regtopk_workspace_bytes(1, ds[i], ds[i])) ++bad;
  }
  if (regtopk_workspace_bytes(0, 10, 1) != 0 || regtopk_workspace_bytes(65536, 10, 1) != 0 ||
      regtopk_workspace_bytes(1, 2147483648LL, 1) != 0) ++bad;
  /* argument checks that return before any GPU call */
  regtopk_ctx* c = 0;
  int rc[8];
  rc[0] = regtopk_create(&c, 0, 10, 1, 1.0f);
  rc[1] = regtopk_create(&c, 2, 10, 11, 1.0f);
  rc[2] = regtopk_create(0, 2, 10, 1, 1.0f);
  rc[3] = regtopk_create(&c, 2, 10, 1, -1.0f);
  rc[4] = regtopk_create_in(&c, 2, 10, 1, 1.0f, 0, 1 << 20, 0);
  rc[5] = regtopk_create_in(&c, 2, 10, 1, 1.0f, (void*)256, 16, 0);
  rc[6] = regtopk_set_option(0, 1, 1.0);
  rc[7] = regtopk_sgd_update(0, 0, 0.1f, -1, 0);
  for (int i = 0; i < 8; ++i) if (rc[i] >= 0) ++bad;
  if (regtopk_last_error()[0] == 0) ++bad;
  printf("host logic under sanitizers: bad=%ld\n", bad);
  return bad != 0;
}
'''


def test_host_logic_of_the_hip_library_under_asan_and_ubsan(tmp_path):
    # the library's host code (layout arithmetic, argument checks) compiled with the sanitizers on the
    # host side only; the driver never reaches a GPU call
    from paper_2501_05633_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("ROCm compilers not present")
    lib = tmp_path / "libregtopk_san.so"
    flags = [f for f in build.HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g"]
    for s in ("address", "undefined"):
        flags += ["-Xarch_host", "-fsanitize=" + s]
    subprocess.check_call([hipcc, *flags, *build.sources(), "-o", str(lib)], stderr=subprocess.DEVNULL)
    src = tmp_path / "driver.c"
    src.write_text(HOST_DRIVER)
    exe = tmp_path / "driver"
    subprocess.check_call([clang, "-fsanitize=address,undefined", "-g", "-I", os.path.join(ROOT, "include"), str(src),
                           str(lib), "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)])
    env = dict(ENV, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0")
    out = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "bad=0" in out.stdout
