"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU needed):

  - the oracle's C part (oracle/gemm_i64.c) with a brute-force driver on small ragged shapes;
  - the library's C entry points: a build of the HIP sources whose *host* code is instrumented
    (the GPU code is not, and nothing is launched), driven by a C program that calls every entry point
    with arguments that fail validation or are no-ops, and the host-only planning queries over a grid
    of shapes.

Both drivers live in tests/sanitize/; a sanitizer report makes the run exit non-zero.
"""

import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23", UBSAN_OPTIONS="halt_on_error=1:exitcode=24",
           OMP_NUM_THREADS="4")


def _run(exe):
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, "exit %d\n%s\n%s" % (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_c_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_check")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    os.path.join(ROOT, "oracle", "gemm_i64.c"), os.path.join(SAN, "oracle_check.c"), "-o", exe], check=True)
    assert "oracle_check: ok" in _run(exe)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_library_host_code_under_sanitizers(tmp_path):
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2410_05265_amd", "csrc", "*.hip")))
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    flags = ["--offload-arch=gfx950", "-O1", "-g0", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", *san]
    objs = []
    procs = []
    for s in srcs:                       # (device code at -O1: this build is never run on a GPU)
        o = str(tmp_path / (os.path.basename(s) + ".o"))
        objs.append(o)
        procs.append(subprocess.Popen([HIPCC, *flags, "-c", s, "-o", o], stderr=subprocess.PIPE, text=True))
    for pr in procs:
        _, err = pr.communicate()
        assert pr.returncode == 0, err[-4000:]
    drv = str(tmp_path / "abi_check.o")
    subprocess.run(["gcc", "-O1", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c",
                    os.path.join(SAN, "abi_check.c"), "-o", drv], check=True)
    exe = str(tmp_path / "abi_check")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", *objs, drv, "-o", exe],
                   check=True)
    assert "abi_check: ok" in _run(exe)
    shutil.rmtree(tmp_path, ignore_errors=True)
