"""CPU sanitizer leg: the oracle's C routines and the host side of the C ABI (argument checks, plans, kernel names)
run under AddressSanitizer and UndefinedBehaviorSanitizer.  No GPU is involved: the drivers under tests/sanitizer/
make only queries and calls that are rejected before any launch."""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", *SAN, "-static-libasan",
                           os.path.join(ROOT, "tests", "sanitizer", "oracle_driver.c"), os.path.join(ROOT, "oracle", "gemm_oracle.c"),
                           os.path.join(ROOT, "oracle", "transpose_oracle.c"), "-lm", "-o", exe])
    assert "ok" in _run(exe)


def test_host_dispatch_under_sanitizers(tmp_path):
    from paper_2506_09092_amd import build

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    # the library's other objects, as the build leaves them beside the library
    objs = [os.path.join(os.path.dirname(build.CSRC), "_build", src.replace(".hip", ".o")) for src in build.SOURCES if src != "api.hip"]
    newest_source = max(os.path.getmtime(p) for p in glob.glob(os.path.join(build.CSRC, "*")))
    if not all(os.path.exists(o) and os.path.getmtime(o) >= newest_source for o in objs):
        build.build_library()
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]          # the sanitizers instrument the host pass only
    api, drv, exe = str(tmp_path / "api_san.o"), str(tmp_path / "host_driver.o"), str(tmp_path / "host_driver")
    subprocess.check_call([hipcc, *build.HIPCC_FLAGS, "-O1", "-g", *host_san, "-c", os.path.join(build.CSRC, "api.hip"), "-o", api],
                          stderr=subprocess.DEVNULL)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host_san, "-I", os.path.join(ROOT, "include"), "-x", "c++", "-c",
                           os.path.join(ROOT, "tests", "sanitizer", "host_driver.cpp"), "-o", drv], stderr=subprocess.DEVNULL)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", api, drv, *objs, "-o", exe],
                          stderr=subprocess.DEVNULL)
    assert "ok" in _run(exe)
