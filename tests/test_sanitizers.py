"""CPU jobs under sanitizers (host code only; GPU code cannot be sanitized on this pool).

1. The oracle, compiled with AddressSanitizer + UndefinedBehaviorSanitizer into a standalone program
   (tests/sanitize_oracle_main.c calls every exported function on small ragged shapes with exact-size heap buffers).
2. The oracle as a UBSan-instrumented shared library, with the oracle pin tests run against it in a child process.
3. The host side of the C ABI (csrc/api.hip: argument checks, workspace arithmetic, launch plans) compiled with
   -Xarch_host -fsanitize=address,undefined and driven through its refusal paths and host-only queries by a small
   program; no kernel is launched and no GPU is needed.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_C = os.path.join(ROOT, "oracle", "lrnnx_oracle.c")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-std=c99", "-Wall", *SAN, "-fopenmp", "-o", str(exe),
           os.path.join(ROOT, "tests", "sanitize_oracle_main.c"), ORACLE_C, "-lm"]
    subprocess.run(cmd, check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=dict(ENV, OMP_NUM_THREADS="4"), timeout=300)
    assert r.returncode == 0 and "sanitized oracle run ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]


def test_oracle_pins_against_a_ubsan_build(tmp_path):
    """The pins of tests/test_oracle_pins.py and the golden anchors, run against a UBSan build of the oracle library
    (UBSan needs no preloaded runtime, so the instrumented library loads into an ordinary Python)."""
    lib = tmp_path / "liblrnnx_oracle_ubsan.so"
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-fsanitize=undefined",
           "-fno-sanitize-recover=all", "-o", str(lib), ORACLE_C, "-lm"]
    subprocess.run(cmd, check=True)
    code = (
        "import sys, pytest\n"
        f"sys.path.insert(0, {ROOT!r})\n"
        "import oracle\n"
        f"oracle._LIB = {str(lib)!r}\n"          # newer than the source: build() keeps it
        "oracle._lib = None\n"
        f"sys.exit(pytest.main(['-q', '-x', '-p', 'no:cacheprovider', {os.path.join(ROOT, 'tests', 'test_oracle_pins.py')!r},"
        f" {os.path.join(ROOT, 'tests', 'test_oracle_golden.py')!r}]))\n"
    )
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=ENV, timeout=900, cwd=str(tmp_path))
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stdout + r.stderr


HIPCC = "/opt/rocm/bin/hipcc"
CSRC = os.path.join(ROOT, "paper_2602_08810_amd", "csrc")
OBJ = os.path.join(ROOT, "paper_2602_08810_amd", "_build")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_c_abi_host_paths_under_sanitizers(tmp_path):
    """api.hip's host code instrumented, linked with the library's other (uninstrumented) objects and a driver that
    walks the refusal paths and the host-only queries.  Needs the objects of a previous library build."""
    from paper_2602_08810_amd import build as _build
    others = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in _build.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in others):
        pytest.skip("library objects missing: run python -m paper_2602_08810_amd.build first")
    api_o = tmp_path / "api_san.o"
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    subprocess.run([HIPCC, *[f for f in _build.FLAGS if f != "-O3"], "-O1", "-g", *host_san, "-c",
                    os.path.join(CSRC, "api.hip"), "-o", str(api_o)], check=True, capture_output=True)
    drv_o = tmp_path / "drv.o"
    # the driver is plain host C++: g++ compiles it; hipcc only links (host sanitizer runtimes, no device sanitizer)
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", *SAN, "-c", os.path.join(ROOT, "tests", "sanitize_cabi_main.cpp"),
                    "-o", str(drv_o)], check=True, capture_output=True)
    exe = tmp_path / "cabi_san"
    subprocess.run([HIPCC, "--offload-arch=gfx950", *host_san, "-o", str(exe), str(drv_o), str(api_o), *others],
                   check=True, capture_output=True)
    # the HIP runtime's own start-up allocations are not ours to judge: no leak report
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300,
                       env=dict(ENV, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0"))
    assert r.returncode == 0 and "sanitized C ABI run ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
