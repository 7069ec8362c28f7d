"""CPU-only sanitizer runs over everything here that executes on the host: the C oracle (AddressSanitizer +
UndefinedBehaviorSanitizer over every entry point, then its pins once more under UBSan) and the host side of
the HIP library (size queries and argument validation of every entry point, ASan + UBSan).  GPU code is not
instrumented (device sanitizers are not available on the machines this runs on)."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "paper_2506_07900_amd", "_build", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-4000:], r.stderr[-4000:])
    return r


def test_oracle_entry_points_under_asan_and_ubsan():
    if shutil.which("gcc") is None:
        pytest.skip("no host C compiler")
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_san")
    run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp",
         "-ffp-contract=off", os.path.join(ROOT, "oracle", "infllmv2_oracle.c"), os.path.join(SAN, "oracle_san.c"),
         "-o", exe, "-lm"])
    r = run([exe], env=ENV, timeout=600)
    assert "oracle_san ok" in r.stdout


def test_oracle_pins_under_ubsan():
    # the same pins as tests/test_oracle_pins.py, over a UBSan build of the oracle: a report aborts the run
    env = dict(ENV, INFLLMV2_ORACLE_SANITIZE="undefined")
    r = run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
             os.path.join(ROOT, "tests", "test_oracle_pins.py")], env=env, cwd=ROOT, timeout=1200)
    assert " passed" in r.stdout and "failed" not in r.stdout


def test_library_host_code_under_asan_and_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no hipcc")
    from paper_2506_07900_amd import build as hip_build
    os.makedirs(OUT, exist_ok=True)
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                "-fno-sanitize-recover=all"]
    flags = [f for f in hip_build.FLAGS if f != "-O3"] + ["-O1", "-g"] + host_san
    objs = [os.path.join(OUT, s[:-4] + ".o") for s in hip_build.SOURCES]
    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(lambda so: run([hipcc] + flags + ["-c", os.path.join(hip_build.CSRC, so[0]), "-o", so[1]]),
                      zip(hip_build.SOURCES, objs)))
    lib = os.path.join(OUT, "libinfllmv2_san.so")
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
         "-fno-gpu-sanitize"] + objs + ["-o", lib])
    exe = os.path.join(OUT, "abi_san")
    run([clang, "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "abi_san.c"), "-o", exe,
         "-L", OUT, "-l:libinfllmv2_san.so", "-L", "/opt/rocm/lib", "-lamdhip64",
         "-Wl,-rpath," + OUT, "-Wl,-rpath,/opt/rocm/lib"])
    r = run([exe], env=ENV, timeout=300)
    assert "abi_san ok" in r.stdout
