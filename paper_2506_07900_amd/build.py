"""Build step: compile the HIP sources under csrc/ for gfx950 with hipcc into
  libinfllmv2.so        the library (the entry points of include/infllmv2.h)
  libinfllmv2_bench.so  the same sources compiled with INFLLMV2_TIMING, plus per-kernel event timing and the
                        probe kernels (include/infllmv2_bench.h); loaded by bench.py only.

Run as `python -m paper_2506_07900_amd.build`.  hipcc cross-compiles, so no GPU is needed."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libinfllmv2.so")
BENCH_LIB = os.path.join(HERE, "libinfllmv2_bench.so")
SOURCES = ["api.hip", "compress_keys.hip", "select_prefill.hip", "select_prefill16.hip", "attn_prefill.hip",
           "attn_bwd.hip", "decode.hip", "noalloc.hip"]
BENCH_SOURCES = SOURCES + ["timing.hip", "probes.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 VALU forms are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results go to ordinary vector registers: the softmax arithmetic consumes them
         # directly, with no copies out of the accumulation registers
         "-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("hipcc failed with exit code %d: %s" % (res.returncode, " ".join(cmd[-3:])))


def build(verbose=False, jobs=None):
    """Compiles every source (always: no staleness check), one hipcc process per object, then links both
    libraries and moves them into place."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    units = [(s, [], os.path.join(OBJ, s[:-4] + ".o")) for s in SOURCES]
    units += [(s, ["-DINFLLMV2_TIMING"], os.path.join(OBJ, s[:-4] + ".bench.o")) for s in BENCH_SOURCES]
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda u: _run([hipcc] + FLAGS + u[1] + ["-c", os.path.join(CSRC, u[0]), "-o", u[2]], verbose),
                      units))
    for lib, objs in ((LIB, [u[2] for u in units if not u[1]]), (BENCH_LIB, [u[2] for u in units if u[1]])):
        tmp = lib + ".tmp%d" % os.getpid()
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp], verbose)
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
