"""Build step: compile the HIP sources under csrc/ into libinfllmv2.so for gfx950 with hipcc.

Run as `python -m paper_2506_07900_amd.build`.  hipcc cross-compiles, so no GPU is needed."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libinfllmv2.so")
SOURCES = ["api.hip", "compress_keys.hip", "select_prefill.hip", "select_prefill16.hip", "attn_prefill.hip", "attn_bwd.hip", "decode.hip", "noalloc.hip", "probes.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # packed fp32 VALU forms are kept out of the generated code on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results go to ordinary vector registers: the softmax arithmetic consumes them
         # directly, with no copies out of the accumulation registers
         "-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("hipcc failed with exit code %d" % res.returncode)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
