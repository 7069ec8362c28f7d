"""Builds tests/c_client/abi_client: a plain C99 client of the C ABI (no Python, no torch), linked against
the in-tree libinfllmv2.so and the HIP runtime.  Run by __graft_entry__.build(); the GPU tests run the binary."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BIN = os.path.join(HERE, "abi_client")
LIBDIR = os.path.join(ROOT, "paper_2506_07900_amd")


def build(verbose=False):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           os.path.join(HERE, "abi_client.c"), "-o", BIN,
           "-L", LIBDIR, "-l:libinfllmv2.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2506_07900_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("gcc failed with exit code %d" % res.returncode)
    return BIN


if __name__ == "__main__":
    print(build(verbose=True))
