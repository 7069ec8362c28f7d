"""fp64 CPU oracle for InfLLM v2 block-sparse attention (MiniCPM4 report, section 2.1).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
cpu_baseline leg of the benchmark.  The product package never imports this.

`ref` is a thin ctypes wrapper around `infllmv2_oracle.c` (argument marshalling
only).  Arrays of bf16 values travel as numpy uint16 bit patterns.
"""
from . import ref  # noqa: F401
