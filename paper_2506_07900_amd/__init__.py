"""InfLLM v2 block-sparse attention (MiniCPM4 report, section 2.1) for MI355X / gfx950.

`paper_2506_07900_amd.binding` is the thin Python layer over the C-ABI library built
from `csrc/` (hand-written HIP kernels); `paper_2506_07900_amd.synth` draws the seeded
synthetic inputs.  Importing the package loads nothing: the HIP library is loaded on the
first call into `binding`, and a missing library is an error, never a fallback.
"""
__all__ = ["binding", "synth"]
