"""HCCS (Head-Calibrated Clipped-Linear Softmax) for gfx950: HIP kernels behind
a C ABI, and a thin Python binding.  Importing the package loads nothing; the
binding opens the shared library on first use and raises if it is missing."""
__all__ = ["binding", "synth"]
