"""Tucker-attention forward pass for MI355X (gfx950): hand-written HIP kernels behind a
C-ABI library, plus a thin ctypes binding.  Importing the package loads nothing; the
binding loads the shared library on first use and fails loudly if it is missing."""

__all__ = ["workloads", "binding"]
