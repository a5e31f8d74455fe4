"""LFPS decode-step hot path for MI355X (gfx950): hand-written HIP kernels behind a C ABI
(include/lfps.h, liblfps.so) with a thin ctypes binding.  Importing `binding` loads the
shared library and fails if it has not been built; there is no CPU path."""

__all__ = ["binding", "build"]
