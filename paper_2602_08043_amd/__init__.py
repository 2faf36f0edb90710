"""V-ABFT verified GEMM for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI.

  binding  - ctypes mirror of include/vabft.h (vabft_encode, vabft_threshold,
             vabft_gemm_verified, ...)
  session  - PyTorch-backed device buffers around those calls
  build    - in-tree hipcc build of libvabft.so

There is no CPU fallback: without the built library every call fails loudly.
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
