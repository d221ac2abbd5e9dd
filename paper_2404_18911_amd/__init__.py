"""MI355X-native hot path of Kangaroo self-speculative decoding (batch-1 draft-and-verify loop).

Sub-modules:
  inputs   seeded synthetic weights / prompts / uniforms (no model arithmetic; serves tests, bench and oracle drivers)
  binding  thin ctypes binding over the C-ABI library libkangaroo.so (HIP kernels for gfx950)
  build    hipcc build of the library

Nothing is imported eagerly so that `inputs` can be used without the HIP library being present.
"""
__all__ = ["inputs", "binding", "build"]
