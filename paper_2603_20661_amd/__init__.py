"""MI355X-native batched decoder inference (paged-KV GQA attention + dense projections).

Sub-modules:
  synth    seeded synthetic inputs (no model arithmetic; shared with the tests' CPU oracle)
  binding  ctypes binding of the C-ABI library declared in include/www.h (needs the built HIP library)
  build    compiles the HIP library for gfx950 with hipcc

Nothing is imported eagerly, so the input generator can be used without the GPU library.
"""
__all__ = ["synth", "binding", "build"]
