"""MI355X-native chunked model-state hot path (pack -> grad norm -> clip -> AdamW -> stream).

Sub-modules:
  binding  - ctypes face of libptchunk.so (same names as include/ptchunk.h)
  build    - hipcc build of the library for gfx950
  shapes   - tensor-size tables of the synthetic model states (integers only)
  synth    - seeded, counter-based input generators (no arithmetic of the method)

Nothing is loaded at import time; `binding` raises if the HIP library is missing.
"""
__all__ = ["binding", "build", "shapes", "synth"]
