"""MI355X-native per-layer optimizer step (fused k-way gradient accumulation, global
gradient-norm reduction, AdamW with bf16 weight emission) behind a C-ABI HIP library.

Sub-modules:
  gs      -- thin ctypes binding of the C ABI declared in include/gs.h (loads the HIP library;
             importing it fails loudly if the library has not been built)
  inputs  -- seeded synthetic workloads (no arithmetic of the method)
  build   -- hipcc build of the library for gfx950
"""
__all__ = ["gs", "inputs", "build"]
