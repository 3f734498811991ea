"""MI355X-native coalesced MoE-layer hot path (route -> permute -> grouped SwiGLU
expert GEMMs -> combine) behind a C-ABI library, with a thin ctypes binding.

Sub-modules:
  synth    seeded synthetic input generators (no MoE arithmetic; shared by tests/bench)
  build    hipcc driver that compiles csrc/ into libmoe.so for gfx950
  binding  ctypes marshalling onto the C-ABI entry points declared in include/moe.h

Nothing here falls back to a CPU implementation: if libmoe.so is missing or no GPU is
present, the binding raises.
"""

__all__ = ["synth", "build", "binding"]
