"""MI355X-native branched SwiGLU MLP forward (MLPMoE, Sec. 3.1-3.3).

Submodules:
    synth    seeded synthetic layer inputs (numpy only)
    build    hipcc build of the C-ABI library (gfx950)
    binding  ctypes binding of the C-ABI library; importing it loads the
             shared object and fails loudly if it has not been built

Nothing is imported eagerly, so that the input generators can be used without
the GPU library being present.
"""
__all__ = ["synth", "build", "binding"]
