"""MI355X-native GXPO active-step update engine.

`paper_2605_06755_amd.binding` is the thin ctypes layer over the C-ABI library
(`libgxpo.so`, hand-written HIP for gfx950); importing it fails loudly when
the library has not been built.  `paper_2605_06755_amd.synth` holds the seeded
synthetic workloads.  Nothing is imported eagerly here so that CPU-only tools
can use `synth` without the GPU library.
"""
__all__ = ["binding", "synth", "build"]
