"""MI355X-native FP8 hot path of LoKA-style low-precision linear layers.

`binding` exposes the C ABI of libloka.so (include/loka.h); `synth` draws the seeded
synthetic workloads; `build` compiles the HIP sources.  Importing the package does
not load the library: `binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["binding", "synth", "build"]
