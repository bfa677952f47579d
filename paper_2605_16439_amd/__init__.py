"""KVCapsule hot path for AMD MI355X: HIP kernels behind a C ABI, with a ctypes binding.

`kvcapsule` is the binding (loads libkvcapsule.so lazily and fails loudly when it is not
built), `synth` draws the seeded synthetic workloads, `build` compiles the library.
"""
__all__ = ["kvcapsule", "synth", "build"]
