"""W4A4 quantized linear layer for MI355X: HIP kernels behind a C ABI (libw4a4.so).

`binding` is the ctypes face of the library; `synth` draws the seeded synthetic
workloads; `build` compiles the library with hipcc.  Importing this package does not
load the library: `binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["binding", "synth", "build"]
