"""Pruned-FFT 3D convolutional layer for AMD MI355X (gfx950): HIP kernels behind a C ABI, plus a thin binding.

`workloads` (seeded synthetic layers) imports without the compiled library; `binding` loads
libznni.so on first use and raises if it is missing -- there is no CPU fallback.
"""
__all__ = ["workloads", "binding"]
