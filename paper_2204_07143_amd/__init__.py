"""MI355X-native 2D Neighborhood Attention: HIP kernels behind a C ABI, plus a thin binding.

Importing the package does not load the GPU library; ``paper_2204_07143_amd.binding``
loads ``libna2d.so`` on first use and raises if it has not been built.
"""
__all__ = ["binding", "synth", "build"]
