"""MI355X-native SEKA / AdaSEKA prefill attention: HIP kernels behind a C ABI, plus a thin binding.

Importing the package does not load the shared library; `paper_2603_01281_amd.binding`
does, and raises if it has not been built.
"""
__all__ = ["inputs", "binding", "build"]
