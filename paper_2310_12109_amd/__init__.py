"""MI355X-native Monarch Mixer hot path: HIP kernels behind a C ABI plus a thin binding.

Importing the package does not load the HIP library; `paper_2310_12109_amd.binding`
does, and fails loudly when the library has not been built.
"""
