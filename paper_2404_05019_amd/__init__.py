"""MI355X-native ScMoE forward pass: hand-written HIP kernels behind a C ABI.

Importing the package loads nothing; `paper_2404_05019_amd.binding` loads the shared library
and raises when it has not been built (there is no CPU fallback).
"""
