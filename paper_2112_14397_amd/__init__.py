"""MI355X-native DTS-Gate MoE layer (EvoMoE, arXiv 2112.14397): HIP kernels behind a C ABI.

Importing the package does not load the HIP library; `paper_2112_14397_amd.binding`
does, and fails loudly if it has not been built.
"""
__all__ = ["binding"]
