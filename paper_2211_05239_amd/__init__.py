"""MI355X-native RecD deduplicated-embedding hot path (HIP kernels behind a C ABI).

Importing the package does not load the HIP library; `paper_2211_05239_amd.recd` does, and it
fails loudly when the library has not been built.
"""
