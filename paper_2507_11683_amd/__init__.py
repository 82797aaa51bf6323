"""MI355X-native index-batched snapshot construction (PGT-I, arXiv 2507.11683).

`paper_2507_11683_amd.pgti` is the Python binding of the C-ABI HIP library (argument
marshalling only); `paper_2507_11683_amd.workloads` generates the seeded synthetic inputs.
Importing the package itself loads neither, so input generation works without a GPU.
"""
__version__ = "0.1.0"
