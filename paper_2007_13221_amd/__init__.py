"""MI355X-native CSER optimizer update (arxiv 2007.13221): HIP kernels behind a C ABI.

`binding` loads the compiled library (paper_2007_13221_amd/libcser_hip.so) on first use and
raises if it is missing; there is no CPU fallback.  `inputs` only describes workloads and
draws seeded synthetic tensors.
"""
__all__ = ["binding", "inputs", "build"]
