"""MI355X-native hot path of Oases (arXiv 2305.16121): one tensor-model-parallel rank's share of a
transformer layer, forward and backward, under the sub-batch schedule of Algorithm 1.

`binding` is a thin ctypes layer over the C ABI declared in include/oases.h; every step of the path
runs in the HIP kernels of csrc/.  There is no CPU fallback: importing `binding` fails if the
library has not been built (python paper_2305_16121_amd/csrc/build.py).
"""
