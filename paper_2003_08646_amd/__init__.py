"""liblance for AMD MI355X: quantized Winograd 3x3 convolution (LANCE, arXiv 2003.08646).

``binding`` wraps the C ABI of ``include/lance.h`` one to one; ``layer`` adds buffer management
on torch device memory; ``workloads`` names the seeded synthetic benchmark layers.
"""
from . import workloads  # noqa: F401  (no GPU, no library needed)

__all__ = ["workloads", "binding", "layer"]
