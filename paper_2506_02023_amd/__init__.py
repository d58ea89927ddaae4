"""MI355X-native graph-partitioned inference of a radial message-passing interatomic potential.

The compute path is the HIP library libmlip.so (csrc/, C ABI in include/mlip.h); this package is
its thin ctypes binding.  There is no CPU or PyTorch fallback: importing the binding's functions
and calling them without the built library raises ImportError.
"""
from .binding import (MODE_SLABS, MODE_WHOLE, PRECISION_BF16, PRECISION_FP32, PRECISION_FP32_SPLIT, BondWeights, Graph, MlipError, TorchAllocator, Weights, lib,  # noqa: F401
                      mlip_build_graph, mlip_forward, mlip_forward_bonds, mlip_forward_static)
