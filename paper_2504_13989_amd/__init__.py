"""MI355X-native online Hadamard rotate-and-quantize (arXiv 2504.13989 hot path).

`binding` wraps the C ABI of librotq.so (HIP kernels for gfx950); `workloads` holds the
seeded synthetic input generators; `build` compiles the library in-tree.
"""
from . import workloads  # noqa: F401
from .binding import (Hadamard, RotqError, hadamard_build, next_order, quant_error,  # noqa: F401
                      quant_error_workspace, rotate_quantize)
