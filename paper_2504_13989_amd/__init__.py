"""MI355X-native online Hadamard rotate-and-quantize (arXiv 2504.13989 hot path).

`binding` wraps the C ABI of librotq.so (HIP kernels for gfx950); `workloads` holds the
seeded synthetic input generators; `build` compiles the library in-tree.
"""
from . import workloads  # noqa: F401
from .binding import (Hadamard, RotqError, dequantize_rotate, expand_limit, gbs_search, hadamard_build, next_order,  # noqa: F401
                      quant_error, quant_error_workspace, quantize, quantize_asym, rotate, rotate_quantize,
                      rotate_quantize_asym)
