"""ocn: a strided n-dimensional tensor engine for AMD MI355X (gfx950).

Elementwise unary/binary operations, type-casting copies, axis/full reductions and reductions
of an elementwise result (inner products, norms, counts) over strided, broadcast and reversed views, after the Ocean Tensor Package (arXiv 1810.08723).
All computation happens in hand-written HIP kernels behind the C ABI of include/ocn.h; this
package only marshals arguments.
"""
from .binding import (BINARY_OPS, DTYPES, REDUCE_OPS, STRICT_TYPES, UNARY_OPS, OcnError, Tensor,
                      binary, binary_reduce, binary_reduce_workspace_bytes, cast_copy, domain_check, dtype_size,
                      gather, index_offsets, mask_offsets, scatter,
                      plan_binary, plan_binary_reduce, plan_reduce, plan_unary, promote, reduce,
                      reduce_scratch, reduce_workspace_bytes, unary, unary_mode)

__all__ = ["BINARY_OPS", "DTYPES", "REDUCE_OPS", "STRICT_TYPES", "UNARY_OPS", "OcnError", "Tensor",
           "binary", "binary_reduce", "binary_reduce_workspace_bytes", "cast_copy", "domain_check", "dtype_size",
           "gather", "index_offsets", "mask_offsets", "scatter",
           "plan_binary", "plan_binary_reduce", "plan_reduce", "plan_unary", "promote", "reduce",
           "reduce_scratch", "reduce_workspace_bytes", "unary", "unary_mode"]
