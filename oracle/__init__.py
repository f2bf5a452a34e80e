"""CPU oracle for the vector-quantised matrix-vector path (TEST INFRASTRUCTURE).

Only tests, the smoke check and the bench's CPU-baseline leg may import this
package.  It shares no code with the GPU library and never calls it.
"""
from .vq_oracle import (  # noqa: F401
    VQFormat, bits_per_value, canonical_sizes, unpack_indices, decode_dense,
    gemv, gemm, decode_element, normwise_rel_err, dequantise_codebooks, canonical_sizes_i8,
    em_assign, em_update, em_objective, apply_block_scales, canonical_sizes_bn,
    read_tables_i8, read_tables_bn, gemv_lora,
)
