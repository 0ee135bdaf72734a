"""CPU oracle for the fine-grained weight-only quantisation path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition of what
the GPU library computes.  It shares no code with the HIP path and neither
side imports the other.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.
"""
from .fq_oracle import (  # noqa: F401
    qmax_of,
    levels_of,
    group_absmax,
    scale_from_absmax,
    quantize,
    dequantize,
    gemm_ref,
    gemm_ref_grouped,
    choose_group,
    bits_per_weight,
    quant_error,
    bf16_scale_bits,
)
from .fq_oracle_int import (  # noqa: F401
    quantize_int_scales,
    dequantize_int_scales,
    quantize_activations_int8,
    gemm_ref_int,
)
