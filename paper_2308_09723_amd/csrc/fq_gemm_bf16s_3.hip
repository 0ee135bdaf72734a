// Instantiation of the product kernels for bf16 activations with bf16 scales and 3-bit codes.
#include "fq_gemm_dispatch.h"

FQ_INSTANTIATE_GEMM(2, 3)
