// Instantiation of the product kernels for fp16 activations and 3-bit codes.
#include "fq_gemm_dispatch.h"

FQ_INSTANTIATE_GEMM(0, 3)
