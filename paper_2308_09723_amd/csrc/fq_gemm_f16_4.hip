// Instantiation of the product kernels for f16 activations and 4-bit codes.
#include "fq_gemm_dispatch.h"

FQ_INSTANTIATE_GEMM(0, 4)
