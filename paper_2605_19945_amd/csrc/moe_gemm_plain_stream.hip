// Instantiations of the grouped GEMM kernel for the second expert GEMM (down projection), weight loads with the non-temporal hint.
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(plain_stream, EPI_PLAIN, true)
