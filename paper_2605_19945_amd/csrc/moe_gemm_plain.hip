// Instantiations of the grouped GEMM kernel for the second expert GEMM (down projection).
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(plain, EPI_PLAIN, false)
