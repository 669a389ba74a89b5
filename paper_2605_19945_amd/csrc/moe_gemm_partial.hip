// Instantiations of the grouped GEMM kernel for reduction splits of the second expert GEMM (fp32 partial sums).
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(partial, EPI_PARTIAL_F32, false)
