// Instantiations of the grouped GEMM kernel for the router-logit GEMM (high + low bf16 term of Wg, fp32 out).
#define MOE_GEMM_NO_TALL_TILE
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(pairsum, EPI_PAIR_SUM_F32, false)
