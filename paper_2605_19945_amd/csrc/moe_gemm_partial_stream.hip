// Instantiations of the grouped GEMM kernel for reduction splits of the second expert GEMM (fp32 partial sums), weight loads with the non-temporal hint.
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(partial_stream, EPI_PARTIAL_F32, true)
