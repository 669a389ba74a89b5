// Instantiations of the grouped GEMM kernel for the first expert GEMM (gate/up projections + SwiGLU epilogue).
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(swiglu, EPI_SWIGLU, false)
