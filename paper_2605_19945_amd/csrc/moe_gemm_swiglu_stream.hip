// Instantiations of the grouped GEMM kernel for the first expert GEMM (gate/up projections + SwiGLU epilogue), weight loads with the non-temporal hint.
#include "moe_gemm_kernel.h"

MOE_GEMM_INSTANTIATE(swiglu_stream, EPI_SWIGLU, true)
