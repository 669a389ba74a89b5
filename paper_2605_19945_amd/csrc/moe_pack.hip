// Load-time repacking of the expert weights (the analogue of the paper's deployment step, which
// places each expert's weights on its GPU once, Sec. 3.3.4).  Not on the hot path.
//
// Packed layout (bf16), MFMA-fragment order: [ W13f : E_local x 2f/32 x d/16 x 64 x 8 ]
//                                            [ W2f  : E_local x d/32  x f/16 x 64 x 8 ]
//   Wf[e][nb][kc][l][j] = (packed weight row 32*nb + l%32, reduction element 16*kc + 8*(l/32) + j)
// where packed row n of W13 is column c = 32*(n/64) + n%32 of W1 (n%64 < 32) or of W3 (n%64 >= 32)
// -- gate and up projection interleaved in blocks of 32 columns, so that one 32x32 accumulator pair
// of the first GEMM holds both for the same (row, column) -- and packed row c of W2f is column c of
// W2.  One (nb, kc) fragment is the 1 KB a wavefront loads for one MFMA operand.
#include "moe_internal.h"

// in [K][C] (per expert, K = reduction index) ->
//   out[e][nb][k / 16][l][j] = in[e][16*(k/16) + 8*(l/32) + j][c],   c = cb*32 + l % 32,
// where nb = cb (plain) or 2*cb + slot (gate/up interleave: even row blocks W1, odd row blocks W3).
__global__ __launch_bounds__(256) void fragment_pack_kernel(const uint16_t* __restrict__ in, int K, int C,
                                                            uint16_t* __restrict__ out, int n_blocks /* per expert */,
                                                            int interleave, int slot) {
    __shared__ uint16_t tile[64][66];  // [k][c]
    const int e = blockIdx.z;
    const int c0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const uint16_t* src = in + (size_t)e * K * C;
    for (int kk = ty; kk < 64; kk += 4) tile[kk][tx] = src[(size_t)(k0 + kk) * C + c0 + tx];
    __syncthreads();
    // 2 column blocks x 4 K chunks = 8 fragments of 64 lanes x 8 elements
    for (int frag = ty; frag < 8; frag += 4) {
        const int cb = frag >> 2, kc = frag & 3, l = tx;
        const int nb_plain = c0 / 32 + cb;
        const int nb = interleave ? 2 * nb_plain + slot : nb_plain;
        uint16_t* dst = out + (((size_t)e * n_blocks + nb) * (K / 16) + (k0 / 16 + kc)) * 512 + l * 8;
        uint16_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = tile[kc * 16 + 8 * (l >> 5) + j][cb * 32 + (l & 31)];
        u32x4_t o;
        o.x = v[0] | ((uint32_t)v[1] << 16);
        o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16);
        o.w = v[6] | ((uint32_t)v[7] << 16);
        *(u32x4_t*)dst = o;
    }
}

hipError_t launch_pack_experts(const uint16_t* W1, const uint16_t* W3, const uint16_t* W2, int E_local, int d,
                               int f, uint16_t* packed, hipStream_t st) {
    uint16_t* w13f = packed;
    uint16_t* w2f = packed + (size_t)E_local * 2 * f * d;
    dim3 g13(f / 64, d / 64, E_local), g2(d / 64, f / 64, E_local);
    hipLaunchKernelGGL(fragment_pack_kernel, g13, dim3(256), 0, st, W1, d, f, w13f, 2 * f / 32, 1, 0);
    hipLaunchKernelGGL(fragment_pack_kernel, g13, dim3(256), 0, st, W3, d, f, w13f, 2 * f / 32, 1, 1);
    hipLaunchKernelGGL(fragment_pack_kernel, g2, dim3(256), 0, st, W2, f, d, w2f, d / 32, 0, 0);
    return hipGetLastError();
}
