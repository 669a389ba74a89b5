// Load-time repacking of the expert weights (the analogue of the paper's deployment step, which
// places each expert's weights on its GPU once, Sec. 3.3.4).  Not on the hot path.
//
// Packed layout (bf16), MFMA-fragment order: [ W13f : E_local x 2f/64 x d/64 x 8 x 64 x 8 ]
//                                            [ W2f  : E_local x d/64  x f/64 x 8 x 64 x 8 ]
//   Wf[e][nb][kt][4*q + a][l][j] = (packed weight row 64*nb + 16*a + l%16,
//                                   reduction element 64*kt + 32*q + 8*(l/16) + j)
// where packed row n of W13 is column c = 32*(n/64) + n%32 of W1 (n%64 < 32) or of W3 (n%64 >= 32)
// -- gate and up projection interleaved in blocks of 32 columns, so that the accumulators of one wavefront
// (64 packed rows) hold both for the same (row, column) -- and packed row c of W2f is column c of
// W2.  One fragment is the 1 KB a wavefront loads for one v_mfma_f32_16x16x32_bf16 operand; the eight
// fragments of a wavefront's 64 rows and one 64-element K step lie together, so every wavefront reads one
// sequential stream.
#include "moe_internal.h"

// in [K][C] (per expert, K = reduction index), one 64 x 64 tile per workgroup -> its eight fragments.
// Plain: packed row = column.  Gate/up interleave: column c goes to packed row 64*(c/32) + 32*slot + c%32
// (slot 0: W1, slot 1: W3).
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
    // 4 column blocks of 16 x 2 K halves = 8 fragments of 64 lanes x 8 elements
    for (int frag = ty; frag < 8; frag += 4) {
        const int cb = frag >> 1, q = frag & 1, l = tx;
        const int nb = interleave ? c0 / 32 + (cb >> 1) : c0 / 64;   // 64-row block of the packed rows
        const int a = interleave ? 2 * slot + (cb & 1) : cb;         // 16-row block inside it
        uint16_t* dst = out + ((((size_t)e * n_blocks + nb) * (K / 64) + k0 / 64) * 8 + (4 * q + a)) * 512 + l * 8;
        uint16_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = tile[q * 32 + 8 * (l >> 4) + j][cb * 16 + (l & 15)];
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
    hipLaunchKernelGGL(fragment_pack_kernel, g13, dim3(256), 0, st, W1, d, f, w13f, 2 * f / 64, 1, 0);
    hipLaunchKernelGGL(fragment_pack_kernel, g13, dim3(256), 0, st, W3, d, f, w13f, 2 * f / 64, 1, 1);
    hipLaunchKernelGGL(fragment_pack_kernel, g2, dim3(256), 0, st, W2, f, d, w2f, d / 64, 0, 0);
    return hipGetLastError();
}
