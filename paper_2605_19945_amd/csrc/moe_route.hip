// Router: logits = x * Wg (+ bias) on the matrix cores, top-k per token in one wavefront,
// softmax over the selected logits, per-expert counts.
//
// The paper describes the router only as "selects a subset of experts for each token" (Sec. 2.1)
// and notes that its top-k output is where the expert-utilisation trace comes from (Sec. 3.3.1).
//
// Precision: x is bf16 (exact), Wg is fp32.  Wg is split once, at load time, into two bf16 terms
// hi = rne(Wg), lo = rne(Wg - hi); both products accumulate into the same fp32 MFMA accumulator,
// which leaves a relative weight error of 2^-18 -- far below the 1e-3 logit gap at which two
// implementations are expected to agree on the selected experts.
#include "moe_internal.h"

static __device__ inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static __device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// rp layout: [2 terms][R rows][d], row r < E holds column r of Wg, rows >= E are zero.
__global__ void pack_router_kernel(const float* __restrict__ Wg, int d, int E, int R,
                                   uint16_t* __restrict__ rp) {
    size_t n = (size_t)R * d;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        int r = (int)(o / d), i = (int)(o % d);
        float v = r < E ? Wg[(size_t)i * E + r] : 0.f;
        uint16_t hi = f32_to_bf16_rne(v);
        uint16_t lo = f32_to_bf16_rne(v - bf16_to_f32(hi));
        rp[o] = hi;
        rp[n + o] = lo;
    }
}

// GEMM-path layout (E >= MOE_ROUTER_GEMM_MIN_E), MFMA-fragment order like the expert weights:
//   rp[nb][kc][l][j] = term (nb % 2) of Wg[16*kc + 8*(l/32) + j][32*(nb/2) + l%32]
// (term 0 = high bf16 part, term 1 = low part; experts padded to a multiple of 32 with zeros).
__global__ void pack_router_gemm_kernel(const float* __restrict__ Wg, int d, int E, int Ep,
                                        uint16_t* __restrict__ rp) {
    const size_t n = (size_t)(2 * Ep / 32) * (d / 16) * 64;  // 16-byte chunks
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        const int l = (int)(o % 64);
        const int kc = (int)((o / 64) % (d / 16));
        const int nb = (int)(o / 64 / (d / 16));
        const int e = 32 * (nb / 2) + (l & 31), term = nb & 1;
        uint16_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = 16 * kc + 8 * (l >> 5) + j;
            const float x = e < E ? Wg[(size_t)i * E + e] : 0.f;
            const uint16_t hi = f32_to_bf16_rne(x);
            v[j] = term == 0 ? hi : f32_to_bf16_rne(x - bf16_to_f32(hi));
        }
        u32x4_t q;
        q.x = v[0] | ((uint32_t)v[1] << 16);
        q.y = v[2] | ((uint32_t)v[3] << 16);
        q.z = v[4] | ((uint32_t)v[5] << 16);
        q.w = v[6] | ((uint32_t)v[7] << 16);
        *(u32x4_t*)(rp + o * 8) = q;
    }
}

hipError_t launch_pack_router(const float* Wg, int d, int E, uint16_t* rp, hipStream_t st) {
    if (E >= MOE_ROUTER_GEMM_MIN_E) {
        int Ep = moe_router_cols(E);
        size_t n = (size_t)Ep * d / 4;
        int blocks = (int)((n + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(pack_router_gemm_kernel, dim3(blocks), dim3(256), 0, st, Wg, d, E, Ep, rp);
        return hipGetLastError();
    }
    int R = moe_router_rows(E);
    size_t n = (size_t)R * d;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(pack_router_kernel, dim3(blocks), dim3(256), 0, st, Wg, d, E, R, rp);
    return hipGetLastError();
}

// Order-preserving map float -> uint32 (larger float <=> larger unsigned).
static __device__ inline uint32_t float_order_bits(float v) {
    if (v == 0.f) v = 0.f;  // -0 and +0 compare equal; give them one key
    uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
static __device__ inline float float_from_order_bits(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

constexpr int ROUTE_TOK = 16;  // tokens per workgroup = N of the 16x16x32 MFMA

// NB: blocks of 16 packed router rows; NW: wavefronts per workgroup (they split the reduction).
template <int NB, int NW>
__global__ __launch_bounds__(NW * 64) void route_kernel(const uint16_t* __restrict__ x,
                                                        const uint16_t* __restrict__ rp,
                                                        const float* __restrict__ bias, int T, int d,
                                                        int E, int k, int32_t* __restrict__ idx,
                                                        float* __restrict__ w,
                                                        int32_t* __restrict__ counts) {
    constexpr int R = NB * 16;
    constexpr int EPL = (R + 63) / 64;  // logits per lane during selection
    extern __shared__ float smem[];
    float* part = smem;                               // [NW][R][16]
    float* logit = smem + NW * R * ROUTE_TOK;         // [16][R + 1]
    int32_t* hist = (int32_t*)(logit + ROUTE_TOK * (R + 1));  // [R]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * ROUTE_TOK;
    const uint16_t* rp_lo = rp + (size_t)R * d;

    for (int e = tid; e < R; e += NW * 64) hist[e] = 0;

    // ---- logits: MFMA 16x16x32, first operand = router rows (i), second = tokens (j) ----------
    // lane l feeds row/token (l % 16) with the 8 reduction elements starting at 8 * (l / 16).
    f32x4_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int steps = d / 32;
    const int per_wave = (steps + NW - 1) / NW;
    const int s_begin = wave * per_wave;
    const int s_end = min(steps, s_begin + per_wave);
    int tok = t0 + (lane & 15);
    if (tok >= T) tok = T - 1;  // clamp: rows past T are computed and dropped
    const uint16_t* xrow = x + (size_t)tok * d + 8 * (lane >> 4);
    const uint16_t* hrow = rp + (size_t)(lane & 15) * d + 8 * (lane >> 4);
    const uint16_t* lrow = rp_lo + (size_t)(lane & 15) * d + 8 * (lane >> 4);

#pragma unroll 8
    for (int s = s_begin; s < s_end; ++s) {
        bf16x8_t xf = __builtin_bit_cast(bf16x8_t, *(const uint4*)(xrow + s * 32));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            bf16x8_t hf = __builtin_bit_cast(bf16x8_t, *(const uint4*)(hrow + (size_t)nb * 16 * d + s * 32));
            bf16x8_t lf = __builtin_bit_cast(bf16x8_t, *(const uint4*)(lrow + (size_t)nb * 16 * d + s * 32));
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hf, xf, acc[nb], 0, 0, 0);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lf, xf, acc[nb], 0, 0, 0);
        }
    }
    // accumulator element v of lane l is (router row 4 * (l / 16) + v, token l % 16)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            part[(wave * R + nb * 16 + 4 * (lane >> 4) + v) * ROUTE_TOK + (lane & 15)] = acc[nb][v];
    __syncthreads();

    // ---- reduce the per-wave partial sums in a fixed order, add the bias ------------------------
    for (int o = tid; o < R * ROUTE_TOK; o += NW * 64) {
        int e = o / ROUTE_TOK, t = o % ROUTE_TOK;
        float s = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) s += part[(ww * R + e) * ROUTE_TOK + t];
        if (bias != nullptr && e < E) s += bias[e];
        logit[t * (R + 1) + e] = s;
    }
    __syncthreads();

    // ---- top-k: one wavefront per token, k rounds of a wave-wide maximum over 64-bit keys
    //      (order bits of the logit << 32 | ~expert): larger logit wins, then the lower index ----
    for (int t = wave; t < ROUTE_TOK; t += NW) {
        if (t0 + t >= T) break;  // wave-uniform
        unsigned long long key[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            int e = lane + 64 * i;
            key[i] = 0ull;
            if (e < E)
                key[i] = ((unsigned long long)float_order_bits(logit[t * (R + 1) + e]) << 32) |
                         (unsigned long long)(0xFFFFFFFFu - (uint32_t)e);
        }
        float my_val = 0.f;
        int my_e = 0;
        for (int j = 0; j < k; ++j) {
            unsigned long long best = key[0];
#pragma unroll
            for (int i = 1; i < EPL; ++i) best = key[i] > best ? key[i] : best;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                unsigned long long o = __shfl_xor(best, off, 64);
                best = o > best ? o : best;
            }
            uint32_t e_sel = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
#pragma unroll
            for (int i = 0; i < EPL; ++i)
                if ((int)e_sel == lane + 64 * i) key[i] = 0ull;  // remove the winner
            if (lane == j) {
                my_e = (int)e_sel;
                my_val = float_from_order_bits((uint32_t)(best >> 32));
            }
        }
        // softmax over the k selected logits (slot 0 holds the largest)
        float l0 = __shfl(my_val, 0, 64);
        float ex = lane < k ? expf(my_val - l0) : 0.f;
        float sum = ex;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane < k) {
            size_t o = (size_t)(t0 + t) * k + lane;
            idx[o] = my_e;
            w[o] = ex / sum;
            atomicAdd(&hist[my_e], 1);
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += NW * 64)
        if (hist[e] != 0) atomicAdd(&counts[e], hist[e]);
}

// Top-k / softmax / counts from fp32 logits in global memory (the GEMM router path): one wavefront
// per token, same key construction and tie-break as route_kernel.
template <int EPL>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int ldl,
                                                   const float* __restrict__ bias, int T, int E, int k,
                                                   int32_t* __restrict__ idx, float* __restrict__ w,
                                                   int32_t* __restrict__ counts) {
    __shared__ int32_t hist[64 * EPL];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int e = tid; e < 64 * EPL; e += 256) hist[e] = 0;
    __syncthreads();
    const int tokens_per_block = 16;
    for (int i = wave; i < tokens_per_block; i += 4) {
        const int t = blockIdx.x * tokens_per_block + i;
        if (t >= T) break;
        unsigned long long key[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            int e = lane + 64 * j;
            key[j] = 0ull;
            if (e < E) {
                float v = logits[(size_t)t * ldl + e];
                if (bias != nullptr) v += bias[e];
                key[j] = ((unsigned long long)float_order_bits(v) << 32) |
                         (unsigned long long)(0xFFFFFFFFu - (uint32_t)e);
            }
        }
        float my_val = 0.f;
        int my_e = 0;
        for (int j = 0; j < k; ++j) {
            unsigned long long best = key[0];
#pragma unroll
            for (int q = 1; q < EPL; ++q) best = key[q] > best ? key[q] : best;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                unsigned long long o = __shfl_xor(best, off, 64);
                best = o > best ? o : best;
            }
            uint32_t e_sel = 0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull);
#pragma unroll
            for (int q = 0; q < EPL; ++q)
                if ((int)e_sel == lane + 64 * q) key[q] = 0ull;
            if (lane == j) {
                my_e = (int)e_sel;
                my_val = float_from_order_bits((uint32_t)(best >> 32));
            }
        }
        float l0 = __shfl(my_val, 0, 64);
        float ex = lane < k ? expf(my_val - l0) : 0.f;
        float sum = ex;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane < k) {
            size_t o = (size_t)t * k + lane;
            idx[o] = my_e;
            w[o] = ex / sum;
            atomicAdd(&hist[my_e], 1);
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256)
        if (hist[e] != 0) atomicAdd(&counts[e], hist[e]);
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <int NB, int NW>
static hipError_t route_launch_t(const uint16_t* x, const uint16_t* rp, const float* bias, int T, int d,
                                 int E, int k, int32_t* idx, float* w, int32_t* counts, hipStream_t st) {
    constexpr int R = NB * 16;
    size_t smem = (size_t)(NW * R * ROUTE_TOK + ROUTE_TOK * (R + 1)) * sizeof(float) + R * sizeof(int32_t);
    int blocks = (T + ROUTE_TOK - 1) / ROUTE_TOK;
    hipLaunchKernelGGL((route_kernel<NB, NW>), dim3(blocks), dim3(NW * 64), smem, st, x, rp, bias, T, d, E,
                       k, idx, w, counts);
    return hipGetLastError();
}

hipError_t launch_route(const uint16_t* x, const uint16_t* rp, const float* bias, int T, int d, int E, int k,
                        int32_t* idx, float* w, int32_t* counts, float* logits_ws, TileDesc* table_ws,
                        hipStream_t st) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((E + 255) / 256), dim3(256), 0, st, counts, E);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (E >= MOE_ROUTER_GEMM_MIN_E) {
        // logits on the tiled GEMM kernel (reduction over d, two bf16 terms of Wg), then top-k
        const int Ep = moe_router_cols(E);
        err = launch_router_gemm(x, rp, T, d, 2 * Ep, logits_ws, Ep, table_ws, st);
        if (err != hipSuccess) return err;
        const int blocks = (T + 15) / 16;
        const int epl = (E + 63) / 64;
        if (epl <= 1) hipLaunchKernelGGL(topk_kernel<1>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, bias, T, E, k, idx, w, counts);
        else if (epl == 2) hipLaunchKernelGGL(topk_kernel<2>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, bias, T, E, k, idx, w, counts);
        else hipLaunchKernelGGL(topk_kernel<4>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, bias, T, E, k, idx, w, counts);
        return hipGetLastError();
    }
    int nb = moe_router_rows(E) / 16;
    switch (nb) {
        case 1: return route_launch_t<1, 16>(x, rp, bias, T, d, E, k, idx, w, counts, st);
        case 2: return route_launch_t<2, 8>(x, rp, bias, T, d, E, k, idx, w, counts, st);
        case 4: return route_launch_t<4, 4>(x, rp, bias, T, d, E, k, idx, w, counts, st);
        case 8: return route_launch_t<8, 4>(x, rp, bias, T, d, E, k, idx, w, counts, st);
        case 16: return route_launch_t<16, 2>(x, rp, bias, T, d, E, k, idx, w, counts, st);
        default: return hipErrorInvalidValue;
    }
}
