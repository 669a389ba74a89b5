// Router: logits = x * Wg (+ bias) on the matrix cores, top-k per token in one wavefront,
// softmax over the selected logits, per-expert counts.
//
// The paper describes the router in one sentence (it picks a few of the experts per token, Sec. 2.1)
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

// Resident-path layout (moe_router_resident): [16][d], rows 0..7 the high terms of experts 0..7, rows
// 8..15 their low terms (zero rows for experts >= E): one 16-row MFMA block carries both terms.
__global__ void pack_router_resident_kernel(const float* __restrict__ Wg, int d, int E, uint16_t* __restrict__ rp) {
    size_t n = (size_t)8 * d;
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        int e = (int)(o / d), i = (int)(o % d);
        float v = e < E ? Wg[(size_t)i * E + e] : 0.f;
        uint16_t hi = f32_to_bf16_rne(v);
        rp[o] = hi;
        rp[n + o] = f32_to_bf16_rne(v - bf16_to_f32(hi));
    }
}

// GEMM-path layout (E >= MOE_ROUTER_GEMM_MIN_E), MFMA-fragment order like the expert weights:
//   rp[nb][kt][4*q + a][l][j] = term ((n / 32) % 2) of Wg[64*kt + 32*q + 8*(l/16) + j][32*(n/64) + n%32],
//   n = 64*nb + 16*a + l%16
// (packed rows in blocks of 32: term 0 = high bf16 part, term 1 = low part of the same 32 experts; experts
// padded to a multiple of 32 with zeros).
__global__ void pack_router_gemm_kernel(const float* __restrict__ Wg, int d, int E, int Ep,
                                        uint16_t* __restrict__ rp) {
    const size_t n = (size_t)(2 * Ep / 64) * (d / 64) * 8 * 64;  // 16-byte chunks
    for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        const int l = (int)(o % 64);
        const int frag = (int)((o / 64) % 8), q = frag >> 2, a = frag & 3;
        const int kt = (int)((o / 512) % (d / 64));
        const int nb = (int)(o / 512 / (d / 64));
        const int prow = 64 * nb + 16 * a + (l & 15);
        const int e = 32 * (prow / 64) + (prow & 31), term = (prow >> 5) & 1;
        uint16_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int i = 64 * kt + 32 * q + 8 * (l >> 4) + j;
            const float x = e < E ? Wg[(size_t)i * E + e] : 0.f;
            const uint16_t hi = f32_to_bf16_rne(x);
            v[j] = term == 0 ? hi : f32_to_bf16_rne(x - bf16_to_f32(hi));
        }
        u32x4_t qv;
        qv.x = v[0] | ((uint32_t)v[1] << 16);
        qv.y = v[2] | ((uint32_t)v[3] << 16);
        qv.z = v[4] | ((uint32_t)v[5] << 16);
        qv.w = v[6] | ((uint32_t)v[7] << 16);
        *(u32x4_t*)(rp + o * 8) = qv;
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
    if (moe_router_resident(E, d)) {
        hipLaunchKernelGGL(pack_router_resident_kernel, dim3((8 * d + 255) / 256), dim3(256), 0, st, Wg, d, E, rp);
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

// ---- wave-wide selection ------------------------------------------------------------------------
// Maximum of an unsigned value over the 64 lanes with data-parallel-primitive moves (register
// crossbar, no LDS traffic): an inclusive "max scan" inside each row of 16 lanes, then the row
// results are folded into lane 63.  Lanes without a source take the identity 0.
static __device__ inline uint32_t wave_max_u32(uint32_t v) {
#define DPP_MAX(ctrl, row_mask)                                                                      \
    {                                                                                                \
        uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, row_mask, 0xf, false);   \
        v = o > v ? o : v;                                                                           \
    }
    DPP_MAX(0x111, 0xf)  // row_shr:1
    DPP_MAX(0x112, 0xf)  // row_shr:2
    DPP_MAX(0x114, 0xf)  // row_shr:4
    DPP_MAX(0x118, 0xf)  // row_shr:8   -> lane 15 of every row holds the row maximum
    DPP_MAX(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
    DPP_MAX(0x143, 0xc)  // row_bcast:31 into rows 2 and 3 -> lane 63 holds the wave maximum
#undef DPP_MAX
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
// Sum over lanes 0..15 (the first row), returned to all lanes.
static __device__ inline float row0_sum_f32(float v) {
#define DPP_ADD(ctrl) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, 0xf, 0xf, false));
    DPP_ADD(0x111) DPP_ADD(0x112) DPP_ADD(0x114) DPP_ADD(0x118)
#undef DPP_ADD
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
}

// Top-k of the E logits a wavefront holds as order-preserving keys (lane l keeps the keys of experts
// l, l + 64, ...; 0 = no expert): k rounds of a wave-wide maximum, the larger logit wins, equal
// logits go to the lower expert index.  Slot j's expert and logit end up in lane j; then the softmax
// over the k selected logits (slot 0 holds the largest).  Returns the gate weight of lane < k.
template <int EPL>
static __device__ inline float wave_topk_softmax(uint32_t (&key)[EPL], int k, int lane, int& my_e) {
    float my_val = 0.f;
    my_e = 0;
    for (int j = 0; j < k; ++j) {
        uint32_t bv = key[0];
        int bq = 0;
#pragma unroll
        for (int q = 1; q < EPL; ++q)
            if (key[q] > bv) {  // strict: ties keep the lower expert of this lane
                bv = key[q];
                bq = q;
            }
        const uint32_t m = wave_max_u32(bv);
        // the lowest expert index among the lanes that hold the maximum: lowest q first, then lowest lane
        int e_sel = -1;
#pragma unroll
        for (int q = 0; q < EPL; ++q) {
            const unsigned long long mask = __ballot(bv == m && bq == q);
            if (e_sel < 0 && mask != 0ull) e_sel = q * 64 + (int)__builtin_ctzll(mask);
        }
#pragma unroll
        for (int q = 0; q < EPL; ++q)
            if (e_sel == lane + 64 * q) key[q] = 0u;  // remove the winner
        if (lane == j) {
            my_e = e_sel;
            my_val = float_from_order_bits(m);
        }
    }
    const float l0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_val), 0));
    const float ex = lane < k ? expf(my_val - l0) : 0.f;
    return ex / row0_sum_f32(ex);  // k <= 16: all selected logits sit in the first row of lanes
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

    // ---- top-k and gate weights: one wavefront per token ------------------------------------------
    for (int t = wave; t < ROUTE_TOK; t += NW) {
        if (t0 + t >= T) break;  // wave-uniform
        uint32_t key[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + 64 * i;
            key[i] = e < E ? float_order_bits(logit[t * (R + 1) + e]) : 0u;
        }
        int my_e;
        const float gate = wave_topk_softmax<EPL>(key, k, lane, my_e);
        if (lane < k) {
            size_t o = (size_t)(t0 + t) * k + lane;
            idx[o] = my_e;
            w[o] = gate;
            atomicAdd(&hist[my_e], 1);
        }
    }
    __syncthreads();
    if (counts == nullptr) return;  // the caller counts the assignments itself
    for (int e = tid; e < E; e += NW * 64)
        if (hist[e] != 0) atomicAdd(&counts[e], hist[e]);
}


// Small routers (E <= 8, d a multiple of 512 up to 4096): a persistent kernel, one workgroup of 16
// wavefronts per compute unit.  Each wavefront keeps the router fragments of its slice of the
// reduction dimension in registers for the whole launch and streams 16-token groups past them
// (the next group's activations are in flight while the current one is reduced and ranked), so
// the router matrix is read once per workgroup instead of once per 16 tokens.  Per-expert counts are
// accumulated per workgroup and summed by the last workgroup to finish (ticket in ws[0], partial
// counts behind it): no zeroing launch, no spinning.
constexpr int RR_NW = 16, RR_MAXS = 8, RR_MAX_GRID = 256;
__global__ __launch_bounds__(RR_NW * 64) void route_resident_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ rp, const float* __restrict__ bias, int T, int d,
    int E, int k, int32_t* __restrict__ idx, float* __restrict__ w, int32_t* __restrict__ counts,
    int32_t* __restrict__ ws) {
    __shared__ float part[RR_NW][16][17];  // [wave][router row][token]
    __shared__ float logit[ROUTE_TOK][9];  // [token][expert]
    __shared__ int32_t hist[8];
    __shared__ int32_t is_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int steps = d / (32 * RR_NW);  // K steps of 32 per wavefront, <= RR_MAXS
    const int groups = (T + ROUTE_TOK - 1) / ROUTE_TOK;
    if (tid < 8) hist[tid] = 0;
    // fetched up front: read where it is added, it would be one more memory round trip behind the reduction
    const float bias_mine = (bias != nullptr && tid < 8 * ROUTE_TOK && (tid >> 4) < E) ? bias[tid >> 4] : 0.f;

    const size_t koff = (size_t)wave * steps * 32 + 8 * (lane >> 4);
    bf16x8_t wf[RR_MAXS], xf[RR_MAXS], xn[RR_MAXS];
#pragma unroll
    for (int s = 0; s < RR_MAXS; ++s)
        if (s < steps) wf[s] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(rp + (size_t)(lane & 15) * d + koff + s * 32));
    auto load_group = [&](int g, bf16x8_t* dst) {
        int tok = g * ROUTE_TOK + (lane & 15);
        if (tok >= T) tok = T - 1;  // clamp: rows past T are computed and dropped
        const uint16_t* xrow = x + (size_t)tok * d + koff;
#pragma unroll
        for (int s = 0; s < RR_MAXS; ++s)
            if (s < steps) dst[s] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(xrow + s * 32));
    };
    int g = blockIdx.x;
    if (g < groups) load_group(g, xf);
    for (; g < groups; g += gridDim.x) {
        const int gn = g + gridDim.x;
        if (gn < groups) load_group(gn, xn);
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < RR_MAXS; ++s)
            if (s < steps) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[s], xf[s], acc, 0, 0, 0);
        // accumulator element v of lane l is (router row 4 * (l / 16) + v, token l % 16)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave][4 * (lane >> 4) + v][lane & 15] = acc[v];
        __syncthreads();
        if (tid < 8 * ROUTE_TOK) {
            const int e = tid >> 4, t = tid & 15;
            float s = 0.f;
#pragma unroll
            for (int ww = 0; ww < RR_NW; ++ww) s += part[ww][e][t] + part[ww][e + 8][t];  // high + low term
            s += bias_mine;
            logit[t][e] = s;
        }
        __syncthreads();
        // top-k: one wavefront per token (same keys and tie-break as route_kernel)
        const int t = wave, tok = g * ROUTE_TOK + t;
        if (tok < T) {
            uint32_t key[1] = {lane < E ? float_order_bits(logit[t][lane]) : 0u};
            int my_e;
            const float gate = wave_topk_softmax<1>(key, k, lane, my_e);
            if (lane < k) {
                const size_t o = (size_t)tok * k + lane;
                idx[o] = my_e;
                w[o] = gate;
                atomicAdd(&hist[my_e], 1);
            }
        }
#pragma unroll
        for (int s = 0; s < RR_MAXS; ++s) xf[s] = xn[s];
    }
    if (counts == nullptr) return;  // (kernel argument, uniform) the caller counts the assignments itself
    __syncthreads();
    // per-workgroup counts -> workspace; the last workgroup to arrive sums them.  Device-scope
    // atomics only (they are performed at the memory side, past the per-XCD L2s): the partial counts
    // are exchanged in and their returns awaited before the ticket is taken, so no device-wide fence
    // (an L2 write-back that costs more than the whole kernel) is needed.
    if (tid < 8) {
        int old = __hip_atomic_exchange(&ws[1 + blockIdx.x * 8 + tid], hist[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("" ::"v"(old));  // the exchange has been performed once its return value is here
    }
    __syncthreads();
    if (tid == 0) is_last = __hip_atomic_fetch_add(&ws[0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1;
    __syncthreads();
    if (is_last) {
        // all threads fetch the partial counts side by side (the loads bypass the caches; one thread
        // walking them one after the other would take longer than the rest of the kernel)
        if (tid < 8) hist[tid] = 0;
        __syncthreads();
        const int n = (int)gridDim.x * 8;
        int s = 0;
        for (int i = tid; i < n; i += RR_NW * 64)  // i % 8 == tid % 8: every thread sums one expert
            s += __hip_atomic_load(&ws[1 + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (s != 0) atomicAdd(&hist[tid & 7], s);
        __syncthreads();
        if (tid < E) counts[tid] = hist[tid];
        if (tid == 0) __hip_atomic_store(&ws[0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    }
}

// Top-k / softmax / counts from fp32 logits in global memory (the GEMM router path): one wavefront
// per token, same keys and tie-break as route_kernel.  Counts go to TOPK_SUB sub-counters per expert
// (picked by workgroup) so that the atomics on one address stay few; reduce_counts_kernel folds them
// into counts[] and leaves them zero for the next call.
constexpr int TOPK_SUB = 32;
template <int EPL>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int ldl, int nsplit,
                                                   const float* __restrict__ bias, int T, int E, int k,
                                                   int32_t* __restrict__ idx, float* __restrict__ w,
                                                   int32_t* __restrict__ sub_counts) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x * 4 + wave;
    if (t >= T) return;  // wave-uniform
    uint32_t key[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
        const int e = lane + 64 * j;
        key[j] = 0u;
        if (e < E) {
            // partial logits of the split reduction, added in slab order
            float v = logits[(size_t)t * ldl + e];
            for (int sp = 1; sp < nsplit; ++sp) v += logits[((size_t)sp * T + t) * ldl + e];
            if (bias != nullptr) v += bias[e];
            key[j] = float_order_bits(v);
        }
    }
    int my_e;
    const float gate = wave_topk_softmax<EPL>(key, k, lane, my_e);
    if (lane < k) {
        const size_t o = (size_t)t * k + lane;
        idx[o] = my_e;
        w[o] = gate;
        if (sub_counts != nullptr) atomicAdd(&sub_counts[(blockIdx.x % TOPK_SUB) * E + my_e], 1);
    }
}

__global__ __launch_bounds__(256) void reduce_counts_kernel(int32_t* __restrict__ sub_counts, int E,
                                                            int32_t* __restrict__ counts) {
    const int e = threadIdx.x;
    if (e >= E) return;
    int s = 0;
#pragma unroll 8
    for (int i = 0; i < TOPK_SUB; ++i) {
        s += sub_counts[i * E + e];
        sub_counts[i * E + e] = 0;
    }
    counts[e] = s;
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
                        int32_t* idx, float* w, int32_t* counts, float* logits_ws, int logits_slabs,
                        TileDesc* table_ws, int* table_T, int32_t* route_ws, hipStream_t st) {
    if (moe_router_resident(E, d)) {
        const int groups = (T + ROUTE_TOK - 1) / ROUTE_TOK;
        const int grid = groups < RR_MAX_GRID ? groups : RR_MAX_GRID;
        hipLaunchKernelGGL(route_resident_kernel, dim3(grid), dim3(RR_NW * 64), 0, st, x, rp, bias, T, d, E, k, idx, w,
                           counts, route_ws);
        return hipGetLastError();
    }
    hipError_t err;
    if (E >= MOE_ROUTER_GEMM_MIN_E) {
        // logits on the tiled GEMM kernel (reduction over d, two bf16 terms of Wg), then top-k
        const int Ep = moe_router_cols(E);
        int nsplit = 1;
        err = launch_router_gemm(x, rp, T, d, 2 * Ep, logits_ws, Ep, logits_slabs, &nsplit, table_ws, table_T, st);
        if (err != hipSuccess) return err;
        const int blocks = (T + 3) / 4;
        const int epl = (E + 63) / 64;
        int32_t* sub = counts != nullptr ? route_ws + MOE_ROUTE_WS_SUBCOUNTS : nullptr;
        if (epl <= 1) hipLaunchKernelGGL(topk_kernel<1>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, nsplit, bias, T, E, k, idx, w, sub);
        else if (epl == 2) hipLaunchKernelGGL(topk_kernel<2>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, nsplit, bias, T, E, k, idx, w, sub);
        else hipLaunchKernelGGL(topk_kernel<4>, dim3(blocks), dim3(256), 0, st, logits_ws, Ep, nsplit, bias, T, E, k, idx, w, sub);
        if (counts != nullptr) hipLaunchKernelGGL(reduce_counts_kernel, dim3(1), dim3(256), 0, st, sub, E, counts);
        return hipGetLastError();
    }
    if (counts != nullptr) hipLaunchKernelGGL(zero_i32_kernel, dim3((E + 255) / 256), dim3(256), 0, st, counts, E);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
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
