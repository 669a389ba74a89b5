// Device helpers shared by the grouped-GEMM kernels (gfx950 only): bf16 packing, the epilogues, the
// LDS swizzle, explicitly scheduled LDS reads and wait-count helpers.
#pragma once
#include <type_traits>
#include <utility>

#include "moe_internal.h"

static __device__ inline uint32_t pack2_bf16(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}
static __device__ inline float silu_f32(float g) { return g / (1.f + __expf(-g)); }

enum { EPI_PLAIN = 0, EPI_SWIGLU = 1, EPI_PAIR_SUM_F32 = 2 };

// Epilogue shared by the GEMM kernels.  Accumulator element v of lane l in block (a, b) is
//   weight row  a*32 + 8*(v/4) + 4*(l/32) + v%4,   token row  b*32 + l%32,
// so a lane owns 4 consecutive output columns of one token row per accumulator quad.
template <int FM, int FN, int TM, int TN, int EPI>
static __device__ inline void gemm_epilogue(f32x16_t (&acc)[FN][FM], const TileDesc& td, int Np,
                                            uint16_t* __restrict__ C, int ldc, int wm, int wn, int lane) {
    const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        const int trow = wm * TM + b * 32 + frow;
        if (trow >= td.rows) continue;
        uint16_t* crow = C + (size_t)(td.row0 + trow) * ldc;
        if constexpr (EPI == EPI_PAIR_SUM_F32) {
            // router logits: the even block holds the products with the high bf16 term of Wg, the odd
            // block those with the low term; their sum is stored as fp32 (C is a float matrix)
            float* frow_out = (float*)C + (size_t)(td.row0 + trow) * ldc;
#pragma unroll
            for (int a2 = 0; a2 < FN / 2; ++a2) {
                const int prow = td.n0 + wn * TN + a2 * 64;
                if (prow >= Np) continue;
                const int col = prow / 2 + 4 * fhalf;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4_t o;
#pragma unroll
                    for (int v = 0; v < 4; ++v) o[v] = acc[2 * a2][b][4 * q + v] + acc[2 * a2 + 1][b][4 * q + v];
                    *(f32x4_t*)(frow_out + col + 8 * q) = o;
                }
            }
        } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int a2 = 0; a2 < FN / 2; ++a2) {
                const int prow = td.n0 + wn * TN + a2 * 64;  // packed row of the gate block
                if (prow >= Np) continue;
                const int hcol = prow / 2 + 4 * fhalf;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float h[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        h[v] = silu_f32(acc[2 * a2][b][4 * q + v]) * acc[2 * a2 + 1][b][4 * q + v];
                    u32x2_t o;
                    o.x = pack2_bf16(h[0], h[1]);
                    o.y = pack2_bf16(h[2], h[3]);
                    *(u32x2_t*)(crow + hcol + 8 * q) = o;
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                const int col = td.n0 + wn * TN + a * 32;
                if (col >= Np) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u32x2_t o;
                    o.x = pack2_bf16(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]);
                    o.y = pack2_bf16(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                    *(u32x2_t*)(crow + col + 4 * fhalf + 8 * q) = o;
                }
            }
        }
    }
}

template <int CH>
static __device__ inline int swz_of(int r) {
    // LDS: 64 banks x 4 B; a ds_read_b128 is served 16 lanes (256 B) per cycle.  The 16 rows a
    // lane group reads at one logical chunk must land in 16 distinct 16-byte slots of a 256-byte
    // bank line: rows sharing a bank-line position (r mod (16/CH)) get distinct XOR masks.
    return (CH == 8) ? ((r >> 1) & 7) : ((r >> 2) & 3);
}

// ---- explicitly scheduled LDS reads -------------------------------------------------------------
// The compiler's own placement of ds_read / s_waitcnt leaves every MFMA group waiting for the LDS
// reads issued just before it.  For the software-pipelined K loop the reads are issued through
// inline asm (invisible to the compiler's wait-count pass) and waited for with exact counts:
// the LDS returns data in order, so "lgkmcnt(N)" = everything but the N newest reads has landed.
template <int OFF>
static __device__ inline bf16x8_t lds_read_b128(uint32_t byte_addr) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(byte_addr), "n"(OFF) : "memory");
    return __builtin_bit_cast(bf16x8_t, v);
}
static __device__ inline bf16x8_t lds_read_b128_rt(uint32_t byte_addr) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(byte_addr) : "memory");
    return __builtin_bit_cast(bf16x8_t, v);
}
template <int STRIDE, int... I>
static __device__ inline void lds_read_frags(bf16x8_t* f, uint32_t byte_addr, std::integer_sequence<int, I...>) {
    ((f[I] = lds_read_b128<I * STRIDE>(byte_addr)), ...);
}
template <int N>
static __device__ inline void wait_lgkmcnt() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
// makes the fragment "depend" on the preceding wait so that its consumers stay behind it
static __device__ inline void tie(bf16x8_t& f) { asm volatile("" : "+v"(f)); }

template <int N>
static __device__ inline void wait_vmcnt() {
    // s_waitcnt vmcnt(N) only: expcnt = 7, lgkmcnt = 15 are left unconstrained (gfx9 encoding)
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 0xF) | ((N >> 4) << 14));
}

