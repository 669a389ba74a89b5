// Grouped expert GEMMs on the gfx950 matrix cores -- the expert kernel the paper profiles in isolation
// (Sec. 3.3.2), whose latency over token count is the staircase GEM samples at tile boundaries.
//
//   GEMM1 + SwiGLU:  H[r, c] = silu(sum_i X[r,i] W1[e][i,c]) * (sum_i X[r,i] W3[e][i,c])
//   GEMM2:           Y[r, c] = sum_j H[r,j] W2[e][j,c]
// for the rows r of expert e (ragged, device-side counts), bf16 operands, fp32 accumulation.
// The router logits of large routers (E >= 32) run on the same kernel as one group.
//
// Design (CDNA4):
//   * work item = up to BM rows of ONE expert x 256 packed weight rows; the list of work items is
//     built on the device from the per-expert offsets (no host sync), experts with no rows get
//     none, row tiles have a run-time height (a multiple of 32 rows, the last one of an expert
//     possibly ragged: loads clamped, stores masked) -- no padding to the largest expert.
//   * v_mfma_f32_16x16x32_bf16 with the WEIGHT rows as the first operand and the TOKEN rows as the
//     second, so a lane's accumulator holds 4 consecutive output columns of one token row.  Under this
//     device's power limit the 16x16x32 shape sustains a higher clock than 32x32x16 (a quarter of the
//     accumulator registers read and written per flop): the same loop on 32x32x16 ran at 1.55 GHz and
//     1.28 PFLOP/s on the Mixtral shape, this one reaches 1.35.
//   * only the token rows go through LDS.  The weights are stored at load time in MFMA-fragment
//     order
//        Wf[e][n / 64][k / 64][4*q + a][lane][8],  lane l <-> packed weight row 64*(n/64) + 16*a + l % 16,
//                                                 reduction elements 64*(k/64) + 32*q + 8*(l/16) .. +8,
//     so a wavefront fetches one 16x32 operand fragment with ONE fully coalesced 1 KB load straight
//     into the registers the MFMA reads, two K steps ahead of its use (three register buffers), and the
//     eight fragments of its 64 weight rows for one K step are 8 KB in a row: one sequential stream per
//     wavefront (with a stream per row block the weight-streaming launches were 3 to 7 % slower).
//     The token rows are staged by global_load_lds into an NSX-deep LDS ring (XOR-swizzled 16-byte
//     chunks, see swz_of) and every wavefront multiplies ALL rows of the tile by its own 64 weight
//     rows (1 x 4 wave layout): no weight byte is loaded twice or touches LDS, and the LDS ring is
//     deep because it only holds the tokens (NSX-1 token stages and two weight stages, about
//     150 KB per compute unit, are in flight towards L2).
//   * one wavefront per SIMD (256 threads, up to 512 registers per lane, accumulators in AGPRs),
//     so all latency hiding is explicit: LDS fragment reads run one MFMA sub-step ahead, the
//     barrier that publishes stage kt+1 sits before the LAST sub-step of stage kt so that the first
//     fragments of the next stage are read under those MFMAs, and the loads of a K step are spread
//     one by one over its MFMA slots (bursts from four lockstep wavefronts overrun the compute
//     unit's single vector-memory pipe and stall MFMA issue).
//   * a K step of 64 is four sub-steps (K half q, token half th): the MFMAs of sub-step (q, th) multiply the
//     four 16-row weight blocks by the 16-row token blocks of half th, so the token fragments held in
//     registers at a time are those of half a tile.
//   * the tallest tile has 288 rows: 18 token blocks x 4 weight blocks of 4 accumulator registers: the 256
//     AGPRs hold sixteen token blocks, blocks 8 and 17 (the ninth of either half) accumulate in VGPRs.
//     Left to itself the compiler shuffles the 72 small accumulators between the two files inside the K
//     loop, so the tall tiles (256 and 288 rows) issue EVERY MFMA through inline asm with the register file
//     in the constraint (mfma_pinned_agpr / mfma_pinned_vgpr); what the compiler then no longer does for
//     these MFMAs -- keep writers of their operands and readers of their results at a distance -- the
//     kernel arranges itself and tests/test_isa_hazards.py checks on the compiled code.
//   * work items are ordered so that the workgroups running concurrently on one XCD share weight
//     panels through that XCD's L2, and so that each XCD's queue of work items is dense.
#pragma once
#include <stdlib.h>

#include <type_traits>
#include <utility>

#include "moe_internal.h"

// two floats rounded to nearest even and packed, a in the low half: one v_cvt_pk_bf16_f32
static __device__ inline uint32_t pack2_bf16(float a, float b) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// g * sigmoid(g) with the hardware reciprocal (1 ulp): an IEEE division costs about ten more instructions
// per element, 144 elements per lane and tile, all of them after the last MFMA
static __device__ inline float silu_f32(float g) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)); }

enum { EPI_PLAIN = 0, EPI_SWIGLU = 1, EPI_PAIR_SUM_F32 = 2, EPI_PARTIAL_F32 = 3 };

// Epilogues.  Accumulator element v of lane l in block (a, t) -- a: 16 packed weight rows, t: 16 token rows -- is
//   weight row  a*16 + 4*(l/16) + v,   token row  t*16 + l%16,
// so a lane owns 4 consecutive output columns of one token row per accumulator.  The wavefront's 64 packed
// weight rows are blocks a = 0..3; in the interleaved layouts (gate/up, high/low router term) rows 0..31 are
// the first and rows 32..63 the second member of the pair, i.e. block a pairs with block a + 2.
//
// Storage.  A tile of up to 256 rows keeps token block t in acc[.][t] (AGPRs).  The 288-row tile has 18 token
// blocks and 16 AGPR slots: when all nine 32-row blocks are valid (NINE), blocks 8 and 17 -- the last of either
// token half -- live in accv[.][0] and accv[.][1] (VGPRs) and the others close ranks; with fewer valid blocks
// everything fits the AGPR slots.  Every accumulator thus has ONE register file for the whole kernel: sharing
// a variable between an AGPR use in one case and a VGPR use in another makes the compiler keep it in one file
// and copy it around every MFMA of the other, right behind the MFMA that writes it.
template <int FT>
struct AccShape {
    static constexpr int NA = FT < 16 ? FT : 16;  // token blocks accumulating in AGPRs
    static constexpr int NV = FT > 16 ? FT - 16 : 1;  // in VGPRs (one unused slot keeps the type valid)
};
template <bool NINE, int FA, int NA, int NV>
static __device__ __forceinline__ const f32x4_t& acc_at(const f32x4_t (&acc)[FA][NA], const f32x4_t (&accv)[FA][NV],
                                                        int a, int t) {
    if (NINE) {
        if (t == 8) return accv[a][0];
        if (t == 17) return accv[a][NV - 1];
        return acc[a][t < 8 ? t : t - 1];
    }
    return acc[a][t < NA ? t : 0];  // (t >= NA is never reached at run time: fewer than nine valid blocks)
}

template <int FT, int FA, int TM, int TN, int EPI, bool NINE>
static __device__ inline void gemm_epilogue(const f32x4_t (&acc_)[FA][AccShape<FT>::NA],
                                            const f32x4_t (&accv_)[FA][AccShape<FT>::NV], const TileDesc& td, int Np,
                                            uint16_t* __restrict__ C, int ldc, int wm, int wn, int lane) {
    static_assert(FA == 4 && TN == 64, "wave tile");
    auto A = [&](int a, int t) -> const f32x4_t& {
        return acc_at<NINE, FA, AccShape<FT>::NA, AccShape<FT>::NV>(acc_, accv_, a, t);
    };
    const int frow = lane & 15, fq = lane >> 4;
#pragma unroll
    for (int t = 0; t < FT; ++t) {
        const int trow = wm * TM + t * 16 + frow;
        if (trow >= td.rows) continue;
        uint16_t* crow = C + (size_t)(td.row0 + trow) * ldc;
        const int prow = td.n0 + wn * TN;  // first packed weight row of this wavefront (Np is a multiple of 64)
        if (prow >= Np) continue;
        if constexpr (EPI == EPI_PAIR_SUM_F32) {
            // router logits: blocks 0, 1 hold the products with the high bf16 term of Wg, blocks 2, 3 those
            // with the low term of the same experts; their sum is stored as fp32 (C is a float matrix)
            float* frow_out = (float*)C + (size_t)(td.row0 + trow) * ldc;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                f32x4_t o;
#pragma unroll
                for (int v = 0; v < 4; ++v) o[v] = A(a, t)[v] + A(a + 2, t)[v];
                *(f32x4_t*)(frow_out + prow / 2 + 16 * a + 4 * fq) = o;
            }
        } else if constexpr (EPI == EPI_PARTIAL_F32) {
            // partial sums of a reduction split, fp32 (C is a float matrix, one slab per split)
            float* frow_out = (float*)C + (size_t)(td.row0 + trow) * ldc;
#pragma unroll
            for (int a = 0; a < FA; ++a) *(f32x4_t*)(frow_out + prow + 16 * a + 4 * fq) = A(a, t);
        } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                float h[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) h[v] = silu_f32(A(a, t)[v]) * A(a + 2, t)[v];
                u32x2_t o;
                o.x = pack2_bf16(h[0], h[1]);
                o.y = pack2_bf16(h[2], h[3]);
                *(u32x2_t*)(crow + prow / 2 + 16 * a + 4 * fq) = o;
            }
        } else {
#pragma unroll
            for (int a = 0; a < FA; ++a) {
                u32x2_t o;
                o.x = pack2_bf16(A(a, t)[0], A(a, t)[1]);
                o.y = pack2_bf16(A(a, t)[2], A(a, t)[3]);
                *(u32x2_t*)(crow + prow + 16 * a + 4 * fq) = o;
            }
        }
    }
}

// bf16 epilogues (EPI_PLAIN, EPI_SWIGLU) through LDS.  Stored straight from the accumulators, a wave-level
// store would write 16 bytes to each of 32 rows; instead every wavefront parks its 64 output columns (32 after SwiGLU) of all rows in its own quarter of
// the token ring, which nobody reads any more, and writes them back out row-contiguously: 16 bytes per
// lane, whole 128-byte (64-byte) runs per row.  Rows are ROWB bytes apart in LDS with the 16-byte chunks
// XOR-swizzled by row so that both the 8-byte writes (32 rows at one column) and the 16-byte reads (8 or
// 16 rows at all columns) are spread over the banks.  Worth 0.2 % (Mixtral shape, 64 to 224 K steps per
// tile) to 1.8 % (f = 768: 12 K steps per tile) of the layer time; most of the cost of the scattered
// stores was their completion, which the wavefronts never waited for.
// The caller has made sure that no wavefront still reads the ring.
template <int FT, int FA, int BM, int TN, int EPI, bool NINE>
static __device__ inline void gemm_epilogue_staged(const f32x4_t (&acc_)[FA][AccShape<FT>::NA],
                                                   const f32x4_t (&accv_)[FA][AccShape<FT>::NV], const TileDesc& td,
                                                   int Np, uint16_t* __restrict__ C, int ldc, int wn, int lane,
                                                   char* lds_base) {
    auto A = [&](int a, int t) -> const f32x4_t& {
        return acc_at<NINE, FA, AccShape<FT>::NA, AccShape<FT>::NV>(acc_, accv_, a, t);
    };
    static_assert(EPI == EPI_PLAIN || EPI == EPI_SWIGLU, "bf16 outputs");
    static_assert(FA == 4 && TN == 64, "wave tile");
    constexpr int OUTC = EPI == EPI_SWIGLU ? TN / 2 : TN;  // output columns of this wavefront per row
    constexpr int ROWB = OUTC * 2;                         // 128 or 64 bytes per row
    constexpr int NCH = ROWB / 16;                         // 16-byte chunks per row: 8 or 4
    char* stage = lds_base + wn * (BM * ROWB);
    const int frow = lane & 15, fq = lane >> 4;
    auto swz = [](int r) { return EPI == EPI_SWIGLU ? (r >> 2) & 3 : (r ^ (r >> 3)) & 7; };
#pragma unroll
    for (int t = 0; t < FT; ++t) {
        if (t * 16 >= td.rows) break;  // uniform
        const int r = t * 16 + frow;
        // the lane's 4 columns of block a start at byte 32*a + 8*fq of the row: chunk 2*a + fq/2, half fq%2
        char* srow = stage + r * ROWB + 8 * (fq & 1);
        const int x = swz(r);
        if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                float h[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) h[v] = silu_f32(A(a, t)[v]) * A(a + 2, t)[v];
                u32x2_t o;
                o.x = pack2_bf16(h[0], h[1]);
                o.y = pack2_bf16(h[2], h[3]);
                *(u32x2_t*)(srow + (((2 * a + (fq >> 1)) ^ x) << 4)) = o;
            }
        } else {
#pragma unroll
            for (int a = 0; a < FA; ++a) {
                u32x2_t o;
                o.x = pack2_bf16(A(a, t)[0], A(a, t)[1]);
                o.y = pack2_bf16(A(a, t)[2], A(a, t)[3]);
                *(u32x2_t*)(srow + (((2 * a + (fq >> 1)) ^ x) << 4)) = o;
            }
        }
    }
    // the wavefront reads back only what it wrote itself
    const int prow = td.n0 + wn * TN;  // first packed weight row of this wavefront
    if (prow >= Np) return;            // Np is a multiple of 64
    constexpr int RPI = 64 / NCH;      // rows per wave-level store
    const int ch = lane % NCH;
    uint16_t* cbase = C + (size_t)td.row0 * ldc + (EPI == EPI_SWIGLU ? prow / 2 : prow) + ch * 8;
    for (int r = lane / NCH; r < td.rows; r += RPI) {
        const u32x4_t v = *(const u32x4_t*)(stage + r * ROWB + ((ch ^ swz(r)) << 4));
        *(u32x4_t*)(cbase + (size_t)r * ldc) = v;
    }
}

template <int CH>
static __device__ inline int swz_of(int r) {
    // LDS: 64 banks x 4 B; a ds_read_b128 is served 16 lanes (256 B) per cycle.  The 16 rows a
    // lane group reads at one logical chunk must land in 16 distinct 16-byte slots of a 256-byte
    // bank line: rows sharing a bank-line position (r mod (16/CH)) get distinct XOR masks.
    static_assert(CH == 8, "128-byte staged rows");
    return (r >> 1) & 7;
}

// ---- explicitly scheduled LDS reads -------------------------------------------------------------
// The compiler's own placement of ds_read / s_waitcnt leaves every MFMA group waiting for the LDS
// reads issued just before it.  The reads of the software-pipelined K loop are issued through
// inline asm (invisible to the compiler's wait-count pass) and waited for explicitly.
template <int OFF>
static __device__ inline bf16x8_t lds_read_b128(uint32_t byte_addr) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(byte_addr), "n"(OFF) : "memory");
    return __builtin_bit_cast(bf16x8_t, v);
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


template <int... I, class F>
static __device__ inline void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
static __device__ inline void static_for(F&& f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Row tiles of more than 256 rows need more than the 256 accumulator registers (AGPRs) of a lane: two of
// the eighteen token blocks accumulate in ordinary VGPRs.  The MFMAs of the tall tiles are issued through
// inline asm that names the register file of the accumulator.  The asm is opaque to the compiler's hazard
// recogniser, which would otherwise keep a reader of an MFMA result, and a writer of an MFMA operand, the
// required wait states away: the caller places the VGPR ones first in a sub-step (the others follow before
// anything can read their result), reads accumulators only after the K loop, and claims the zeroed
// accumulators in their register file before the prologue (claim_agpr / claim_vgpr).
static __device__ inline void mfma_pinned_vgpr(f32x4_t& acc, const bf16x8_t& w, const bf16x8_t& x) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(w), "v"(x));
}
// the value exists in a register of that file from here on (see the use in gemm_tile)
static __device__ inline void claim_vgpr(f32x4_t& acc) { asm volatile("" : "+v"(acc)); }
static __device__ inline void claim_agpr(f32x4_t& acc) { asm volatile("" : "+a"(acc)); }
static __device__ inline void mfma_pinned_agpr(f32x4_t& acc, const bf16x8_t& w, const bf16x8_t& x) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(x));
}

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (the instruction takes an immediate)
static __device__ inline void wait_vmcnt_rt(int n) {
    switch (n) {
#define C(i) case i: wait_vmcnt<i>(); break;
        C(1) C(2) C(3) C(4) C(5) C(6) C(7) C(8) C(9) C(10) C(11) C(12) C(13) C(14) C(15) C(16) C(17) C(18)
        C(19) C(20) C(21) C(22) C(23) C(24) C(25) C(26) C(27) C(28) C(29) C(30) C(31) C(32)
#undef C
        default: wait_vmcnt<0>(); break;
    }
}

// Split K (gridDim.y > 1, used by the router-logit GEMM whose output is tiny next to its reduction
// length): workgroup (x, y) reduces over elements [y*K, (y+1)*K) of the K_total = gridDim.y * K long
// reduction dimension and writes its partial result c_split_bytes behind that of split y-1; the
// consumer adds the partial results in a fixed order.
// W_STREAM: the weight loads carry the non-temporal hint.  A launch in which every expert has a single row
// tile reads each weight once; plain loads then reach about 6.4 TB/s of the 8 TB/s HBM peak on this device and
// hinted ones about 7.2 TB/s (read-only streaming kernel, 1.9 GB).  Launches whose row tiles share weight
// panels through the L2 lose with the hint (Mixtral shape, 1024 rows per expert: +2.8 % time), so it is a
// variant picked per launch.
// gemm_tile: one work item (table entry bx) by one workgroup.
template <int BM, int NSX, int EPI, int NW, bool W_STREAM>
static __device__ __forceinline__ void gemm_tile(int bx, const uint16_t* __restrict__ X, int ldx,
                                                 const int32_t* __restrict__ row_map,
                                                 const uint16_t* __restrict__ Wf, int Np, int K,
                                                 uint16_t* __restrict__ C, int ldc,
                                                 const TileDesc* __restrict__ table, size_t c_split_bytes) {
    constexpr int BN = 64 * NW, BK = 64, TN = BN / NW, FA = TN / 16, FM = BM / 32, FT = 2 * FM;
    constexpr int CH = BK / 8;   // 16-byte chunks per staged token row
    constexpr int RPL = 64 / CH; // rows covered by one wave-level load
    constexpr int XP = 32 / (NW * RPL);  // wave-level token loads of one wavefront per 32-row block
    constexpr int KQ = BK / 32;  // K halves of a K step: one v_mfma_f32_16x16x32_bf16 reduces over 32 elements
    constexpr int KK = 2 * KQ;   // MFMA sub-steps per K step: (K half q, token half th), kk = 2*q + th
    constexpr int DX = NSX - 1;  // token prefetch distance (K steps)
    constexpr int WPF = 2;       // weight prefetch distance (K steps); WPF + 1 register buffers
    constexpr int WL = FA * KQ;  // weight loads per lane per K step
    constexpr int STAGE = BM * CH;            // 16-byte chunks per token stage
    constexpr int BLK = 16 * CH * 16;         // bytes between consecutive 16-row blocks in a stage
    static_assert(FA == 4 && KK == 4, "wave tile");
    static_assert(BM % 32 == 0 && FM >= 1 && FM <= 9, "row tile");
    static_assert(NW == 4 || NW == 2, "wavefronts per workgroup");
    static_assert(NSX >= 3 && (2 * FM * XP + WL) <= 48, "pipeline depth");

    extern __shared__ u32x4_t lds[];  // [NSX][STAGE]

    const TileDesc td = table[bx];
    if (td.rows <= 0) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane / CH, lphys = lane % CH;
    const int frow = lane & 15, fq = lane >> 4;
    const int KT = K / BK;
    const int fmv = (td.rows + 31) / 32;  // valid 32-row blocks: the same for all four wavefronts
    const int K_total = K * (int)gridDim.y;
    X += (size_t)blockIdx.y * K;
    C = (uint16_t*)((char*)C + (size_t)blockIdx.y * c_split_bytes);

    // token sources: pass p of a wavefront brings rows 8*(NW*p + wave) .. +8 of the tile (XP passes per
    // 32-row block), 32-bit byte offsets from the wave-uniform base X + kt*BK
    uint32_t xo[FM * XP];
#pragma unroll
    for (int p = 0; p < FM * XP; ++p) {
        const int r = (p * NW + wave) * RPL + lrow;
        const int rr = r < td.rows ? r : td.rows - 1;  // clamp: rows past the end are never stored
        int grow = td.row0 + rr;
        if (row_map != nullptr) grow = row_map[grow];
        xo[p] = (uint32_t)grow * (uint32_t)(ldx * 2) + (uint32_t)((lphys ^ swz_of<CH>(r)) * 16);
    }
    // weight source: the eight fragments a wavefront needs for one K step (4 row blocks x 2 K halves) are the
    // 8 KB at ((e*Np/64 + nb)*K/64 + kt)*8 KB, fragment j = 4*q + a at j KB: ONE sequential stream per
    // wavefront.  Wave-uniform base (scalar registers) plus the lane's 16 bytes.
    const int nbt = Np / 64;
    int nb = (td.n0 + wave * TN) / 64;
    if (nb >= nbt) nb = nbt - 1;  // past the last weight row: computed, never stored
    const char* wsrc = (const char*)(Wf + ((size_t)td.expert * nbt + nb) * ((size_t)K_total * 64) + (size_t)blockIdx.y * K * 64);
    const uint32_t wlane = (uint32_t)lane * 16u;
    // LDS byte address (inside a stage) of this lane's chunk of 16-row block 0 for either K half: token row
    // frow, reduction elements 32*q + 8*fq .. +8 (the swizzle of a row depends on row % 16 only)
    uint32_t fx_addr[KQ];
#pragma unroll
    for (int q = 0; q < KQ; ++q)
        fx_addr[q] = (uint32_t)((frow * CH + ((q * 4 + fq) ^ swz_of<CH>(frow))) * 16);

    // block (a, t): 16 packed weight rows x 16 token rows (storage: see AccShape)
    constexpr int NA = AccShape<FT>::NA, NV = AccShape<FT>::NV;
    f32x4_t acc[FA][NA], accv[FA][NV];
#pragma unroll
    for (int a = 0; a < FA; ++a) {
#pragma unroll
        for (int t = 0; t < NA; ++t) acc[a][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < NV; ++t) accv[a][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }

    auto main_loop = [&](auto fmv_c) {
        constexpr int FMV = decltype(fmv_c)::value;  // valid 32-row blocks (compile time)
        constexpr int NM = FMV * FA;                 // MFMAs per sub-step: FMV 16-row token blocks x 4 weight blocks
        constexpr int XV = FMV * XP;                 // token loads per lane per K step
        constexpr int NL = WL + XV;                  // loads per lane per K step

        bf16x8_t wr[WPF + 1][KQ][FA];
        bf16x8_t xf[2][FMV];  // sub-step (q, th): the 16-row token blocks th*FMV .. th*FMV + FMV - 1, K half q

        // The tall tiles issue every MFMA through inline asm (see mfma_pinned_agpr).  The compiler then does
        // not know that the first MFMA reads the accumulator it has just zeroed and would put the zeroing
        // writes directly in front of it, closer than the wait states a matrix instruction needs behind a
        // write of its third operand.  Claiming every accumulator here, in the register file its MFMAs use,
        // makes the zeros exist now; the prologue's loads, waits and barrier follow before the first MFMA.
        if constexpr (FM >= 8) {
            static_for<2 * FMV>([&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                static_for<FA>([&](auto a_c) {
                    constexpr int a = decltype(a_c)::value;
                    if constexpr (FMV == 9 && (t == 8 || t == 17)) {
                        claim_vgpr(accv[a][t == 8 ? 0 : NV - 1]);
                    } else {
                        claim_agpr(acc[a][FMV == 9 && t > 8 ? t - 1 : t]);
                    }
                });
            });
        }

        auto issue_x_one = [&](int kt, int p) {
            u32x4_t* base = lds + (kt % NSX) * STAGE;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)((const char*)(X + (size_t)kt * BK) + xo[p]),
                (__attribute__((address_space(3))) void*)(base + (p * NW + wave) * RPL * CH), 16, 0, 0);
        };
        // Weight loads go through inline asm: the compiler's own wait-count pass would otherwise put a
        // nearly-zero vmcnt in front of the MFMAs that consume them (it cannot see through the
        // unrolled, branched loop) and collapse the prefetch distance.  They are waited for together
        // with the token loads, with exact counts, before the barrier that precedes their use.
        auto load_w_one = [&](int kt, auto buf_c, auto j_c) {  // j = q * FA + a
            constexpr int BUF = decltype(buf_c)::value;
            constexpr int kk = decltype(j_c)::value / FA, a = decltype(j_c)::value % FA;  // kk: K half here
            u32x4_t v;
            const char* base = wsrc + (size_t)kt * (WL * 1024) + kk * (FA * 1024);  // (offsets reach 4 KB)
            if constexpr (W_STREAM) {
                asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt"
                             : "=v"(v)
                             : "v"(wlane), "s"(base), "n"(a * 1024)
                             : "memory");
            } else {
                asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3"
                             : "=v"(v)
                             : "v"(wlane), "s"(base), "n"(a * 1024)
                             : "memory");
            }
            wr[BUF][kk][a] = __builtin_bit_cast(bf16x8_t, v);
        };
        // prologue: weights of stages 0, 1 and tokens of stages 0 .. DX-1, oldest needs first
        static_for<WL>([&](auto j) { load_w_one(0, std::integral_constant<int, 0>{}, j); });
        static_for<XV>([&](auto p) { issue_x_one(0, p); });
        int after0 = 0;  // loads issued after those of stage 0
        if (1 < KT) {
            static_for<WL>([&](auto j) { load_w_one(1, std::integral_constant<int, 1>{}, j); });
            after0 += WL;
        }
#pragma unroll
        for (int s = 1; s < DX; ++s)
            if (s < KT) {
                static_for<XV>([&](auto p) { issue_x_one(s, p); });
                after0 += XV;
            }
        wait_vmcnt_rt(after0);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        static_for<FMV>([&](auto b) { xf[0][b] = lds_read_b128<b * BLK>(fx_addr[0]); });  // sub-step (0, 0)

        // one K step; BUF = kt % (WPF + 1) is a compile-time register-buffer index.  STEADY: the step
        // is neither among the first nor the last ones, so every prefetch of it exists and nothing
        // in it is conditional.
        auto step = [&](int kt, auto buf_c, auto steady_c) {
            constexpr int BUF = decltype(buf_c)::value;
            constexpr bool STEADY = decltype(steady_c)::value;
            constexpr int NBUF = (BUF + WPF) % (WPF + 1);  // buffer of stage kt + WPF
            const bool more_w = STEADY || kt + WPF < KT;
            const bool more_x = STEADY || kt + DX < KT;
            const bool next = STEADY || kt + 1 < KT;
            const uint32_t sbase = (uint32_t)((kt % NSX) * STAGE * 16);
            const uint32_t nbase = (uint32_t)(((kt + 1) % NSX) * STAGE * 16);
            // the weights of this stage landed before the barrier that published it
            static_for<WL>([&](auto j) { tie(wr[BUF][decltype(j)::value / FA][decltype(j)::value % FA]); });
            static_for<KK>([&](auto kk_c) {
                constexpr int kk = decltype(kk_c)::value;
                constexpr int cur = kk & 1, nxt = cur ^ 1;
                constexpr int q = kk >> 1, th = kk & 1;          // K half, token half of this sub-step
                constexpr int qn = (kk + 1) >> 1, thn = (kk + 1) & 1;  // of the next one (same K step)
                if constexpr (kk == KK - 1) {
                    // publish stage kt+1 before the last sub-step: own loads of stage kt+1 have landed
                    // (what may stay in flight: the tokens issued one step ago, after the weights of
                    // stage kt+1, and everything issued during this step), all wavefronts have issued
                    // and completed every LDS read of stage kt
                    if constexpr (STEADY) {
                        wait_vmcnt<WL + 2 * XV>();
                    } else {
                        int pending = (more_w ? WL : 0) + (more_x ? XV : 0);
                        if (kt >= 1) {
                            pending += kt - 1 + DX < KT ? XV : 0;
                        } else {
#pragma unroll
                            for (int s = 2; s < DX; ++s) pending += s < KT ? XV : 0;  // issued by the prologue
                        }
                        if (next) wait_vmcnt_rt(pending);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                } else {
                    wait_lgkmcnt<0>();
                }
                static_for<FMV>([&](auto b) { tie(xf[cur][b]); });
                __builtin_amdgcn_sched_barrier(0);
                static_for<NM>([&](auto m_c) {
                    constexpr int m = decltype(m_c)::value;
                    // a block that accumulates in VGPRs goes first: whatever reads its result next (the compiler may
                    // copy it at the end of a basic block) then sits behind the sub-step's other MFMAs
                    constexpr int a = m % FA;
                    constexpr int b = FMV <= 8 ? m / FA : (m / FA + 8) % 9;
                    constexpr int t = th * FMV + b;  // 16-row token block
                    if constexpr (b < 8) {
                        constexpr int slot = FMV == 9 && t > 8 ? t - 1 : t;
                        if constexpr (FM >= 8) mfma_pinned_agpr(acc[a][slot], wr[BUF][q][a], xf[cur][b]);
                        else acc[a][slot] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr[BUF][q][a], xf[cur][b], acc[a][slot], 0, 0, 0);
                    } else {
                        mfma_pinned_vgpr(accv[a][th == 0 ? 0 : NV - 1], wr[BUF][q][a], xf[cur][b]);
                    }
                    // first half of the slots: LDS reads of the next sub-step's token fragments, early
                    // enough that their latency is covered by the MFMAs of the second half
                    if constexpr (m < FMV) {
                        if constexpr (kk + 1 < KK) {
                            xf[nxt][m] = lds_read_b128<(thn * FMV + m) * BLK>(sbase + fx_addr[qn]);
                        } else {
                            if (next) xf[nxt][m] = lds_read_b128<m * BLK>(nbase + fx_addr[0]);
                        }
                    }
                    // the step's NL loads (weights of stage kt+WPF first, then tokens of stage kt+DX)
                    // are spread evenly over the MFMA slots of all sub-steps but the last: the four
                    // wavefronts run in lockstep, and bursts of back-to-back loads from all of them
                    // exceed what the compute unit's one vector-memory pipe takes per cycle
                    if constexpr (kk < KK - 1) {
                        constexpr int slot = kk * NM + m, S = (KK - 1) * NM;
                        static_for<NL>([&](auto i_c) {
                            constexpr int i = decltype(i_c)::value;
                            if constexpr ((i * S) / NL == slot) {
                                if constexpr (i < WL) {
                                    if (more_w) load_w_one(kt + WPF, std::integral_constant<int, NBUF>{}, std::integral_constant<int, i>{});
                                } else {
                                    if (more_x) issue_x_one(kt + DX, i - WL);
                                }
                            }
                        });
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        };
        using T_ = std::true_type;
        using F_ = std::false_type;
        using B0 = std::integral_constant<int, 0>;
        using B1 = std::integral_constant<int, 1>;
        using B2 = std::integral_constant<int, 2>;
        static_assert(WPF == 2, "the loops below rotate three weight buffers");
        // first step, then the steady steps three at a time, then whatever is left (generic)
        step(0, B0{}, F_{});
        int kt = 1;
        for (; kt + 2 + DX < KT; kt += 3) {
            step(kt, B1{}, T_{});
            step(kt + 1, B2{}, T_{});
            step(kt + 2, B0{}, T_{});
        }
        for (; kt < KT; kt += 3) {
            step(kt, B1{}, F_{});
            if (kt + 1 < KT) step(kt + 1, B2{}, F_{});
            if (kt + 2 < KT) step(kt + 2, B0{}, F_{});
        }
    };

    switch (fmv) {
#define CASE(n)                                                        \
    case n:                                                            \
        if constexpr (n <= FM) main_loop(std::integral_constant<int, (n <= FM ? n : 1)>{}); \
        break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9)
#undef CASE
        default: break;
    }

    if constexpr (EPI == EPI_PLAIN || EPI == EPI_SWIGLU) {
        static_assert(NSX >= 4, "the staged epilogue uses four quarters of BM x 128 bytes");
        // every wavefront has issued and completed its last reads of the token ring
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (FM == 9 && fmv == 9) gemm_epilogue_staged<FT, FA, BM, TN, EPI, FM == 9>(acc, accv, td, Np, C, ldc, wave, lane, (char*)lds);
        else gemm_epilogue_staged<FT, FA, BM, TN, EPI, false>(acc, accv, td, Np, C, ldc, wave, lane, (char*)lds);
    } else {
        if (FM == 9 && fmv == 9) gemm_epilogue<FT, FA, BM, TN, EPI, FM == 9>(acc, accv, td, Np, C, ldc, 0, wave, lane);
        else gemm_epilogue<FT, FA, BM, TN, EPI, false>(acc, accv, td, Np, C, ldc, 0, wave, lane);
    }
}



// ---- per-epilogue instantiation units ----------------------------------------------------------
// Classes 0 and 1 are the production token-tile classes of ordinary loads (row tiles of up to 128 rows for
// low loads, up to 288 rows otherwise), class 5 the one of decode-sized loads (see below); the other ids are
// alternatives kept for tuning runs (moe_set_tile_class).
// Class 5: two wavefronts per workgroup, 128 packed weight rows and up to 64 token rows per work item.  At a
// few rows per expert the kernel only streams weights, and what bounds it is the number of bytes a compute
// unit has in flight: a 4-wavefront workgroup with all its registers keeps 64 KB of weights under way and
// occupies the compute unit alone; these workgroups need under 256 registers per lane and 33 KB of LDS, four
// of them share a compute unit, together they keep 128 KB under way, and the weight panels are half as large,
// so a launch has four times as many workgroups to spread over the device (Mixtral shape, 64 tokens: 1792
// instead of 896 for 256 compute units).
// A unit that defines MOE_GEMM_NO_TALL_TILE before including this file leaves out the 288-row class (its
// launcher then rejects class 1): the router-logit GEMM never uses it, and with that unit's epilogue the
// compiler copies the VGPR accumulators right behind their MFMAs (see mfma_pinned_vgpr).
//   V(id, BM, NSX, NW)
#ifdef MOE_GEMM_NO_TALL_TILE
#define FOR_EACH_VARIANT(V) \
    V(0, 128, 4, 4)         \
    V(2, 64, 4, 4)          \
    V(3, 32, 4, 4)          \
    V(4, 256, 4, 4)         \
    V(5, 64, 4, 2)
#else
#define FOR_EACH_VARIANT(V) \
    V(0, 128, 4, 4)         \
    V(1, 288, 4, 4)         \
    V(2, 64, 4, 4)          \
    V(3, 32, 4, 4)          \
    V(4, 256, 4, 4)         \
    V(5, 64, 4, 2)
#endif

// Workgroup x takes the entries x, x + gridDim.x, ... of the work list.  Every class but the decode class is
// launched with one workgroup per entry: the hardware then hands the next entry to whichever compute unit is
// free, which balances tiles of unequal height (looping over a fixed share instead costs 3.5 % on the Mixtral
// shape at 1024 rows per expert and 13 % on ragged fine-grained loads).  The decode class has equal items
// that only stream weights; there a workgroup that stays resident saves the placement of a new one (about
// 5 us each): first expert GEMM of the Mixtral shape at 16 rows per expert, 1792 items on 1024 resident
// workgroups, 310 -> 298 us.  The barrier between two items keeps the next item's token loads out of the ring
// until every wavefront has read back its staged output.
template <int BM, int NSX, int EPI, int NW, bool W_STREAM>
__global__ __launch_bounds__(NW * 64) void grouped_gemm_kernel(const uint16_t* __restrict__ X, int ldx,
                                                               const int32_t* __restrict__ row_map,
                                                               const uint16_t* __restrict__ Wf, int Np, int K,
                                                               uint16_t* __restrict__ C, int ldc,
                                                               const TileDesc* __restrict__ table,
                                                               size_t c_split_bytes, int n_entries) {
    if constexpr (NW == 2) {
        for (int b = blockIdx.x; b < n_entries; b += gridDim.x) {
            gemm_tile<BM, NSX, EPI, NW, W_STREAM>(b, X, ldx, row_map, Wf, Np, K, C, ldc, table, c_split_bytes);
            // LDS reads only: the output stores need not have completed (a full __syncthreads() would also
            // wait for them, and a workgroup that waits for its last stores holds its compute unit longer)
            if (b + (int)gridDim.x < n_entries) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
    } else {
        // no loop in the code of the other classes: the compiler would keep the lane-dependent values it can
        // hoist out of it in registers for the whole kernel, and the tall tiles have none to spare
        gemm_tile<BM, NSX, EPI, NW, W_STREAM>(blockIdx.x, X, ldx, row_map, Wf, Np, K, C, ldc, table, c_split_bytes);
    }
}

template <int BM, int NSX, int EPI, int NW, bool WS>
struct Variant {
    static constexpr size_t smem = (size_t)NSX * BM * 64 * 2;
    static hipError_t set_attr() {
        return hipFuncSetAttribute((const void*)grouped_gemm_kernel<BM, NSX, EPI, NW, WS>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    // K is the reduction length of ONE split; nsplit = 1 for the expert GEMMs
    static hipError_t launch(int grid, const uint16_t* X, int ldx, const int32_t* row_map, const uint16_t* Wf,
                             int Np, int K, uint16_t* C, int ldc, const TileDesc* table, int nsplit,
                             size_t c_split_bytes, hipStream_t st) {
        constexpr int RESIDENT = 256 * 4;  // decode class: four workgroups fit a compute unit
        const int gx = (NW == 2 && grid > RESIDENT) ? RESIDENT : grid;
        hipLaunchKernelGGL((grouped_gemm_kernel<BM, NSX, EPI, NW, WS>), dim3(gx, nsplit), dim3(NW * 64), smem, st,
                           X, ldx, row_map, Wf, Np, K, C, ldc, table, c_split_bytes, grid);
        return hipGetLastError();
    }
};

template <int EPI, bool WS>
static hipError_t gemm_set_attr_all() {
    hipError_t err;
#define V(id, bm, ns, nw)                               \
    err = Variant<bm, ns, EPI, nw, WS>::set_attr();     \
    if (err != hipSuccess) return err;
    FOR_EACH_VARIANT(V)
#undef V
    return hipSuccess;
}

template <int EPI, bool WS>
static hipError_t gemm_launch_any(int cls, int grid, const uint16_t* X, int ldx, const int32_t* row_map,
                                  const uint16_t* Wf, int Np, int K, uint16_t* C, int ldc, const TileDesc* table,
                                  int nsplit, size_t c_split_bytes, hipStream_t st) {
    switch (cls) {
#define V(id, bm, ns, nw)                                                                                     \
    case id:                                                                                                  \
        return Variant<bm, ns, EPI, nw, WS>::launch(grid, X, ldx, row_map, Wf, Np, K, C, ldc, table, nsplit,  \
                                                    c_split_bytes, st);
        FOR_EACH_VARIANT(V)
#undef V
    }
    return hipErrorInvalidValue;
}

// Defines gemm_set_attr_<name>() and gemm_launch_<name>(cls, ...) for one epilogue and one kind of weight load;
// each is compiled in a translation unit of its own so that the units build in parallel.
#define MOE_GEMM_INSTANTIATE(name, EPI, WS)                                                                   \
    hipError_t gemm_set_attr_##name() { return gemm_set_attr_all<EPI, WS>(); }                                \
    hipError_t gemm_launch_##name(int cls, int grid, const uint16_t* X, int ldx, const int32_t* row_map,      \
                                  const uint16_t* Wf, int Np, int K, uint16_t* C, int ldc,                    \
                                  const TileDesc* table, int nsplit, size_t c_split_bytes, hipStream_t st) {  \
        return gemm_launch_any<EPI, WS>(cls, grid, X, ldx, row_map, Wf, Np, K, C, ldc, table, nsplit,         \
                                        c_split_bytes, st);                                                   \
    }
