// Grouped expert GEMMs on the gfx950 matrix cores -- the paper's "isolated MoE expert kernel"
// (Sec. 3.3.2), whose latency over token count is the staircase GEM samples at tile boundaries.
//
//   GEMM1 + SwiGLU:  H[r, c] = silu(sum_i X[r,i] W1[e][i,c]) * (sum_i X[r,i] W3[e][i,c])
//   GEMM2:           Y[r, c] = sum_j H[r,j] W2[e][j,c]
// for the rows r of expert e (ragged, device-side counts), bf16 operands, fp32 accumulation.
//
// Design (CDNA4):
//   * work item = BM rows of ONE expert x BN packed weight rows; the list of work items is built
//     on the device from the per-expert offsets (no host sync), experts with no rows get none,
//     the last row tile of an expert is partial (loads clamped, stores masked) -- no padding to
//     the largest expert.
//   * both operands are reduction-contiguous (weights are pre-transposed at load time), staged
//     through LDS in 16-byte chunks with an XOR swizzle, double buffered over the K loop;
//     v_mfma_f32_32x32x16_bf16 with the WEIGHT rows as the first operand and the TOKEN rows as
//     the second, so a lane's accumulator holds 4 consecutive output columns of one token row.
//   * work items are ordered so that the workgroups running concurrently on one XCD (ids equal
//     modulo 8) share weight panels and row panels through that XCD's L2.
#include "moe_internal.h"

static __device__ inline uint32_t pack2_bf16(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}
static __device__ inline float silu_f32(float g) { return g / (1.f + __expf(-g)); }

template <int BM, int BN, int BK, int WM, int WN, bool SWIGLU>
__global__ __launch_bounds__(WM* WN * 64) void grouped_gemm_kernel(
    const uint16_t* __restrict__ X, int ldx, const int32_t* __restrict__ row_map,
    const uint16_t* __restrict__ Wp, int Np, int K, uint16_t* __restrict__ C, int ldc,
    const TileDesc* __restrict__ table) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;  // wave tile: TM token rows x TN weight rows
    constexpr int FM = TM / 32, FN = TN / 32;  // 32x32 accumulator blocks per wave
    constexpr int CH = BK / 8;                 // 16-byte chunks per staged row
    constexpr int RPP = NT / CH;               // rows staged per pass of the whole workgroup
    constexpr int XPASS = BM / RPP, WPASS = BN / RPP;
    constexpr int SWZ_SHIFT = (CH == 8) ? 0 : (CH == 4 ? 1 : 2);
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert(!SWIGLU || FN % 2 == 0, "SwiGLU needs gate/up block pairs in one wave");
    static_assert(BM % RPP == 0 && BN % RPP == 0 && XPASS >= 1 && WPASS >= 1, "staging shape");
    static_assert(BK == 32 || BK == 64, "BK");
    constexpr int STAGE = (BM + BN) * CH;  // 16-byte chunks per stage

    extern __shared__ u32x4_t lds[];  // [2][STAGE]: X rows then W rows

    const TileDesc td = table[blockIdx.x];
    if (td.rows <= 0) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lc = tid % CH, lr = tid / CH;

    // ---- per-thread staging sources (fixed over the K loop) ------------------------------------
    const u32x4_t* xsrc[XPASS];
    int xdst[XPASS];
#pragma unroll
    for (int p = 0; p < XPASS; ++p) {
        int r = lr + p * RPP;
        int rr = r < td.rows ? r : td.rows - 1;
        int grow = td.row0 + rr;
        if (row_map != nullptr) grow = row_map[grow];
        xsrc[p] = (const u32x4_t*)(X + (size_t)grow * ldx) + lc;
        xdst[p] = r * CH + (lc ^ ((r >> SWZ_SHIFT) & (CH - 1)));
    }
    const u32x4_t* wsrc[WPASS];
    int wdst[WPASS];
#pragma unroll
    for (int p = 0; p < WPASS; ++p) {
        int r = lr + p * RPP;
        int n = td.n0 + r;
        if (n >= Np) n = Np - 1;
        wsrc[p] = (const u32x4_t*)(Wp + ((size_t)td.expert * Np + n) * K) + lc;
        wdst[p] = BM * CH + r * CH + (lc ^ ((r >> SWZ_SHIFT) & (CH - 1)));
    }

    f32x16_t acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int KT = K / BK;
    u32x4_t xreg[XPASS], wreg[WPASS];
#pragma unroll
    for (int p = 0; p < XPASS; ++p) xreg[p] = xsrc[p][0];
#pragma unroll
    for (int p = 0; p < WPASS; ++p) wreg[p] = wsrc[p][0];
#pragma unroll
    for (int p = 0; p < XPASS; ++p) lds[xdst[p]] = xreg[p];
#pragma unroll
    for (int p = 0; p < WPASS; ++p) lds[wdst[p]] = wreg[p];
    __syncthreads();

    // fragment rows of this lane inside the staged tile
    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) {
#pragma unroll
            for (int p = 0; p < XPASS; ++p) xreg[p] = xsrc[p][(size_t)(kt + 1) * CH];
#pragma unroll
            for (int p = 0; p < WPASS; ++p) wreg[p] = wsrc[p][(size_t)(kt + 1) * CH];
        }
        const u32x4_t* xs = lds + cur * STAGE;
        const u32x4_t* ws = xs + BM * CH;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int c = kk * 2 + fhalf;
            bf16x8_t xf[FM], wf[FN];
#pragma unroll
            for (int b = 0; b < FM; ++b) {
                int r = wm * TM + b * 32 + frow;
                xf[b] = __builtin_bit_cast(bf16x8_t, xs[r * CH + (c ^ ((r >> SWZ_SHIFT) & (CH - 1)))]);
            }
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                int r = wn * TN + a * 32 + frow;
                wf[a] = __builtin_bit_cast(bf16x8_t, ws[r * CH + (c ^ ((r >> SWZ_SHIFT) & (CH - 1)))]);
            }
#pragma unroll
            for (int a = 0; a < FN; ++a)
#pragma unroll
                for (int b = 0; b < FM; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
        }
        if (kt + 1 < KT) {
            u32x4_t* nxt = lds + (cur ^ 1) * STAGE;
#pragma unroll
            for (int p = 0; p < XPASS; ++p) nxt[xdst[p]] = xreg[p];
#pragma unroll
            for (int p = 0; p < WPASS; ++p) nxt[wdst[p]] = wreg[p];
        }
        __syncthreads();
    }

    // ---- epilogue: accumulator element v of lane l in block (a, b) is
    //      weight row  a*32 + 8*(v/4) + 4*(l/32) + v%4,  token row  b*32 + l%32 --------------------
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        const int trow = wm * TM + b * 32 + frow;
        if (trow >= td.rows) continue;
        uint16_t* crow = C + (size_t)(td.row0 + trow) * ldc;
        if constexpr (SWIGLU) {
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
                    uint2 o;
                    o.x = pack2_bf16(h[0], h[1]);
                    o.y = pack2_bf16(h[2], h[3]);
                    *(uint2*)(crow + hcol + 8 * q) = o;
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < FN; ++a) {
                const int col = td.n0 + wn * TN + a * 32;
                if (col >= Np) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 o;
                    o.x = pack2_bf16(acc[a][b][4 * q + 0], acc[a][b][4 * q + 1]);
                    o.y = pack2_bf16(acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                    *(uint2*)(crow + col + 4 * fhalf + 8 * q) = o;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Device-side work list.  Work-item id b runs on XCD b % 8 (workgroups are dealt round-robin to
// the 8 XCDs); XCD x owns the weight-row tiles x, x+8, ...; inside an XCD the order is
// expert-major, then weight-row tile, then row tile (fastest), so the ~32 workgroups resident on
// an XCD cover all row tiles of one expert times a handful of its weight tiles.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void schedule_kernel(const int32_t* __restrict__ offsets, int E_local,
                                                       int bm, int bn, int nt1, int grid1,
                                                       TileDesc* __restrict__ t1, int nt2, int grid2,
                                                       TileDesc* __restrict__ t2) {
    __shared__ int32_t pre[257];  // exclusive prefix of row tiles per expert; pre[E_local] = total
    __shared__ int32_t off[257];
    const int tid = threadIdx.x;
    int mt = 0;
    if (tid < E_local) {
        int n = offsets[tid + 1] - offsets[tid];
        mt = (n + bm - 1) / bm;
    }
    for (int i = tid; i <= E_local; i += 256) off[i] = offsets[i];
    __shared__ int32_t scan[256];
    scan[tid] = mt;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
        int v = tid >= o ? scan[tid - o] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    pre[tid + 1] = scan[tid];
    if (tid == 0) pre[0] = 0;
    __syncthreads();
    const int MT = pre[E_local];

    for (int which = 0; which < 2; ++which) {
        const int nt = which ? nt2 : nt1;
        const int grid = which ? grid2 : grid1;
        TileDesc* table = which ? t2 : t1;
        for (int b = blockIdx.x * 256 + tid; b < grid; b += gridDim.x * 256) {
            const int x = b & 7, j = b >> 3;
            const int cnt = nt > x ? (nt - x + 7) / 8 : 0;  // weight-row tiles owned by XCD x
            TileDesc td;
            td.expert = 0; td.row0 = 0; td.rows = 0; td.n0 = 0;
            if (j < MT * cnt) {
                // largest e with pre[e] * cnt <= j
                int lo = 0, hi = E_local;
                while (hi - lo > 1) {
                    int mid = (lo + hi) >> 1;
                    if (pre[mid] * cnt <= j) lo = mid; else hi = mid;
                }
                const int e = lo;
                const int mte = pre[e + 1] - pre[e];
                const int r = j - pre[e] * cnt;
                const int mi = r % mte, nl = r / mte;
                const int e_rows = off[e + 1] - off[e];
                td.expert = e;
                td.row0 = off[e] + mi * bm;
                td.rows = min(bm, e_rows - mi * bm);
                td.n0 = (nl * 8 + x) * bn;
            }
            table[b] = td;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Host side: tile classes, plans, launches.
// ------------------------------------------------------------------------------------------------
struct ClassDef { int bm, bn, bk, wm, wn; };
static const ClassDef kClass[GEMM_NUM_CLASSES] = {
    {32, 256, 64, 1, 4},    // GEMM_BM32
    {64, 256, 64, 1, 4},    // GEMM_BM64
    {128, 128, 64, 2, 2},   // GEMM_BM128
    {256, 256, 64, 2, 4},   // GEMM_BM256
};

int gemm_class_rows(int cls) { return kClass[cls].bm; }

int gemm_pick_class(double rows_per_expert) {
    if (rows_per_expert > 384.0) return GEMM_BM256;
    if (rows_per_expert > 96.0) return GEMM_BM128;
    if (rows_per_expert > 40.0) return GEMM_BM64;
    return GEMM_BM32;
}

GemmPlan gemm_make_plan(int cls, int64_t n_rows_cap, int E_local, int d, int f) {
    GemmPlan p;
    p.cls = cls;
    p.bm = kClass[cls].bm;
    p.bn = kClass[cls].bn;
    int64_t extra = n_rows_cap < E_local ? n_rows_cap : E_local;
    p.mt_max = (int)(n_rows_cap / p.bm + extra);
    p.nt1 = (2 * f + p.bn - 1) / p.bn;
    p.nt2 = (d + p.bn - 1) / p.bn;
    p.grid1 = 8 * p.mt_max * ((p.nt1 + 7) / 8);
    p.grid2 = 8 * p.mt_max * ((p.nt2 + 7) / 8);
    return p;
}

template <int BM, int BN, int BK, int WM, int WN, bool SW>
static hipError_t set_attr_t() {
    size_t smem = (size_t)2 * (BM + BN) * BK * 2;
    return hipFuncSetAttribute((const void*)grouped_gemm_kernel<BM, BN, BK, WM, WN, SW>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
}

#define FOR_EACH_CLASS(M)      \
    M(GEMM_BM32, 32, 256, 64, 1, 4)   \
    M(GEMM_BM64, 64, 256, 64, 1, 4)   \
    M(GEMM_BM128, 128, 128, 64, 2, 2) \
    M(GEMM_BM256, 256, 256, 64, 2, 4)

hipError_t gemm_init_attributes() {
    hipError_t err;
#define M(cls, bm, bn, bk, wm, wn)                                       \
    err = set_attr_t<bm, bn, bk, wm, wn, true>();                        \
    if (err != hipSuccess) return err;                                   \
    err = set_attr_t<bm, bn, bk, wm, wn, false>();                       \
    if (err != hipSuccess) return err;
    FOR_EACH_CLASS(M)
#undef M
    return hipSuccess;
}

hipError_t launch_schedule(const GemmPlan& p, const int32_t* offsets, int E_local, TileDesc* t1, TileDesc* t2,
                           hipStream_t st) {
    int g = p.grid1 > p.grid2 ? p.grid1 : p.grid2;
    int blocks = (g + 1023) / 1024;
    if (blocks < 1) blocks = 1;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(schedule_kernel, dim3(blocks), dim3(256), 0, st, offsets, E_local, p.bm, p.bn, p.nt1,
                       p.grid1, t1, p.nt2, p.grid2, t2);
    return hipGetLastError();
}

template <int BM, int BN, int BK, int WM, int WN, bool SW>
static hipError_t gemm_launch_t(int grid, const uint16_t* X, int ldx, const int32_t* row_map,
                                const uint16_t* Wp, int Np, int K, uint16_t* C, int ldc, const TileDesc* table,
                                hipStream_t st) {
    size_t smem = (size_t)2 * (BM + BN) * BK * 2;
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, BK, WM, WN, SW>), dim3(grid), dim3(WM * WN * 64), smem, st,
                       X, ldx, row_map, Wp, Np, K, C, ldc, table);
    return hipGetLastError();
}

hipError_t launch_gemm1(const GemmPlan& p, const uint16_t* X, int ldx, const int32_t* row_map,
                        const uint16_t* W13p, int d, int f, uint16_t* H, const TileDesc* table, hipStream_t st) {
    if (p.grid1 <= 0) return hipSuccess;
    switch (p.cls) {
#define M(cls, bm, bn, bk, wm, wn) \
    case cls: return gemm_launch_t<bm, bn, bk, wm, wn, true>(p.grid1, X, ldx, row_map, W13p, 2 * f, d, H, f, table, st);
        FOR_EACH_CLASS(M)
#undef M
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm2(const GemmPlan& p, const uint16_t* H, const uint16_t* W2p, int d, int f, uint16_t* Y,
                        const TileDesc* table, hipStream_t st) {
    if (p.grid2 <= 0) return hipSuccess;
    switch (p.cls) {
#define M(cls, bm, bn, bk, wm, wn) \
    case cls: return gemm_launch_t<bm, bn, bk, wm, wn, false>(p.grid2, H, f, nullptr, W2p, d, f, Y, d, table, st);
        FOR_EACH_CLASS(M)
#undef M
    }
    return hipErrorInvalidValue;
}
