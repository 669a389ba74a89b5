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
//     the last row tile of an expert is partial (loads clamped or skipped, stores masked) -- no
//     padding to the largest expert.
//   * both operands are reduction-contiguous (weights are pre-transposed at load time), staged in
//     LDS in 16-byte chunks with an XOR swizzle, multi-buffered over the K loop;
//     v_mfma_f32_32x32x16_bf16 with the WEIGHT rows as the first operand and the TOKEN rows as
//     the second, so a lane's accumulator holds 4 consecutive output columns of one token row.
//   * work items are ordered so that the workgroups running concurrently on one XCD (ids equal
//     modulo 8) share weight panels and row panels through that XCD's L2.
#include <stdlib.h>

#include "moe_gemm_common.h"

// ------------------------------------------------------------------------------------------------
// The GEMM kernel.  Operands go global -> LDS with global_load_lds_dwordx4 (no VGPR staging, no
// ds_write): one wave-level load writes 64 lanes x 16 bytes contiguously at a wave-uniform LDS
// address (lane l lands at base + 16*l), so the bank-conflict-avoiding XOR swizzle is applied on
// the *global* side: the lane that owns physical chunk p of a row fetches logical chunk
// p ^ swz(row).  NSTAGE-deep LDS ring, prefetch distance D = NSTAGE-1, one barrier per K step:
//   wait own loads of stage kt | barrier | issue loads of stage kt+D into the slot read at kt-1 |
//   MFMAs on stage kt.
// SPREAD >= 1 issues the next stage's loads between the MFMAs of the first SPREAD sub-steps instead
// of one burst after the barrier.  SWP >= 1 software-pipelines the LDS->register fragment reads one
// MFMA sub-step ahead: explicitly scheduled reads (SWP per MFMA slot) and explicit waits.
// Row tiles have a run-time height (a multiple of 32 rows up to BM, the last one of an expert
// possibly ragged): 32-row blocks past the last valid row are neither loaded nor multiplied.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, int NSTAGE, int SPREAD, int SWP, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void grouped_gemm_kernel(
    const uint16_t* __restrict__ X, int ldx, const int32_t* __restrict__ row_map,
    const uint16_t* __restrict__ Wp, int ldw, int Np, int K, uint16_t* __restrict__ C, int ldc,
    const TileDesc* __restrict__ table) {
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;  // wave tile: TM token rows x TN weight rows
    constexpr int FM = TM / 32, FN = TN / 32;  // 32x32 accumulator blocks per wave
    constexpr int CH = BK / 8;                 // 16-byte chunks per staged row
    constexpr int RPL = 64 / CH;               // rows covered by one wave-level load
    constexpr int XPASS = BM / (NW * RPL), WPASS = BN / (NW * RPL);
    constexpr int LPT = XPASS + WPASS;         // loads per thread per stage
    constexpr int STAGE = (BM + BN) * CH;      // 16-byte chunks per stage
    constexpr int D = NSTAGE - 1;
    constexpr int KK = BK / 16;                // MFMA sub-steps per K step
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 blocks");
    static_assert(EPI == EPI_PLAIN || FN % 2 == 0, "paired epilogues need both blocks of a pair in one wave");
    static_assert(BM % (NW * RPL) == 0 && BN % (NW * RPL) == 0, "staging shape");
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4 && D * LPT < 64, "pipeline depth");
    static_assert(TM % 16 == 0 && TN % 16 == 0 && (FM > FN ? FM : FN) * 32 * CH * 16 < 65536, "fragment addressing");

    extern __shared__ u32x4_t lds[];  // [NSTAGE][STAGE]: X rows then W rows

    const TileDesc td = table[blockIdx.x];
    if (td.rows <= 0) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in an SGPR
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = lane / CH, lphys = lane % CH;
    const int frow = lane & 31, fhalf = lane >> 5;
    const int KT = K / BK;

    // per-thread global sources: 32-bit byte offsets from wave-uniform bases (the bases advance by
    // BK elements per K step in scalar registers, the offsets never change)
    const uint16_t* wbase = Wp + (size_t)td.expert * Np * ldw;
    uint32_t xo[XPASS], wo[WPASS];
#pragma unroll
    for (int p = 0; p < XPASS; ++p) {
        const int r = (p * NW + wave) * RPL + lrow;
        const int rr = r < td.rows ? r : td.rows - 1;  // clamp: rows past the end are never stored
        int grow = td.row0 + rr;
        if (row_map != nullptr) grow = row_map[grow];
        xo[p] = (uint32_t)grow * (uint32_t)(ldx * 2) + (uint32_t)((lphys ^ swz_of<CH>(r)) * 16);
    }
#pragma unroll
    for (int p = 0; p < WPASS; ++p) {
        const int r = (p * NW + wave) * RPL + lrow;
        int n = td.n0 + r;
        if (n >= Np) n = Np - 1;
        wo[p] = (uint32_t)n * (uint32_t)(ldw * 2) + (uint32_t)((lphys ^ swz_of<CH>(r)) * 16);
    }
    // LDS fragment addresses of this lane (in 16-byte chunks) and their XOR masks
    int xoff[FM], xswz[FM], woff[FN], wswz[FN];
#pragma unroll
    for (int b = 0; b < FM; ++b) {
        const int r = wm * TM + b * 32 + frow;
        xoff[b] = r * CH;
        xswz[b] = swz_of<CH>(r);
    }
#pragma unroll
    for (int a = 0; a < FN; ++a) {
        const int r = wn * TN + a * 32 + frow;
        woff[a] = BM * CH + r * CH;
        wswz[a] = swz_of<CH>(r);
    }

    // byte addresses (inside a stage) of this lane's fragment chunk for every MFMA sub-step; the
    // 32-row blocks of a wave are a constant 32*CH*16 bytes apart and share the XOR mask (the wave
    // tile starts at a multiple of 16 rows)
    uint32_t fx_addr[KK], fw_addr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int c = kk * 2 + fhalf;
        fx_addr[kk] = (uint32_t)((xoff[0] + (c ^ xswz[0])) * 16);
        fw_addr[kk] = (uint32_t)((woff[0] + (c ^ wswz[0])) * 16);
    }

    f32x16_t acc[FN][FM];
#pragma unroll
    for (int a = 0; a < FN; ++a)
#pragma unroll
        for (int b = 0; b < FM; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // wave-uniform extents of the valid part of the tile (in 32-row blocks / load passes)
    const int rows32 = (td.rows + 31) & ~31;
    const bool full = td.rows == BM;
    int fm_valid = (rows32 - wm * TM) / 32;  // valid 32-row blocks of this wave
    fm_valid = fm_valid < 0 ? 0 : (fm_valid > FM ? FM : fm_valid);

    // loads [lo, hi) of the LPT loads that bring in stage kt (X passes first, then W passes);
    // X passes whose rows all lie past the last valid 32-row block are skipped
    auto issue = [&](int kt, auto lo_c, auto hi_c) {
        constexpr int lo = decltype(lo_c)::value, hi = decltype(hi_c)::value;
        u32x4_t* base = lds + (kt % NSTAGE) * STAGE;
#pragma unroll
        for (int q = lo; q < hi; ++q) {
            if (q < XPASS) {
                if ((q * NW + wave) * RPL < rows32)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)((const char*)(X + (size_t)kt * BK) + xo[q]),
                        (__attribute__((address_space(3))) void*)(base + (q * NW + wave) * RPL * CH), 16, 0, 0);
            } else {
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)((const char*)(wbase + (size_t)kt * BK) + wo[q - XPASS]),
                    (__attribute__((address_space(3))) void*)(base + BM * CH + ((q - XPASS) * NW + wave) * RPL * CH),
                    16, 0, 0);
            }
        }
    };
    auto issue_one = [&](int kt, int q) {  // q is a compile-time constant after unrolling
        u32x4_t* base = lds + (kt % NSTAGE) * STAGE;
        if (q < XPASS) {
            if ((q * NW + wave) * RPL < rows32)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)((const char*)(X + (size_t)kt * BK) + xo[q]),
                    (__attribute__((address_space(3))) void*)(base + (q * NW + wave) * RPL * CH), 16, 0, 0);
        } else {
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)((const char*)(wbase + (size_t)kt * BK) + wo[q - XPASS]),
                (__attribute__((address_space(3))) void*)(base + BM * CH + ((q - XPASS) * NW + wave) * RPL * CH), 16,
                0, 0);
        }
    };
    using IC0 = std::integral_constant<int, 0>;
    using ICL = std::integral_constant<int, LPT>;

    // The K loop, specialised on the number of valid 32-row blocks of this wave: FMV >= 0 is a
    // compile-time count (no per-MFMA branches); FMV < 0 reads it at run time.  Waves of one
    // workgroup may take different specialisations; all of them execute one barrier per K step.
    auto main_loop = [&](auto fmv_c) {
        constexpr int FMV = decltype(fmv_c)::value;
        auto live = [&](int b) { return FMV >= 0 ? b < FMV : b < fm_valid; };
        const bool any = FMV >= 0 ? FMV > 0 : fm_valid > 0;
#pragma unroll
        for (int s = 0; s < D; ++s)
            if (s < KT) issue(s, IC0{}, ICL{});

        for (int kt = 0; kt < KT; ++kt) {
            // loads that may stay in flight: those of the already issued stages after kt (the
            // count per stage is only known at compile time for full tiles)
            const int ahead = full ? min(D - 1, KT - 1 - kt) : 0;
            if (ahead <= 0) wait_vmcnt<0>();
            else if (ahead == 1) wait_vmcnt<LPT>();
            else wait_vmcnt<2 * LPT>();
            // barrier without the workgroup fence of __syncthreads(): the fence would wait for ALL
            // outstanding loads (vmcnt(0)) and collapse the prefetch distance to one stage
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const bool more = kt + D < KT;
            if constexpr (SPREAD == 0) {
                if (more) issue(kt + D, IC0{}, ICL{});
            }
            const u32x4_t* st = lds + (kt % NSTAGE) * STAGE;
            auto spread_issue = [&](int kk) {
                if constexpr (SPREAD >= 1) {
                    // feed the vector-memory pipe a slice of the next stage's loads per sub-step
                    // (all but the last sub-step) instead of one burst right after the barrier
                    constexpr int PH = KK > 1 ? KK - 1 : 1;
                    if (more) {
                        if (kk == 0) issue(kt + D, std::integral_constant<int, 0>{}, std::integral_constant<int, (LPT * 1) / PH>{});
                        if (kk == 1 && PH > 1) issue(kt + D, std::integral_constant<int, (LPT * 1) / PH>{}, std::integral_constant<int, (LPT * 2) / PH>{});
                        if (kk == 2 && PH > 2) issue(kt + D, std::integral_constant<int, (LPT * 2) / PH>{}, std::integral_constant<int, (LPT * 3) / PH>{});
                    }
                }
            };
            if constexpr (SWP >= 1 && FMV > 0) {
                // fragments of sub-step kk+1 are read while the MFMAs of sub-step kk run
                constexpr int BLK = 32 * CH * 16;  // bytes between consecutive 32-row blocks
                using XS = std::make_integer_sequence<int, FMV>;
                using WS = std::make_integer_sequence<int, FN>;
                const uint32_t sbase = (uint32_t)((kt % NSTAGE) * STAGE * 16);
                bf16x8_t xf[2][FM], wf[2][FN];
                lds_read_frags<BLK>(xf[0], sbase + fx_addr[0], XS{});
                lds_read_frags<BLK>(wf[0], sbase + fw_addr[0], WS{});
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    const int cur = kk & 1, nxt = cur ^ 1;
                    // everything read for this sub-step was issued during the previous one
                    wait_lgkmcnt<0>();
#pragma unroll
                    for (int b = 0; b < FMV; ++b) tie(xf[cur][b]);
#pragma unroll
                    for (int a = 0; a < FN; ++a) tie(wf[cur][a]);
                    __builtin_amdgcn_sched_barrier(0);
                    // one memory instruction after each MFMA: first the LDS reads of the next
                    // sub-step's fragments, then this sub-step's share of the next stage's loads
                    constexpr int NM = FMV * FN;
                    constexpr int PHL = SPREAD < 1 ? 1 : (SPREAD > KK ? KK : SPREAD);  // sub-steps carrying loads
                    constexpr int LPP = (LPT + PHL - 1) / PHL;                         // loads per such sub-step
                    constexpr int RPS0 = (FMV + FN + NM - 1) / NM;
                    constexpr int RPS = SWP > RPS0 ? SWP : RPS0;                       // LDS reads per MFMA slot
                    constexpr int LPS = (LPP + NM - 1) / NM;                           // loads per MFMA slot
#pragma unroll
                    for (int m = 0; m < NM; ++m) {
                        const int b = m / FN, a = m % FN;
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][a], xf[cur][b], acc[a][b], 0, 0, 0);
                        if (kk + 1 < KK) {
#pragma unroll
                            for (int r = m * RPS; r < (m + 1) * RPS; ++r) {
                                if (r < FN) wf[nxt][r] = lds_read_b128_rt(sbase + fw_addr[kk + 1] + r * BLK);
                                else if (r < FN + FMV) xf[nxt][r - FN] = lds_read_b128_rt(sbase + fx_addr[kk + 1] + (r - FN) * BLK);
                            }
                        }
                        if constexpr (SPREAD >= 1) {
                            // loads of the next stage, one after each of the first MFMAs of the first
                            // PHL sub-steps (a different issue port than the LDS reads)
#pragma unroll
                            for (int l = m * LPS; l < (m + 1) * LPS; ++l) {
                                const int q = kk * LPP + l;
                                if (kk < PHL && l < LPP && q < LPT && more) issue_one(kt + D, q);
                            }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    const int c = kk * 2 + fhalf;
                    spread_issue(kk);
                    bf16x8_t wf[FN];
#pragma unroll
                    for (int a = 0; a < FN; ++a)
                        if (any) wf[a] = __builtin_bit_cast(bf16x8_t, st[woff[a] + (c ^ wswz[a])]);
#pragma unroll
                    for (int b = 0; b < FM; ++b)
                        if (live(b)) {
                            bf16x8_t xf = __builtin_bit_cast(bf16x8_t, st[xoff[b] + (c ^ xswz[b])]);
#pragma unroll
                            for (int a = 0; a < FN; ++a)
                                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf, acc[a][b], 0, 0, 0);
                        }
                }
            }
        }
    };
    if (fm_valid == FM) main_loop(std::integral_constant<int, FM>{});
    else if (FM > 1 && fm_valid == FM - 1) main_loop(std::integral_constant<int, (FM > 1 ? FM - 1 : 0)>{});
    else main_loop(std::integral_constant<int, -1>{});

    gemm_epilogue<FM, FN, TM, TN, EPI>(acc, td, Np, C, ldc, wm, wn, lane);
}

// ------------------------------------------------------------------------------------------------
// Device-side work list.  The rows of expert e are cut into ceil(n_e / bm) row tiles of nearly
// equal height (a multiple of 32 rows, at most bm): an expert slightly larger than a multiple of
// the tile height does not get a nearly empty extra tile, its rows are spread over taller tiles.
// The list order is expert-major, then weight-row tile, then row tile (fastest); chunks of 4
// consecutive items (row tiles sharing a weight panel) are dealt round-robin to the 8 XCDs, so the
// workgroups resident on one XCD reuse weight panels in that XCD's L2 and every XCD gets the same
// amount of work whatever the number of weight-row tiles.
// ------------------------------------------------------------------------------------------------
constexpr int SCHED_CHUNK = 4;
static inline int sched_grid(int mt_max, int nt) {
    const int chunks = (mt_max * nt + SCHED_CHUNK - 1) / SCHED_CHUNK;
    return 8 * SCHED_CHUNK * ((chunks + 7) / 8);
}

__global__ __launch_bounds__(256) void schedule_kernel(const int32_t* __restrict__ offsets, int E_local,
                                                       int bm, int bn, int nt1, int grid1,
                                                       TileDesc* __restrict__ t1, int nt2, int grid2,
                                                       TileDesc* __restrict__ t2, int host_rows) {
    __shared__ int32_t pre[257];  // exclusive prefix of row tiles per expert; pre[E_local] = total
    __shared__ int32_t off[257];
    __shared__ int32_t scan[256];
    const int tid = threadIdx.x;
    int mt = 0;
    // host_rows >= 0: one group of host_rows rows (the router GEMM), no offsets array to read
    if (tid < E_local) {
        int n = host_rows >= 0 ? host_rows : offsets[tid + 1] - offsets[tid];
        mt = (n + bm - 1) / bm;
    }
    for (int i = tid; i <= E_local; i += 256) off[i] = host_rows >= 0 ? i * host_rows : offsets[i];
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
            // XCD-aware order: the linear list (expert-major, then weight-row tile, then row tile) is
            // cut into chunks of SCHED_CHUNK consecutive items -- row tiles that share one weight
            // panel -- and the chunks are dealt round-robin to the 8 XCDs (work item b runs on XCD b % 8)
            const int x = b & 7, slot = b >> 3;
            const int L = ((slot / SCHED_CHUNK) * 8 + x) * SCHED_CHUNK + slot % SCHED_CHUNK;
            TileDesc td;
            td.expert = 0; td.row0 = 0; td.rows = 0; td.n0 = 0;
            if (L < MT * nt) {
                // largest e with pre[e] * nt <= L  (that expert has at least one row tile)
                int lo = 0, hi = E_local;
                while (hi - lo > 1) {
                    int mid = (lo + hi) >> 1;
                    if (pre[mid] * nt <= L) lo = mid; else hi = mid;
                }
                const int e = lo;
                const int mte = pre[e + 1] - pre[e];
                const int r = L - pre[e] * nt;
                const int mi = r % mte, ni = r / mte;
                const int e_rows = off[e + 1] - off[e];
                // 32-row blocks of the expert, dealt evenly to its mte tiles
                const int nblk = (e_rows + 31) / 32;
                const int base = nblk / mte, rem = nblk % mte;
                const int blk0 = mi * base + min(mi, rem);
                const int nb = base + (mi < rem ? 1 : 0);
                td.expert = e;
                td.row0 = off[e] + blk0 * 32;
                td.rows = min(nb * 32, e_rows - blk0 * 32);
                td.n0 = ni * bn;
            }
            table[b] = td;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Host side: tile variants, plans, launches.
// Variant ids 0 and 1 are the production token-tile classes (row tiles of up to 128 rows for low
// loads, up to 320 rows otherwise); higher ids are alternatives kept for tuning runs
// (moe_set_tile_class).
//   V(id, BM, BN, BK, WM, WN, NSTAGE, SPREAD, SWP)
// ------------------------------------------------------------------------------------------------
#define FOR_EACH_VARIANT(V)                \
    V(0, 128, 256, 64, 2, 4, 3, 0, 0)      \
    V(1, 320, 256, 64, 2, 4, 2, 3, 0)      \
    V(2, 256, 256, 64, 2, 4, 2, 2, 1)      \
    V(3, 320, 256, 64, 2, 4, 2, 2, 1)      \
    V(4, 32, 256, 64, 1, 4, 4, 0, 0)       \
    V(5, 64, 256, 64, 1, 4, 3, 0, 0)       \
    V(6, 128, 128, 64, 2, 2, 3, 0, 0)      \
    V(7, 256, 256, 64, 2, 4, 2, 0, 0)      \
    V(8, 192, 256, 64, 2, 4, 2, 3, 0)      \
    V(9, 128, 256, 64, 2, 4, 3, 2, 1)      \
    V(10, 256, 256, 64, 2, 2, 2, 2, 1)

struct VariantDef { int bm, bn, bk, wm, wn, nstage; };
static const VariantDef kVariant[GEMM_NUM_CLASSES] = {
#define V(id, bm, bn, bk, wm, wn, ns, spread, swp) {bm, bn, bk, wm, wn, ns},
    FOR_EACH_VARIANT(V)
#undef V
};

int gemm_class_rows(int cls) {
    return cls >= GEMM_NUM_CLASSES ? gemm_dw_class_rows(cls - GEMM_NUM_CLASSES) : kVariant[cls].bm;
}

int gemm_pick_class(double rows_per_expert) {
    // Measured on the expert-parallel share (32 experts, Zipf loads): the 320-row class with balanced,
    // block-skipping tiles wins from ~1 K rows upwards; below that the 128-row class streams the
    // weights slightly faster (three LDS stages).
    return rows_per_expert < 24.0 ? GEMM_LOW : GEMM_MAIN;
}

GemmPlan gemm_make_plan(int cls, int64_t n_rows_cap, int E_local, int d, int f) {
    GemmPlan p;
    p.cls = cls;
    p.bm = gemm_class_rows(cls);
    p.bn = cls >= GEMM_NUM_CLASSES ? 256 : kVariant[cls].bn;
    int64_t extra = n_rows_cap < E_local ? n_rows_cap : E_local;
    p.mt_max = (int)(n_rows_cap / p.bm + extra);
    p.nt1 = (2 * f + p.bn - 1) / p.bn;
    p.nt2 = (d + p.bn - 1) / p.bn;
    p.grid1 = sched_grid(p.mt_max, p.nt1);
    p.grid2 = sched_grid(p.mt_max, p.nt2);
    return p;
}

template <int BM, int BN, int BK, int WM, int WN, int NS, int SPREAD, int SWP, int EPI>
struct Variant {
    static constexpr size_t smem = (size_t)NS * (BM + BN) * BK * 2;
    static hipError_t set_attr() {
        return hipFuncSetAttribute((const void*)grouped_gemm_kernel<BM, BN, BK, WM, WN, NS, SPREAD, SWP, EPI>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    static hipError_t launch(int grid, const uint16_t* X, int ldx, const int32_t* row_map, const uint16_t* Wp,
                             int ldw, int Np, int K, uint16_t* C, int ldc, const TileDesc* table, hipStream_t st) {
        hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, BK, WM, WN, NS, SPREAD, SWP, EPI>), dim3(grid),
                           dim3(WM * WN * 64), smem, st, X, ldx, row_map, Wp, ldw, Np, K, C, ldc, table);
        return hipGetLastError();
    }
};

hipError_t gemm_init_attributes() {
    hipError_t err;
#define V(id, bm, bn, bk, wm, wn, ns, spread, swp)                        \
    err = Variant<bm, bn, bk, wm, wn, ns, spread, swp, EPI_SWIGLU>::set_attr();        \
    if (err != hipSuccess) return err;                                    \
    err = Variant<bm, bn, bk, wm, wn, ns, spread, swp, EPI_PLAIN>::set_attr();       \
    if (err != hipSuccess) return err;
    FOR_EACH_VARIANT(V)
#undef V
    return hipSuccess;
}

hipError_t launch_schedule(const GemmPlan& p, const int32_t* offsets, int E_local, TileDesc* t1, TileDesc* t2,
                           hipStream_t st) {
    int g = p.grid1 > p.grid2 ? p.grid1 : p.grid2;
    int blocks = (g + 1023) / 1024;
    if (blocks < 1) blocks = 1;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(schedule_kernel, dim3(blocks), dim3(256), 0, st, offsets, E_local, p.bm, p.bn, p.nt1,
                       p.grid1, t1, p.nt2, p.grid2, t2, -1);
    return hipGetLastError();
}

hipError_t launch_gemm1(const GemmPlan& p, const uint16_t* X, int ldx, const int32_t* row_map,
                        const uint16_t* W13p, int d, int f, uint16_t* H, const TileDesc* table, hipStream_t st) {
    if (p.grid1 <= 0) return hipSuccess;
    switch (p.cls) {
#define V(id, bm, bn, bk, wm, wn, ns, spread, swp) \
    case id:                                \
        return Variant<bm, bn, bk, wm, wn, ns, spread, swp, EPI_SWIGLU>::launch(p.grid1, X, ldx, row_map, W13p, moe_ld_pad(d), 2 * f, d, H, moe_ld_pad(f), table, st);
        FOR_EACH_VARIANT(V)
#undef V
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm2(const GemmPlan& p, const uint16_t* H, const uint16_t* W2p, int d, int f, uint16_t* Y,
                        const TileDesc* table, hipStream_t st) {
    if (p.grid2 <= 0) return hipSuccess;
    switch (p.cls) {
#define V(id, bm, bn, bk, wm, wn, ns, spread, swp) \
    case id:                                \
        return Variant<bm, bn, bk, wm, wn, ns, spread, swp, EPI_PLAIN>::launch(p.grid2, H, moe_ld_pad(f), nullptr, W2p, moe_ld_pad(f), d, f, Y, d, table, st);
        FOR_EACH_VARIANT(V)
#undef V
    }
    return hipErrorInvalidValue;
}

// ---- router logits as a one-group GEMM (E >= 32): logits[T, Ep] = x[T, d] * Wg, fp32 ------------
// Router rows are packed like W1|W3: 32-row blocks alternate between the high and the low bf16 term
// of the same 32 experts, and the epilogue adds the two accumulators.
#define FOR_EACH_ROUTER_VARIANT(V)  \
    V(0, 32, 256, 64, 1, 4, 4, 0)   \
    V(1, 64, 256, 64, 1, 4, 3, 0)   \
    V(2, 128, 256, 64, 2, 4, 3, 0)  \
    V(3, 320, 256, 64, 2, 4, 2, 3)

static const int kRouterBm[4] = {32, 64, 128, 320};

hipError_t router_gemm_init_attributes() {
    hipError_t err;
#define V(id, bm, bn, bk, wm, wn, ns, spread)                                   \
    err = Variant<bm, bn, bk, wm, wn, ns, spread, 0, EPI_PAIR_SUM_F32>::set_attr(); \
    if (err != hipSuccess) return err;
    FOR_EACH_ROUTER_VARIANT(V)
#undef V
    return hipSuccess;
}

int router_gemm_pick(int T, int Rp) {
    // smallest row tile that still gives every CU a work item
    const int nt = (Rp + 255) / 256;
    for (int v = 3; v > 0; --v)
        if ((T / kRouterBm[v]) * nt >= 256) return v;
    return 0;
}

int router_gemm_grid(int v, int T_max, int Rp) {
    const int nt = (Rp + 255) / 256;
    return sched_grid(T_max / kRouterBm[v] + 1, nt);
}

hipError_t launch_router_gemm(const uint16_t* x, const uint16_t* rp, int T, int d, int Rp, float* logits, int ldl,
                              TileDesc* table, hipStream_t st) {
    const int v = router_gemm_pick(T, Rp);
    const int nt = (Rp + 255) / 256;
    const int grid = router_gemm_grid(v, T, Rp);
    hipLaunchKernelGGL(schedule_kernel, dim3((grid + 1023) / 1024), dim3(256), 0, st, (const int32_t*)nullptr, 1,
                       kRouterBm[v], 256, nt, grid, table, 0, 0, (TileDesc*)nullptr, T);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    switch (v) {
#define V(id, bm, bn, bk, wm, wn, ns, spread) \
    case id:                                  \
        return Variant<bm, bn, bk, wm, wn, ns, spread, 0, EPI_PAIR_SUM_F32>::launch(grid, x, d, nullptr, rp, moe_ld_pad(d), Rp, d, (uint16_t*)logits, ldl, table, st);
        FOR_EACH_ROUTER_VARIANT(V)
#undef V
    }
    return hipErrorInvalidValue;
}
