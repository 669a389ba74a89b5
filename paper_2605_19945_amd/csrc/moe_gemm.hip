// Work list, tile classes, plans and launches of the grouped GEMMs (the kernel itself lives in
// moe_gemm_kernel.h and is instantiated per epilogue in moe_gemm_{swiglu,plain,pairsum,partial}.hip).
#include "moe_internal.h"

#include "moe_schedule.h"

// The work lists of both expert GEMMs from the per-expert offsets (or, host_rows >= 0, of a launch with one
// group of host_rows rows: the router-logit GEMM).
__global__ __launch_bounds__(256) void schedule_kernel(const int32_t* __restrict__ offsets, int host_rows, SchedArgs a) {
    __shared__ int32_t s_off[257];
    for (int i = threadIdx.x; i <= a.E_local; i += 256) s_off[i] = host_rows >= 0 ? i * host_rows : offsets[i];
    __syncthreads();
    schedule_tables(a, s_off, blockIdx.x, gridDim.x);
}

// ------------------------------------------------------------------------------------------------
// Host side: tile classes, plans, launches.  Class ids index the variants listed in
// moe_gemm_kernel.h: 0 = 128-row tiles (very low loads), 1 = 288-row tiles (main), 2 = 64, 3 = 32,
// 4 = 256.
// ------------------------------------------------------------------------------------------------
static const int kClassRows[GEMM_NUM_CLASSES] = {128, 288, 64, 32, 256, 64};
static const int kClassBn[GEMM_NUM_CLASSES] = {256, 256, 256, 256, 256, 128};   // packed weight rows per work item
static const int kClassPerCu[GEMM_NUM_CLASSES] = {1, 1, 2, 3, 1, 4};            // workgroups that share a compute unit
constexpr int GEMM_BN = 256;  // of the classes the router-logit GEMM uses

#define DECL(name)                                                                                         \
    hipError_t gemm_set_attr_##name();                                                                     \
    hipError_t gemm_launch_##name(int cls, int grid, const uint16_t* X, int ldx, const int32_t* row_map,   \
                                  const uint16_t* Wf, int Np, int K, uint16_t* C, int ldc,                 \
                                  const TileDesc* table, int nsplit, size_t c_split_bytes, hipStream_t st);
DECL(swiglu) DECL(plain) DECL(pairsum) DECL(partial)
DECL(swiglu_stream) DECL(plain_stream) DECL(partial_stream)  // weight loads with the non-temporal hint
#undef DECL

int gemm_class_rows(int cls) { return kClassRows[cls]; }

// Weight loads with the non-temporal hint (see grouped_gemm_kernel): when the mean load says that an expert's
// rows fit one row tile, so that nearly every weight is read once.  Measured on layer time, hint against no
// hint: Mixtral shape 16 rows per expert (decode class) 0.505 against 0.556 ms, 64 rows per expert (288-row
// class) 0.539 against 0.590, 1024 rows per expert 2.38 against 2.31; expert-parallel share, 4 rows per expert
// (128-row class) 0.205 against 0.215, 530 rows per expert 1.40 against 1.41; fine-grained experts with 512
// rows on average and up to 1500, 0.859 against 0.826.
bool gemm_pick_stream(int cls, double rows_per_expert) { return rows_per_expert <= (double)kClassRows[cls]; }

int gemm_pick_class(double rows_per_expert) {
    // Measured on the layer time of the Mixtral shape, near-uniform loads (ms; classes 5 / 0 / 1 = decode,
    // 128-row, 288-row):
    //     8 rows per expert   0.481 / 0.484 / 0.495        64 rows   0.656 / 0.527 / 0.539
    //    32                   0.501 / 0.501 / 0.516        96        0.820 / 0.554 / 0.571
    //    48                   0.515 / 0.515 / 0.528       128        0.980 / 0.657 / 0.587
    // and of the expert-parallel share at 4 to 8 rows per expert: 0.225 / 0.238 / 0.235 for 0 / 5 / 1.
    // A class loses as soon as experts need a second row tile of it (their weights are then streamed twice).
    // On uniform loads the small classes would win by 2 to 3 % up to about three quarters of their tile
    // height; but the host only knows the MEAN load, and under the skew this library is built for they lose
    // more than that (expert-parallel share with Zipf loads, mean 64 rows per expert: 0.559 ms with the
    // 128-row class against 0.517 with the tall one).  So the small classes are used only where even a hot
    // expert stays inside one tile: below 12 rows per expert the 128-row class, up to 24 the decode class.
    if (rows_per_expert < 12.0) return GEMM_LOW;
    return rows_per_expert <= 24.0 ? GEMM_DECODE : GEMM_MAIN;
}

GemmPlan gemm_make_plan(int cls, int64_t n_rows_cap, int E_local, int d, int f) {
    GemmPlan p;
    p.cls = cls;
    p.bm = kClassRows[cls];
    p.bn = kClassBn[cls];
    int64_t extra = n_rows_cap < E_local ? n_rows_cap : E_local;
    // Row tiles at the tallest cap number at most rows / bm + one per loaded expert; a quarter more lets the
    // scheduler pick lower caps (it only considers caps whose tiles fit the list).
    const int64_t mt_tall = n_rows_cap / p.bm + extra + 1;
    p.mt_max = (int)(mt_tall + mt_tall / 4);
    p.nt1 = (2 * f + p.bn - 1) / p.bn;
    p.nt2 = (d + p.bn - 1) / p.bn;
    p.grid1 = sched_grid(p.mt_max, p.nt1);
    p.grid2 = sched_grid(p.mt_max, p.nt2);
    p.w_stream = false;  // the caller decides from the load it expects (gemm_pick_stream)
    return p;
}

hipError_t gemm_init_attributes() {
    hipError_t err = gemm_set_attr_swiglu();
    if (err == hipSuccess) err = gemm_set_attr_plain();
    if (err == hipSuccess) err = gemm_set_attr_pairsum();
    if (err == hipSuccess) err = gemm_set_attr_partial();
    if (err == hipSuccess) err = gemm_set_attr_swiglu_stream();
    if (err == hipSuccess) err = gemm_set_attr_plain_stream();
    if (err == hipSuccess) err = gemm_set_attr_partial_stream();
    return err;
}

SchedArgs gemm_sched_args(const GemmPlan& p, int E_local, TileDesc* t1, TileDesc* t2, int nsplit2, int64_t rows_cap,
                          int32_t* refused) {
    SchedArgs a;
    a.E_local = E_local;
    a.bm = p.bm; a.bn = p.bn;
    a.nt1 = p.nt1; a.grid1 = p.grid1; a.t1 = t1;
    a.nt2 = p.nt2; a.grid2 = p.grid2; a.t2 = t2;
    a.nsplit1 = 1; a.nsplit2 = nsplit2;
    a.rows_cap = (int)rows_cap;
    a.refused_out = refused;
    return a;
}

int gemm_sched_blocks(const GemmPlan& p) {
    int g = p.grid1 > p.grid2 ? p.grid1 : p.grid2;
    int blocks = (g + 255) / 256;  // one entry per thread: an entry is a few thousand cycles of dependent integer work
    if (blocks < 1) blocks = 1;
    if (blocks > 64) blocks = 64;
    return blocks;
}

hipError_t launch_schedule(const GemmPlan& p, const int32_t* offsets, int E_local, TileDesc* t1, TileDesc* t2,
                           int nsplit2, int64_t rows_cap, int32_t* refused, hipStream_t st) {
    hipLaunchKernelGGL(schedule_kernel, dim3(gemm_sched_blocks(p)), dim3(256), 0, st, offsets, -1,
                       gemm_sched_args(p, E_local, t1, t2, nsplit2, rows_cap, refused));
    return hipGetLastError();
}

hipError_t launch_gemm1(const GemmPlan& p, const uint16_t* X, int ldx, const int32_t* row_map,
                        const uint16_t* W13f, int d, int f, uint16_t* H, const TileDesc* table, hipStream_t st) {
    if (p.grid1 <= 0) return hipSuccess;
    return (p.w_stream ? gemm_launch_swiglu_stream : gemm_launch_swiglu)(p.cls, p.grid1, X, ldx, row_map, W13f, 2 * f, d, H, moe_ld_pad(f), table, 1, 0, st);
}

// Reduction splits of the second expert GEMM.  With few resident experts and few rows it has far fewer
// work items than the device has compute units (Mixtral shape: 16 weight-row tiles x 8 experts = 128), and
// each item streams a 256 x f weight panel at what ONE compute unit can pull.  Cutting the reduction into
// nsplit ranges multiplies the items; the partial sums go to fp32 slabs and are added in slab order.
// Estimated time of a launch in units of one unsplit item: rounds * (1 / nsplit + fixed cost per item),
// plus the slab traffic relative to the weights.  The row tiles are estimated from the mean load (the
// host does not know the per-expert counts).  Only for launches that are bound by weight streaming: with
// more rows per expert the idle compute units are not a loss, the busy ones run at a higher clock within
// the same power (Mixtral shape, both expert GEMMs together, split against unsplit: 0.642 against 0.694
// ms at 176 rows per expert, 0.656 against 0.705 at 192, 0.712 against 0.679 at 208, 0.757 against
// 0.739 at 256).
int gemm_pick_split2(const GemmPlan& p, int64_t n_rows, int E_local, int d, int f, size_t part_bytes) {
    if (n_rows <= 0) return 1;
    const int64_t e_loaded = n_rows < E_local ? n_rows : E_local;
    if (n_rows > 192 * e_loaded) return 1;
    const int64_t tiles = e_loaded * ((n_rows / e_loaded + p.bm - 1) / p.bm);
    const double items = (double)tiles * p.nt2;
    const double w_bytes = (double)e_loaded * d * f * 2;
    const int KT = f / 64;
    if (p.cls == GEMM_DECODE) {
        // decode class: the launch only streams weights.  Two wavefronts that read one sequential stream each
        // keep a compute unit's share of the memory system busy, so the reduction is only split until every
        // compute unit has a work item (Mixtral shape, 16 rows per expert, 256 items unsplit: 146 us; 2 splits
        // 149; 4 splits, one item per resident workgroup, 156; 8 splits 164)
        const double want = (double)SCHED_CU;
        int pick = 1;
        for (int s = 1; s <= 8; ++s) {
            if (KT % s != 0 || KT / s < 16) continue;
            if ((double)s * n_rows * d * 4 > (double)part_bytes) continue;
            pick = s;
            if (items * s >= want) break;
        }
        return pick;
    }
    auto cost = [&](int s) {
        const double rounds = (double)(((int64_t)(items * s) + SCHED_CU - 1) / SCHED_CU);
        double c = rounds * (1.0 / s + 0.06);
        if (s > 1) c += 0.02 + 2.0 * s * (double)n_rows * d * 4 / w_bytes * (items / SCHED_CU);
        return c;
    };
    int best = 1;
    double best_cost = cost(1) * 0.9;  // a split has to win by 10 %
    for (int s = 2; s <= 8; ++s) {
        if (KT % s != 0 || KT / s < 16) continue;
        if ((double)s * n_rows * d * 4 > (double)part_bytes) continue;
        const double c = cost(s);
        if (c < best_cost) {
            best_cost = c;
            best = s;
        }
    }
    return best;
}

// Y[r, c] = bf16(sum over the slabs of part[s][r][c]) for the rows r < *n_rows_dev
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ part, int nsplit,
                                                            size_t slab_elems, const int32_t* __restrict__ n_rows_dev,
                                                            int n_rows_cap, int d, uint16_t* __restrict__ Y) {
    const int rows = *n_rows_dev;
    if (rows > n_rows_cap) return;  // refused by the scheduler: nothing was computed
    const size_t n = (size_t)rows * d / 4;  // quads of columns
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        f32x4_t acc = *(const f32x4_t*)(part + 4 * i);
        for (int s = 1; s < nsplit; ++s) {
            const f32x4_t v = *(const f32x4_t*)(part + s * slab_elems + 4 * i);
            acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
        }
        u32x2_t o;
        o.x = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)acc[0]) | ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)acc[1]) << 16);
        o.y = (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)acc[2]) | ((uint32_t)__builtin_bit_cast(uint16_t, (__bf16)acc[3]) << 16);
        *(u32x2_t*)(Y + 4 * i) = o;
    }
}

hipError_t launch_gemm2(const GemmPlan& p, const uint16_t* H, const uint16_t* W2f, int d, int f, uint16_t* Y,
                        const TileDesc* table, int nsplit, float* part, int64_t n_rows, const int32_t* n_rows_dev,
                        hipStream_t st) {
    if (p.grid2 <= 0) return hipSuccess;
    if (nsplit <= 1)
        return (p.w_stream ? gemm_launch_plain_stream : gemm_launch_plain)(p.cls, p.grid2, H, moe_ld_pad(f), nullptr, W2f, d, f, Y, d, table, 1, 0, st);
    const size_t slab_elems = (size_t)n_rows * d;
    hipError_t e = (p.w_stream ? gemm_launch_partial_stream : gemm_launch_partial)(p.cls, p.grid2, H, moe_ld_pad(f), nullptr, W2f, d, f / nsplit, (uint16_t*)part, d,
                                       table, nsplit, slab_elems * 4, st);
    if (e != hipSuccess || Y == nullptr) return e;  // Y == nullptr: the caller consumes the partial slabs
    size_t blocks = (slab_elems / 4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)part, nsplit,
                       slab_elems, n_rows_dev, (int)n_rows, d, Y);
    return hipGetLastError();
}

// ---- router logits as a one-group GEMM (E >= 32): logits[T, Ep] = x[T, d] * Wg, fp32 ------------
// Router rows are packed like W1|W3: 32-row blocks alternate between the high and the low bf16 term
// of the same 32 experts, and the epilogue adds the two accumulators.  The output is tiny next to the
// reduction length, so the reduction is split over up to 8 workgroups per tile (partial logits in
// consecutive [T, ldl] slabs, added in order by the top-k kernel) until every compute unit has work.
struct RouterPick { int cls, nsplit; };
static RouterPick router_gemm_pick(int T, int d, int Rp, int max_split) {
    const int nt = (Rp + GEMM_BN - 1) / GEMM_BN, KT = d / 64;
    static const int order[4] = {4, 0, 2, 3};  // tallest tile first (256, 128, 64, 32 rows)
    for (int i = 0; i < 4; ++i) {
        const int c = order[i];
        const int mt = (T + kClassRows[c] - 1) / kClassRows[c];
        for (int s = 1; s <= 8 && s <= max_split; ++s)
            if (KT % s == 0 && KT / s >= 8 && mt * nt * s >= SCHED_CU) return {c, s};
    }
    // not enough work for the whole device whatever the shape: the 128-row tile, deepest allowed split
    int s = 1;
    for (int t = 2; t <= 8 && t <= max_split; ++t)
        if (KT % t == 0 && KT / t >= 8) s = t;
    return {0, s};
}

int router_gemm_grid_max(int T_max, int Rp) {
    const int nt = (Rp + GEMM_BN - 1) / GEMM_BN;
    int g = 0;
    for (int c = 0; c < GEMM_NUM_CLASSES; ++c) {
        int gc = sched_grid(T_max / (32 * sched_min_cap_blocks(kClassRows[c])) + 1, nt);
        if (gc > g) g = gc;
    }
    return g;
}

// *table_T: the token count the work list in `table` was last built for (it depends on nothing else for a
// given context), so that steps with an unchanged batch size skip that launch.
hipError_t launch_router_gemm(const uint16_t* x, const uint16_t* rp, int T, int d, int Rp, float* logits, int ldl,
                              int max_split, int* nsplit_out, TileDesc* table, int* table_T, hipStream_t st) {
    const RouterPick pk = router_gemm_pick(T, d, Rp, max_split);
    const int c = pk.cls;
    const int nt = (Rp + GEMM_BN - 1) / GEMM_BN;
    const int grid = sched_grid(T / (32 * sched_min_cap_blocks(kClassRows[c])) + 1, nt);
    *nsplit_out = pk.nsplit;
    // Under stream capture the launch goes into the graph, and a replay may then rebuild the list at any
    // later time: from the first captured call on, the list is rebuilt by every call (-2 = never skip).
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &capture) != hipSuccess) return hipGetLastError();
    if (capture != hipStreamCaptureStatusNone) *table_T = -2;
    if (*table_T != T) {
        SchedArgs a;
        a.E_local = 1;
        a.bm = kClassRows[c]; a.bn = GEMM_BN;
        a.nt1 = nt; a.grid1 = grid; a.t1 = table;
        a.nt2 = 0; a.grid2 = 0; a.t2 = nullptr;
        a.nsplit1 = pk.nsplit; a.nsplit2 = 1;
        a.rows_cap = -1;
        a.refused_out = nullptr;
        hipLaunchKernelGGL(schedule_kernel, dim3((grid + 1023) / 1024), dim3(256), 0, st, (const int32_t*)nullptr, T, a);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        if (*table_T != -2) *table_T = T;
    }
    return gemm_launch_pairsum(c, grid, x, d, nullptr, rp, Rp, d / pk.nsplit, (uint16_t*)logits, ldl, table, pk.nsplit,
                               (size_t)T * ldl * sizeof(float), st);
}

// ---- sustained matrix-core rate (measurement aid) ------------------------------------------------
// Every wavefront issues iters * 64 MFMAs on 8 independent accumulator blocks and touches no memory until
// its single predicated store; 4 wavefronts per workgroup, 8 workgroups per compute unit in the grid.
// The operands are 8 + 8 registers of pseudo-random bf16 values (random sign and mantissa, magnitudes
// 0.5 .. 2) paired differently in every MFMA, so that the multipliers see changing inputs as they do in a
// GEMM: with constant operands the same kernel runs at the full 2.4 GHz, with these it does not.
__device__ float g_mfma_rate_sink;  // where the (never taken) store below goes: a real address
// SHAPE 0: v_mfma_f32_32x32x16_bf16 (the grouped GEMM's instruction); SHAPE 1: v_mfma_f32_16x16x32_bf16 (half
// the flop per instruction, a quarter of the accumulator registers: iters * 128 per wavefront for the same work).
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters) {
    const uint32_t lane = threadIdx.x & 63;
    bf16x8_t a[8], b[8];
    uint32_t h = lane * 0x9E3779B1u + 0x7F4A7C15u;
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            h = h * 1664525u + 1013904223u;
            // sign | exponent 126 or 127 | 7 mantissa bits
            a[r][i] = __builtin_bit_cast(__bf16, (uint16_t)(((h >> 16) & 0x8000u) | ((126u + ((h >> 8) & 1u)) << 7) | ((h >> 20) & 0x7Fu)));
            h = h * 1664525u + 1013904223u;
            b[r][i] = __builtin_bit_cast(__bf16, (uint16_t)(((h >> 16) & 0x8000u) | ((126u + ((h >> 8) & 1u)) << 7) | ((h >> 20) & 0x7Fu)));
        }
    float s = 0.f;
    if constexpr (SHAPE == 0) {
        f32x16_t acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + u) & 7], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[j][j];
    } else {
        f32x4_t acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < 2 * iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j], b[(j + u) & 7], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[j][j & 3];
    }
    if (s == 1.2345e-30f) g_mfma_rate_sink = s;  // practically never taken: keeps the sums live
}

// Read-only streaming over a buffer: every thread has eight 16-byte loads in flight, grid-stride; plain or with
// the non-temporal hint.  The value read only feeds a store that is practically never taken.
__device__ uint32_t g_read_rate_sink;
template <bool NT>
__global__ __launch_bounds__(256) void read_rate_kernel(const uint4* __restrict__ p, size_t n16) {
    constexpr int U = 8;
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    for (size_t base = (size_t)blockIdx.x * 256 * U + threadIdx.x; base < n16; base += stride) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = base + (size_t)u * 256;
            v[u] = i < n16 ? (NT ? load_stream(p + i) : p[i]) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u && n16 == 1) g_read_rate_sink = acc;
}

hipError_t launch_read_rate(const void* buf, size_t bytes, bool nontemporal, hipStream_t st) {
    const size_t n16 = bytes / 16;
    if (nontemporal)
        hipLaunchKernelGGL(read_rate_kernel<true>, dim3(SCHED_CU * 2), dim3(256), 0, st, (const uint4*)buf, n16);
    else
        hipLaunchKernelGGL(read_rate_kernel<false>, dim3(SCHED_CU * 2), dim3(256), 0, st, (const uint4*)buf, n16);
    return hipGetLastError();
}

hipError_t launch_mfma_rate(int shape, int iters_per_wave, double* flop, hipStream_t st) {
    const int grid = SCHED_CU * 8;
    if (shape == 0) hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(grid), dim3(256), 0, st, iters_per_wave);
    else hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(grid), dim3(256), 0, st, iters_per_wave);
    *flop = (double)grid * 4 * (double)iters_per_wave * 64 * (2.0 * 32 * 32 * 16);
    return hipGetLastError();
}
