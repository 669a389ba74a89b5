// Work list, tile classes, plans and launches of the grouped GEMMs (the kernel itself lives in
// moe_gemm_kernel.h and is instantiated per epilogue in moe_gemm_{swiglu,plain,pairsum,partial}.hip).
#include "moe_internal.h"

// ------------------------------------------------------------------------------------------------
// Device-side work list.  The rows of expert e are cut into ceil(n_e / cap) row tiles of nearly
// equal height (a multiple of 32 rows, at most cap): an expert slightly larger than a multiple of
// the cap does not get a nearly empty extra tile, its rows are spread over its tiles.
//
// The cap itself is chosen per GEMM on the device from the tallest tile and the next five heights down
// (as far as their row tiles fit the work list), from the actual
// loads: a launch runs in ceil(work items / compute units) rounds of roughly one tile time each, so
// when there are only a few rounds (the second expert GEMM has few weight-row tiles) a slightly
// lower cap that fills the last round beats the tallest tile -- the tile-boundary staircase of
// Sec. 3.3.2, seen from the scheduler's side.  Estimated time of a cap, in units of one 32-row
// block of MFMA work: rounds * (mean tile height in blocks + SCHED_TILE_OVERHEAD); a launch with reduction
// splits has that many workgroups per work item.
//
// Order of the work list.  The hardware hands out the workgroups of a launch in index order:
// workgroup b goes to XCD b % 8, and within an XCD to shader engine (b / 8) % 4, whose eight compute
// units take whatever arrives there; the XCD's dispatcher does not move on while the engine whose
// turn it is has no free compute unit (measured with per-workgroup time stamps: an engine that
// keeps receiving workgroups with nothing to do idles, it cannot run ahead of the other three).
// So each XCD's queue -- the entries b = x, x + 8, x + 16, ... of the table -- is dense: real tiles
// only, empty entries follow after the last one.
//
// A "piece" is up to SCHED_PIECE_MAX row tiles of one expert and one weight-row tile, consecutive in
// one XCD's queue: they run side by side and share that weight panel in the XCD's L2.  An expert
// with more row tiles is cut into pp > 1 row ranges of nearly equal length (the first mte % pp one
// tile longer).  Pieces are numbered expert-major, then row range, then weight-row tile, and dealt
// round-robin to the XCDs.  The workgroups resident on one XCD at a time are then consecutive
// weight-row tiles of one expert times the row tiles of one row range: they share the token panels
// of that range, all eight XCDs work on the same range (it stays in the Infinity Cache), and every
// XCD gets its share of every range.  An expert's weights are streamed once per row range.  With few
// work items the pieces are made shorter so that there are at least 64 of them.
// ------------------------------------------------------------------------------------------------
constexpr int SCHED_CU = 256;    // compute units of the device (one workgroup each)
constexpr int SCHED_PIECE_MAX = 8;  // row tiles per piece, at most
// Per-tile cost that does not scale with the tile's height, in 32-row blocks of MFMA work.  In launches
// where every row tile has the same height and the workgroups run in step the cost is about one block
// (Mixtral shape, tiles forced to 6, 7, 8, 9 blocks: 28 rounds of GEMM1 take 2331, 2656, 2993, 3333 us).
// On ragged loads a tile costs more than that -- its weight panel is shared with fewer neighbours the
// further the workgroups drift apart -- and 3.5 picks caps that are as fast or up to 2 % faster than
// those picked with 1.0 on every benchmark workload.
constexpr float SCHED_TILE_OVERHEAD = 3.5f;
constexpr int SCHED_CAPS = 6;  // candidate caps: the tallest tile and the next five heights down
static __host__ __device__ inline int sched_min_cap_blocks(int bm) {
    const int h = bm / 32 - (SCHED_CAPS - 1);
    return h < 1 ? 1 : h;
}
// Entries of a work list (= workgroups of the launch) for at most mt row tiles: the eight queues together
// hold (row tiles * weight-row tiles) entries; dealing whole pieces can leave them unequal, and the
// scheduler falls back to single-tile pieces, whose queues differ by at most one entry, when eight times
// the longest would not fit.  Workgroups past the end of their queue exit at once, but each still has to
// be placed on a compute unit with its full LDS and register allotment (about 0.5 us): the list is kept
// as short as the bound allows.
static inline int sched_grid(int mt, int nt) { return mt * nt + 64; }

// inclusive prefix sum over the 64 lanes with data-parallel-primitive moves: a Kogge-Stone scan inside
// each row of 16 lanes, then the row totals are carried into the following rows
static __device__ inline int wave_scan_incl(int v) {
#define DPP_ADD(ctrl, row_mask) v += __builtin_amdgcn_update_dpp(0, v, ctrl, row_mask, 0xf, false);
    DPP_ADD(0x111, 0xf)  // row_shr:1
    DPP_ADD(0x112, 0xf)  // row_shr:2
    DPP_ADD(0x114, 0xf)  // row_shr:4
    DPP_ADD(0x118, 0xf)  // row_shr:8
    DPP_ADD(0x142, 0xa)  // row_bcast:15 into rows 1 and 3
    DPP_ADD(0x143, 0xc)  // row_bcast:31 into rows 2 and 3
#undef DPP_ADD
    return v;
}
// inclusive scan of one int per thread over the 256 threads of the workgroup; part: 4 ints of LDS
// scratch; two barriers
static __device__ inline int block_scan_incl(int v, int32_t* part) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_scan_incl(v);
    __syncthreads();  // part[] may still be read from a previous call
    if (lane == 63) part[wave] = v;
    __syncthreads();
    for (int ww = 0; ww < wave; ++ww) v += part[ww];
    return v;
}

// Number of integers in [a, a + len) that are congruent to x modulo 8 (a >= 0, 0 <= x < 8)
static __device__ inline int sched_count_mod8(int a, int len, int x) {
    return ((a + len - 1 - x) >> 3) - ((a - 1 - x) >> 3);  // arithmetic shifts: floor division
}

__global__ __launch_bounds__(256) void schedule_kernel(const int32_t* __restrict__ offsets, int E_local,
                                                       int bm, int bn, int nt1, int grid1,
                                                       TileDesc* __restrict__ t1, int nt2, int grid2,
                                                       TileDesc* __restrict__ t2, int host_rows, int nsplit1,
                                                       int nsplit2, int rows_cap, int32_t* __restrict__ refused_out) {
    __shared__ int32_t s_off[257];
    __shared__ int32_t s_mte[256];     // row tiles of expert e
    __shared__ int32_t s_pre[257];     // pieces per weight-row tile of the experts before e; [E_local] = total
    __shared__ int32_t s_len[8][257];  // tiles in XCD x's queue before those of expert e; [E_local] = length
    __shared__ int32_t s_wave[8][4];
    __shared__ int32_t s_part[4];
    __shared__ int32_t s_tot[SCHED_CAPS + 2][4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // host_rows >= 0: one group of host_rows rows (the router GEMM), no offsets array to read
    int nblk_e = 0;  // 32-row blocks of expert tid
    if (tid < E_local) {
        const int n = host_rows >= 0 ? host_rows : offsets[tid + 1] - offsets[tid];
        nblk_e = (n + 31) / 32;
    }
    for (int i = tid; i <= E_local; i += 256) s_off[i] = host_rows >= 0 ? i * host_rows : offsets[i];
    const int hmax = bm / 32, hmin = sched_min_cap_blocks(bm);
    // totals over the experts: 32-row blocks, loaded experts, row tiles for every candidate cap
    int tot[SCHED_CAPS + 2];
    tot[0] = nblk_e;
    tot[SCHED_CAPS + 1] = nblk_e > 0 ? 1 : 0;
#pragma unroll
    for (int c = 0; c < SCHED_CAPS; ++c) {
        const int h = hmax - c;
        tot[c + 1] = (h >= hmin && nblk_e > 0) ? (nblk_e + h - 1) / h : 0;
    }
    {
#pragma unroll
        for (int c = 0; c < SCHED_CAPS + 2; ++c) {
            const int incl = wave_scan_incl(tot[c]);
            if (lane == 63) s_tot[c][wave] = incl;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < SCHED_CAPS + 2; ++c) tot[c] = s_tot[c][0] + s_tot[c][1] + s_tot[c][2] + s_tot[c][3];
    }

    for (int which = 0; which < 2; ++which) {
        const int nt = which ? nt2 : nt1;
        const int grid = which ? grid2 : grid1;
        TileDesc* table = which ? t2 : t1;
        if (grid <= 0) continue;  // uniform
        // ---- pick the cap --------------------------------------------------------------------
        int cap = hmax, MT = 0;
        float best = 3.0e38f;
        const int nsplit = which ? nsplit2 : nsplit1;  // reduction splits: workgroups per table entry
#pragma unroll
        for (int c = 0; c < SCHED_CAPS; ++c) {
            const int tiles = tot[c + 1];
            if (tiles > 0 && (long long)tiles * nt + 8 <= grid) {
                const int rounds = (tiles * nt * nsplit + SCHED_CU - 1) / SCHED_CU;
                const float est = (float)rounds * ((float)tot[0] / (float)tiles + SCHED_TILE_OVERHEAD);
                if (est < best) {  // ties keep the taller tile
                    best = est;
                    cap = hmax - c;
                    MT = tiles;
                }
            }
        }
        // ---- pieces and the dense queue of every XCD -------------------------------------------
        const int mte_mine = (nblk_e + cap - 1) / cap;
        // second attempt: single-tile pieces, whose queues (at most ceil(MT * nt / 8) long) always fit
        for (int attempt = 0; attempt < 2; ++attempt) {
            int cmax = 1;
            if (attempt == 0) {
                const long long per64 = (long long)MT * nt / 64;
                cmax = per64 < 1 ? 1 : (per64 > SCHED_PIECE_MAX ? SCHED_PIECE_MAX : (int)per64);
            }
            int pp = (mte_mine + cmax - 1) / cmax;
            const int pp_incl = block_scan_incl(pp, s_part);
            int mine[8];
            if (pp > 0) {
                // the expert's pieces are S .. S + pp * nt - 1; those of its first prem row ranges are
                // one tile longer
                const int S = (pp_incl - pp) * nt, pbase = mte_mine / pp, prem = mte_mine % pp;
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    mine[x] = (pbase + 1) * sched_count_mod8(S, prem * nt, x) +
                              pbase * sched_count_mod8(S + prem * nt, (pp - prem) * nt, x);
            } else {
#pragma unroll
                for (int x = 0; x < 8; ++x) mine[x] = 0;
            }
            __syncthreads();  // the tables of the previous attempt or GEMM are no longer read
            s_mte[tid] = mte_mine;
            s_pre[tid + 1] = pp_incl;
            if (tid == 0) s_pre[0] = 0;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                mine[x] = wave_scan_incl(mine[x]);
                if (lane == 63) s_wave[x][wave] = mine[x];
            }
            __syncthreads();
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                int v = mine[x];
                for (int ww = 0; ww < wave; ++ww) v += s_wave[x][ww];
                s_len[x][tid + 1] = v;
                if (tid == 0) s_len[x][0] = 0;
            }
            __syncthreads();
            int longest = 0;
#pragma unroll
            for (int x = 0; x < 8; ++x) longest = max(longest, s_len[x][E_local]);
            if (8 * longest <= grid) break;  // uniform
        }

        // Offsets beyond the bound the launches and the buffers were sized for: nothing is scheduled (every
        // entry stays empty, so no kernel touches a row) and the refusal is recorded for the caller.
        const bool refused = host_rows < 0 && s_off[E_local] > rows_cap;
        if (which == 0 && refused_out != nullptr && blockIdx.x == 0 && tid == 0) *refused_out = refused ? 1 : 0;
        for (int b = blockIdx.x * 256 + tid; b < grid; b += gridDim.x * 256) {
            const int x = b & 7, j = b >> 3;
            TileDesc td;
            td.expert = 0; td.row0 = 0; td.rows = 0; td.n0 = 0;
            if (!refused && j < s_len[x][E_local]) {
                // the expert e with s_len[x][e] <= j < s_len[x][e + 1]
                int lo = 0, hi = E_local;
                while (hi - lo > 1) {
                    int mid = (lo + hi) >> 1;
                    if (s_len[x][mid] <= j) lo = mid; else hi = mid;
                }
                const int e = lo;
                const int mte = s_mte[e], pp = s_pre[e + 1] - s_pre[e];
                const int S = s_pre[e] * nt;
                const int pbase = mte / pp, prem = mte % pp;
                // this queue's pieces of the expert: first + 8 i, the long ones come first
                const int first = S + ((x - S) & 7);
                const int n_long = sched_count_mod8(S, prem * nt, x);
                const int r = j - s_len[x][e];
                int i, pos;
                if (r < n_long * (pbase + 1)) {
                    i = r / (pbase + 1);
                    pos = r % (pbase + 1);
                } else {
                    const int rs = r - n_long * (pbase + 1);
                    i = n_long + rs / pbase;
                    pos = rs % pbase;
                }
                const int q = first + 8 * i - S;
                const int pc = q / nt, ni = q % nt;
                const int mi = pc * pbase + min(pc, prem) + pos;
                const int e_rows = s_off[e + 1] - s_off[e];
                // 32-row blocks of the expert, dealt evenly to its mte tiles
                const int nblk = (e_rows + 31) / 32;
                const int base = nblk / mte, rem = nblk % mte;
                const int blk0 = mi * base + min(mi, rem);
                const int nb = base + (mi < rem ? 1 : 0);
                td.expert = e;
                td.row0 = s_off[e] + blk0 * 32;
                td.rows = min(nb * 32, e_rows - blk0 * 32);
                td.n0 = ni * bn;
            }
            table[b] = td;
        }
    }
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
#undef DECL

int gemm_class_rows(int cls) { return kClassRows[cls]; }

int gemm_pick_class(double rows_per_expert) {
    // Measured (Mixtral shape and the expert-parallel share, layer time): below 12 rows per expert the
    // 128-row class is the fastest of the weight-streaming launches (4 to 8 rows per expert: 0.225 / 0.238 /
    // 0.235 ms for the classes 0 / 5 / 1 on the expert-parallel share); from 12 to 24 rows per expert the
    // decode class (16 and 24 rows per expert on the Mixtral shape: 0.562 against 0.572 and 0.566 against
    // 0.580 ms); above that the tall class (it wins from about 32 rows per expert upwards).
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
    return p;
}

hipError_t gemm_init_attributes() {
    hipError_t err = gemm_set_attr_swiglu();
    if (err == hipSuccess) err = gemm_set_attr_plain();
    if (err == hipSuccess) err = gemm_set_attr_pairsum();
    if (err == hipSuccess) err = gemm_set_attr_partial();
    return err;
}

hipError_t launch_schedule(const GemmPlan& p, const int32_t* offsets, int E_local, TileDesc* t1, TileDesc* t2,
                           int nsplit2, int64_t rows_cap, int32_t* refused, hipStream_t st) {
    int g = p.grid1 > p.grid2 ? p.grid1 : p.grid2;
    int blocks = (g + 1023) / 1024;
    if (blocks < 1) blocks = 1;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(schedule_kernel, dim3(blocks), dim3(256), 0, st, offsets, E_local, p.bm, p.bn, p.nt1,
                       p.grid1, t1, p.nt2, p.grid2, t2, -1, 1, nsplit2, (int)rows_cap, refused);
    return hipGetLastError();
}

hipError_t launch_gemm1(const GemmPlan& p, const uint16_t* X, int ldx, const int32_t* row_map,
                        const uint16_t* W13f, int d, int f, uint16_t* H, const TileDesc* table, hipStream_t st) {
    if (p.grid1 <= 0) return hipSuccess;
    return gemm_launch_swiglu(p.cls, p.grid1, X, ldx, row_map, W13f, 2 * f, d, H, moe_ld_pad(f), table, 1, 0, st);
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
        // decode class: the launch only streams weights; split until every compute unit holds as many workgroups
        // as fit on it (each keeps two K steps of its weight panel in flight)
        const double want = (double)SCHED_CU * kClassPerCu[GEMM_DECODE];
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
        return gemm_launch_plain(p.cls, p.grid2, H, moe_ld_pad(f), nullptr, W2f, d, f, Y, d, table, 1, 0, st);
    const size_t slab_elems = (size_t)n_rows * d;
    hipError_t e = gemm_launch_partial(p.cls, p.grid2, H, moe_ld_pad(f), nullptr, W2f, d, f / nsplit, (uint16_t*)part, d,
                                       table, nsplit, slab_elems * 4, st);
    if (e != hipSuccess) return e;
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
        hipLaunchKernelGGL(schedule_kernel, dim3((grid + 1023) / 1024), dim3(256), 0, st, (const int32_t*)nullptr, 1,
                           kClassRows[c], GEMM_BN, nt, grid, table, 0, 0, (TileDesc*)nullptr, T, pk.nsplit, 1, T,
                           (int32_t*)nullptr);
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
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][j];
    if (s == 1.2345e-30f) g_mfma_rate_sink = s;  // practically never taken: keeps the sums live
}

hipError_t launch_mfma_rate(int iters_per_wave, double* flop, hipStream_t st) {
    const int grid = SCHED_CU * 8;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(256), 0, st, iters_per_wave);
    *flop = (double)grid * 4 * (double)iters_per_wave * 64 * (2.0 * 32 * 32 * 16);
    return hipGetLastError();
}
