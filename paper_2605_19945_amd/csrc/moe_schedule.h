// Device-side work list of the grouped GEMMs: shared by the stand-alone scheduling kernel (moe_gemm.hip) and the
// dispatch kernels that build the work lists in the same launch as the permutation (moe_permute.hip).
#pragma once
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

// Builds this workgroup's share (entries part*256 + tid, + parts*256, ...) of both work lists.  s_off: the
// exclusive prefix of the experts' rows, [E_local + 1] entries in SHARED memory, written by the caller and
// published by a barrier before the call.  All 256 threads of the workgroup must call.
static __device__ inline void schedule_tables(const SchedArgs& a, const int32_t* s_off, int part, int parts) {
    __shared__ int32_t s_mte[256];     // row tiles of expert e
    __shared__ int32_t s_pre[257];     // pieces per weight-row tile of the experts before e; [E_local] = total
    __shared__ int32_t s_len[8][257];  // tiles in XCD x's queue before those of expert e; [E_local] = length
    __shared__ int32_t s_wave[8][4];
    __shared__ int32_t s_part[4];
    __shared__ int32_t s_tot[SCHED_CAPS + 2][4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int E_local = a.E_local;
    int nblk_e = 0;  // 32-row blocks of expert tid
    if (tid < E_local) nblk_e = (s_off[tid + 1] - s_off[tid] + 31) / 32;
    const int hmax = a.bm / 32, hmin = sched_min_cap_blocks(a.bm);
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
        const int nt = which ? a.nt2 : a.nt1;
        const int grid = which ? a.grid2 : a.grid1;
        TileDesc* table = which ? a.t2 : a.t1;
        if (grid <= 0) continue;  // uniform
        // ---- pick the cap --------------------------------------------------------------------
        int cap = hmax, MT = 0;
        float best = 3.0e38f;
        const int nsplit = which ? a.nsplit2 : a.nsplit1;  // reduction splits: workgroups per table entry
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
        const bool refused = a.rows_cap >= 0 && s_off[E_local] > a.rows_cap;
        if (which == 0 && a.refused_out != nullptr && part == 0 && tid == 0) *a.refused_out = refused ? 1 : 0;
        for (int b = part * 256 + tid; b < grid; b += parts * 256) {
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
                td.n0 = ni * a.bn;
            }
            table[b] = td;
        }
    }
}

