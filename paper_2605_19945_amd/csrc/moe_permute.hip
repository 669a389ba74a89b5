// Dispatch by expert: a stable counting sort of the (token, slot) assignments by resident expert.
//
// The paper says only that every token is sent to the GPUs that host its experts (Sec. 2.1);
// inside one GPU that is the grouping of rows by expert computed here.
// Order inside an expert is ascending token id, so the result is unique and reproducible.
//
// Three small kernels, no atomics on global memory, no waiting between workgroups (up to 512 tokens:
// one kernel, one workgroup, the same steps):
//   1. per-256-token block histogram of resident experts,
//   2. one workgroup: exclusive scan over blocks (per expert) and over experts -> offsets,
//   3. per block: rank of every assignment among the block's earlier tokens, from per-wavefront
//      64-bit membership masks in LDS -> row_of, tok_of.
// The row copy itself (xp[row_of[t, j]] = x[t]) is a separate streaming kernel.
#include <stdio.h>

#include <mutex>

#include "moe_internal.h"
#include "moe_schedule.h"

constexpr int PB = 256;  // tokens per block (one token per thread)
constexpr int PW = PB / 64;
// A token's selected experts are fetched into registers in one go (all loads in flight together) before any
// of them is used for an LDS atomic: written as load-then-atomic per entry, the k loads run one after the
// other, a full memory round trip each.  Entries past KREG are read where they are used.
constexpr int KREG = 8;
static __device__ inline void load_topk(const int32_t* __restrict__ p, int k, int (&ev)[KREG]) {
#pragma unroll
    for (int j = 0; j < KREG; ++j) ev[j] = j < k ? p[j] : 0;
}
// f(j, expert) for every entry j < k of a token
template <class F>
static __device__ inline void for_topk(const int (&ev)[KREG], const int32_t* __restrict__ p, int k, F&& f) {
#pragma unroll
    for (int j = 0; j < KREG; ++j)
        if (j < k) f(j, ev[j]);
    for (int j = KREG; j < k; ++j) f(j, p[j]);
}

__global__ __launch_bounds__(PB) void permute_hist_kernel(const int32_t* __restrict__ idx, int T, int k,
                                                          int e_lo, int E_local,
                                                          int32_t* __restrict__ blockhist) {
    extern __shared__ int32_t hist[];  // [E_local]
    for (int e = threadIdx.x; e < E_local; e += PB) hist[e] = 0;
    __syncthreads();
    int t = blockIdx.x * PB + threadIdx.x;
    if (t < T)
        for (int j = 0; j < k; ++j) {
            int e = idx[(size_t)t * k + j] - e_lo;
            if (e >= 0 && e < E_local) atomicAdd(&hist[e], 1);
        }
    __syncthreads();
    for (int e = threadIdx.x; e < E_local; e += PB) blockhist[(size_t)blockIdx.x * E_local + e] = hist[e];
}

// One workgroup of 256 threads; E_local <= 256.  blockhist[b][e] becomes the number of
// assignments to e in blocks before b; offsets[e] the exclusive prefix over experts.
__global__ __launch_bounds__(256) void permute_scan_kernel(int32_t* __restrict__ blockhist, int nblk,
                                                           int E_local, int32_t* __restrict__ offsets) {
    __shared__ int32_t tot[256];
    int e = threadIdx.x;
    int run = 0;
    if (e < E_local)
        for (int b = 0; b < nblk; ++b) {
            int c = blockhist[(size_t)b * E_local + e];
            blockhist[(size_t)b * E_local + e] = run;
            run += c;
        }
    tot[e] = e < E_local ? run : 0;
    __syncthreads();
    // inclusive Hillis-Steele scan over 256 entries
    for (int off = 1; off < 256; off <<= 1) {
        int v = e >= off ? tot[e - off] : 0;
        __syncthreads();
        tot[e] += v;
        __syncthreads();
    }
    if (e < E_local) offsets[e + 1] = tot[e];
    if (e == 0) offsets[0] = 0;
}

__global__ __launch_bounds__(PB) void permute_rank_kernel(const int32_t* __restrict__ idx, int T, int k,
                                                          int e_lo, int E_local,
                                                          const int32_t* __restrict__ blockhist,
                                                          const int32_t* __restrict__ offsets,
                                                          int32_t* __restrict__ row_of,
                                                          int32_t* __restrict__ tok_of) {
    extern __shared__ unsigned long long masks[];  // [PW][E_local] lanes of wave w that selected e
    int32_t* wbase = (int32_t*)(masks + PW * E_local);  // [PW][E_local] rows of e in earlier waves
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int o = tid; o < PW * E_local; o += PB) masks[o] = 0ull;
    __syncthreads();
    const int t = blockIdx.x * PB + tid;
    if (t < T)
        for (int j = 0; j < k; ++j) {
            int e = idx[(size_t)t * k + j] - e_lo;
            if (e >= 0 && e < E_local) atomicOr(&masks[wave * E_local + e], 1ull << lane);
        }
    __syncthreads();
    for (int e = tid; e < E_local; e += PB) {
        int run = offsets[e] + blockhist[(size_t)blockIdx.x * E_local + e];
#pragma unroll
        for (int ww = 0; ww < PW; ++ww) {
            wbase[ww * E_local + e] = run;
            run += __popcll(masks[ww * E_local + e]);
        }
    }
    __syncthreads();
    if (t < T) {
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int j = 0; j < k; ++j) {
            int e = idx[(size_t)t * k + j] - e_lo;
            int r = -1;
            if (e >= 0 && e < E_local) {
                r = wbase[wave * E_local + e] + __popcll(masks[wave * E_local + e] & below);
                tok_of[r] = t;
            }
            row_of[(size_t)t * k + j] = r;
        }
    }
}

// The same three steps in ONE workgroup, for up to PF_BLOCKS blocks of 256 tokens: at decode-sized
// batches the three launches and the gaps between them cost more than the work (permute + work-list
// stage at 64 tokens: 29 -> 17 us; from about four blocks on the three kernels are faster).
constexpr int PF_BLOCKS = 2;
// PLAN (plan_small_kernel of the layer): workgroup 0 also counts the assignments of all E experts (counts_out,
// may be null); the workgroups after it build the work lists of the expert GEMMs, each from a histogram of
// its own over the few hundred tokens (cheaper than a second launch that waits for workgroup 0's offsets; one
// work-list entry costs a thread about as long as the whole permutation, so they are spread over many
// workgroups).
template <bool PLAN>
__global__ __launch_bounds__(PB) void permute_fused_kernel(const int32_t* __restrict__ idx, int T, int k, int e_lo,
                                                           int E_local, int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ row_of,
                                                           int32_t* __restrict__ tok_of, int E,
                                                           int32_t* __restrict__ counts_out, SchedArgs a) {
    __shared__ int32_t hist[PF_BLOCKS * 256];         // [block][E_local] -> assignments to e in earlier blocks
    __shared__ unsigned long long masks[PW * 256];   // [wave][E_local]
    __shared__ int32_t wbase[PW * 256];
    __shared__ int32_t tot[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblk = (T + PB - 1) / PB;
    if constexpr (PLAN) {
        if (blockIdx.x > 0) {
            __shared__ int32_t s_scan[4];
            int32_t* s_off = hist;  // [E_local + 1]
            tot[tid] = 0;
            __syncthreads();
            int evs[PF_BLOCKS][KREG];
#pragma unroll
            for (int b = 0; b < PF_BLOCKS; ++b)
                if (b * PB + tid < T) load_topk(idx + (size_t)(b * PB + tid) * k, k, evs[b]);
#pragma unroll
            for (int b = 0; b < PF_BLOCKS; ++b)
                if (b * PB + tid < T)
                    for_topk(evs[b], idx + (size_t)(b * PB + tid) * k, k, [&](int, int eg) {
                        const int e = eg - e_lo;
                        if (e >= 0 && e < E_local) atomicAdd(&tot[e], 1);
                    });
            __syncthreads();
            const int incl = block_scan_incl(tot[tid], s_scan);  // tot is 0 beyond E_local
            if (tid < E_local) s_off[tid + 1] = incl;
            if (tid == 0) s_off[0] = 0;
            __syncthreads();
            schedule_tables(a, s_off, blockIdx.x - 1, gridDim.x - 1);
            return;
        }
    }
    int evs[PF_BLOCKS][KREG];  // this thread's tokens (one per block of PB) stay in registers throughout
#pragma unroll
    for (int b = 0; b < PF_BLOCKS; ++b)
        if (b * PB + tid < T) load_topk(idx + (size_t)(b * PB + tid) * k, k, evs[b]);
    for (int o = tid; o < nblk * E_local; o += PB) hist[o] = 0;
    if (PLAN && counts_out != nullptr) wbase[tid] = 0;  // (free until the ranks) assignments per expert, all E
    __syncthreads();
#pragma unroll
    for (int b = 0; b < PF_BLOCKS; ++b) {
        const int t = b * PB + tid;
        if (t < T)
            for_topk(evs[b], idx + (size_t)t * k, k, [&](int, int eg) {
                if (PLAN && counts_out != nullptr) atomicAdd(&wbase[eg], 1);
                const int e = eg - e_lo;
                if (e >= 0 && e < E_local) atomicAdd(&hist[b * E_local + e], 1);
            });
    }
    __syncthreads();
    if (PLAN && counts_out != nullptr && tid < E) counts_out[tid] = wbase[tid];
    int run = 0;
    if (tid < E_local)
        for (int b = 0; b < nblk; ++b) {
            const int c = hist[b * E_local + tid];
            hist[b * E_local + tid] = run;
            run += c;
        }
    tot[tid] = run;  // 0 beyond E_local
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {  // inclusive Hillis-Steele scan
        const int v = tid >= off ? tot[tid - off] : 0;
        __syncthreads();
        tot[tid] += v;
        __syncthreads();
    }
    if (tid < E_local) offsets[tid + 1] = tot[tid];
    if (tid == 0) offsets[0] = 0;
#pragma unroll
    for (int b = 0; b < PF_BLOCKS; ++b) {
        if (b >= nblk) break;  // uniform
        for (int o = tid; o < PW * E_local; o += PB) masks[o] = 0ull;
        __syncthreads();
        const int t = b * PB + tid;
        if (t < T)
            for_topk(evs[b], idx + (size_t)t * k, k, [&](int, int eg) {
                const int e = eg - e_lo;
                if (e >= 0 && e < E_local) atomicOr(&masks[wave * E_local + e], 1ull << lane);
            });
        __syncthreads();
        for (int e = tid; e < E_local; e += PB) {
            int r = (e > 0 ? tot[e - 1] : 0) + hist[b * E_local + e];  // tot is the inclusive scan
#pragma unroll
            for (int ww = 0; ww < PW; ++ww) {
                wbase[ww * E_local + e] = r;
                r += __popcll(masks[ww * E_local + e]);
            }
        }
        __syncthreads();
        if (t < T) {
            const unsigned long long below = (1ull << lane) - 1ull;
            for_topk(evs[b], idx + (size_t)t * k, k, [&](int j, int eg) {
                const int e = eg - e_lo;
                int r = -1;
                if (e >= 0 && e < E_local) {
                    r = wbase[wave * E_local + e] + __popcll(masks[wave * E_local + e] & below);
                    tok_of[r] = t;
                }
                row_of[(size_t)t * k + j] = r;
            });
        }
        __syncthreads();  // masks and wbase are rewritten for the next block
    }
}

// ---- dispatch inside moe_layer_forward: permutation and GEMM work lists together -------------------------
// The router has already counted the assignments per expert, and the work lists of the expert GEMMs depend on
// nothing else; only the ranks need the per-block histograms.  So the layer runs
//     plan_kernel:           blocks [0, nblk): block histograms (as permute_hist_kernel)
//                            the other blocks: offsets from the router's counts, both work lists
//     permute_rank2_kernel:  per block, the prefix over the earlier blocks' histograms (the scan of
//                            permute_scan_kernel, redone by every block: nblk * E_local integers), then the ranks
// two launches between the router and the first GEMM instead of four (histogram, scan, ranks, work lists), and
// the work lists, the longest of them, are built next to the histograms instead of after the ranks.  Up to
// PF_BLOCKS blocks of tokens everything happens in ONE launch (plan_small_kernel) whose first workgroup also
// counts the assignments itself, so that the router can skip its cross-workgroup count reduction.
constexpr int PLAN_COPIES = 32;
constexpr int PLAN_OWN_COUNT_MAX = 16384;  // indices a work-list workgroup counts itself (64 per thread)
__global__ __launch_bounds__(PB) void plan_kernel(const int32_t* __restrict__ idx, int T, int k, int e_lo, int nblk,
                                                  int32_t* __restrict__ blockhist,
                                                  const int32_t* __restrict__ counts_in, int E,
                                                  int32_t* __restrict__ counts_out,
                                                  int32_t* __restrict__ offsets, SchedArgs a) {
    const int E_local = a.E_local;
    const int tid = threadIdx.x;
    if ((int)blockIdx.x < nblk) {
        __shared__ int32_t hist[256];
        const int t = blockIdx.x * PB + tid;
        int ev[KREG];
        if (t < T) load_topk(idx + (size_t)t * k, k, ev);
        hist[tid] = 0;
        __syncthreads();
        if (t < T)
            for_topk(ev, idx + (size_t)t * k, k, [&](int, int eg) {
                const int e = eg - e_lo;
                if (e >= 0 && e < E_local) atomicAdd(&hist[e], 1);
            });
        __syncthreads();
        if (tid < E_local) blockhist[(size_t)blockIdx.x * E_local + tid] = hist[tid];
        return;
    }
    __shared__ int32_t s_off[257];
    __shared__ int32_t s_scan[4];
    const int part = blockIdx.x - nblk, parts = gridDim.x - nblk;
    int rows;
    if (counts_in != nullptr) {
        rows = tid < E_local ? counts_in[e_lo + tid] : 0;
    } else {
        // No counts from the router (it skips its cross-workgroup reduction for batches this small): every
        // work-list workgroup counts all T * k indices itself, into PLAN_COPIES histograms picked by thread
        // so that few lanes meet on one address even with a handful of experts.
        __shared__ int32_t h[PLAN_COPIES * 257];
        int Ep = 8;
        while (Ep < E) Ep <<= 1;
        const int C = 2048 / Ep < PLAN_COPIES ? 2048 / Ep : PLAN_COPIES, stride = Ep + 1;
        for (int o = tid; o < C * stride; o += PB) h[o] = 0;
        __syncthreads();
        int32_t* mine = h + (tid % C) * stride;
        const int n = T * k, n4 = n >> 2;
        const int4* idx4 = (const int4*)idx;  // (256-byte aligned workspace)
        for (int base = 0; base < n4; base += 8 * PB) {
            int4 v[8];  // eight 16-byte loads in flight per thread, then the atomics
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = base + u * PB + tid;
                v[u] = i < n4 ? idx4[i] : make_int4(-1, -1, -1, -1);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (v[u].x >= 0) {
                    atomicAdd(&mine[v[u].x], 1);
                    atomicAdd(&mine[v[u].y], 1);
                    atomicAdd(&mine[v[u].z], 1);
                    atomicAdd(&mine[v[u].w], 1);
                }
        }
        for (int i = 4 * n4 + tid; i < n; i += PB) atomicAdd(&mine[idx[i]], 1);
        __syncthreads();
        int all = 0;  // assignments to expert tid, resident or not
        if (tid < E)
            for (int c = 0; c < C; ++c) all += h[c * stride + tid];
        if (part == 0 && counts_out != nullptr && tid < E) counts_out[tid] = all;
        __syncthreads();
        if (tid < E) h[tid] = all;
        __syncthreads();
        rows = tid < E_local ? h[e_lo + tid] : 0;
    }
    const int incl = block_scan_incl(rows, s_scan);
    if (tid < E_local) s_off[tid + 1] = incl;
    if (tid == 0) s_off[0] = 0;
    __syncthreads();
    if (part == 0)
        for (int i = tid; i <= E_local; i += PB) offsets[i] = s_off[i];
    schedule_tables(a, s_off, part, parts);
}

__global__ __launch_bounds__(PB) void permute_rank2_kernel(const int32_t* __restrict__ idx, int T, int k, int e_lo,
                                                           int E_local, const int32_t* __restrict__ blockhist,
                                                           const int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ row_of, int32_t* __restrict__ tok_of) {
    extern __shared__ unsigned long long masks[];          // [PW][E_local] lanes of wave w that selected e
    int32_t* wbase = (int32_t*)(masks + PW * E_local);     // [PW][E_local] rows of e in earlier waves
    int32_t* before = wbase + PW * E_local;                // [E_local] assignments to e in earlier blocks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.x * PB + tid;
    int ev[KREG];
    if (t < T) load_topk(idx + (size_t)t * k, k, ev);
    const int off_mine = tid < E_local ? offsets[tid] : 0;
    for (int o = tid; o < PW * E_local; o += PB) masks[o] = 0ull;
    for (int e = tid; e < E_local; e += PB) before[e] = 0;
    __syncthreads();
    // prefix over the earlier blocks: thread (g, e) adds the blocks g, g + G, ... and the G partial sums meet in LDS
    int Ep = 1;
    while (Ep < E_local) Ep <<= 1;
    const int G = PB / Ep, e_mine = tid % Ep, g = tid / Ep;
    if (e_mine < E_local) {
        int sum = 0;
        for (int b = g; b < (int)blockIdx.x; b += G) sum += blockhist[(size_t)b * E_local + e_mine];
        if (sum != 0) atomicAdd(&before[e_mine], sum);
    }
    if (t < T)
        for_topk(ev, idx + (size_t)t * k, k, [&](int, int eg) {
            const int e = eg - e_lo;
            if (e >= 0 && e < E_local) atomicOr(&masks[wave * E_local + e], 1ull << lane);
        });
    __syncthreads();
    for (int e = tid; e < E_local; e += PB) {  // (E_local <= PB: e == tid)
        int run = off_mine + before[e];
#pragma unroll
        for (int ww = 0; ww < PW; ++ww) {
            wbase[ww * E_local + e] = run;
            run += __popcll(masks[ww * E_local + e]);
        }
    }
    __syncthreads();
    if (t < T) {
        const unsigned long long below = (1ull << lane) - 1ull;
        for_topk(ev, idx + (size_t)t * k, k, [&](int j, int eg) {
            const int e = eg - e_lo;
            int r = -1;
            if (e >= 0 && e < E_local) {
                r = wbase[wave * E_local + e] + __popcll(masks[wave * E_local + e] & below);
                tok_of[r] = t;
            }
            row_of[(size_t)t * k + j] = r;
        });
    }
}

hipError_t launch_permute(const int32_t* idx, int T, int k, int e_lo, int E_local, int32_t* blockhist,
                          int32_t* offsets, int32_t* row_of, int32_t* tok_of, hipStream_t st) {
    int nblk = (T + PB - 1) / PB;
    if (nblk <= PF_BLOCKS) {
        hipLaunchKernelGGL(permute_fused_kernel<false>, dim3(1), dim3(PB), 0, st, idx, T, k, e_lo, E_local, offsets,
                           row_of, tok_of, 0, (int32_t*)nullptr, SchedArgs{});
        return hipGetLastError();
    }
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nblk), dim3(PB), E_local * sizeof(int32_t), st, idx, T, k,
                       e_lo, E_local, blockhist);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(256), 0, st, blockhist, nblk, E_local, offsets);
    size_t smem = (size_t)PW * E_local * (sizeof(unsigned long long) + sizeof(int32_t));
    hipLaunchKernelGGL(permute_rank_kernel, dim3(nblk), dim3(PB), smem, st, idx, T, k, e_lo, E_local,
                       blockhist, offsets, row_of, tok_of);
    return hipGetLastError();
}

bool dispatch_plan_counts_itself(int T, int k) { return (long long)T * k <= PLAN_OWN_COUNT_MAX; }

// Permutation plus work lists of the layer (see plan_kernel).  counts: the router's per-expert counts over all E
// experts; with dispatch_plan_counts_itself(T, k) they are an OUTPUT here (or null), otherwise an input.
hipError_t launch_dispatch_plan(const int32_t* idx, int T, int k, int E, int e_lo, int32_t* blockhist, int32_t* counts,
                                int32_t* offsets, int32_t* row_of, int32_t* tok_of, const SchedArgs& a, int sched_blocks,
                                hipStream_t st) {
    const int nblk = (T + PB - 1) / PB, E_local = a.E_local;
    if (nblk <= PF_BLOCKS) {
        hipLaunchKernelGGL(permute_fused_kernel<true>, dim3(1 + sched_blocks), dim3(PB), 0, st, idx, T, k, e_lo, E_local, offsets,
                           row_of, tok_of, E, counts, a);
        return hipGetLastError();
    }
    const bool own = dispatch_plan_counts_itself(T, k);
    hipLaunchKernelGGL(plan_kernel, dim3(nblk + sched_blocks), dim3(PB), 0, st, idx, T, k, e_lo, nblk, blockhist,
                       own ? (const int32_t*)nullptr : (const int32_t*)counts, E, own ? counts : (int32_t*)nullptr,
                       offsets, a);
    const size_t smem = (size_t)PW * E_local * (sizeof(unsigned long long) + sizeof(int32_t)) + (size_t)E_local * 4;
    hipLaunchKernelGGL(permute_rank2_kernel, dim3(nblk), dim3(PB), smem, st, idx, T, k, e_lo, E_local,
                       (const int32_t*)blockhist, (const int32_t*)offsets, row_of, tok_of);
    return hipGetLastError();
}

// xp[row_of[t, j], :] = x[t, :] for every local assignment: one wavefront per token reads the row once
// (16 bytes per lane, four chunks in flight) and stores it to its up-to-k destination rows; rows of xp
// that no assignment maps to are left untouched.  Grid-stride over tokens.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4* __restrict__ x,
                                                           const int32_t* __restrict__ row_of, int T, int k,
                                                           int chunks /* d / 8 */, uint4* __restrict__ xp) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int t = blockIdx.x * 4 + wave; t < T; t += gridDim.x * 4) {
        const uint4* src = x + (size_t)t * chunks;
        const int32_t* dst_rows = row_of + (size_t)t * k;
        for (int c0 = 0; c0 < chunks; c0 += 256) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 64 + lane;
                if (c < chunks) v[u] = load_stream(src + c);
            }
            for (int j = 0; j < k; ++j) {
                const int r = dst_rows[j];
                if (r < 0) continue;  // expert not resident (wave-uniform)
                uint4* dst = xp + (size_t)r * chunks;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u * 64 + lane;
                    if (c < chunks) store_stream(dst + c, v[u]);
                }
            }
        }
    }
}

hipError_t launch_gather(const uint16_t* x, const int32_t* row_of, int T, int k, int d, uint16_t* xp,
                         hipStream_t st) {
    int blocks = (T + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks), dim3(256), 0, st, (const uint4*)x, row_of, T, k, d / 8,
                       (uint4*)xp);
    return hipGetLastError();
}

// out[t, :] = sum_j w[t, j] * y[row_of[t, j], :], fp32, slot order, one 16-byte store per lane.
static __device__ inline float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
static __device__ inline float bf16hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
static __device__ inline uint32_t pack_bf16x2(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}

// STREAM: non-temporal loads and stores, for expert outputs too large to still sit in the last-level cache
// (2 x 268 MB + 537 MB moved: 263 against 270 us; at 34 + 67 MB, straight behind the GEMM that wrote the
// rows, plain accesses are faster: 16.0 against 17.9 us).
template <bool STREAM>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y,
                                                      const int32_t* __restrict__ row_of,
                                                      const float* __restrict__ w, int T, int k,
                                                      int chunks /* d / 8 */, uint4* __restrict__ out) {
    const int chunks_per_block = blockDim.x;
    const int blocks_per_row = (chunks + chunks_per_block - 1) / chunks_per_block;
    const int t = blockIdx.x / blocks_per_row;
    const int c = (blockIdx.x % blocks_per_row) * chunks_per_block + threadIdx.x;
    if (t >= T || c >= chunks) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < k; ++j) {
        int r = row_of[(size_t)t * k + j];
        if (r < 0) continue;
        float g = w[(size_t)t * k + j];
        const uint4 v = STREAM ? load_stream(y + (size_t)r * chunks + c) : y[(size_t)r * chunks + c];
        acc[0] += g * bf16lo(v.x); acc[1] += g * bf16hi(v.x);
        acc[2] += g * bf16lo(v.y); acc[3] += g * bf16hi(v.y);
        acc[4] += g * bf16lo(v.z); acc[5] += g * bf16hi(v.z);
        acc[6] += g * bf16lo(v.w); acc[7] += g * bf16hi(v.w);
    }
    uint4 o;
    o.x = pack_bf16x2(acc[0], acc[1]);
    o.y = pack_bf16x2(acc[2], acc[3]);
    o.z = pack_bf16x2(acc[4], acc[5]);
    o.w = pack_bf16x2(acc[6], acc[7]);
    if (STREAM) store_stream(out + (size_t)t * chunks + c, o);
    else out[(size_t)t * chunks + c] = o;
}

// The same sum when the second GEMM ran as nsplit reduction ranges: the expert output row is first formed from
// its partial sums (added in slab order, rounded to bf16 exactly as reduce_splits_kernel stores it), so the
// result equals moe_combine on the reduced rows bit for bit and the reduced rows are never written.
__global__ __launch_bounds__(256) void combine_split_kernel(const float* __restrict__ part, int nsplit,
                                                            size_t slab_elems, const int32_t* __restrict__ row_of,
                                                            const float* __restrict__ w, int T, int k, int chunks,
                                                            uint4* __restrict__ out) {
    const int chunks_per_block = blockDim.x;
    const int blocks_per_row = (chunks + chunks_per_block - 1) / chunks_per_block;
    const int t = blockIdx.x / blocks_per_row;
    const int c = (blockIdx.x % blocks_per_row) * chunks_per_block + threadIdx.x;
    if (t >= T || c >= chunks) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < k; ++j) {
        const int r = row_of[(size_t)t * k + j];
        if (r < 0) continue;
        const float g = w[(size_t)t * k + j];
        const float* src = part + ((size_t)r * chunks + c) * 8;
        f32x4_t lo = *(const f32x4_t*)src, hi = *(const f32x4_t*)(src + 4);
        for (int sp = 1; sp < nsplit; ++sp) {
            const f32x4_t l2 = *(const f32x4_t*)(src + sp * slab_elems), h2 = *(const f32x4_t*)(src + sp * slab_elems + 4);
            lo[0] += l2[0]; lo[1] += l2[1]; lo[2] += l2[2]; lo[3] += l2[3];
            hi[0] += h2[0]; hi[1] += h2[1]; hi[2] += h2[2]; hi[3] += h2[3];
        }
        for (int q = 0; q < 4; ++q) {
            acc[q] += g * (float)(__bf16)lo[q];
            acc[4 + q] += g * (float)(__bf16)hi[q];
        }
    }
    uint4 o;
    o.x = pack_bf16x2(acc[0], acc[1]);
    o.y = pack_bf16x2(acc[2], acc[3]);
    o.z = pack_bf16x2(acc[4], acc[5]);
    o.w = pack_bf16x2(acc[6], acc[7]);
    out[(size_t)t * chunks + c] = o;
}

hipError_t launch_combine_split(const float* part, int nsplit, size_t slab_elems, const int32_t* row_of, const float* w,
                                int T, int k, int d, uint16_t* out, hipStream_t st) {
    int chunks = d / 8;
    int threads = chunks >= 256 ? 256 : (chunks + 63) / 64 * 64;
    int blocks_per_row = (chunks + threads - 1) / threads;
    hipLaunchKernelGGL(combine_split_kernel, dim3(T * blocks_per_row), dim3(threads), 0, st, part, nsplit, slab_elems,
                       row_of, w, T, k, chunks, (uint4*)out);
    return hipGetLastError();
}

constexpr size_t COMBINE_STREAM_MIN_BYTES = (size_t)128 << 20;  // of expert output rows (upper bound T * k rows)
hipError_t launch_combine(const uint16_t* y, const int32_t* row_of, const float* w, int T, int k, int d,
                          uint16_t* out, hipStream_t st) {
    int chunks = d / 8;
    int threads = chunks >= 256 ? 256 : (chunks + 63) / 64 * 64;
    int blocks_per_row = (chunks + threads - 1) / threads;
    if ((size_t)T * k * d * 2 > COMBINE_STREAM_MIN_BYTES)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(T * blocks_per_row), dim3(threads), 0, st, (const uint4*)y,
                           row_of, w, T, k, chunks, (uint4*)out);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(T * blocks_per_row), dim3(threads), 0, st, (const uint4*)y,
                           row_of, w, T, k, chunks, (uint4*)out);
    return hipGetLastError();
}

// ---- dispatch without a context or a workspace ------------------------------------------------------
// For callers that can neither allocate device memory nor hand over a workspace.  The only scratch the
// three-kernel path needs, the per-block expert histograms, lives in a static device array: every device
// the library runs on holds its own copy, at its own address, until the process ends.  The array's name is
// only a host-side handle; its device address is looked up once per device and the kernels get that address
// as an ordinary argument.  Every entry the scan and rank kernels read is first written by the histogram
// kernel of the same call, so nothing has to be cleared between calls; calls that overlap in time on one
// device share the array and race.
constexpr int PERMUTE_STATIC_INTS = 262144;  // 1 MiB: ceil(T / 256) * E_local block-histogram entries
static __device__ __align__(256) int32_t g_permute_static_scratch[PERMUTE_STATIC_INTS];

constexpr int PERMUTE_MAX_DEVICES = 64;
static int32_t* g_permute_static_ptr[PERMUTE_MAX_DEVICES];  // device address of the array, per device
static std::mutex g_permute_static_mutex;

// Device address of the current device's copy of the static scratch array (looked up on first use).
static hipError_t permute_static_scratch(int32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= PERMUTE_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_permute_static_mutex);
    if (g_permute_static_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_permute_static_scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_permute_static_ptr[dev] = (int32_t*)p;
    }
    *out = g_permute_static_ptr[dev];
    return hipSuccess;
}

extern "C" moe_status moe_permute_noalloc(const void* x, const int32_t* topk_idx, int32_t T, int32_t d, int32_t E,
                                          int32_t k, int32_t e_lo, int32_t E_local, void* xp, int32_t* offsets,
                                          int32_t* row_of, int32_t* tok_of, void* stream) {
    auto misaligned = [](const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; };
    if (T < 0 || T > (1 << 20) || E < 1 || E > 256 || k < 1 || k > 16 || k > E || e_lo < 0 || E_local < 1 ||
        (int64_t)e_lo + E_local > E)
        return MOE_ERR_INVALID_ARG;
    if (topk_idx == nullptr || offsets == nullptr || row_of == nullptr || tok_of == nullptr) return MOE_ERR_INVALID_ARG;
    if (misaligned(topk_idx, 4) || misaligned(offsets, 4) || misaligned(row_of, 4) || misaligned(tok_of, 4))
        return MOE_ERR_INVALID_ARG;
    if (xp != nullptr && (x == nullptr || d < 8 || d % 8 != 0 || misaligned(x, 16) || misaligned(xp, 16)))
        return MOE_ERR_INVALID_ARG;
    const int64_t nblk = ((int64_t)T + PB - 1) / PB;
    if (nblk * E_local > PERMUTE_STATIC_INTS) {
        char msg[200];
        snprintf(msg, sizeof(msg),
                 "moe_permute_noalloc: T = %d tokens and %d resident experts need %lld scratch entries, the static "
                 "array holds %d", T, E_local, (long long)(nblk * E_local), PERMUTE_STATIC_INTS);
        moe_note_error(msg);
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    }
    if (T == 0) return MOE_OK;
    hipStream_t st = (hipStream_t)stream;
    int32_t* scratch = nullptr;
    hipError_t e = permute_static_scratch(&scratch);
    if (e == hipSuccess) e = launch_permute(topk_idx, T, k, e_lo, E_local, scratch, offsets, row_of, tok_of, st);
    if (e == hipSuccess && xp != nullptr) e = launch_gather((const uint16_t*)x, row_of, T, k, d, (uint16_t*)xp, st);
    if (e != hipSuccess) {
        moe_note_error(hipGetErrorString(e));
        return MOE_ERR_DEVICE;
    }
    return MOE_OK;
}
