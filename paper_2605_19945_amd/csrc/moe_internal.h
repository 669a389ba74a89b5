// Internal declarations shared by the translation units of libmoe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// 16-byte accesses with the non-temporal hint, for data a kernel touches once: a read-only streaming kernel
// reaches about 7.2 TB/s with them on this device against 6.4 TB/s with plain loads.
#ifdef __HIPCC__
static __device__ inline uint4 load_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
static __device__ inline void store_stream(uint4* p, const uint4& v) {
    const u32x4_t u = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(u, (u32x4_t*)p);
}
#endif

// One work item of a grouped GEMM launch: BM rows of one expert times BN packed weight rows.
struct TileDesc {
    int32_t expert;  // local expert index
    int32_t row0;    // first row (in the expert-contiguous row space)
    int32_t rows;    // valid rows in this tile (0: nothing to do)
    int32_t n0;      // first packed weight row
};

// What a work-list build needs besides the per-expert rows.
struct SchedArgs {
    int E_local;
    int bm, bn;            // tallest row tile, packed weight rows per work item
    int nt1, grid1;        // weight-row tiles and work-list entries of the first GEMM
    TileDesc* t1;
    int nt2, grid2;        // of the second GEMM (grid2 = 0: none)
    TileDesc* t2;
    int nsplit1, nsplit2;  // reduction splits (workgroups per entry) of the two launches
    int rows_cap;          // host bound on the total rows (-1: none); exceeded -> nothing is scheduled
    int32_t* refused_out;  // where that refusal is recorded (or nullptr)
};

// Token-tile classes of the grouped GEMM.
enum GemmClass { GEMM_LOW = 0, GEMM_MAIN = 1, GEMM_DECODE = 5, GEMM_NUM_CLASSES = 6 };

struct GemmPlan {
    int cls;         // GemmClass
    int bm, bn;      // tile: bm rows x bn packed weight rows
    int mt_max;      // upper bound on the number of row tiles
    int nt1, nt2;    // weight-row tiles of GEMM1 (2f packed rows) and GEMM2 (d rows)
    int grid1, grid2;
    bool w_stream;   // weight loads carry the non-temporal hint (gemm_pick_stream)
};

constexpr int MOE_EVENT_RING = 64;

struct moe_ctx {
    moe_shape s;
    int device;
    char* ws;
    size_t ws_bytes;
    // workspace carve-up (device pointers)
    int32_t* idx;        // [T_max, k]
    float* w;            // [T_max, k]
    int32_t* counts;     // [E]
    int32_t* offsets;    // [E_local + 1]
    int32_t* row_of;     // [T_max, k]
    int32_t* tok_of;     // [rows_cap]
    int32_t* blockhist;  // [nblk_max, E_local]
    TileDesc* table1;    // [grid1_max]
    TileDesc* table2;    // [grid2_max]
    TileDesc* table_r;   // router GEMM work list (E >= MOE_ROUTER_GEMM_MIN_E)
    int table_r_T;       // token count table_r was built for; -1: none yet; -2: rebuild at every call
    float* logits;       // [T_max, router cols] fp32 (E >= MOE_ROUTER_GEMM_MIN_E)
    int32_t* route_ws;   // [MOE_ROUTE_WS_INTS] resident router: ticket (zero between launches) + partial counts
    int32_t* refused;    // [1] 1 if the most recent work list was refused: offsets[E_local] exceeded the host's row bound
    uint16_t* H;         // [rows_cap, f] bf16
    uint16_t* Y;         // [rows_cap, d] bf16
    float* part;         // fp32 partial sums of a reduction split of GEMM2: [nsplit][n_rows, d]
    size_t part_bytes;
    int64_t rows_cap;
    int table1_cap, table2_cap;
    hipEvent_t (*ev)[MOE_NUM_STAGES + 1];  // ring of MOE_EVENT_RING event sets, or nullptr
    int ev_count;                          // layer calls recorded since the last read-out
    int last_cls;    // tile class of the most recent expert GEMM launch
    int forced_cls;  // -1: pick by expected rows per expert
};

static inline int64_t moe_round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
// Workspace for the partial sums of a split second GEMM: splits are only worth it at low loads
static inline size_t moe_part_bytes(int64_t rows_cap, int d) {
    const size_t want = (size_t)8 * rows_cap * d * 4, cap = (size_t)64 << 20;
    return want < cap ? want : cap;
}
// Leading dimension (elements) of the intermediate H, which the library lays out itself: rows are
// padded by 128 bytes so that the rows of a tile, which are all read at the same K offset, do not
// fall on one L2 channel when K*2 is a power of two.
static __host__ __device__ inline int moe_ld_pad(int K) { return K + 64; }
// Routers with at least this many experts compute their logits with the tiled GEMM kernel; smaller
// ones with the direct MFMA kernel.
constexpr int MOE_ROUTER_GEMM_MIN_E = 32;
// Routers this small keep their matrix in registers (persistent kernel, see moe_route.hip).
static inline bool moe_router_resident(int E, int d) { return E <= 8 && d % 512 == 0 && d <= 4096; }
// Router scratch (ints, all zero between launches): ticket + per-workgroup partial counts of the
// resident router, then 32 sub-counters per expert of the top-k kernel (GEMM path).
constexpr int MOE_ROUTE_WS_SUBCOUNTS = 1 + 256 * 8 + 63;
constexpr int MOE_ROUTE_WS_INTS = MOE_ROUTE_WS_SUBCOUNTS + 32 * 256;
static inline int moe_router_cols(int E) { return (E + 31) / 32 * 32; }       // logits row length (GEMM path)
static inline int moe_router_packed_rows(int E) { return moe_router_cols(E) * 2; }  // hi/lo interleaved rows
static inline int moe_router_rows(int E) {  // packed router rows: multiple of 16, power-of-two blocks
    int nb = (E + 15) / 16;
    int p = 1;
    while (p < nb) p *= 2;
    return p * 16;
}

// Records the text moe_last_device_error() returns on this thread.
void moe_note_error(const char* text);

// ---- launchers (each validates nothing; the C-ABI layer has done that) -------------------------
hipError_t launch_pack_router(const float* Wg, int d, int E, uint16_t* rp, hipStream_t st);
hipError_t launch_pack_experts(const uint16_t* W1, const uint16_t* W3, const uint16_t* W2, int E_local,
                               int d, int f, uint16_t* packed, hipStream_t st);
hipError_t launch_route(const uint16_t* x, const uint16_t* rp, const float* bias, int T, int d, int E,
                        int k, int32_t* idx, float* w, int32_t* counts, float* logits_ws, int logits_slabs,
                        TileDesc* table_ws, int* table_T, int32_t* route_ws, hipStream_t st);
hipError_t launch_permute(const int32_t* idx, int T, int k, int e_lo, int E_local, int32_t* blockhist,
                          int32_t* offsets, int32_t* row_of, int32_t* tok_of, hipStream_t st);
hipError_t launch_gather(const uint16_t* x, const int32_t* row_of, int T, int k, int d, uint16_t* xp,
                         hipStream_t st);
hipError_t launch_combine(const uint16_t* y, const int32_t* row_of, const float* w, int T, int k, int d,
                          uint16_t* out, hipStream_t st);

GemmPlan gemm_make_plan(int cls, int64_t n_rows_cap, int E_local, int d, int f);
int gemm_pick_class(double expected_rows_per_expert);
int gemm_class_rows(int cls);
bool gemm_pick_stream(int cls, double expected_rows_per_expert);
hipError_t gemm_init_attributes();
int router_gemm_grid_max(int T_max, int Rp);
hipError_t launch_router_gemm(const uint16_t* x, const uint16_t* rp, int T, int d, int Rp, float* logits, int ldl,
                              int max_split, int* nsplit_out, TileDesc* table, int* table_T, hipStream_t st);
// Slabs of partial router logits ([T, cols] fp32 each) the workspace holds for T tokens
static inline int moe_router_split_cap(int T) { return T <= 8192 ? 8 : T <= 16384 ? 4 : T <= 32768 ? 2 : 1; }
hipError_t launch_schedule(const GemmPlan& p, const int32_t* offsets, int E_local, TileDesc* t1,
                           TileDesc* t2, int nsplit2, int64_t rows_cap, int32_t* refused, hipStream_t st);
// Arguments of a work-list build for plan p, and the workgroups worth spending on it
SchedArgs gemm_sched_args(const GemmPlan& p, int E_local, TileDesc* t1, TileDesc* t2, int nsplit2, int64_t rows_cap,
                          int32_t* refused);
int gemm_sched_blocks(const GemmPlan& p);
// Dispatch of the layer: offsets, row_of, tok_of and both work lists from idx (and the router's counts).
// dispatch_plan_counts_itself(T, k): the launch counts the assignments itself (counts is an output, may be null,
// and the router need not count); otherwise counts[E] is the router's and is read.
bool dispatch_plan_counts_itself(int T, int k);
hipError_t launch_dispatch_plan(const int32_t* idx, int T, int k, int E, int e_lo, int32_t* blockhist, int32_t* counts,
                                int32_t* offsets, int32_t* row_of, int32_t* tok_of, const SchedArgs& a, int sched_blocks,
                                hipStream_t st);
// moe_combine on rows that still lie as nsplit fp32 partial slabs (slab_elems floats apart) of the second GEMM
hipError_t launch_combine_split(const float* part, int nsplit, size_t slab_elems, const int32_t* row_of, const float* w,
                                int T, int k, int d, uint16_t* out, hipStream_t st);
hipError_t launch_gemm1(const GemmPlan& p, const uint16_t* X, int ldx, const int32_t* row_map,
                        const uint16_t* W13f, int d, int f, uint16_t* H, const TileDesc* table,
                        hipStream_t st);
int gemm_pick_split2(const GemmPlan& p, int64_t n_rows, int E_local, int d, int f, size_t part_bytes);
hipError_t launch_gemm2(const GemmPlan& p, const uint16_t* H, const uint16_t* W2f, int d, int f, uint16_t* Y,
                        const TileDesc* table, int nsplit, float* part, int64_t n_rows, const int32_t* n_rows_dev,
                        hipStream_t st);
// one launch of the MFMA-only kernel (no loads) on instruction shape 0 (32x32x16) or 1 (16x16x32); *flop: MFMA
// flop of the launch (the same for both shapes)
hipError_t launch_mfma_rate(int shape, int iters_per_wave, double* flop, hipStream_t st);
// one launch of the read-only streaming kernel over bytes / 16 16-byte words of buf
hipError_t launch_read_rate(const void* buf, size_t bytes, bool nontemporal, hipStream_t st);
