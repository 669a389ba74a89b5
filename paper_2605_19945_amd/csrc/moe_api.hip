// C ABI of libmoe: argument validation, workspace carve-up, stage sequencing.  No kernels here.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "moe_internal.h"

namespace {

constexpr size_t kAlign = 256;

bool shape_ok(const moe_shape* s) {
    if (s == nullptr) return false;
    if (s->T_max < 1 || s->T_max > (1 << 20)) return false;
    if (s->d < 64 || s->f < 64 || s->d % 64 != 0 || s->f % 64 != 0) return false;
    if (s->d > (1 << 16) || s->f > (1 << 17)) return false;
    if (s->E < 1 || s->E > 256) return false;
    if (s->k < 1 || s->k > s->E || s->k > 16) return false;
    if (s->e_lo < 0 || s->E_local < 1 || s->E_local > 256) return false;
    if ((int64_t)s->e_lo + s->E_local > s->E) return false;
    if (moe_rows_capacity(s, s->T_max) > (int64_t)1 << 24) return false;
    // the GEMM kernels address their token operands with 32-bit byte offsets from per-tensor bases
    const int64_t lim = (int64_t)1 << 32;
    if ((int64_t)s->T_max * s->d * 2 >= lim) return false;
    if (moe_rows_capacity(s, s->T_max) * moe_ld_pad(s->f) * 2 >= lim) return false;
    if (moe_rows_capacity(s, s->T_max) * s->d * 2 >= lim) return false;
    return true;
}

struct Layout {
    size_t idx, w, counts, offsets, row_of, tok_of, blockhist, table1, table2, table_r, logits, route_ws, refused, H, Y, part, total;
    int table1_cap, table2_cap;
    int64_t rows_cap;
};

Layout make_layout(const moe_shape* s) {
    Layout L;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o += (bytes + kAlign - 1) / kAlign * kAlign;
        return at;
    };
    const int64_t A = (int64_t)s->T_max * s->k;
    L.rows_cap = moe_rows_capacity(s, s->T_max);
    L.idx = take(A * 4);
    L.w = take(A * 4);
    L.counts = take((size_t)s->E * 4);
    L.offsets = take((size_t)(s->E_local + 1) * 4);
    L.row_of = take(A * 4);
    L.tok_of = take((size_t)L.rows_cap * 4);
    const int nblk = (s->T_max + 255) / 256;
    L.blockhist = take((size_t)nblk * s->E_local * 4);
    L.table1_cap = L.table2_cap = 0;
    for (int c = 0; c < GEMM_NUM_CLASSES; ++c) {
        GemmPlan p = gemm_make_plan(c, L.rows_cap, s->E_local, s->d, s->f);
        if (p.grid1 > L.table1_cap) L.table1_cap = p.grid1;
        if (p.grid2 > L.table2_cap) L.table2_cap = p.grid2;
    }
    L.table1 = take((size_t)L.table1_cap * sizeof(TileDesc));
    L.table2 = take((size_t)L.table2_cap * sizeof(TileDesc));
    if (s->E >= MOE_ROUTER_GEMM_MIN_E) {
        const int cap = router_gemm_grid_max(s->T_max, moe_router_packed_rows(s->E));
        L.table_r = take((size_t)cap * sizeof(TileDesc));
        L.logits = take((size_t)moe_router_split_cap(s->T_max) * s->T_max * moe_router_cols(s->E) * 4);
    } else {
        L.table_r = L.logits = 0;
    }
    L.route_ws = take((size_t)MOE_ROUTE_WS_INTS * 4);
    L.refused = take(4);
    L.H = take((size_t)L.rows_cap * moe_ld_pad(s->f) * 2);
    L.Y = take((size_t)L.rows_cap * s->d * 2);
    L.part = take(moe_part_bytes(L.rows_cap, s->d));
    L.total = o;
    return L;
}

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }
inline bool bad_bf16(const void* p) { return p == nullptr || !aligned(p, 16); }
inline bool bad_i32(const void* p) { return p == nullptr || !aligned(p, 4); }

thread_local char g_last_error[256] = "";

inline moe_status note_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return MOE_OK;
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(e));
    return MOE_ERR_DEVICE;
}
inline moe_status from_hip(hipError_t e) { return note_hip(e, "kernel launch"); }

}  // namespace

void moe_note_error(const char* text) { snprintf(g_last_error, sizeof(g_last_error), "%s", text); }

extern "C" {

const char* moe_last_device_error(void) { return g_last_error; }

const char* moe_status_string(moe_status s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
        case MOE_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case MOE_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

int64_t moe_rows_capacity(const moe_shape* s, int32_t T) {
    if (s == nullptr || T < 0) return 0;
    int kk = s->k < s->E_local ? s->k : s->E_local;
    return (int64_t)T * kk;
}

size_t moe_workspace_bytes(const moe_shape* s) {
    if (!shape_ok(s)) return 0;
    return make_layout(s).total;
}

size_t moe_packed_router_bytes(const moe_shape* s) {
    if (!shape_ok(s)) return 0;
    if (s->E >= MOE_ROUTER_GEMM_MIN_E) return (size_t)moe_router_packed_rows(s->E) * s->d * 2;
    if (moe_router_resident(s->E, s->d)) return (size_t)16 * s->d * 2;
    return (size_t)2 * moe_router_rows(s->E) * s->d * 2;
}

size_t moe_packed_weight_bytes(const moe_shape* s) {
    if (!shape_ok(s)) return 0;
    return (size_t)s->E_local * 3 * s->d * s->f * 2;
}

moe_status moe_create(moe_ctx** out, const moe_shape* s, void* workspace, size_t bytes) {
    if (out == nullptr) return MOE_ERR_INVALID_ARG;
    *out = nullptr;
    if (s == nullptr) return MOE_ERR_INVALID_ARG;
    if (!shape_ok(s)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (workspace == nullptr || !aligned(workspace, kAlign)) return MOE_ERR_INVALID_ARG;
    Layout L = make_layout(s);
    if (bytes < L.total) return MOE_ERR_WORKSPACE_TOO_SMALL;

    int dev = -1;
    moe_status ds = note_hip(hipGetDevice(&dev), "hipGetDevice");
    if (ds != MOE_OK) return ds;
    hipDeviceProp_t prop;
    ds = note_hip(hipGetDeviceProperties(&prop, dev), "hipGetDeviceProperties");
    if (ds != MOE_OK) return ds;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {  // kernels exist for gfx950 only
        snprintf(g_last_error, sizeof(g_last_error), "device is %s, this library is built for gfx950",
                 prop.gcnArchName);
        return MOE_ERR_DEVICE;
    }
    ds = note_hip(gemm_init_attributes(), "hipFuncSetAttribute(max dynamic LDS)");
    if (ds != MOE_OK) return ds;

    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (c == nullptr) return MOE_ERR_INVALID_ARG;
    c->s = *s;
    c->device = dev;
    c->ws = (char*)workspace;
    c->ws_bytes = bytes;
    c->idx = (int32_t*)(c->ws + L.idx);
    c->w = (float*)(c->ws + L.w);
    c->counts = (int32_t*)(c->ws + L.counts);
    c->offsets = (int32_t*)(c->ws + L.offsets);
    c->row_of = (int32_t*)(c->ws + L.row_of);
    c->tok_of = (int32_t*)(c->ws + L.tok_of);
    c->blockhist = (int32_t*)(c->ws + L.blockhist);
    c->table1 = (TileDesc*)(c->ws + L.table1);
    c->table2 = (TileDesc*)(c->ws + L.table2);
    c->table_r = (TileDesc*)(c->ws + L.table_r);
    c->route_ws = (int32_t*)(c->ws + L.route_ws);
    c->refused = (int32_t*)(c->ws + L.refused);
    c->logits = (float*)(c->ws + L.logits);
    c->H = (uint16_t*)(c->ws + L.H);
    c->Y = (uint16_t*)(c->ws + L.Y);
    c->part = (float*)(c->ws + L.part);
    c->part_bytes = moe_part_bytes(L.rows_cap, s->d);
    c->rows_cap = L.rows_cap;
    c->table1_cap = L.table1_cap;
    c->table2_cap = L.table2_cap;
    c->ev = nullptr;
    c->ev_count = 0;
    c->last_cls = -1;
    c->forced_cls = -1;
    c->table_r_T = -1;
    // the resident router's ticket counter must be zero before the first launch (each launch leaves
    // it at zero again); synchronous, creation is not on the hot path
    if (note_hip(hipMemset(c->route_ws, 0, (size_t)MOE_ROUTE_WS_INTS * 4), "hipMemset(workspace)") != MOE_OK) {
        delete c;
        return MOE_ERR_DEVICE;
    }
    if (s->flags & MOE_FLAG_STAGE_EVENTS) {
        c->ev = new (std::nothrow) hipEvent_t[MOE_EVENT_RING][MOE_NUM_STAGES + 1];
        if (c->ev == nullptr) {
            delete c;
            return MOE_ERR_INVALID_ARG;
        }
        for (int r = 0; r < MOE_EVENT_RING; ++r)
            for (int i = 0; i <= MOE_NUM_STAGES; ++i) c->ev[r][i] = nullptr;
        for (int r = 0; r < MOE_EVENT_RING; ++r)
            for (int i = 0; i <= MOE_NUM_STAGES; ++i)
                if (hipEventCreate(&c->ev[r][i]) != hipSuccess) {
                    moe_destroy(c);
                    return MOE_ERR_DEVICE;
                }
    }
    *out = c;
    return MOE_OK;
}

void moe_destroy(moe_ctx* c) {
    if (c == nullptr) return;
    if (c->ev != nullptr) {
        for (int r = 0; r < MOE_EVENT_RING; ++r)
            for (int i = 0; i <= MOE_NUM_STAGES; ++i)
                if (c->ev[r][i] != nullptr) (void)hipEventDestroy(c->ev[r][i]);
        delete[] c->ev;
    }
    delete c;
}

moe_status moe_measure_mfma_rate(int32_t iters_per_wave, int32_t launches, float* tflops, void* stream) {
    return moe_measure_mfma_rate_of(1, iters_per_wave, launches, tflops, stream);  // the grouped GEMM's shape
}

moe_status moe_measure_mfma_rate_of(int32_t shape, int32_t iters_per_wave, int32_t launches, float* tflops,
                                    void* stream) {
    if (tflops == nullptr || iters_per_wave < 1 || launches < 1 || shape < 0 || shape > 1) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (note_hip(hipEventCreate(&e0), "hipEventCreate") != MOE_OK) return MOE_ERR_DEVICE;
    if (note_hip(hipEventCreate(&e1), "hipEventCreate") != MOE_OK) {
        (void)hipEventDestroy(e0);
        return MOE_ERR_DEVICE;
    }
    double flop = 0;
    moe_status rc = note_hip(launch_mfma_rate(shape, iters_per_wave, &flop, st), "mfma_rate_kernel");  // warm-up
    if (rc == MOE_OK) rc = note_hip(hipEventRecord(e0, st), "hipEventRecord");
    for (int i = 0; i < launches && rc == MOE_OK; ++i)
        rc = note_hip(launch_mfma_rate(shape, iters_per_wave, &flop, st), "mfma_rate_kernel");
    if (rc == MOE_OK) rc = note_hip(hipEventRecord(e1, st), "hipEventRecord");
    if (rc == MOE_OK) rc = note_hip(hipEventSynchronize(e1), "hipEventSynchronize");
    float ms = 0.f;
    if (rc == MOE_OK) rc = note_hip(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime");
    if (rc == MOE_OK) *tflops = ms > 0.f ? (float)(flop * launches / (ms * 1e9)) : 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

moe_status moe_measure_hbm_read_rate(const void* buf, size_t bytes, int32_t nontemporal, int32_t launches,
                                     float* gb_per_s, void* stream) {
    if (buf == nullptr || gb_per_s == nullptr || bytes < 16 || launches < 1 || !aligned(buf, 16))
        return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (note_hip(hipEventCreate(&e0), "hipEventCreate") != MOE_OK) return MOE_ERR_DEVICE;
    if (note_hip(hipEventCreate(&e1), "hipEventCreate") != MOE_OK) {
        (void)hipEventDestroy(e0);
        return MOE_ERR_DEVICE;
    }
    moe_status rc = note_hip(launch_read_rate(buf, bytes, nontemporal != 0, st), "read_rate_kernel");  // warm-up
    if (rc == MOE_OK) rc = note_hip(hipEventRecord(e0, st), "hipEventRecord");
    for (int i = 0; i < launches && rc == MOE_OK; ++i)
        rc = note_hip(launch_read_rate(buf, bytes, nontemporal != 0, st), "read_rate_kernel");
    if (rc == MOE_OK) rc = note_hip(hipEventRecord(e1, st), "hipEventRecord");
    if (rc == MOE_OK) rc = note_hip(hipEventSynchronize(e1), "hipEventSynchronize");
    float ms = 0.f;
    if (rc == MOE_OK) rc = note_hip(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime");
    if (rc == MOE_OK) *gb_per_s = ms > 0.f ? (float)((double)(bytes / 16 * 16) * launches / (ms * 1e6)) : 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

moe_status moe_set_tile_class(moe_ctx* c, int32_t cls) {
    if (c == nullptr || cls < -1 || cls >= GEMM_NUM_CLASSES) return MOE_ERR_INVALID_ARG;
    c->forced_cls = cls;
    return MOE_OK;
}

int32_t moe_tile_rows(const moe_ctx* c) {
    if (c == nullptr) return 0;
    int cls = c->forced_cls >= 0 ? c->forced_cls : c->last_cls;
    if (cls < 0) cls = gemm_pick_class((double)c->s.T_max * c->s.k / c->s.E);
    return gemm_class_rows(cls);
}

moe_status moe_pack_router(moe_ctx* c, const float* Wg, void* rp, void* stream) {
    if (c == nullptr || bad_i32(Wg) || bad_bf16(rp)) return MOE_ERR_INVALID_ARG;
    return from_hip(launch_pack_router(Wg, c->s.d, c->s.E, (uint16_t*)rp, (hipStream_t)stream));
}

moe_status moe_pack_weights(moe_ctx* c, const void* W1, const void* W3, const void* W2, void* packed,
                            void* stream) {
    if (c == nullptr || bad_bf16(W1) || bad_bf16(W3) || bad_bf16(W2) || bad_bf16(packed))
        return MOE_ERR_INVALID_ARG;
    return from_hip(launch_pack_experts((const uint16_t*)W1, (const uint16_t*)W3, (const uint16_t*)W2,
                                        c->s.E_local, c->s.d, c->s.f, (uint16_t*)packed,
                                        (hipStream_t)stream));
}

// partial-logit slabs of T tokens that fit the workspace sized for T_max
static int logits_slabs(const moe_ctx* c, int T) {
    int64_t n = (int64_t)moe_router_split_cap(c->s.T_max) * c->s.T_max / (T > 0 ? T : 1);
    return n > 8 ? 8 : (int)n;
}

moe_status moe_route(moe_ctx* c, const void* x, const void* rp, const float* bias, int32_t T,
                     int32_t* topk_idx, float* topk_w, int32_t* counts, void* stream) {
    if (c == nullptr || T < 0 || T > c->s.T_max) return MOE_ERR_INVALID_ARG;
    if (bad_bf16(x) || bad_bf16(rp) || bad_i32(topk_idx) || bad_i32(topk_w) || bad_i32(counts))
        return MOE_ERR_INVALID_ARG;
    if (bias != nullptr && !aligned(bias, 4)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    return from_hip(launch_route((const uint16_t*)x, (const uint16_t*)rp, bias, T, c->s.d, c->s.E, c->s.k,
                                 topk_idx, topk_w, counts, c->logits, logits_slabs(c, T), c->table_r, &c->table_r_T, c->route_ws,
                                 (hipStream_t)stream));
}

moe_status moe_permute(moe_ctx* c, const void* x, const int32_t* topk_idx, int32_t T, void* xp,
                       int32_t* offsets, int32_t* row_of, int32_t* tok_of, void* stream) {
    if (c == nullptr || T < 0 || T > c->s.T_max) return MOE_ERR_INVALID_ARG;
    if (bad_i32(topk_idx) || bad_i32(offsets) || bad_i32(row_of) || bad_i32(tok_of)) return MOE_ERR_INVALID_ARG;
    if (xp != nullptr && (bad_bf16(xp) || bad_bf16(x))) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = launch_permute(topk_idx, T, c->s.k, c->s.e_lo, c->s.E_local, c->blockhist, offsets, row_of,
                                  tok_of, st);
    if (e == hipSuccess && xp != nullptr)
        e = launch_gather((const uint16_t*)x, row_of, T, c->s.k, c->s.d, (uint16_t*)xp, st);
    return from_hip(e);
}

// The two expert GEMMs.  plan == nullptr: the work lists are built here from offsets (one more launch);
// otherwise they have been built for *plan with nsplit reduction ranges of the second GEMM.  Y == nullptr
// with nsplit > 1 leaves the second GEMM's partial sums in c->part for the caller.
static moe_status run_ffn(moe_ctx* c, int cls, const uint16_t* X, const int32_t* row_map,
                          const int32_t* offsets, int64_t n_rows_cap, const uint16_t* packed, uint16_t* Y,
                          hipStream_t st, hipEvent_t* events, const GemmPlan* plan = nullptr, int nsplit = 1) {
    const moe_shape& s = c->s;
    GemmPlan p;
    hipError_t e;
    if (plan != nullptr) {
        p = *plan;
    } else {
        p = gemm_make_plan(cls, n_rows_cap, s.E_local, s.d, s.f);
        if (p.grid1 > c->table1_cap || p.grid2 > c->table2_cap) return MOE_ERR_WORKSPACE_TOO_SMALL;
        p.w_stream = gemm_pick_stream(cls, (double)n_rows_cap / s.E_local);
        nsplit = gemm_pick_split2(p, n_rows_cap, s.E_local, s.d, s.f, c->part_bytes);
        // offsets[E_local] = the rows actually present
        e = launch_schedule(p, offsets, s.E_local, c->table1, c->table2, nsplit, n_rows_cap, c->refused, st);
        if (e != hipSuccess) return MOE_ERR_DEVICE;
    }
    c->last_cls = cls;
    const uint16_t* w13f = packed;
    const uint16_t* w2f = packed + (size_t)s.E_local * 2 * s.f * s.d;
    if (events) (void)hipEventRecord(events[MOE_STAGE_GEMM1], st);
    e = launch_gemm1(p, X, s.d, row_map, w13f, s.d, s.f, c->H, c->table1, st);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    if (events) (void)hipEventRecord(events[MOE_STAGE_GEMM2], st);
    e = launch_gemm2(p, c->H, w2f, s.d, s.f, Y, c->table2, nsplit, c->part, n_rows_cap, offsets + s.E_local, st);
    return from_hip(e);
}

moe_status moe_grouped_ffn(moe_ctx* c, const void* xp, const int32_t* offsets, int32_t n_rows_cap,
                           const void* packed, void* y, void* stream) {
    if (c == nullptr || n_rows_cap < 0 || n_rows_cap > c->rows_cap) return MOE_ERR_INVALID_ARG;
    if (bad_bf16(xp) || bad_i32(offsets) || bad_bf16(packed) || bad_bf16(y)) return MOE_ERR_INVALID_ARG;
    if (n_rows_cap == 0) return MOE_OK;
    int cls = c->forced_cls >= 0 ? c->forced_cls : gemm_pick_class((double)n_rows_cap / c->s.E_local);
    return run_ffn(c, cls, (const uint16_t*)xp, nullptr, offsets, n_rows_cap, (const uint16_t*)packed,
                   (uint16_t*)y, (hipStream_t)stream, nullptr);
}

moe_status moe_profile_ffn(moe_ctx* c, const void* xp, const void* packed, void* y, const int32_t* token_counts,
                           int32_t n_points, int32_t warmup, int32_t iters, float* ms, void* stream) {
    if (c == nullptr || token_counts == nullptr || ms == nullptr || n_points < 0 || warmup < 0 || iters < 1)
        return MOE_ERR_INVALID_ARG;
    if (bad_bf16(xp) || bad_bf16(packed) || bad_bf16(y)) return MOE_ERR_INVALID_ARG;
    for (int i = 0; i < n_points; ++i)
        if (token_counts[i] < 0 || token_counts[i] > c->rows_cap) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int E_local = c->s.E_local;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (note_hip(hipEventCreate(&e0), "hipEventCreate") != MOE_OK) return MOE_ERR_DEVICE;
    if (note_hip(hipEventCreate(&e1), "hipEventCreate") != MOE_OK) {
        (void)hipEventDestroy(e0);
        return MOE_ERR_DEVICE;
    }
    int32_t host_off[257];
    moe_status rc = MOE_OK;
    for (int i = 0; i < n_points && rc == MOE_OK; ++i) {
        const int n = token_counts[i];
        ms[i] = 0.f;
        if (n == 0) continue;
        // n rows spread evenly over the resident experts, the first n % E_local get one more
        host_off[0] = 0;
        for (int e = 0; e < E_local; ++e) host_off[e + 1] = host_off[e] + n / E_local + (e < n % E_local ? 1 : 0);
        rc = note_hip(hipMemcpyAsync(c->offsets, host_off, (size_t)(E_local + 1) * 4, hipMemcpyHostToDevice, st),
                      "hipMemcpyAsync(offsets)");
        if (rc != MOE_OK) break;
        rc = note_hip(hipStreamSynchronize(st), "hipStreamSynchronize");  // host_off is reused
        if (rc != MOE_OK) break;
        const int cls = c->forced_cls >= 0 ? c->forced_cls : gemm_pick_class((double)n / E_local);
        for (int r = 0; r < warmup + iters && rc == MOE_OK; ++r) {
            if (r == warmup) rc = note_hip(hipEventRecord(e0, st), "hipEventRecord");
            if (rc == MOE_OK)
                rc = run_ffn(c, cls, (const uint16_t*)xp, nullptr, c->offsets, n, (const uint16_t*)packed,
                             (uint16_t*)y, st, nullptr);
        }
        if (rc != MOE_OK) break;
        rc = note_hip(hipEventRecord(e1, st), "hipEventRecord");
        if (rc == MOE_OK) rc = note_hip(hipEventSynchronize(e1), "hipEventSynchronize");
        float t = 0.f;
        if (rc == MOE_OK) rc = note_hip(hipEventElapsedTime(&t, e0, e1), "hipEventElapsedTime");
        ms[i] = t / (float)iters;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

moe_status moe_combine(moe_ctx* c, const void* y, const int32_t* row_of, const float* topk_w, int32_t T,
                       void* out, void* stream) {
    if (c == nullptr || T < 0 || T > c->s.T_max) return MOE_ERR_INVALID_ARG;
    if (bad_bf16(y) || bad_i32(row_of) || bad_i32(topk_w) || bad_bf16(out)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    return from_hip(launch_combine((const uint16_t*)y, row_of, topk_w, T, c->s.k, c->s.d, (uint16_t*)out,
                                   (hipStream_t)stream));
}

moe_status moe_layer_forward(moe_ctx* c, const void* x, const void* rp, const float* bias, const void* packed,
                             int32_t T, void* out, int32_t* counts_out, void* stream) {
    if (c == nullptr || T < 0 || T > c->s.T_max) return MOE_ERR_INVALID_ARG;
    if (bad_bf16(x) || bad_bf16(rp) || bad_bf16(packed) || bad_bf16(out)) return MOE_ERR_INVALID_ARG;
    if (bias != nullptr && !aligned(bias, 4)) return MOE_ERR_INVALID_ARG;
    if (counts_out != nullptr && !aligned(counts_out, 4)) return MOE_ERR_INVALID_ARG;
    if (T == 0) return MOE_OK;
    const moe_shape& s = c->s;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t* ev = c->ev != nullptr ? c->ev[c->ev_count % MOE_EVENT_RING] : nullptr;
    int32_t* counts = counts_out != nullptr ? counts_out : c->counts;

    // everything the host decides is decided before the first launch: tile class, work-list sizes, splits
    const int64_t cap = moe_rows_capacity(&s, T);
    const int cls = c->forced_cls >= 0 ? c->forced_cls : gemm_pick_class((double)T * s.k / s.E);
    GemmPlan p = gemm_make_plan(cls, cap, s.E_local, s.d, s.f);
    if (p.grid1 > c->table1_cap || p.grid2 > c->table2_cap) return MOE_ERR_WORKSPACE_TOO_SMALL;
    p.w_stream = gemm_pick_stream(cls, (double)T * s.k / s.E);
    const int nsplit = gemm_pick_split2(p, cap, s.E_local, s.d, s.f, c->part_bytes);
    const SchedArgs sa = gemm_sched_args(p, s.E_local, c->table1, c->table2, nsplit, cap, c->refused);
    // small batches: the dispatch launch counts the assignments itself and the router skips its count reduction
    const bool plan_counts = dispatch_plan_counts_itself(T, s.k);

    if (ev) (void)hipEventRecord(ev[MOE_STAGE_ROUTE], st);
    hipError_t e = launch_route((const uint16_t*)x, (const uint16_t*)rp, bias, T, s.d, s.E, s.k, c->idx, c->w,
                                plan_counts ? nullptr : counts, c->logits, logits_slabs(c, T), c->table_r,
                                &c->table_r_T, c->route_ws, st);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    if (ev) (void)hipEventRecord(ev[MOE_STAGE_PERMUTE], st);
    e = launch_dispatch_plan(c->idx, T, s.k, s.E, s.e_lo, c->blockhist, plan_counts ? counts_out : counts, c->offsets,
                             c->row_of, c->tok_of, sa, gemm_sched_blocks(p), st);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    // the row copy is folded into GEMM1: it reads x through tok_of; the split second GEMM leaves fp32
    // partial sums that the combine adds up itself
    moe_status ms = run_ffn(c, cls, (const uint16_t*)x, c->tok_of, c->offsets, cap, (const uint16_t*)packed,
                            nsplit > 1 ? nullptr : c->Y, st, ev, &p, nsplit);
    if (ms != MOE_OK) return ms;
    if (ev) (void)hipEventRecord(ev[MOE_STAGE_COMBINE], st);
    if (nsplit > 1)
        e = launch_combine_split(c->part, nsplit, (size_t)cap * s.d, c->row_of, c->w, T, s.k, s.d, (uint16_t*)out, st);
    else
        e = launch_combine(c->Y, c->row_of, c->w, T, s.k, s.d, (uint16_t*)out, st);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    if (ev) {
        (void)hipEventRecord(ev[MOE_NUM_STAGES], st);
        c->ev_count++;
    }
    return MOE_OK;
}

moe_status moe_stage_times(moe_ctx* c, float* ms) {
    if (c == nullptr || ms == nullptr || c->ev == nullptr || c->ev_count == 0) return MOE_ERR_INVALID_ARG;
    const int n = c->ev_count < MOE_EVENT_RING ? c->ev_count : MOE_EVENT_RING;
    const int last = (c->ev_count - 1) % MOE_EVENT_RING;
    c->ev_count = 0;
    if (hipEventSynchronize(c->ev[last][MOE_NUM_STAGES]) != hipSuccess) return MOE_ERR_DEVICE;
    double sum[MOE_NUM_STAGES] = {0};
    for (int r = 0; r < n; ++r)
        for (int i = 0; i < MOE_NUM_STAGES; ++i) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, c->ev[r][i], c->ev[r][i + 1]) != hipSuccess) return MOE_ERR_DEVICE;
            sum[i] += t;
        }
    for (int i = 0; i < MOE_NUM_STAGES; ++i) ms[i] = (float)(sum[i] / n);
    return MOE_OK;
}

moe_status moe_ffn_refused_flag(moe_ctx* c, const int32_t** flag) {
    if (c == nullptr || flag == nullptr) return MOE_ERR_INVALID_ARG;
    *flag = c->refused;
    return MOE_OK;
}

moe_status moe_layer_intermediates(moe_ctx* c, const int32_t** topk_idx, const float** topk_w,
                                   const int32_t** offsets, const int32_t** row_of) {
    if (c == nullptr) return MOE_ERR_INVALID_ARG;
    if (topk_idx) *topk_idx = c->idx;
    if (topk_w) *topk_w = c->w;
    if (offsets) *offsets = c->offsets;
    if (row_of) *row_of = c->row_of;
    return MOE_OK;
}

}  // extern "C"
