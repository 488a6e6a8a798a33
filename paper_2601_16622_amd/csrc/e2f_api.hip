// C ABI of libe2f.so: argument checks, workspace layout, and the sequence of launches per entry point.
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <new>

#include "e2f_internal.h"

// Workspace of e2f_attn_forward_static: device memory that belongs to the loaded library, one copy per GPU.  In host
// code this name only stands for the symbol; the address on a device comes from hipGetSymbolAddress (static_scratch).
static __device__ __align__(256) unsigned char scratch[E2F_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on every GPU that has asked for it
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
e2f_status static_scratch(void** ptr) {
    int dev = -1;
    E2F_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return E2F_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        E2F_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return E2F_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return E2F_OK;
}

bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

// Clebsch-Gordan coefficient <j1 m1; j2 m2 | j m> (Condon-Shortley phases) by Racah's closed formula, in double.
// Only the m2 = 0 column is needed: it holds the non-zero entries of the re-indexing operator P (Sec. 3.3,
// Def. of P; App. C): for even l_i+l_f+l_o the order m is kept, for odd it is taken from -m with the sign of m.
double factorial(int n) {
    double f = 1.0;
    for (int x = 2; x <= n; ++x) f *= x;
    return f;
}
double clebsch_gordan(int j1, int m1, int j2, int m2, int j, int m) {
    if (m1 + m2 != m || j > j1 + j2 || j < abs(j1 - j2) || abs(m1) > j1 || abs(m2) > j2 || abs(m) > j) return 0.0;
    const double delta = factorial(j1 + j2 - j) * factorial(j1 - j2 + j) * factorial(-j1 + j2 + j) / factorial(j1 + j2 + j + 1);
    const double norm = (2.0 * j + 1.0) * delta * factorial(j1 + m1) * factorial(j1 - m1) * factorial(j2 + m2) *
                        factorial(j2 - m2) * factorial(j + m) * factorial(j - m);
    double sum = 0.0;
    for (int t = 0; t <= j1 + j2 - j; ++t) {
        const int d1 = j1 + j2 - j - t, d2 = j1 - m1 - t, d3 = j2 + m2 - t, d4 = j - j2 + m1 + t, d5 = j - j1 - m2 + t;
        if (d1 < 0 || d2 < 0 || d3 < 0 || d4 < 0 || d5 < 0) continue;
        const double term = 1.0 / (factorial(t) * factorial(d1) * factorial(d2) * factorial(d3) * factorial(d4) * factorial(d5));
        sum += (t % 2) ? -term : term;
    }
    return sqrt(norm) * sum;
}

size_t cells_ws_layout(int32_t N, int32_t S, void* ws, e2f_cells* c) {
    const int32_t max_cells = 27 * S + 2 * N + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = ws ? static_cast<char*>(ws) + off : nullptr;
        off += e2f_align_up(bytes);
        return p;
    };
    char* grid = take((size_t)((S > 0 ? S : 1) + 1) * sizeof(E2fSegGrid));   // one more: the cells-in-use sentinel
    char* cell_start = take((size_t)(max_cells + 1) * 4);
    char* perm = take((size_t)N * 4);
    char* scell = take((size_t)N * 4);
    char* sseg = take((size_t)N * 4);
    char* atom_slot = take((size_t)N * 4);
    char* bbox = take((size_t)(S > 0 ? S : 1) * 6 * 4);
    char* atom_seg = take((size_t)N * 4);
    char* atom_cell = take((size_t)N * 4);
    char* cell_fill = take((size_t)max_cells * 4);
    char* tmp_slot = take((size_t)N * 4);
    char* atom_sub = take((size_t)N * 4);
    char* box = take((size_t)(S > 0 ? S : 1) * 6 * 4);
    char* sinfo = take((size_t)N * 2 * sizeof(int4));
    if (c) {
        c->view.sinfo = (const int4*)sinfo;
        c->box = (float*)box;
        c->host_box = nullptr;
        c->view.periodic = 0;
        c->view.grid = (const E2fSegGrid*)grid;
        c->view.cell_start = (const int32_t*)cell_start;
        c->view.perm = (const int32_t*)perm;
        c->view.scell = (const int32_t*)scell;
        c->view.sseg = (const int32_t*)sseg;
        c->view.atom_slot = (const int32_t*)atom_slot;
        c->view.N = N;
        c->view.S = S;
        c->bbox = (int32_t*)bbox;
        c->atom_seg = (int32_t*)atom_seg;
        c->atom_cell = (int32_t*)atom_cell;
        c->cell_fill = (int32_t*)cell_fill;
        c->tmp_slot = (int32_t*)tmp_slot;
        c->atom_sub = (int32_t*)atom_sub;
        c->max_cells = max_cells;
    }
    return off;
}

e2f_status check_forward_args(const e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                              const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, const float* out,
                              const void* ws, size_t ws_bytes) {
    if (!ctx || !cells || !w || N < 0 || S < 0) return E2F_ERR_INVALID_ARG;
    if (cells->view.N != N || cells->view.S != S) return E2F_ERR_INVALID_ARG;
    if (N == 0) return E2F_OK;
    if (!pos || !h || !seg_offsets || !out || !ws) return E2F_ERR_INVALID_ARG;
    if (cells->pos != pos) return E2F_ERR_INVALID_ARG;
    if (!w->WQ1 || !w->WQ2 || !w->WK1 || !w->WK2 || !w->WV || !w->Wb || !w->w_path) return E2F_ERR_INVALID_ARG;
    if (!aligned256(ws)) return E2F_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(h) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u)) return E2F_ERR_INVALID_ARG;
    if (ws_bytes < e2f_attn_workspace_bytes(ctx, N)) return E2F_ERR_WORKSPACE_TOO_SMALL;
    return E2F_OK;
}

}  // namespace

E2fAttnWs e2f_attn_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, int v_layout) {
    E2fAttnWs L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = ws ? static_cast<char*>(ws) + off : nullptr;
        off += e2f_align_up(bytes);
        return p;
    };
    const size_t esz = ctx->cfg.feat_dtype == E2F_BF16 ? 2 : 4;
    L.spos = (float4*)take((size_t)N * sizeof(float4));
    L.q = L.k = nullptr;
    L.v = nullptr;
    L.q16 = L.k16 = L.v4 = nullptr;
    L.qf = L.kf = L.vf = nullptr;
    L.G = nullptr;
    L.lists_hdr = nullptr;
    L.lists_ent = nullptr;
    L.lists_pos = nullptr;
    L.lists_mask = nullptr;
    if (v_layout == 2) {
        const size_t H = ctx->cfg.H, DKP = ((size_t)(ctx->cfg.L_max + 1) * 16 + 31) / 32 * 32;
        const size_t N4 = ((size_t)N + 3) / 4 * 4;
        L.q16 = (uint16_t*)take((size_t)N * H * DKP * 2);
        L.k16 = (uint16_t*)take(N4 * H * DKP * 2);
        L.v4 = (uint16_t*)take(N4 / 4 * H * ctx->n * 64 * 2);
        L.G = (float*)take((size_t)(3 * E2F_MAX_N * E2F_MAX_N + 256) * 4);   // full form, then the packed non-zeros
        const size_t n_tiles = ((size_t)N + 15) / 16;
        L.lists_hdr = (int4*)take(n_tiles * sizeof(int4));
        L.lists_ent = (int*)take(n_tiles * E2F_TILE_LCAP * 4);
        L.lists_pos = (float4*)take(n_tiles * E2F_TILE_LCAP * 4 * sizeof(float4));
        L.lists_mask = (unsigned long long*)take(n_tiles * E2F_TILE_LCAP * 8);
        if (!e2f_tile_layouts_direct(ctx)) {   // the projection's plain layouts, turned into the ones above by a relayout kernel
            L.q = (float*)take((size_t)N * (ctx->cfg.L_max + 1) * ctx->cfg.C * 4);
            L.k = (float*)take((size_t)N * (ctx->cfg.L_max + 1) * ctx->cfg.C * 4);
            L.v = (void*)take((size_t)N * ctx->n * ctx->cfg.C * esz);
        }
    } else {
        if (v_layout == 3) {
            const size_t H = ctx->cfg.H, DK = (size_t)(ctx->cfg.L_max + 1) * 16, N4 = ((size_t)N + 3) / 4 * 4;
            L.qf = (float*)take((size_t)N * H * DK * 4);
            L.kf = (float*)take(N4 * H * DK * 4);
            L.vf = (float*)take(N4 * H * ctx->n * 16 * 4);
            L.G = (float*)take((size_t)(3 * E2F_MAX_N * E2F_MAX_N + 256) * 4);
            const size_t n_tiles = ((size_t)N + 15) / 16;
            L.lists_hdr = (int4*)take(n_tiles * sizeof(int4));
            L.lists_ent = (int*)take(n_tiles * E2F_TILE_LCAP * 4);
            L.lists_pos = (float4*)take(n_tiles * E2F_TILE_LCAP * 4 * sizeof(float4));
            L.lists_mask = (unsigned long long*)take(n_tiles * E2F_TILE_LCAP * 8);
        }
        L.q = (float*)take((size_t)N * (ctx->cfg.L_max + 1) * ctx->cfg.C * 4);
        L.k = (float*)take((size_t)N * (ctx->cfg.L_max + 1) * ctx->cfg.C * 4);
        // tiled v of the per-pair MFMA attention kernel: 16-row tiles per head, two tiles when L_max >= 3
        const size_t v_elems = v_layout == 1 ? (size_t)ctx->cfg.H * (ctx->cfg.L_max >= 3 ? 2 : 1) * 256
                                             : (size_t)ctx->n * ctx->cfg.C;
        L.v = (void*)take((size_t)N * v_elems * esz);
    }
    L.cw = (float*)take((size_t)E2F_MAX_N * E2F_NP * 4);
    L.wbT = (float*)take((size_t)ctx->cfg.B * ctx->cfg.H * 4);
    L.cap_d2 = nullptr;
    L.cap_idx = nullptr;
    L.bytes = off;
    return L;
}

extern "C" {

const char* e2f_status_string(e2f_status s) {
    switch (s) {
        case E2F_OK: return "ok";
        case E2F_ERR_INVALID_ARG: return "invalid argument";
        case E2F_ERR_UNSUPPORTED: return "unsupported configuration";
        case E2F_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case E2F_ERR_HIP: return "HIP runtime error";
        case E2F_ERR_OOM: return "out of device memory";
        case E2F_ERR_SCRATCH_EXCEEDED: return "problem exceeds the library's static scratch (E2F_STATIC_SCRATCH_BYTES)";
    }
    return "unknown status";
}

e2f_status e2f_create(const e2f_config* cfg, e2f_ctx** ctx_out) {
    if (!cfg || !ctx_out) return E2F_ERR_INVALID_ARG;
    if (cfg->L_max < 0 || cfg->C <= 0 || cfg->H <= 0 || cfg->B <= 0 || cfg->lf < 0) return E2F_ERR_INVALID_ARG;
    if (!(cfg->cutoff > 0.0f) || !isfinite(cfg->cutoff)) return E2F_ERR_INVALID_ARG;
    if (cfg->C % cfg->H != 0) return E2F_ERR_INVALID_ARG;
    if (cfg->feat_dtype != E2F_F32 && cfg->feat_dtype != E2F_BF16) return E2F_ERR_INVALID_ARG;
    if (cfg->attention < E2F_ATTN_AUTO || cfg->attention > E2F_ATTN_VALU) return E2F_ERR_INVALID_ARG;
    if (cfg->flags & ~(E2F_FLAG_TILE_LISTS_PER_HEAD | E2F_FLAG_PROJECT_PER_CHANNEL_TILE)) return E2F_ERR_INVALID_ARG;
    if (cfg->lf > cfg->L_max && cfg->lf != 0) return E2F_ERR_INVALID_ARG;
    if (cfg->L_max > E2F_MAX_L || cfg->lf > E2F_MAX_LF || cfg->H > E2F_MAX_H) return E2F_ERR_UNSUPPORTED;
    // channel tiling of the kernels: 16-wide MFMA tiles (32-deep for bf16), lanes over channels in the fused kernel
    if (cfg->C % 16 != 0 || cfg->C > 256 || (cfg->C > 64 && cfg->C % 64 != 0)) return E2F_ERR_UNSUPPORTED;
    if (cfg->feat_dtype == E2F_BF16 && cfg->C % 32 != 0) return E2F_ERR_UNSUPPORTED;
    const int cpl = cfg->C <= 64 ? 1 : cfg->C / 64;
    const int Ch = cfg->C / cfg->H;
    if (Ch % cpl != 0) return E2F_ERR_UNSUPPORTED;
    const int lph = Ch / cpl;  // lanes per head must be a power of two (butterfly reduction of q.k)
    if ((lph & (lph - 1)) != 0) return E2F_ERR_UNSUPPORTED;

    e2f_ctx* c = new (std::nothrow) e2f_ctx;
    if (!c) return E2F_ERR_OOM;
    c->cfg = *cfg;
    c->n = (cfg->L_max + 1) * (cfg->L_max + 1);
    c->Ch = Ch;
    c->cpl = cpl;
    c->tau = (float)(1.0 / sqrt((double)((cfg->L_max + 1) * Ch)));
    c->rc2 = cfg->cutoff * cfg->cutoff;  // binary32 product, as the predicate defines it
    const double bm1 = cfg->B > 1 ? (double)(cfg->B - 1) : 1.0;
    c->rbf_gamma = (float)(0.5 * bm1 * bm1 / ((double)cfg->cutoff * (double)cfg->cutoff));
    c->rbf_step = (float)((double)cfg->cutoff / bm1);
    for (int x = 0; x < E2F_MAX_N; ++x)
        for (int t = 0; t < E2F_NP; ++t) c->coefP[x][t] = 0.0f;
    const int lf = cfg->lf;
    for (int lo = 0; lo <= cfg->L_max; ++lo)
        for (int m = -lo; m <= lo; ++m) {
            const int comp = lo * lo + lo + m, am = m < 0 ? -m : m;
            for (int kk = 0; kk <= 2 * lf; ++kk) {
                const int li = lo - lf + kk;
                if (li < 0 || li > cfg->L_max || am > li) continue;
                const double cg = clebsch_gordan(li, am, lf, 0, lo, am);
                // odd l_i + l_f + l_o (odd kk): the entry couples order -m to m and carries the sign of m
                c->coefP[comp][kk] = (float)((kk % 2) ? (m > 0 ? cg : (m < 0 ? -cg : 0.0)) : cg);
            }
        }
    // Attention kernel: the tile kernel where it applies, else the per-pair matrix-core kernel, else the ALU kernel,
    // unless the configuration names one.
    const int pick = cfg->attention;
    c->use_tile_attn = e2f_tile_supported(c) && (pick == E2F_ATTN_AUTO || pick == E2F_ATTN_TILE);
    c->use_tile_f32 = e2f_tile_f32_supported(c) && (pick == E2F_ATTN_AUTO || pick == E2F_ATTN_TILE);
    c->use_mfma_attn = !c->use_tile_attn && e2f_fused_mfma_supported(c) && (pick == E2F_ATTN_AUTO || pick == E2F_ATTN_PAIR);
    if ((pick == E2F_ATTN_TILE && !c->use_tile_attn && !c->use_tile_f32) || (pick == E2F_ATTN_PAIR && !c->use_mfma_attn)) {
        delete c;
        return E2F_ERR_UNSUPPORTED;
    }
    c->prof_events = nullptr;
    c->prof_capacity = 0;
    c->prof_calls = 0;
    *ctx_out = c;
    return E2F_OK;
}

void e2f_destroy(e2f_ctx* ctx) {
    if (!ctx) return;
    if (ctx->prof_events) {
        for (int i = 0; i < ctx->prof_capacity * (E2F_N_STAGES + 1); ++i) (void)hipEventDestroy(ctx->prof_events[i]);
        delete[] ctx->prof_events;
    }
    delete ctx;
}

e2f_status e2f_profile_begin(e2f_ctx* ctx, int32_t max_calls) {
    if (!ctx || max_calls <= 0 || max_calls > 4096 || ctx->prof_events) return E2F_ERR_INVALID_ARG;
    const int ne = max_calls * (E2F_N_STAGES + 1);
    hipEvent_t* ev = new (std::nothrow) hipEvent_t[ne];
    if (!ev) return E2F_ERR_OOM;
    for (int i = 0; i < ne; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
            delete[] ev;
            return E2F_ERR_HIP;
        }
    ctx->prof_events = ev;
    ctx->prof_capacity = max_calls;
    ctx->prof_calls = 0;
    return E2F_OK;
}

e2f_status e2f_profile_read(e2f_ctx* ctx, float* call_ms, int32_t capacity, int32_t* calls) {
    if (!ctx || !call_ms || !calls || capacity < 0 || !ctx->prof_events) return E2F_ERR_INVALID_ARG;
    const int nc = ctx->prof_calls < capacity ? ctx->prof_calls : capacity;
    for (int c = 0; c < nc; ++c) {
        hipEvent_t* ev = ctx->prof_events + c * (E2F_N_STAGES + 1);
        E2F_HIP_CHECK(hipEventSynchronize(ev[E2F_N_STAGES]));
        for (int s = 0; s < E2F_N_STAGES; ++s) E2F_HIP_CHECK(hipEventElapsedTime(&call_ms[c * E2F_N_STAGES + s], ev[s], ev[s + 1]));
    }
    *calls = nc;
    return E2F_OK;
}

e2f_status e2f_profile_end(e2f_ctx* ctx, float* stage_ms, int32_t* calls) {
    if (!ctx || !stage_ms || !calls || !ctx->prof_events) return E2F_ERR_INVALID_ARG;
    e2f_status rc = E2F_OK;
    double sum[E2F_N_STAGES] = {0.0, 0.0, 0.0};
    for (int c = 0; c < ctx->prof_calls && rc == E2F_OK; ++c) {
        hipEvent_t* ev = ctx->prof_events + c * (E2F_N_STAGES + 1);
        if (hipEventSynchronize(ev[E2F_N_STAGES]) != hipSuccess) rc = E2F_ERR_HIP;
        for (int s = 0; s < E2F_N_STAGES && rc == E2F_OK; ++s) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, ev[s], ev[s + 1]) != hipSuccess) rc = E2F_ERR_HIP;
            sum[s] += ms;
        }
    }
    *calls = ctx->prof_calls;
    for (int s = 0; s < E2F_N_STAGES; ++s) stage_ms[s] = ctx->prof_calls > 0 ? (float)(sum[s] / ctx->prof_calls) : 0.0f;
    for (int i = 0; i < ctx->prof_capacity * (E2F_N_STAGES + 1); ++i) (void)hipEventDestroy(ctx->prof_events[i]);
    delete[] ctx->prof_events;
    ctx->prof_events = nullptr;
    ctx->prof_capacity = 0;
    ctx->prof_calls = 0;
    return rc;
}

size_t e2f_cells_workspace_bytes(const e2f_ctx* ctx, int32_t N, int32_t S) {
    if (!ctx || N < 0 || S < 0) return 0;
    return cells_ws_layout(N, S, nullptr, nullptr);
}

e2f_status e2f_build_cells(e2f_ctx* ctx, const float* pos, const int32_t* seg_offsets, int32_t N, int32_t S, void* ws,
                           size_t ws_bytes, e2f_cells** cells, void* hip_stream) {
    return e2f_build_cells_periodic(ctx, pos, seg_offsets, N, S, nullptr, ws, ws_bytes, cells, hip_stream);
}

e2f_status e2f_build_cells_periodic(e2f_ctx* ctx, const float* pos, const int32_t* seg_offsets, int32_t N, int32_t S,
                                    const float* box, void* ws, size_t ws_bytes, e2f_cells** cells,
                                    void* hip_stream) {
    if (!ctx || !cells || N < 0 || S < 0) return E2F_ERR_INVALID_ARG;
    bool periodic = false;
    if (box)
        for (int64_t i = 0; i < (int64_t)3 * S; ++i) {
            if (!(box[i] > 0.0f)) continue;   // open axis (also NaN)
            // three cells along a periodic axis: an atom then has at most one image inside the cutoff
            if (isinf(box[i]) || box[i] < 3.0f * e2f_cell_edge(ctx->cfg.cutoff)) return E2F_ERR_UNSUPPORTED;
            periodic = true;
        }
    if (N > 0 && (S < 1 || !pos || !seg_offsets || !ws)) return E2F_ERR_INVALID_ARG;
    if ((int64_t)27 * S + (int64_t)2 * N + 1 > 0x7fffffff) return E2F_ERR_UNSUPPORTED;
    if (N > 0 && !aligned256(ws)) return E2F_ERR_INVALID_ARG;
    if (N > 0 && ws_bytes < cells_ws_layout(N, S, nullptr, nullptr)) return E2F_ERR_WORKSPACE_TOO_SMALL;
    e2f_cells* c = new (std::nothrow) e2f_cells;
    if (!c) return E2F_ERR_OOM;
    cells_ws_layout(N, S, ws, c);
    c->pos = pos;
    if (periodic && N > 0) {
        c->host_box = new (std::nothrow) float[(size_t)6 * S];
        if (!c->host_box) {
            delete c;
            return E2F_ERR_OOM;
        }
        for (int32_t s = 0; s < S; ++s)
            for (int k = 0; k < 3; ++k) {
                const float len = box[3 * s + k] > 0.0f ? box[3 * s + k] : 0.0f;
                c->host_box[6 * s + k] = len;
                c->host_box[6 * s + 3 + k] = len > 0.0f ? 1.0f / len : 0.0f;
            }
        c->view.periodic = 1;
        if (hipMemcpyAsync(c->box, c->host_box, sizeof(float) * 6 * S, hipMemcpyHostToDevice,
                           static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
            e2f_cells_destroy(c);
            return E2F_ERR_HIP;
        }
    }
    const e2f_status rc = e2f_launch_build_cells(ctx, c, pos, seg_offsets, static_cast<hipStream_t>(hip_stream));
    if (rc != E2F_OK) {
        e2f_cells_destroy(c);
        return rc;
    }
    *cells = c;
    return E2F_OK;
}

void e2f_cells_destroy(e2f_cells* cells) {
    if (!cells) return;
    delete[] cells->host_box;
    delete cells;
}

e2f_status e2f_count_neighbors(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, int32_t N, int32_t* degree,
                               void* hip_stream) {
    if (!ctx || !cells || N != cells->view.N) return E2F_ERR_INVALID_ARG;
    if (N > 0 && (!pos || !degree || pos != cells->pos)) return E2F_ERR_INVALID_ARG;
    return e2f_launch_count_neighbors(ctx, cells->view, pos, degree, static_cast<hipStream_t>(hip_stream));
}

e2f_status e2f_count_edges(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, int32_t N, int64_t* n_edges,
                           int32_t* degree, void* hip_stream) {
    if (!n_edges) return E2F_ERR_INVALID_ARG;
    *n_edges = 0;
    e2f_status rc = e2f_count_neighbors(ctx, cells, pos, N, degree, hip_stream);
    if (rc != E2F_OK || N == 0) return rc;
    int32_t* host = new (std::nothrow) int32_t[(size_t)N];
    if (!host) return E2F_ERR_OOM;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(host, degree, (size_t)N * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        delete[] host;
        return E2F_ERR_HIP;
    }
    int64_t sum = 0;
    for (int32_t i = 0; i < N; ++i) sum += host[i];
    delete[] host;
    *n_edges = sum;
    return E2F_OK;
}

e2f_status e2f_list_neighbors(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, int32_t N, const int64_t* offsets,
                              int32_t* idx, void* hip_stream) {
    if (!ctx || !cells || N != cells->view.N) return E2F_ERR_INVALID_ARG;
    if (N > 0 && (!pos || !offsets || !idx || pos != cells->pos)) return E2F_ERR_INVALID_ARG;
    return e2f_launch_list_neighbors(ctx, cells->view, pos, offsets, idx, static_cast<hipStream_t>(hip_stream));
}

size_t e2f_attn_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    return e2f_attn_ws_layout(ctx, N, nullptr, e2f_v_layout(ctx)).bytes;
}

// The fused call, optionally with a neighbour cap K > 0 (threshold keys in two more [N] arrays after the workspace)
// or over the caller's padded table.
static e2f_status forward_impl(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                               const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, float* out,
                               void* ws, size_t ws_bytes, void* hip_stream, int32_t cap_K, const int32_t* table,
                               int32_t table_K) {
    e2f_status rc = check_forward_args(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, ws_bytes);
    if (rc != E2F_OK || N == 0) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (cells->view.periodic && table) return E2F_ERR_UNSUPPORTED;   // the table names atoms, not images
    // the table form runs on the tile kernel where that applies, else on the ALU kernel, which reads the plain layout
    // (the fp32 tile kernel takes neither a cap nor a table: those calls run on the ALU kernel)
    const bool tile_f32 = ctx->use_tile_f32 && !table && cap_K <= 0;
    const int v_layout = tile_f32 ? 3 : ((table && !ctx->use_tile_attn) || ctx->use_tile_f32) ? 0 : e2f_v_layout(ctx);
    E2fAttnWs L = e2f_attn_ws_layout(ctx, N, ws, v_layout);
    if (cap_K > 0) {
        if (ws_bytes < L.bytes + 2 * e2f_align_up((size_t)N * 4)) return E2F_ERR_WORKSPACE_TOO_SMALL;
        uint32_t* cd = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + L.bytes);
        int32_t* ci = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.bytes + e2f_align_up((size_t)N * 4));
        if ((rc = e2f_launch_select_neighbors(ctx, cells->view, pos, cap_K, cd, ci, nullptr, nullptr, st)) != E2F_OK)
            return rc;
        L.cap_d2 = cd;
        L.cap_idx = ci;
    }
    hipEvent_t* ev = (ctx->prof_events && ctx->prof_calls < ctx->prof_capacity)
                         ? ctx->prof_events + ctx->prof_calls * (E2F_N_STAGES + 1) : nullptr;
    if (ev) E2F_HIP_CHECK(hipEventRecord(ev[0], st));
    if ((rc = e2f_launch_prepare(ctx, cells->view, pos, w, L, st)) != E2F_OK) return rc;
    if (ev) E2F_HIP_CHECK(hipEventRecord(ev[1], st));
    if ((rc = e2f_launch_project_mfma(ctx, cells->view, h, w, L, v_layout == 3 ? 0 : v_layout, st)) != E2F_OK) return rc;
    if (ev) E2F_HIP_CHECK(hipEventRecord(ev[2], st));
    if (tile_f32) {
        // candidate lists, the fp32 tile kernel for the tiles whose list fits, the ALU kernel for the atoms of the others
        if ((rc = e2f_launch_tile_lists(ctx, cells->view, L, st)) != E2F_OK) return rc;
        if ((rc = e2f_launch_tile_f32(ctx, cells->view, L, out, st)) != E2F_OK) return rc;
    }
    rc = tile_f32             ? e2f_launch_fused_crowded(ctx, cells->view, w, L, out, st)
         : ctx->use_tile_attn ? e2f_launch_tile(ctx, cells->view, L, table, table_K, out, st)
         : table              ? e2f_launch_fused_table(ctx, cells->view, w, L, table, table_K, out, st)
         : ctx->use_mfma_attn ? e2f_launch_fused_mfma(ctx, cells->view, w, L, out, st)
                              : e2f_launch_fused(ctx, cells->view, w, L, out, st);
    if (rc != E2F_OK) return rc;
    if (ev) {
        E2F_HIP_CHECK(hipEventRecord(ev[3], st));
        ctx->prof_calls++;
    }
    return E2F_OK;
}

e2f_status e2f_attn_forward(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                            const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, float* out,
                            void* ws, size_t ws_bytes, void* hip_stream) {
    return forward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, ws_bytes, hip_stream, 0, nullptr, 0);
}

e2f_status e2f_attn_forward_static(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                   const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, float* out,
                                   void* hip_stream) {
    if (!ctx || N < 0) return E2F_ERR_INVALID_ARG;
    if (e2f_attn_workspace_bytes(ctx, N) > (size_t)E2F_STATIC_SCRATCH_BYTES) return E2F_ERR_SCRATCH_EXCEEDED;
    void* ws = nullptr;
    if (N > 0) {
        const e2f_status rc = static_scratch(&ws);
        if (rc != E2F_OK) return rc;
    }
    // Nothing in the workspace has to start at zero: every stage writes all that the next one reads (padding rows of
    // k and v and the tiles' list headers included), so what an earlier, larger call left behind is never read.
    return forward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, (size_t)E2F_STATIC_SCRATCH_BYTES, hip_stream, 0,
                        nullptr, 0);
}

size_t e2f_attn_capped_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    return e2f_attn_ws_layout(ctx, N, nullptr, e2f_v_layout(ctx)).bytes + 2 * e2f_align_up((size_t)N * 4);
}

e2f_status e2f_attn_forward_capped(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                   const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                   int32_t max_neighbors, float* out, void* ws, size_t ws_bytes, void* hip_stream) {
    if (max_neighbors <= 0) return E2F_ERR_INVALID_ARG;
    return forward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, ws_bytes, hip_stream, max_neighbors, nullptr, 0);
}

e2f_status e2f_build_neighbor_table(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, int32_t N, int32_t K,
                                    int32_t* table, int32_t* count, void* hip_stream) {
    if (!ctx || !cells || N != cells->view.N || K <= 0) return E2F_ERR_INVALID_ARG;
    if (N > 0 && (!pos || !table || pos != cells->pos)) return E2F_ERR_INVALID_ARG;
    return e2f_launch_select_neighbors(ctx, cells->view, pos, K, nullptr, nullptr, table, count,
                                       static_cast<hipStream_t>(hip_stream));
}

size_t e2f_attn_table_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    const size_t a = e2f_attn_ws_layout(ctx, N, nullptr, 0).bytes, b = e2f_attn_workspace_bytes(ctx, N);
    return a > b ? a : b;
}

e2f_status e2f_attn_forward_table(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                  const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                  const int32_t* table, int32_t K, float* out, void* ws, size_t ws_bytes,
                                  void* hip_stream) {
    if (K <= 0 || (N > 0 && !table)) return E2F_ERR_INVALID_ARG;
    if (ctx && ws_bytes < e2f_attn_table_workspace_bytes(ctx, N)) return E2F_ERR_WORKSPACE_TOO_SMALL;
    return forward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, ws_bytes, hip_stream, 0, table, K);
}

static E2fFactWs fact_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, size_t attn_bytes) {
    E2fFactWs F;
    size_t off = attn_bytes;
    auto take = [&](size_t bytes) {
        char* p = ws ? static_cast<char*>(ws) + off : nullptr;
        off += e2f_align_up(bytes);
        return p;
    };
    const size_t rows = (size_t)N * ctx->n * ctx->cfg.C * 4;
    F.hp = (float*)take(rows);
    F.a1 = (float*)take(rows);
    F.a0 = (float*)take(rows);
    F.bytes = off;
    return F;
}

size_t e2f_attn_factorized_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    return fact_ws_layout(ctx, N, nullptr, e2f_attn_ws_layout(ctx, N, nullptr, 0).bytes).bytes;
}

e2f_status e2f_attn_forward_factorized(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                       const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                       float* out, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return E2F_ERR_INVALID_ARG;
    if (!e2f_factorized_supported(ctx)) return E2F_ERR_UNSUPPORTED;
    // same argument checks as the fused call, against this call's own workspace size
    e2f_status rc = check_forward_args(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, (size_t)-1);
    if (rc != E2F_OK || N == 0) return rc;
    // the node-level source and target terms take one position per atom; images would need one per pair
    if (cells->view.periodic) return E2F_ERR_UNSUPPORTED;
    if (ws_bytes < e2f_attn_factorized_workspace_bytes(ctx, N)) return E2F_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const E2fAttnWs L = e2f_attn_ws_layout(ctx, N, ws, 0);
    const E2fFactWs F = fact_ws_layout(ctx, N, ws, L.bytes);
    if ((rc = e2f_launch_prepare(ctx, cells->view, pos, w, L, st)) != E2F_OK) return rc;
    if ((rc = e2f_launch_project_mfma(ctx, cells->view, h, w, L, 0, st)) != E2F_OK) return rc;
    return e2f_launch_factorized(ctx, cells->view, L, F, out, st);
}

// q1 = W_Q1 h in v's plain layout, after the attention workspace
static size_t nonlinear_q1_bytes(const e2f_ctx* ctx, int32_t N) {
    return e2f_align_up((size_t)N * ctx->n * ctx->cfg.C * (ctx->cfg.feat_dtype == E2F_BF16 ? 2 : 4));
}

size_t e2f_attn_nonlinear_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    return e2f_attn_ws_layout(ctx, N, nullptr, 0).bytes + nonlinear_q1_bytes(ctx, N);
}

e2f_status e2f_attn_forward_nonlinear(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                      const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                      float* out, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!ctx) return E2F_ERR_INVALID_ARG;
    if (!e2f_nonlinear_supported(ctx)) return E2F_ERR_UNSUPPORTED;
    e2f_status rc = check_forward_args(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, (size_t)-1);
    if (rc != E2F_OK || N == 0) return rc;
    if (ws_bytes < e2f_attn_nonlinear_workspace_bytes(ctx, N)) return E2F_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const E2fAttnWs L = e2f_attn_ws_layout(ctx, N, ws, 0);
    void* q1 = static_cast<char*>(ws) + L.bytes;
    if ((rc = e2f_launch_prepare(ctx, cells->view, pos, w, L, st)) != E2F_OK) return rc;
    // W_Q1 h of every atom: the projection kernel once more, with W_Q1 in the value's place (it rewrites q and k
    // with the same numbers; the second run below leaves them in place with the values)
    e2f_weights wq = *w;
    wq.WV = w->WQ1;
    E2fAttnWs Lq = L;
    Lq.v = q1;
    if ((rc = e2f_launch_project_mfma(ctx, cells->view, h, &wq, Lq, 0, st)) != E2F_OK) return rc;
    if ((rc = e2f_launch_project_mfma(ctx, cells->view, h, w, L, 0, st)) != E2F_OK) return rc;
    return e2f_launch_fused_nonlinear(ctx, cells->view, w, L, q1, out, st);
}

static E2fBwdWs bwd_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, size_t attn_bytes, bool with_W) {
    E2fBwdWs Bw;
    size_t off = attn_bytes;
    auto take = [&](size_t bytes) {
        char* p = ws ? static_cast<char*>(ws) + off : nullptr;
        off += e2f_align_up(bytes);
        return p;
    };
    Bw.lse = (float*)take((size_t)N * ctx->cfg.H * 4);
    Bw.Dn = (float*)take((size_t)N * ctx->cfg.H * 4);
    Bw.G = (float*)take((size_t)3 * E2F_MAX_N * E2F_MAX_N * 4);
    Bw.cw_unit = (float*)take((size_t)E2F_MAX_N * E2F_NP * 4);
    Bw.Gu = (float*)take((size_t)3 * E2F_MAX_N * E2F_MAX_N * 4);
    Bw.pWb = (float*)take((size_t)N * ctx->cfg.H * ctx->cfg.B * 4);
    Bw.pwp = (float*)take((size_t)N * 32 * 4);
    Bw.wT = ctx->cfg.feat_dtype == E2F_BF16
                ? (uint16_t*)take((size_t)5 * (ctx->cfg.L_max + 1) * ctx->cfg.C * ctx->cfg.C * 2) : nullptr;
    Bw.tbuf = Bw.wpart = nullptr;
    if (with_W) {
        const size_t C = ctx->cfg.C, L1 = ctx->cfg.L_max + 1;
        Bw.tbuf = (float*)take((size_t)5 * N * ctx->n * C * 4);
        Bw.wpart = (float*)take((size_t)8 * L1 * L1 * 5 * C * C * 4);   // 8 (L_max+1)^2 slices of partial sums
    }
    Bw.bytes = off;
    return Bw;
}

// The pair work of the backward pass runs in tile form where the forward pass does (with the gradients of Wb and
// w_path only for up to 8 radial basis functions; beyond that the per-atom kernels form them).
static bool backward_in_tile_form(const e2f_ctx* ctx, bool wgrad) {
    return ctx->use_tile_attn && (!wgrad || e2f_backward_tile_weight_gradients_supported(ctx));
}

size_t e2f_attn_backward_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    size_t bytes = bwd_ws_layout(ctx, N, nullptr, e2f_attn_ws_layout(ctx, N, nullptr, 0).bytes, false).bytes;
    if (backward_in_tile_form(ctx, false)) {   // either form may run, depending on the gradients asked for
        const size_t b2 = bwd_ws_layout(ctx, N, nullptr, e2f_attn_ws_layout(ctx, N, nullptr, 2).bytes, false).bytes;
        const size_t b3 = e2f_bwd_tile_ws_layout(ctx, N, nullptr, b2).bytes;
        if (b3 > bytes) bytes = b3;
    }
    return bytes;
}

size_t e2f_attn_backward_weights_workspace_bytes(const e2f_ctx* ctx, int32_t N) {
    if (!ctx || N < 0) return 0;
    size_t bytes = bwd_ws_layout(ctx, N, nullptr, e2f_attn_ws_layout(ctx, N, nullptr, 0).bytes, true).bytes;
    if (backward_in_tile_form(ctx, false)) {
        const size_t b2 = bwd_ws_layout(ctx, N, nullptr, e2f_attn_ws_layout(ctx, N, nullptr, 2).bytes, true).bytes;
        const size_t b3 = e2f_bwd_tile_ws_layout(ctx, N, nullptr, b2).bytes;
        if (b3 > bytes) bytes = b3;
    }
    return bytes;
}

// saved: the workspace still holds what the forward pass wrote (projections, candidate lists, axis operators)
static e2f_status backward_impl(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, const float* out,
                                const float* grad_out, float* grad_pos, float* grad_q, float* grad_k, float* grad_v,
                                float* grad_h, float* grad_Wb, float* grad_w_path, float* grad_W, void* ws, size_t ws_bytes,
                                void* hip_stream, bool saved) {
    if (!ctx) return E2F_ERR_INVALID_ARG;
    if (!e2f_backward_supported(ctx)) return E2F_ERR_UNSUPPORTED;
    // same argument checks as the fused call (out is read here), against this call's own workspace size
    e2f_status rc = check_forward_args(ctx, cells, pos, h, seg_offsets, N, S, w, const_cast<float*>(out), ws, (size_t)-1);
    if (rc != E2F_OK || N == 0) return rc;
    if (!grad_out || !grad_pos || !grad_q || !grad_k || !grad_v) return E2F_ERR_INVALID_ARG;
    if (ws_bytes < (grad_W ? e2f_attn_backward_weights_workspace_bytes(ctx, N) : e2f_attn_backward_workspace_bytes(ctx, N)))
        return E2F_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool tile = backward_in_tile_form(ctx, grad_Wb || grad_w_path);
    const int v_layout = tile ? 2 : 0;
    const E2fAttnWs L = e2f_attn_ws_layout(ctx, N, ws, v_layout);
    const E2fBwdWs Bw = bwd_ws_layout(ctx, N, ws, L.bytes, grad_W != nullptr);
    E2fBwdTileWs Tw;
    if (tile) Tw = e2f_bwd_tile_ws_layout(ctx, N, ws, Bw.bytes);
    // (the forward pass of a configuration whose backward pass runs in tile form used the same layout of ws)
    const bool reuse = saved && tile && ctx->use_tile_attn && !(ctx->cfg.flags & E2F_FLAG_TILE_LISTS_PER_HEAD);
    if (!reuse) {
        if ((rc = e2f_launch_prepare(ctx, cells->view, pos, w, L, st)) != E2F_OK) return rc;
        if ((rc = e2f_launch_project_mfma(ctx, cells->view, h, w, L, v_layout, st)) != E2F_OK) return rc;
    }
    return e2f_launch_backward(ctx, cells->view, w, L, Bw, out, grad_out, grad_pos, grad_q, grad_k, grad_v, h, grad_h,
                               grad_Wb, grad_w_path, grad_W, tile ? &Tw : nullptr, st, reuse);
}

e2f_status e2f_attn_backward(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                             const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w, const float* out,
                             const float* grad_out, float* grad_pos, float* grad_q, float* grad_k, float* grad_v,
                             float* grad_h, float* grad_Wb, float* grad_w_path, float* grad_W, void* ws, size_t ws_bytes,
                             void* hip_stream) {
    return backward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, grad_out, grad_pos, grad_q, grad_k, grad_v, grad_h,
                         grad_Wb, grad_w_path, grad_W, ws, ws_bytes, hip_stream, false);
}

e2f_status e2f_attn_backward_after_forward(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                           const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                           const float* out, const float* grad_out, float* grad_pos, float* grad_q,
                                           float* grad_k, float* grad_v, float* grad_h, float* grad_Wb,
                                           float* grad_w_path, float* grad_W, void* ws, size_t ws_bytes,
                                           void* hip_stream) {
    return backward_impl(ctx, cells, pos, h, seg_offsets, N, S, w, out, grad_out, grad_pos, grad_q, grad_k, grad_v, grad_h,
                         grad_Wb, grad_w_path, grad_W, ws, ws_bytes, hip_stream, true);
}

e2f_status e2f_eaas_tensor_product(e2f_ctx* ctx, const void* h, const float* r, const float* w_path, float* out,
                                   int32_t T, void* hip_stream) {
    if (!ctx || T < 0) return E2F_ERR_INVALID_ARG;
    if (T > 0 && (!h || !r || !w_path || !out)) return E2F_ERR_INVALID_ARG;
    return e2f_launch_tensor_product(ctx, h, r, w_path, out, T, static_cast<hipStream_t>(hip_stream));
}

e2f_status e2f_attn_forward_materialized(e2f_ctx* ctx, const e2f_cells* cells, const float* pos, const void* h,
                                         const int32_t* seg_offsets, int32_t N, int32_t S, const e2f_weights* w,
                                         float* out, void* ws, size_t ws_bytes, void* hip_stream, size_t* edges_out,
                                         size_t* peak_bytes_out) {
    e2f_status rc = check_forward_args(ctx, cells, pos, h, seg_offsets, N, S, w, out, ws, ws_bytes);
    if (edges_out) *edges_out = 0;
    if (peak_bytes_out) *peak_bytes_out = 0;
    if (rc != E2F_OK || N == 0) return rc;
    if (cells->view.periodic) return E2F_ERR_UNSUPPORTED;   // the edge list carries no images
    const E2fAttnWs L = e2f_attn_ws_layout(ctx, N, ws, e2f_v_layout(ctx));
    hipEvent_t* ev = (ctx->prof_events && ctx->prof_calls < ctx->prof_capacity)
                         ? ctx->prof_events + ctx->prof_calls * (E2F_N_STAGES + 1) : nullptr;
    rc = e2f_run_materialized(ctx, cells->view, pos, h, w, L, out, static_cast<hipStream_t>(hip_stream), edges_out,
                              peak_bytes_out, ev);
    if (rc == E2F_OK && ev) ctx->prof_calls++;
    return rc;
}

}  // extern "C"
