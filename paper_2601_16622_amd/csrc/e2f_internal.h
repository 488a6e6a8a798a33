// Internal declarations shared by the translation units of libe2f.so (host objects, device views, launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/e2f.h"

#define E2F_MAX_L 4
#define E2F_MAX_N ((E2F_MAX_L + 1) * (E2F_MAX_L + 1))
#define E2F_MAX_H 32
#define E2F_MAX_LF 2
#define E2F_NP (2 * E2F_MAX_LF + 1)  // coupling paths per output degree: l_in = l_out - lf + k, k = 0..2 lf

// Per-segment uniform grid: cell (x,y,z) of the segment has global id base + (z*ny + y)*nx + x.
// A periodic axis has box length l* > 0 (r* = 1/l* rounded to binary32), origin 0 and at least 3 cells that
// tile the box exactly; an open axis has l* = 0 and cells laid over the bounding box.
struct E2fSegGrid {
    float ox, oy, oz;
    float ix, iy, iz;   // 1 / cell edge per axis
    int32_t nx, ny, nz, base;
    float lx, ly, lz;
    float rx, ry, rz;
};

// Device view of a cell list (all pointers into the caller's cells workspace).
struct E2fCellsView {
    const E2fSegGrid* grid;     // [S]
    const int32_t* cell_start;  // [max_cells + 1] first sorted slot of each global cell
    const int32_t* perm;        // [N] sorted slot -> caller's atom index
    const int32_t* scell;       // [N] global cell id of the atom in each sorted slot
    const int32_t* sseg;        // [N] segment of the atom in each sorted slot
    const int32_t* atom_slot;   // [N] caller's atom index -> sorted slot
    const int4* sinfo;          // [N][2] per sorted slot: (segment, cell x, cell y, cell z), (nx, ny, nz, first cell id)
                                // of its grid: what a target needs to find its stencil without reading the grid
    int32_t N, S;
    int32_t periodic;           // whether any segment has a periodic axis (selects the kernels that follow images)
};

struct e2f_cells {
    E2fCellsView view;
    // scratch used while building
    int32_t* bbox;       // [S][6] order-preserving integer images of min/max coordinates
    int32_t* atom_seg;   // [N]
    int32_t* atom_cell;  // [N]
    int32_t* cell_fill;  // [max_cells]
    int32_t* tmp_slot;   // [N]
    int32_t* atom_sub;   // [N] position of the atom inside its cell: Morton index over 4x4x4 sub-cells
    float* box;          // [S][6] on the device: periodic box lengths (0 = open axis), then their reciprocals
    int32_t max_cells;
    const float* pos;    // the positions the list was built from (identity check only)
    float* host_box;     // [S][6] copy of the periodic boxes that the upload reads (owned; nullptr without any)
};

struct e2f_ctx {
    e2f_config cfg;
    int32_t n;         // (L_max+1)^2
    int32_t Ch;        // channels per head
    int32_t cpl;       // channels per lane in the fused kernel
    bool use_mfma_attn;  // per-pair attention on the matrix cores (bf16, heads of 16 channels); v is stored tiled
    bool use_tile_attn;  // tile attention kernel (bf16, heads of 16 channels, lf = 1); q, k, v in its group layout
    bool use_tile_f32;   // its fp32 form (fp32 features, heads of 16 channels, lf = 1); plain q, k, v plus fp32 tile layouts
    float tau;         // 1/sqrt(d_k)
    float rc2;         // cutoff*cutoff rounded to binary32
    float rbf_gamma;   // (B-1)^2 / (2 cutoff^2)
    float rbf_step;    // cutoff/(B-1)
    // coupling coefficients of the re-indexing operator P for lf (without path weights): coefP[comp][k] multiplies
    // the aligned input of degree l_in = l_out - lf + k; even k keeps the order m, odd k takes it from -m.
    float coefP[E2F_MAX_N][E2F_NP];
    // optional per-stage timing (e2f_profile_begin / e2f_profile_end)
    hipEvent_t* prof_events;  // [prof_capacity][E2F_N_STAGES + 1]
    int32_t prof_capacity, prof_calls;
};

// Layout of the O(N) attention workspace.
struct E2fAttnWs {
    float4* spos;   // [N] sorted positions (w unused)
    float* q;       // [N][L+1][C] sorted order
    float* k;       // [N][L+1][C]
    void* v;        // [N][n][C] sorted order, float or bf16 (follows feat_dtype)
    float* cw;      // [n][E2F_NP] P coefficients times path weights
    float* wbT;     // [B][H] radial bias weights, transposed
    // neighbour cap: threshold key of every sorted slot (null when the call has no cap); see under_cap()
    const uint32_t* cap_d2;
    const int32_t* cap_idx;
    // layout of the tile attention kernel (v_layout 2; q, k, v above are then unused)
    uint16_t* q16;       // [N][H][DKP] binary16, q * tau * log2(e)
    uint16_t* k16;       // [ceil(N/4)][H][DKP/32][4 slots][32] binary16 (e2f::k16_offset)
    uint16_t* v4;        // [ceil(N/4)][H] blocks of n * 64 bf16, components alone or in pairs (e2f::v4_offset)
    float* G;            // [3][25][25] axis operators of the degree-1 filter, then their 216 pattern entries packed
    // candidate lists of the tile kernel, one per tile of 16 sorted slots (see TileParams)
    int4* lists_hdr;     // [ceil(N/16)]
    int* lists_ent;      // [ceil(N/16)][E2F_TILE_LCAP]
    float4* lists_pos;   // [ceil(N/16)][E2F_TILE_LCAP][4]
    unsigned long long* lists_mask;   // [ceil(N/16)][E2F_TILE_LCAP] the (target, slot) pairs of an entry that count
    // layout of the fp32 tile kernel (v_layout 3: beside the plain q, k, v)
    float* qf;           // [N][H][DK] q * tau * log2(e)
    float* kf;           // [ceil(N/4)][H][4 slots][DK]
    float* vf;           // [ceil(N/4)][H][n][16 channels][4 slots]
    size_t bytes;
};
#define E2F_TILE_LCAP 192
// v_layout: 0 plain [N][n][C], 1 component tiles of the per-pair MFMA kernel, 2 slot groups of the tile kernel,
// 3 plain plus the fp32 tile kernel's layouts and lists
E2fAttnWs e2f_attn_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, int v_layout);
static inline int e2f_v_layout(const e2f_ctx* ctx) {
    return ctx->use_tile_attn ? 2 : ctx->use_tile_f32 ? 3 : (ctx->use_mfma_attn ? 1 : 0);
}

// Extra buffers of the backward pass, placed after the attention workspace (untiled v).
struct E2fBwdWs {
    float* lse;  // [N][H] log of the softmax normaliser per sorted slot and head
    float* Dn;   // [N][H] <dL/d out_i, out_i> per head
    float* G;    // [3][25][25] axis operators of the degree-1 filter
    // for the gradients of Wb and w_path: unit-weight path coefficients and axis operators, per-atom partial sums
    float* cw_unit;  // [n][E2F_NP]
    float* Gu;       // [3][25][25]
    float* pWb;      // [N][H][B]
    float* pwp;      // [N][32]
    uint16_t* wT;    // [5][L+1][C in][C out] the projection matrices transposed (bf16 features: chain rule on the matrix cores)
    // for the gradients of the projection matrices (only in the larger workspace of that form of the call)
    float* tbuf;     // [5][N][n][C] row factors
    float* wpart;    // [8 (L+1)^2 slices][5][C][C] partial sums
    size_t bytes;
};

// Extra buffers of the backward pass's tile kernels (bf16 features, heads of 16 channels), after the ones above: the
// operands in the layouts the forward pass does not keep, the softmax statistics and partial position gradients.
struct E2fBwdTileWs {
    uint16_t* q16g;   // q rows in the grouped layout of k16
    uint16_t *q4, *k4;   // [group][H][DKP/32][16 features][2 feature tiles][4 slots] bf16
    uint16_t *vrow, *grow;   // [group][H][steps][4 slots][32] bf16 rows of v and of dL/d out over (component, channel)
    uint16_t* g4;     // dL/d out in the layout of v4
    float* stat4;     // [group][H][4 slots][2]: lse (base-2 units), <dL/d out_i, out_i>
    float* gp_part;   // [2][H][N][3] partial position gradients per side and head group
    float* pWb_t;     // [tiles][H][B] partial sums of dL/dWb per tile
    float* pwp_t;     // [tiles][H][32] partial sums of dL/dw_path per tile and head group
    float* Gu;        // axis operators with unit path weights: full form, then packed
    size_t bytes;     // end of the last buffer, counted from the start of the workspace
};

// Extra O(N) buffers of the factorized pipeline, placed after the attention workspace (untiled v).
struct E2fFactWs {
    float* hp;   // [N][n][C] source terms h'
    float* a1;   // [N][n][C] aggregated source terms
    float* a0;   // [N][n][C] aggregated values
    size_t bytes;
};

static inline size_t e2f_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
// Cell edge: a hair above the cutoff, since the binary32 predicate can accept a pair whose exact |dx| exceeds the
// cutoff by rounding, and cell coordinates carry rounding of their own.
static inline float e2f_cell_edge(float cutoff) { return cutoff * 1.0001f; }

#define E2F_HIP_CHECK(expr)                      \
    do {                                         \
        hipError_t e__ = (expr);                 \
        if (e__ != hipSuccess) return E2F_ERR_HIP; \
    } while (0)

// ---- launchers (each returns after enqueueing on `st`) ----
e2f_status e2f_launch_build_cells(const e2f_ctx* ctx, e2f_cells* c, const float* pos, const int32_t* seg_offsets,
                                  hipStream_t st);
e2f_status e2f_launch_count_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, int32_t* degree,
                                      hipStream_t st);
e2f_status e2f_launch_list_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos,
                                     const int64_t* offsets, int32_t* idx, hipStream_t st);
e2f_status e2f_launch_prepare(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, const e2f_weights* w,
                              const E2fAttnWs& ws, hipStream_t st);
e2f_status e2f_launch_project_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                                   const E2fAttnWs& ws, int v_layout, hipStream_t st);
bool e2f_factorized_supported(const e2f_ctx* ctx);
e2f_status e2f_launch_factorized(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const E2fFactWs& fw,
                                 float* out, hipStream_t st);
e2f_status e2f_launch_project_simple(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                                     float* q, float* k, float* v, hipStream_t st);
e2f_status e2f_launch_fused(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                            float* out, hipStream_t st);
// The same kernel for the atoms of crowded tiles only (tile headers in ws.lists_hdr, x < 0): every other atom's
// output row is left as it is.
e2f_status e2f_launch_fused_crowded(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                    float* out, hipStream_t st);
bool e2f_tile_f32_supported(const e2f_ctx* ctx);
e2f_status e2f_launch_tile_f32(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, float* out, hipStream_t st);
// The fused call with the non-linear pair feature in the logit; q1 = W_Q1 h in v's plain layout and type.
bool e2f_nonlinear_supported(const e2f_ctx* ctx);
e2f_status e2f_launch_fused_nonlinear(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w,
                                      const E2fAttnWs& ws, const void* q1, float* out, hipStream_t st);
e2f_status e2f_launch_tensor_product(const e2f_ctx* ctx, const void* h, const float* r, const float* w_path, float* out,
                                     int32_t T, hipStream_t st);
bool e2f_fused_mfma_supported(const e2f_ctx* ctx);
// K-th smallest neighbour key of every atom (threshold arrays in sorted-slot order) and / or the padded table of
// the at most K nearest neighbours in the caller's atom order; any of the outputs may be null.
e2f_status e2f_launch_select_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, int32_t K,
                                       uint32_t* cap_d2, int32_t* cap_idx, int32_t* table, int32_t* count,
                                       hipStream_t st);
e2f_status e2f_launch_fused_table(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                  const int32_t* table, int32_t K, float* out, hipStream_t st);
bool e2f_tile_supported(const e2f_ctx* ctx);
// Whether the projection writes the tile kernel's layouts itself (C = 32, 64, 128, 256); for other channel counts it
// writes the plain layouts and a relayout kernel follows (the workspace then holds both).
static inline bool e2f_tile_layouts_direct(const e2f_ctx* ctx) {
    return ctx->cfg.C == 32 || ctx->cfg.C == 64 || ctx->cfg.C == 128 || ctx->cfg.C == 256;
}
// G[mu][x_out][x_in], mu = x, y, z: the degree-1 filter's message for a unit pair vector along mu, from the path
// coefficients cw (tile attention kernel, backward pass).
e2f_status e2f_launch_axis_ops(const e2f_ctx* ctx, const float* cw, float* G, hipStream_t st, bool packed = false);
// Tile form of the backward pass's pair work (e2f_bwd_tile.hip): needs the tile layouts of q, k, v and the candidate
// lists in `ws`; tiles whose list did not fit are left to the per-atom kernels.
E2fBwdTileWs e2f_bwd_tile_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, size_t offset);
e2f_status e2f_launch_backward_tile(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws,
                                    const E2fBwdTileWs& tw, const float* out, const float* grad_out, float* grad_pos,
                                    float* grad_q, float* grad_k, float* grad_v, bool wgrad, hipStream_t st);
bool e2f_backward_tile_weight_gradients_supported(const e2f_ctx* ctx);
e2f_status e2f_launch_backward_tile_wsum(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws,
                                         const E2fBwdTileWs& tw, const float* atom_pWb, const float* atom_pwp,
                                         float* grad_Wb, float* grad_w_path, hipStream_t st);
// The candidate lists of the tile kernels and the axis operators only (a crowded tile gets the header -1 and nothing else).
e2f_status e2f_launch_tile_lists(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, hipStream_t st);
// tw: null for the per-atom pair kernels (plain layouts in `ws`), else the tile form (tile layouts in `ws`).
// lists_ready: the candidate lists and axis operators of the tile form are in `ws` already (left by the forward pass).
bool e2f_backward_supported(const e2f_ctx* ctx);
e2f_status e2f_launch_backward(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                               const E2fBwdWs& bw, const float* out, const float* grad_out, float* grad_pos,
                               float* grad_q, float* grad_k, float* grad_v, const void* h, float* grad_h,
                               float* grad_Wb, float* grad_w_path, float* grad_W, const E2fBwdTileWs* tw, hipStream_t st,
                               bool lists_ready = false);
// cw[comp][t] = P coefficient with every path weight one.
e2f_status e2f_launch_unit_cw(const e2f_ctx* ctx, float* cw, hipStream_t st);
// table: the caller's padded neighbour table [N][table_K], or null (every atom within the cutoff is a neighbour)
e2f_status e2f_launch_tile(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const int32_t* table,
                           int table_K, float* out, hipStream_t st);
e2f_status e2f_launch_fused_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                 float* out, hipStream_t st);
e2f_status e2f_run_materialized(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, const void* h,
                                const e2f_weights* w, const E2fAttnWs& ws, float* out, hipStream_t st,
                                size_t* edges_out, size_t* peak_bytes_out, hipEvent_t* ev);
