/*
 * e2f - node-centric on-the-fly equivariant attention forward pass (E2Former-V2) for AMD MI355X (gfx950).
 *
 * C ABI of libe2f.so.  The operator, for every atom i (paper: Preliminaries, Sec. 3.2-3.4):
 *
 *   N(i)    = { j != i in the same segment with |r_j - r_i| < cutoff }
 *   q_i,k_j = concat_l < W1^(l) h^(l), W2^(l) h^(l) >           (Eq. qk; W acts on channels, <,> sums over m)
 *   s_ij,h  = q_i,h . k_j,h / sqrt(d_k) + b_h(|r_ij|)            (Eq. kernel_score)
 *   a_ij,h  = softmax_j(s_ij,h) * phi(|r_ij|)                    (Eq. attn; the gate is outside the softmax)
 *   out_i   = sum_j a_ij,head(c) * ( v_j (x) R^(lf)(r_ij) )      (m_i = sum_j alpha_ij m_ij, v = W_V h)
 *
 * with the tensor product evaluated through Equivariant Axis-Aligned Sparsification (Sec. 3.3: rotate
 * v_j into the frame whose z-axis is r_ij, apply the sparse re-indexing operator P, rotate back) and the
 * sum over neighbours evaluated as the streaming online-softmax reduction of Algorithm 1, so that no
 * per-pair tensor is written to memory by e2f_attn_forward.
 *
 * Conventions
 *   - Component (l,m) of an irreps feature has index l*l + l + m; features are [atom][component][channel],
 *     channel innermost.  The real basis orders l=1 as (y,z,x); harmonics are Racah-normalised.
 *   - Head h owns channels [h*C/H, (h+1)*C/H) of every degree; d_k = (L_max+1)*C/H.
 *   - b_h(d) = sum_b Wb[h][b] exp(-gamma (d - mu_b)^2), mu_b = b*cutoff/(B-1), gamma = (B-1)^2/(2 cutoff^2);
 *     phi(d) = (1 + cos(pi d/cutoff))/2.
 *   - The neighbour predicate is evaluated in binary32 as d2 = (dx*dx + dy*dy) + dz*dz (each operation
 *     rounded, no fused multiply-add), 0 < d2 < cutoff*cutoff.
 *   - An atom without neighbours gets a zero output.
 *
 * Memory: every pointer marked "device" is GPU memory owned by the caller; the library never frees it.
 * Pointers marked "host" are ordinary process memory.  All work is enqueued on the HIP stream passed in
 * (a hipStream_t cast to void*; NULL is the default stream).  e2f_build_cells, e2f_attn_forward, its capped, table
 * and factorized forms, e2f_build_neighbor_table and e2f_attn_backward allocate no device memory and do not
 * synchronise with the host (e2f_build_cells_periodic enqueues one small host-to-device copy of the boxes from a
 * buffer the cells handle owns); e2f_attn_forward_materialized and e2f_count_edges are measurement/test entry points
 * that do both.
 * Errors are reported through the return code; no entry point aborts or throws.  Arguments are checked
 * before anything is launched.
 */
#ifndef E2F_H
#define E2F_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct e2f_ctx e2f_ctx;     /* configuration + constant tables (host object) */
typedef struct e2f_cells e2f_cells; /* host handle onto a cell list living in caller-provided device memory */

typedef enum {
    E2F_OK = 0,
    E2F_ERR_INVALID_ARG = 1,         /* null pointer, negative size, inconsistent configuration */
    E2F_ERR_UNSUPPORTED = 2,         /* valid in principle, not implemented (e.g. L_max > 4, lf > 2) */
    E2F_ERR_WORKSPACE_TOO_SMALL = 3, /* ws_bytes below the value the matching *_workspace_bytes returns */
    E2F_ERR_HIP = 4,                 /* a HIP runtime call failed */
    E2F_ERR_OOM = 5,                 /* device allocation failed (materialized baseline only) */
    E2F_ERR_SCRATCH_EXCEEDED = 6     /* e2f_attn_forward_static: the problem needs more than E2F_STATIC_SCRATCH_BYTES */
} e2f_status;

typedef enum { E2F_F32 = 0, E2F_BF16 = 1 } e2f_dtype;

/*
 * Which kernel runs the attention stage (Sec. 3.4, Algorithm 1).  All give the same result up to rounding.
 *   AUTO  the fastest form that supports the configuration (the order below)
 *   TILE  16 targets x 32 candidates on the matrix cores, degree-1 filter through its linear factorization
 *         (Eq. e2former_final at l = 1); heads of 16 channels, lf = 1, at most 16 radial basis functions; bf16
 *         features with C = 32, 64, 128 or 256, or fp32 features (every product then in binary32).  With bf16
 *         features q and k are kept in binary16 (values beyond +-65504 are clamped: use PAIR for features that are
 *         not normalised).  fp32 calls with a neighbour cap or a table run on VALU.
 *   PAIR  one wave per target, the aligning rotation and P evaluated per pair (Sec. 3.3), operators applied on the
 *         matrix cores; bf16 features, heads of 16 channels, lf = 1 or 2; q and k in fp32
 *   VALU  the same per-pair form on the vector ALUs; every configuration
 * A choice the configuration does not support makes e2f_create return E2F_ERR_UNSUPPORTED.
 */
typedef enum { E2F_ATTN_AUTO = 0, E2F_ATTN_TILE = 1, E2F_ATTN_PAIR = 2, E2F_ATTN_VALU = 3 } e2f_attn_kernel;

/* e2f_config.flags (for A/B measurements and tests; 0 is the fast setting) */
enum {
    E2F_FLAG_TILE_LISTS_PER_HEAD = 1, /* tile kernel: build the candidate lists per (tile, head), not once per tile */
    E2F_FLAG_PROJECT_PER_CHANNEL_TILE = 2 /* projections of the tile layout by the per-channel-tile kernel */
};

typedef struct {
    int32_t L_max;      /* highest degree, 0..4 */
    int32_t C;          /* channels per degree; multiple of 16; C <= 64 or C a multiple of 64, C <= 256 */
    int32_t H;          /* heads; C % H == 0 */
    int32_t B;          /* radial basis functions, >= 1 */
    int32_t lf;         /* degree of the geometric filter R^(lf)(r_ij): 0, 1 or 2 (lf <= L_max unless 0) */
    float cutoff;       /* > 0 */
    int32_t feat_dtype; /* e2f_dtype of h and of the five projection matrices */
    int32_t attention;  /* e2f_attn_kernel */
    int32_t flags;      /* E2F_FLAG_* */
} e2f_config;

typedef struct {
    /* device; [L_max+1][C_out][C_in], feat_dtype; applied as (W h)[co] = sum_ci W[l][co][ci] h[l,m][ci]  (Eq. qk) */
    const void *WQ1, *WQ2, *WK1, *WK2, *WV;
    const float *Wb;     /* device; [H][B] radial bias weights (b(r) of Eq. attn) */
    const float *w_path; /* device; [L_max+1][L_max+1] indexed [l_in][l_out]; entries off the allowed paths are ignored */
} e2f_weights;

const char *e2f_status_string(e2f_status s);

/* Validate the configuration and build the constant tables.  *ctx is written only on E2F_OK. */
e2f_status e2f_create(const e2f_config *cfg, e2f_ctx **ctx);
void e2f_destroy(e2f_ctx *ctx);

/*
 * Cell lists (not part of the paper, which takes a padded neighbour table as given in Sec. 3.4; here the
 * neighbour sets N(i) are found on the GPU from positions).  Every segment [seg_offsets[s], seg_offsets[s+1])
 * gets its own uniform grid of edge >= cutoff over its bounding box; atoms are ordered by (segment, cell,
 * atom index).  The result is deterministic.
 *   pos          device float [N][3]
 *   seg_offsets  device int32 [S+1], non-decreasing, seg_offsets[0] = 0, seg_offsets[S] = N (not checked on the host)
 *   ws           device, at least e2f_cells_workspace_bytes(ctx, N, S) bytes, 256-byte aligned; the cell list
 *                lives there until the caller reuses the memory
 *   *cells       host handle, release with e2f_cells_destroy (this does not touch ws)
 */
size_t e2f_cells_workspace_bytes(const e2f_ctx *ctx, int32_t N, int32_t S);
e2f_status e2f_build_cells(e2f_ctx *ctx, const float *pos, const int32_t *seg_offsets, int32_t N, int32_t S, void *ws,
                           size_t ws_bytes, e2f_cells **cells, void *hip_stream);
void e2f_cells_destroy(e2f_cells *cells);

/*
 * Cell lists under periodic boundaries (for bulk simulation cells such as the periodic water runs of Sec. 4.3; the
 * paper states the operator for given pair vectors and does not define the convention, which is this library's):
 *   box   host float [S][3]: edge lengths of every segment's orthorhombic box; an entry <= 0 (or NaN) leaves that
 *         axis open, NULL means no periodic axis anywhere (the call is then e2f_build_cells).  Read before the call
 *         returns.
 * On a periodic axis of length len a coordinate x counts as w = x - len*floor(x * (1/len)), every operation rounded
 * to binary32 and one correction step into [0, len), so callers need not fold coordinates themselves.  Atom j is
 * seen from atom i at its nearest image w_j + s*len, s in {-1, 0, 1}; the neighbour predicate and the pair vector
 * r_ij of the operator use fl(w_j + s*len) - w_i per axis.  Every periodic edge must be at least three cell edges
 * (3 * 1.0001 * cutoff), so that an atom has at most one image inside the cutoff: E2F_ERR_UNSUPPORTED otherwise
 * (also for an infinite length).  The cells of a periodic axis tile the box exactly.
 * Cell lists built here are accepted by e2f_count_neighbors, e2f_list_neighbors, e2f_build_neighbor_table,
 * e2f_attn_forward and e2f_attn_forward_capped; the materialized baseline, the factorized pipeline (its node-level
 * terms assume one position per atom, Eq. e2former_final) and the table form return E2F_ERR_UNSUPPORTED for them.
 * Everything else as e2f_build_cells.
 */
e2f_status e2f_build_cells_periodic(e2f_ctx *ctx, const float *pos, const int32_t *seg_offsets, int32_t N, int32_t S,
                                    const float *box, void *ws, size_t ws_bytes, e2f_cells **cells, void *hip_stream);

/*
 * Neighbour sets as the kernels see them, for checking against a reference (test entry points).
 *   degree   device int32 [N]: |N(i)| for every atom, in the caller's atom order
 *   offsets  device int64 [N+1]: exclusive prefix sum of degree
 *   idx      device int32 [offsets[N]]: the members of N(i) (caller's atom indices), unordered within a row
 */
e2f_status e2f_count_neighbors(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, int32_t N, int32_t *degree,
                               void *hip_stream);
e2f_status e2f_list_neighbors(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, int32_t N, const int64_t *offsets,
                              int32_t *idx, void *hip_stream);
/*
 * Number of directed pairs E = sum_i |N(i)| (the edge count of the materialize-per-edge regime, App. A) together with
 * the degrees: e2f_count_neighbors, then the sum on the host.
 *   n_edges  host int64, written on E2F_OK
 *   degree   device int32 [N], required (the call has no memory of its own to count into)
 * Synchronises with the host (one device-to-host copy of the degrees).
 */
e2f_status e2f_count_edges(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, int32_t N, int64_t *n_edges,
                           int32_t *degree, void *hip_stream);

/*
 * The fused forward pass (Sec. 3.4, Algorithm 1, with pair geometry, the edge-frame rotation and the EAAS
 * re-indexing of Sec. 3.3 evaluated inside the kernel).
 *   cells        from e2f_build_cells for the same pos / seg_offsets / N / S
 *   pos          device float [N][3]
 *   h            device feat_dtype [N][(L_max+1)^2][C]
 *   out          device float [N][(L_max+1)^2][C], caller's atom order, fully overwritten
 *   ws           device, at least e2f_attn_workspace_bytes(ctx, N) bytes (a closed-form O(N) size: sorted
 *                positions, q, k, v), 256-byte aligned
 * Peak activation memory of the call is ws_bytes + sizeof(out).
 */
size_t e2f_attn_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_forward(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                            const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w, float *out,
                            void *ws, size_t ws_bytes, void *hip_stream);

/*
 * e2f_attn_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without ws / ws_bytes, same kernels,
 * same result bit for bit; the workspace is a fixed array of E2F_STATIC_SCRATCH_BYTES bytes of device memory that
 * belongs to the loaded library (every GPU the library runs on holds its own copy until the process ends).
 *   - e2f_attn_workspace_bytes(ctx, N) must not exceed E2F_STATIC_SCRATCH_BYTES (about 3 200 atoms at L_max = 4,
 *     C = 128, bf16): E2F_ERR_SCRATCH_EXCEEDED otherwise, before anything is launched.
 *   - The device that hip_stream belongs to must be the current device.  The first call on a device looks up the
 *     array's address there (hipGetSymbolAddress; no allocation): make that first call outside a graph capture.
 *   - All calls on one GPU share the one array and it keeps the last call's contents.  Nothing in it has to be
 *     cleared between calls, but two calls that overlap in time on one GPU (different streams, or graphs replayed
 *     side by side) race on it: serialise them.
 * Calls no hipMalloc / hipFree and no allocating library routine; does not synchronise.  Errors as e2f_attn_forward.
 */
#define E2F_STATIC_SCRATCH_BYTES (32u << 20)
e2f_status e2f_attn_forward_static(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                   const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w, float *out,
                                   void *hip_stream);

/*
 * Edge-centric baseline with the same result: builds the edge list and writes per-edge tensors (geometry,
 * rotation matrices, scores, attention weights, messages) to device memory, then reduces them per atom -
 * the "materialize per edge" regime the paper compares against (App. A; Table triton-role).  It allocates
 * O(E) device memory internally, synchronises with the host, and exists only to compare latency and memory.
 *   edges_out       host, optional: number of directed pairs E
 *   peak_bytes_out  host, optional: bytes of device memory the call allocated on top of ws and out
 */
e2f_status e2f_attn_forward_materialized(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                         const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                         float *out, void *ws, size_t ws_bytes, void *hip_stream, size_t *edges_out,
                                         size_t *peak_bytes_out);

/*
 * Neighbour cap (the max_neighbors setting of the paper's model table): the same operator as e2f_attn_forward with
 * N(i) restricted to the max_neighbors nearest atoms inside the cutoff (distance compared through the binary32 d^2 of
 * the cutoff predicate, ties to the lower atom index).  The thresholds are found by a radix select on the GPU inside
 * the call and kept in two more int32 [N] arrays at the end of the workspace; all three attention kernels apply them.
 * max_neighbors <= 0: E2F_ERR_INVALID_ARG.  Otherwise as e2f_attn_forward.
 */
size_t e2f_attn_capped_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_forward_capped(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                   const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                   int32_t max_neighbors, float *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Padded neighbour table, the input form of Algorithm 1 (Sec. 3.4: a padded N x K table of neighbour indices).
 * e2f_build_neighbor_table fills table[i][0 .. count[i]) (device, int32 [N][K], caller's atom numbering) with the at
 * most K nearest atoms of atom i inside the cutoff (same selection as the cap above, order within a row unspecified
 * but deterministic) and the rest of the row with -1; count (device int32 [N]) may be null.
 * e2f_attn_forward_table evaluates the operator with N(i) = the atoms listed in row i that lie inside the cutoff
 * (Sec. 3.4: neighbours within the cutoff; entries < 0, entries equal to i, entries at zero distance and entries at or
 * beyond the cutoff are skipped; entries must be atoms of the same call and a row must not name an atom twice).  The
 * pair geometry is still built from pos inside the kernel; where the tile kernel applies, the table becomes a mask on
 * the tile's candidate list and the call runs on the matrix cores like e2f_attn_forward.
 * Workspace: e2f_attn_table_workspace_bytes.  Both allocate nothing and do not synchronise.
 */
e2f_status e2f_build_neighbor_table(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, int32_t N, int32_t K,
                                    int32_t *table, int32_t *count, void *hip_stream);
size_t e2f_attn_table_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_forward_table(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                  const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                  const int32_t *table, int32_t K, float *out, void *ws, size_t ws_bytes,
                                  void *hip_stream);

/*
 * The fused call with the non-linear pair feature in the logit (App. "Role of Non-linearity", Eqs. app-nonlin-fea and
 * app-nonlin-alpha; the tp_type QKdotS_alpha of the hyper-parameter table).  The paper gives the feature only in
 * outline; this library computes, with Y^(l) the real harmonics of the unit pair vector (Racah normalisation),
 * Q = W_Q1 h_i and V = W_V h_j,
 *     a[l][c] = sum_m Q[l,m,c] Y^(l)_m,  b[l][c] = sum_m V[l,m,c] Y^(l)_m,  sigma(x) = x / (1 + e^-x),
 *     s_ij,h  = (1/sqrt(d_k)) sum_{l, c in head h} q_i[l][c] k_j[l][c] (sigma(a[l][c]) + sigma(b[l][c])) + b_h(d_ij),
 * and softmax, gate and message exactly as e2f_attn_forward.  Same arguments; open and periodic cells; lf = 0, 1, 2.
 * Workspace: e2f_attn_nonlinear_workspace_bytes (the plain-layout attention workspace plus one [N][(L_max+1)^2][C]
 * array of the feature type), O(N).  Requires C <= 256 and heads of a power-of-two number of channels, at most 64.
 * Allocates nothing, does not synchronise.  Errors: as e2f_attn_forward; E2F_ERR_UNSUPPORTED outside those limits.
 */
size_t e2f_attn_nonlinear_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_forward_nonlinear(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                      const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                      float *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The paper's factorized node-centric pipeline for lf = 1 (Eq. e2former_final with l = 1; Sec. 3.2, three-stage data
 * flow; Sec. 3.4 Algorithm 1): source terms h'_j = v_j (x) R(r_j - o) by node-level EAAS, Algorithm 1 streaming over
 * the precomputed rows [h'_j ; v_j] with scalar weights alpha_ij only, target coupling A1_i - A0_i (x) R(r_i - o).
 * o is the centre of the atom's segment.  Same arguments and result as e2f_attn_forward (up to rounding); the
 * workspace is larger (three more fp32 [N][(L_max+1)^2][C] arrays) but still O(N).  Requires lf = 1 and a
 * power-of-two number of channels per head, at most 64.  Allocates nothing, does not synchronise.
 */
size_t e2f_attn_factorized_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_forward_factorized(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                       const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                       float *out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Backward pass of e2f_attn_forward for the degree-1 filter.  The paper gives the forward pass only (Algorithm 1);
 * this is its derivative by the same rules: pair quantities are recomputed from positions, q, k, v and two per-atom
 * softmax statistics, nothing per pair is stored, every atom's sums are formed by the workgroup that owns the atom.
 * With L = sum(out * grad_out) for the neighbour sets of the forward call held fixed:
 *   out       device float [N][(L_max+1)^2][C]: the result of e2f_attn_forward for the same arguments
 *   grad_out  device float [N][(L_max+1)^2][C]: dL/d out
 *   grad_pos  device float [N][3]: dL/d pos (forces are its negative), fully overwritten
 *   grad_q    device float [N][L_max+1][C]: dL/d q, q the invariants of Eq. qk (before the 1/sqrt(d_k) scaling)
 *   grad_k    device float [N][L_max+1][C]: dL/d k likewise
 *   grad_v    device float [N][(L_max+1)^2][C]: dL/d v, v = W_V h (all three in the caller's atom order, fully
 *             overwritten)
 *   grad_h    device float [N][(L_max+1)^2][C] or NULL: dL/d h, by the chain rule from the three above through the
 *             l-wise linear maps of Eq. qk (what an earlier layer, or a force evaluation through several layers,
 *             needs); skipped when NULL.
 *   grad_Wb      device float [H][B] or NULL: dL/d Wb (radial bias weights), fully overwritten
 *   grad_w_path  device float [L_max+1][L_max+1] or NULL: dL/d w_path, fully overwritten (zero off the allowed paths);
 *             either of the two needs B <= 8 * C/H (E2F_ERR_UNSUPPORTED otherwise) and makes the call slower
 *   grad_W    device float [5][L_max+1][C][C] or NULL: dL/d WQ1, WQ2, WK1, WK2, WV in this order (out channel, in
 *             channel), fully overwritten; needs the larger workspace e2f_attn_backward_weights_workspace_bytes(ctx, N)
 *             (five more [N][(L_max+1)^2][C] float arrays of row factors and partial sums of the result)
 *   ws        device, at least e2f_attn_backward_workspace_bytes(ctx, N) bytes, 256-byte aligned
 * Cell lists from e2f_build_cells and e2f_build_cells_periodic are accepted.  E2F_ERR_UNSUPPORTED: lf != 1, or a
 * head width C/H that is not a power of two <= 64.  Where the forward pass runs on the bf16 TILE kernel the pair work of
 * this call runs in the same form on the matrix cores (with grad_Wb / grad_w_path only for B <= 8; beyond that, and for
 * every other configuration, one workgroup per atom on the vector ALUs); position gradients of a segment then sum to
 * zero to rounding of the bf16 operands, not to the last bit.  A neighbour cap has no backward form here (the capped
 * neighbour relation is not symmetric).  Allocates nothing, does not synchronise.  Otherwise as e2f_attn_forward.
 */
size_t e2f_attn_backward_workspace_bytes(const e2f_ctx *ctx, int32_t N);
size_t e2f_attn_backward_weights_workspace_bytes(const e2f_ctx *ctx, int32_t N);
e2f_status e2f_attn_backward(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                             const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w, const float *out,
                             const float *grad_out, float *grad_pos, float *grad_q, float *grad_k, float *grad_v,
                             float *grad_h, float *grad_Wb, float *grad_w_path, float *grad_W, void *ws,
                             size_t ws_bytes, void *hip_stream);
/*
 * The same backward pass for a caller that has just run the forward pass and kept its workspace, as a training step
 * does (Sec. "Model invocation and force modes": energies first, forces by differentiating them): the projected q, k, v
 * and the candidate lists that e2f_attn_forward left in ws are read instead of being computed again.  Arguments and
 * results as e2f_attn_backward.  The caller guarantees that ws is the buffer (of at least this call's workspace size)
 * that the last e2f_attn_forward on this stream wrote, for the same ctx, cells, pos, h, seg_offsets and w, and that
 * nothing has written to it since; the capped and table forms of the forward pass do not qualify.  Nothing of this
 * can be checked here: with a workspace that holds anything else the gradients are wrong, not an error.  Where the
 * backward pass does not run in the tile form (see above) there is nothing to reuse and the call is e2f_attn_backward.
 */
e2f_status e2f_attn_backward_after_forward(e2f_ctx *ctx, const e2f_cells *cells, const float *pos, const void *h,
                                           const int32_t *seg_offsets, int32_t N, int32_t S, const e2f_weights *w,
                                           const float *out, const float *grad_out, float *grad_pos, float *grad_q,
                                           float *grad_k, float *grad_v, float *grad_h, float *grad_Wb,
                                           float *grad_w_path, float *grad_W, void *ws, size_t ws_bytes,
                                           void *hip_stream);

/*
 * Stand-alone EAAS tensor product (Sec. 3.3, Prop. EAAS; the operation of the paper's tensor-product timing table):
 * out[t] = h[t] (x) R^(lf)(r[t]) for t = 0..T-1, channel-wise with path weights, evaluated as rotate into the frame
 * of r[t], re-index with P, rotate back.  Uses L_max, C, lf and feat_dtype of the context.
 *   h       device feat_dtype [T][(L_max+1)^2][C]
 *   r       device float [T][3]; r[t] = 0 gives out[t] = 0 when lf > 0
 *   w_path  device float [L_max+1][L_max+1] indexed [l_in][l_out]
 *   out     device float [T][(L_max+1)^2][C], fully overwritten
 * Allocates nothing, does not synchronise.
 */
e2f_status e2f_eaas_tensor_product(e2f_ctx *ctx, const void *h, const float *r, const float *w_path, float *out,
                                   int32_t T, void *hip_stream);

/*
 * Per-stage timing of e2f_attn_forward for benchmarks (measurement aid; callers that do not ask for it pay
 * nothing).  e2f_profile_begin creates HIP events for up to max_calls calls; while profiling is on, every
 * e2f_attn_forward records events between its stages on the stream it is given (no synchronisation).
 * e2f_profile_end waits for the recorded events, writes the mean duration in milliseconds of each stage
 * (E2F_STAGE_*) over the recorded calls into stage_ms (host float[E2F_N_STAGES]), the number of calls into
 * *calls (host), destroys the events and switches profiling off.
 */
enum { E2F_STAGE_PREPARE = 0, E2F_STAGE_PROJECT = 1, E2F_STAGE_ATTENTION = 2, E2F_N_STAGES = 3 };
e2f_status e2f_profile_begin(e2f_ctx *ctx, int32_t max_calls);
/* Per-call stage durations of the calls recorded so far: call_ms host float [capacity][E2F_N_STAGES] (milliseconds),
 * *calls = rows written.  Waits for those calls' events; profiling stays on.  e2f_attn_forward_materialized records
 * too: stage 0 its node-level kernels, stage 1 the host synchronisation and allocation in between, stage 2 its edge
 * kernels. */
e2f_status e2f_profile_read(e2f_ctx *ctx, float *call_ms, int32_t capacity, int32_t *calls);
e2f_status e2f_profile_end(e2f_ctx *ctx, float *stage_ms, int32_t *calls);

#ifdef __cplusplus
}
#endif
#endif /* E2F_H */
