// Tile form of the fused on-the-fly attention for a degree-1 filter (Sec. 3.4, Algorithm 1, with the linear
// factorization of the filter, Eq. e2former_final at l = 1): the message is linear in the pair vector,
//     v_j (x) R^(1)(r_ij) = sum_mu (r_ij)_mu  G_mu v_j ,        G_mu = (.) (x) R^(1)(e_mu),  mu = x, y, z,
// so   out_i = (1/z_i) sum_mu G_mu T_i,mu   with   T_i,mu = sum_j e^{s_ij - m_i} phi(d_ij) (r_ij)_mu v_j .
// Both dense pieces run on the matrix cores over tiles of 16 target atoms x 32 candidate atoms:
//     S^T = K Q^T          (logits; q and k in binary16, 11-bit significands)
//     T_mu += W_mu V       (aggregation; W_mu[i][j] = e^{s_ij - m_i} phi(d_ij) (r_ij)_mu in bf16, zero off the
//                           neighbour set, V the value rows of the 32 candidates)
// Candidates are groups of four consecutive sorted slots taken from the 27-cell stencil of the tile; the pair
// geometry (distance, cutoff predicate, radial bias, gate) is evaluated per (target, candidate) in registers, the
// softmax is online with a lazily moved reference m_i, and the three axis operators G_mu (built by the EAAS route,
// D^T P D for the three axis frames, path weights included) are applied once per target in the epilogue, using
// only their non-zero entries.  Nothing per pair is written to global memory.
//
// A workgroup of four waves owns (tile, head); each wave scores a quarter of the candidate chunks and accumulates a
// quarter of the components (see k_tile below).  Register layout notes (v_mfma_f32_16x16x32_bf16, lane = 16 g + i):
//   A operand: lane holds A[i][8g..8g+7]; B operand: lane holds B[8g..8g+7][i]; result: lane holds C[4g..4g+3][i].
// The logits come out as S^T[candidate row 4g+r][target i] for two 16-candidate halves; read as the A operand of the
// aggregation the same registers are W[target i][k = 8g + r'] with k -> (first half, row 4g+r') for r' < 4 and
// (second half, row 4g+r'-4) otherwise, and the V operand is loaded in that same order of k.
#include "e2f_tile_shared.h"

namespace {

struct TileParams {
    E2fCellsView cv;
    const float4* spos;
    const uint16_t *q16, *k16, *v4;
    const float* G;
    const float* WbT;
    const uint32_t* cap_d2;   // neighbour cap thresholds per sorted slot, or null
    const int32_t* cap_idx;
    float* out;
    // candidate lists built once per tile for all heads, or null: header (entries or -1 = build the list in the
    // kernel; pass of every target, 4 bits each), entries, positions of the entries' four slots (images included)
    int4* lists_hdr;
    int* lists_ent;
    float4* lists_pos;
    unsigned long long* lists_mask;   // per list entry: which (target, slot) pairs count, bit 4 * target + slot
    // the caller's padded neighbour table [N][table_K] (atom numbers, < 0 = empty), or null: then N(i) is every atom
    // within the cutoff; with a table it is the listed atoms among those
    const int32_t* table;
    int table_K;
    int hpw;           // heads per workgroup of k_tile_heads
    int lists_only;    // the list kernel leaves crowded tiles to the caller instead of running their heads itself
    const float* cw;   // the list kernel's first workgroup forms the axis operators instead: G_out from cw
    float* G_out;
    int C, H, B, n_tiles, blk;   // blk: tiles per XCD chunk (tile_blk)
    float rc2, cutoff, rbf_step, rbf_gamma;
};

// The three axis operators, column by column: G[mu][x_out][x_in] = (e_{x_in} (x) R^(1)(e_mu))[x_out]; with `packed`
// also as the list of their pattern's entries, behind the full form.
template <int L>
__device__ __forceinline__ void axis_ops(const float* __restrict__ cw, float* __restrict__ G, int tid, bool packed) {
    constexpr int n = (L + 1) * (L + 1), DS = e2f::d_offset(L + 1);
    if (tid >= 3 * n) return;
    const int mu = tid / n, xi = tid % n;
    float D[DS];
    e2f::align_D<L>(mu == 0 ? 1.0f : 0.0f, mu == 1 ? 1.0f : 0.0f, mu == 2 ? 1.0f : 0.0f, 1.0f, D);
    float v[n][1], acc[n][1];
#pragma unroll
    for (int x = 0; x < n; ++x) {
        v[x][0] = x == xi ? 1.0f : 0.0f;
        acc[x][0] = 0.0f;
    }
    e2f::eaas_accumulate<L, 1, 1>(v, D, cw, 1.0f, acc);
#pragma unroll
    for (int xo = 0; xo < n; ++xo) {
        G[(mu * E2F_MAX_N + xo) * E2F_MAX_N + xi] = acc[xo][0];
        if (packed && ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u)) G[AXIS_PACKED_AT + AXIS_INDEX.v[mu][xo][xi]] = acc[xo][0];
    }
}
template <int L>
__global__ void k_axis_ops(const float* __restrict__ cw, float* __restrict__ G, bool packed) {
    axis_ops<L>(cw, G, threadIdx.x, packed);
}

// One workgroup of NW waves per (tile of 16 targets, head).  The waves share the candidate list and the softmax
// weights through LDS and split the rest:
//   list      each wave scans a quarter of the stencil's slot groups and keeps those with a slot within reach of a
//             target; the kept groups are packed in order
//   weights   chunks of 32 candidates are taken four at a time; wave w computes the logits (matrix cores), the pair
//             geometry and the weights W_mu of chunk 4G + w and publishes them (3 KB per chunk)
//   aggregate every wave applies all four chunks' W_mu to its own quarter of the components, T_mu += W_mu V
// The softmax reference of a target is common to the four waves: it is set by the target's first neighbours and
// moved (with a rescale of the accumulator rows) only when a later logit exceeds it by M_STEP.
// PBC: whether segments can have periodic axes (the candidate runs then include the images across the faces).
// MODE 0: lists built here, per (tile, head).  MODE 1: one workgroup per tile only builds the tile's list and writes it
// out (no head, no streaming): the passes' lists one after the other, every entry tagged with its pass, so that a
// candidate counts only for the targets of the pass that found it (k_tile_heads reads those lists; tiles whose list
// does not fit LCAP entries are finished by the list kernel's own workgroup, head by head, in MODE 0).
// CAP: whether a neighbour cap is in force (threshold keys per target).
template <int L, int NW, bool PBC, int MODE, bool CAP, int NB>
__device__ __forceinline__ void tile_item(const TileParams& P, const int tile, const int head) {
    constexpr int n = (L + 1) * (L + 1), NX = (n + NW - 1) / NW;
    constexpr int PADE = 8 * NW;        // the list is padded to whole groups of NW chunks
    constexpr int LU = 64 / NW / 4;     // steps of 16 slot groups per wave and batch (256 groups per batch)
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    // LDS: the list and the weights while streaming; the same bytes hold the partial outputs at the end
    constexpr int LIST_BYTES = (CAPG + PADE) * 4 + (CAPG + PADE) * 4 * 16, W_BYTES = NW * 3 * 64 * 16;
    constexpr int PO_BYTES = n * 64 * 16;   // one mu of the accumulators of all waves
    constexpr int MAIN_BYTES = LIST_BYTES + W_BYTES > PO_BYTES ? LIST_BYTES + W_BYTES : PO_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[MAIN_BYTES];
    __shared__ __attribute__((aligned(16))) uint16_t s_q[16 * DKP];
    __shared__ float s_G[AXIS_NNZ];   // the non-zero entries of the axis operators, read by the epilogue
    __shared__ float s_cmax[NW][16];
    __shared__ float s_z[NW][16];
    __shared__ int s_cnt[NW];
    // which (target, slot) pairs of a list entry count, bit 4 * target + slot: the valid slots for every target of the
    // entry's pass, or, with a neighbour table, the listed atoms
    __shared__ unsigned long long s_mask[CAPG + PADE];
    __shared__ float4 s_tgt[16];   // the pass's targets: position and squared reach (0: not in this pass)
    // periodic boundaries: the pass's candidate runs (first and last slot, slot groups before the run, translation)
    constexpr int NRUN = PBC ? 27 : 9;
    __shared__ int s_rlo[32], s_rhi[32], s_rpre[32];
    __shared__ float4 s_rsh[PBC ? 32 : 1];
    int* s_ent = reinterpret_cast<int*>(s_raw);
    float4* s_pos = reinterpret_cast<float4*>(s_raw + (CAPG + PADE) * 4);
    u32x4* s_W = reinterpret_cast<u32x4*>(s_raw + LIST_BYTES);   // [chunk of the group][mu][lane]
    f32x4* s_po = reinterpret_cast<f32x4*>(s_raw);

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, tn = lane & 15, g = lane >> 4;
    // components [x0, x0 + nxw) belong to this wave: n / NW each, the first n % NW waves one more (NX is the largest).
    // Accumulator slot 0 holds the wave's single component (odd nxw), slots 1 + 2p and 2 + 2p its p-th pair.
    static_assert(NW == 4, "the value rows are laid out for four waves (e2f::v4_offset)");
    constexpr int NP = NX / 2, NS = 1 + 2 * NP;
    constexpr bool HAS_ODD = (NX & 1) || (n % NW != 0 && ((NX - 1) & 1));
    const int nxw = n / NW + (wave < n % NW ? 1 : 0);
    const int x0 = wave * (n / NW) + min(wave, n % NW);
    static_assert((n / NW) / 2 == NP, "every wave has NP pairs of components (a wave with one component more has it unpaired)");
    constexpr int npair = NP;
    const bool single = (nxw & 1) != 0;
    const int N = P.cv.N, H = P.H;
    const int t0 = tile * 16, nt = min(16, N - t0);
    const int tslot = min(t0 + tn, N - 1);
    const float4 tp = P.spos[tslot];
    const float4 origin = make_float4(read_lane(tp.x, 0), read_lane(tp.y, 0), read_lane(tp.z, 0), 0.0f);
    const uint32_t capd = CAP ? P.cap_d2[tslot] : 0xffffffffu;
    const int capi = CAP ? P.cap_idx[tslot] : INT_MAX;
    // the target's segment, cell and grid shape in one record (no dependent read of the grid)
    const int4 ti0 = P.cv.sinfo[2 * tslot], ti1 = P.cv.sinfo[2 * tslot + 1];
    const int tseg = ti0.x, tcx = ti0.y, trow = ti0.w * ti1.y + ti0.z;   // row of cells: cz * ny + cy

    // coefficients of this head's radial bias (bias_value)
    float cb[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) cb[b] = 0.0f;
    if constexpr (MODE != 1) {
        const float mine = lane < P.B ? bias_coefficient<NB>(P.WbT[lane * H + head], lane, P.rbf_step, P.rbf_gamma) : 0.0f;
#pragma unroll
        for (int b = 0; b < NB; ++b) cb[b] = read_lane(mine, b);
    }
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * 1.44269504088896341f;
    const float c_g = -P.rbf_gamma * 1.44269504088896341f;

    // rows of the output that this lane will store (targets 4g..4g+3), fetched early
    int orow[4] = {-1, -1, -1, -1};
    if constexpr (MODE != 1) {
        for (int i = threadIdx.x; i < AXIS_NNZ; i += 64 * NW) s_G[i] = P.G[AXIS_PACKED_AT + i];
#pragma unroll
        for (int r = 0; r < 4; ++r) orow[r] = t0 + 4 * g + r < N ? P.cv.perm[t0 + 4 * g + r] : -1;
        // q of the 16 targets for this head -> LDS (3 KB); every group re-reads its B operands from there
        for (int u = threadIdx.x; u < 16 * (DKP / 8); u += 64 * NW) {
            const int tq = u / (DKP / 8), f8 = u % (DKP / 8);
            reinterpret_cast<u32x4*>(s_q)[u] =
                *reinterpret_cast<const u32x4*>(P.q16 + ((size_t)min(t0 + tq, N - 1) * H + head) * DKP + 8 * f8);
        }
    }
    // MODE 1: entries written so far, whether they still fit, the pass of every target
    int out_cnt = 0, pidx = 0;
    bool overflow = false;
    __shared__ int s_tpass[16];

    f32x4 acc[3][NS];
#pragma unroll
    for (int mu = 0; mu < 3; ++mu)
#pragma unroll
        for (int x = 0; x < NS; ++x) acc[mu][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // Reference of the softmax: M_NONE until the target has met a neighbour.  It is finite, so that a masked logit
    // (-inf) minus the reference is -inf and its weight 2^-inf = 0 without a select.
    constexpr float M_NONE = -1.0e30f;
    float m_ref = M_NONE, z = 0.0f;

    int a = 0;
    while (a < nt) {
        // ---- a pass: the targets [a, b) of the tile that share a row of cells (same segment, same y and z cell)
        const int seg_a = __builtin_amdgcn_readlane(tseg, a), row_a = __builtin_amdgcn_readlane(trow, a);
        const bool same = tseg == seg_a && trow == row_a && lane >= a && lane < nt;   // lanes 0..15 carry the targets
        const unsigned bits = (unsigned)(__ballot(same) & 0xFFFFull);
        const unsigned stop = ~bits & ((1u << nt) - 1u) & ~((1u << a) - 1u);
        const int b = stop ? __builtin_ctz(stop) : nt;
        const bool t_active = tn >= a && tn < b;
        // a one in the lowest bit of every target of this pass: times an entry's valid slots it gives the entry's mask
        const unsigned long long pass_nibbles = 0x1111111111111111ull & ((b == 16 ? ~0ull : (1ull << (4 * b)) - 1ull) & ~((1ull << (4 * a)) - 1ull));
        if (MODE == 1 && t_active && threadIdx.x < 16) s_tpass[threadIdx.x] = pidx;
        const int cxa = __builtin_amdgcn_readlane(tcx, a), cxb = __builtin_amdgcn_readlane(tcx, b - 1);
        // Runs of sorted slots that hold the pass's candidates: rows 0..8 are the stencil rows over the cells
        // [cxa - 1, cxb + 1].  With periodic boundaries there are 27: runs 9..17 are the rows' last cell seen across
        // the low x face, runs 18..26 their first cell seen across the high x face, and rows that leave the grid
        // along a periodic y or z come back in from the other side; candidates of a run are seen at their position
        // plus the run's lattice translation.  The runs are a table in LDS, one thread per run (in registers they
        // push the kernel's value rows into scratch).
        int total = 1;
        {
            __syncthreads();   // every wave has finished with the previous pass's table
            if (threadIdx.x < 16) {
                // |p - t|^2 < reach^2 as |q|^2 + q.(-2u) + (|u|^2 - reach^2) < 0 with q = p - o, u = t - o around the
                // tile's first target o (small numbers, so the expanded square keeps its accuracy); with a
                // neighbour cap a target reaches no further than its threshold distance
                const float reach2 = capd == 0xffffffffu ? P.rc2 : fminf(P.rc2, __uint_as_float(capd));
                const float ux = tp.x - read_lane(tp.x, 0), uy = tp.y - read_lane(tp.y, 0), uz = tp.z - read_lane(tp.z, 0);
                s_tgt[threadIdx.x] = make_float4(-2.0f * ux, -2.0f * uy, -2.0f * uz,
                                                 t_active ? ux * ux + uy * uy + uz * uz - reach2 * 1.001f : INFINITY);
            }
            // shape of the pass's grid from the first target's record; box lengths (periodic only) from the grid
            struct { int nx, ny, nz, base; float lx, ly, lz; } G;
            G.nx = __builtin_amdgcn_readlane(ti1.x, a);
            G.ny = __builtin_amdgcn_readlane(ti1.y, a);
            G.nz = __builtin_amdgcn_readlane(ti1.z, a);
            G.base = __builtin_amdgcn_readlane(ti1.w, a);
            G.lx = G.ly = G.lz = 0.0f;
            if (PBC) {
                const E2fSegGrid gs = P.cv.grid[seg_a];
                G.lx = gs.lx;
                G.ly = gs.ly;
                G.lz = gs.lz;
            }
            if (threadIdx.x < NRUN) {
                const int r = threadIdx.x, rr = r % 9, kind = r / 9;
                int y = row_a % G.ny + (rr % 3) - 1, zc = row_a / G.ny + (rr / 3) - 1;
                float shx = 0.0f, shy = 0.0f, shz = 0.0f;
                if (PBC && G.ly > 0.0f) {
                    if (y < 0) { y += G.ny; shy = -G.ly; }
                    else if (y >= G.ny) { y -= G.ny; shy = G.ly; }
                }
                if (PBC && G.lz > 0.0f) {
                    if (zc < 0) { zc += G.nz; shz = -G.lz; }
                    else if (zc >= G.nz) { zc -= G.nz; shz = G.lz; }
                }
                bool have = y >= 0 && y < G.ny && zc >= 0 && zc < G.nz;
                int x_first = max(cxa - 1, 0), x_last = min(cxb + 1, G.nx - 1);
                if (kind == 1) {
                    have = have && G.lx > 0.0f && cxa == 0;
                    x_first = x_last = G.nx - 1;
                    shx = -G.lx;
                } else if (kind == 2) {
                    have = have && G.lx > 0.0f && cxb == G.nx - 1;
                    x_first = x_last = 0;
                    shx = G.lx;
                }
                const int row = G.base + (zc * G.ny + y) * G.nx;
                const int rlo = have ? P.cv.cell_start[row + x_first] : 0;
                const int rhi = have ? P.cv.cell_start[row + x_last + 1] : 0;
                int inc = rhi > rlo ? ((rhi + 3) >> 2) - (rlo >> 2) : 0;   // -> inclusive scan over the 27 runs
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) {
                    const int up = __shfl_up(inc, off);
                    if (r >= off) inc += up;
                }
                s_rlo[r] = rlo;
                s_rhi[r] = rhi;
                s_rpre[r + 1] = inc;
                if (PBC) s_rsh[r] = make_float4(shx, shy, shz, 0.0f);
                if (r == 0) s_rpre[0] = 0;
                if (r < 32 - (NRUN + 1)) s_rpre[NRUN + 1 + r] = INT_MAX;   // stops of the search below
            }
            __syncthreads();
            total = s_rpre[NRUN];
        }
        // (The targets of the pass and how far each reaches are in s_tgt: a candidate group is kept if one of its
        // slots is within reach of one of them.  Tested slot against target, this keeps 40 % fewer groups than a test
        // against the targets' bounding box and costs about as much as scoring one chunk.)

        for (int fbase = 0; fbase < total; fbase += 256) {
            // ---- a batch of the candidate list: 256 slot groups, 64 per wave, kept groups packed in order into
            // entries (group << 8 | pass << 4 | valid slots) with the slots' positions beside them
            int cnt = 0;
            {
            int grp[LU];
            unsigned near4[LU], valid4[LU];
            unsigned long long leaders[LU];
            float4 pj[LU];
            {
                const int ln = lane;
                bool valid[LU];
#pragma unroll
                for (int u = 0; u < LU; ++u) {
                    const int fg = fbase + 16 * LU * wave + 16 * u + (ln >> 2);
                    int gq = -1, rlo = 0, rhi = 0;
                    float4 sh = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    {
                        int r = 0;   // the last run that starts at or before fg (empty runs start where the next does)
#pragma unroll
                        for (int step = (PBC ? 16 : 8); step >= 1; step >>= 1)   // reaches entry 31 or 15
                            if (s_rpre[r + step] <= fg) r += step;
                        if (fg < total) {
                            rlo = s_rlo[r];
                            rhi = s_rhi[r];
                            gq = (rlo >> 2) + fg - s_rpre[r];
                            if (PBC) sh = s_rsh[r];
                        }
                    }
                    const int slot = 4 * gq + (ln & 3);
                    grp[u] = gq;
                    valid[u] = gq >= 0 && slot >= rlo && slot < rhi;
                    pj[u] = P.spos[valid[u] ? slot : tslot];
                    if (PBC) {   // the image this run sees (the translation is exact; the sum rounds to binary32)
                        pj[u].x += sh.x;
                        pj[u].y += sh.y;
                        pj[u].z += sh.z;
                    }
                }
                bool nearby[LU];
                float qx[LU], qy[LU], qz[LU], qq[LU];
#pragma unroll
                for (int u = 0; u < LU; ++u) {
                    nearby[u] = false;
                    qx[u] = pj[u].x - origin.x;
                    qy[u] = pj[u].y - origin.y;
                    qz[u] = pj[u].z - origin.z;
                    qq[u] = qx[u] * qx[u] + qy[u] * qy[u] + qz[u] * qz[u];
                }
#pragma unroll
                for (int tt = 0; tt < 16; ++tt) {
                    const float4 tg = s_tgt[tt];
#pragma unroll
                    for (int u = 0; u < LU; ++u)
                        nearby[u] |= qx[u] * tg.x + (qy[u] * tg.y + (qz[u] * tg.z + (qq[u] + tg.w))) < 0.0f;
                }
                int mine = 0;
#pragma unroll
                for (int u = 0; u < LU; ++u) {
                    const bool near = valid[u] && nearby[u];
                    const int sh = lane & ~3;
                    near4[u] = (unsigned)(__ballot(near) >> sh) & 0xFu;
                    valid4[u] = (unsigned)(__ballot(valid[u]) >> sh) & 0xFu;
                    leaders[u] = __ballot(near4[u] != 0u && (lane & 3) == 0);
                    mine += __popcll(leaders[u]);
                }
                if (lane == 0) s_cnt[wave] = mine;
            }
            __syncthreads();   // every wave has finished with the previous list
            int e0 = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const int cw_ = s_cnt[w];
                e0 += w < wave ? cw_ : 0;
                cnt += cw_;
            }
#pragma unroll
            for (int u = 0; u < LU; ++u) {
                const int sh = lane & ~3;
                const int e = e0 + __popcll(leaders[u] & ((1ull << sh) - 1ull));
                if (near4[u] != 0u) {
                    if ((lane & 3) == 0) {
                        s_ent[e] = (int)(((unsigned)grp[u] << 8) | ((MODE == 1 ? (unsigned)pidx : 0u) << 4) | valid4[u]);
                        s_mask[e] = P.table ? 0ull : (unsigned long long)valid4[u] * pass_nibbles;
                    }
                    s_pos[e * 4 + (lane & 3)] = pj[u];
                }
                e0 += __popcll(leaders[u]);
            }
            }
            if (P.table) {
                // ---- neighbour table: the listed atoms of the pass's targets, looked up in the batch (an atom outside
                // the cutoff has no entry there and is skipped, like an empty table entry or the target itself)
                __syncthreads();
                const int K = P.table_K;
                for (int x = threadIdx.x; x < (b - a) * K; x += 64 * NW) {
                    const int i = a + x / K;
                    const int ai = P.cv.perm[t0 + i];
                    const int nb = P.table[(size_t)ai * K + x % K];
                    if (nb >= 0 && nb < N && nb != ai) {
                        const int sj = P.cv.atom_slot[nb];
                        for (int e = 0; e < cnt; ++e)   // (a group on the border of two runs has an entry in each)
                            if ((int)((unsigned)s_ent[e] >> 8) == (sj >> 2) && ((s_ent[e] >> (sj & 3)) & 1)) {
                                atomicOr(&s_mask[e], 1ull << (4 * i + (sj & 3)));
                                break;
                            }
                    }
                }
            }
            if constexpr (MODE == 1) {
                // ---- the list kernel: append the batch to the tile's list in memory
                __syncthreads();
                if (out_cnt + cnt > LCAP) overflow = true;
                if (!overflow) {
                    int* ge = P.lists_ent + (size_t)tile * LCAP + out_cnt;
                    float4* gp = P.lists_pos + ((size_t)tile * LCAP + out_cnt) * 4;
                    for (int i = threadIdx.x; i < cnt; i += 64 * NW) ge[i] = s_ent[i];
                    for (int i = threadIdx.x; i < 4 * cnt; i += 64 * NW) gp[i] = s_pos[i];
                    for (int i = threadIdx.x; i < cnt; i += 64 * NW) P.lists_mask[(size_t)tile * LCAP + out_cnt + i] = s_mask[i];
                    out_cnt += cnt;
                }
                continue;
            }
            // pad to whole groups of four chunks: entries of group 0 with no valid slot, finite positions
            for (int i = threadIdx.x; i < PADE; i += 64 * NW) {
                s_ent[cnt + i] = 0;
                s_mask[cnt + i] = 0ull;
            }
            for (int i = threadIdx.x; i < PADE * 4; i += 64 * NW) s_pos[cnt * 4 + i] = tp;
            __syncthreads();
            const int nch = (cnt + 7) >> 3, ngr = (nch + NW - 1) / NW;
            if (ngr > 0) {
                auto load_K = [&](int c, f16x8 (&kf)[2][KS]) {
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
                        const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, DKP, 8 * g);
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) kf[mt][ks] = *reinterpret_cast<const f16x8*>(P.k16 + off + 128 * ks);
                    }
                };
                // v rows of this wave's components for the lane's two entries (k = 8g..8g+3 from entry g of the chunk,
                // 8g+4..8g+7 from entry 4+g): the wave's single component, then its pairs (see e2f::v4_offset)
                VRows<NP> vr;
                auto v_base = [&](int c, const uint16_t*& ba, const uint16_t*& bb) {
                    const unsigned ea = (unsigned)s_ent[8 * c + g] >> 8, eb = (unsigned)s_ent[8 * c + 4 + g] >> 8;
                    ba = P.v4 + (((size_t)ea * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
                    bb = P.v4 + (((size_t)eb * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
                };
                f16x8 kf[2][KS];
                load_K(min(wave, nch - 1), kf);
                {
                    const uint16_t *ba, *bb;
                    v_base(0, ba, bb);
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        if (p < npair) vr.load_pair(p, ba, bb);
                    if (HAS_ODD && single) vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);
                }
                for (int G = 0; G < ngr; ++G) {
                    // ---- logits, pair geometry and cutoff mask of this wave's chunk
                    const int cm = NW * G + wave;
                    f32x4 S[2];
                    {
                        f16x8 qf[KS];
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const f16x8*>(s_q + tn * DKP + 32 * ks + 8 * g);
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt) {
                            S[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int ks = 0; ks < KS; ++ks) S[mt] = mfma(kf[mt][ks], qf[ks], S[mt]);
                        }
                    }
                    load_K(min(cm + NW, nch - 1), kf);   // k rows of this wave's chunk in the next group
                    float s2[8], gate[8];
                    float cmax = -INFINITY;
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        const int ei = 8 * cm + 4 * mt + g;
                        const unsigned mine4 = (unsigned)(s_mask[ei] >> (4 * tn));   // this target's four slots of the entry
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int u = 4 * mt + r;
                            const float4 pc = s_pos[ei * 4 + r];
                            const float d2 = e2f::dist2_exact(tp.x, tp.y, tp.z, pc.x, pc.y, pc.z);
                            // (bitwise on purpose: the eight candidates are evaluated side by side; the target itself
                            // is at distance zero, an image of it at a box length: neither passes)
                            const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f) &
                                            (!CAP || e2f::under_cap(d2, pc.w, capd, capi));
                            const float d = __builtin_amdgcn_sqrtf(d2);
                            float bias = bias_value<NB>(cb, d, d2, c_u, c_g, P.rbf_step);
                            // (evaluated for every candidate, not under its predicate: otherwise each of the eight
                            // candidates becomes a basic block of its own and their LDS reads are issued one by one)
                            asm("" : "+v"(bias));
                            s2[u] = ok ? S[mt][r] + bias : -INFINITY;
                            gate[u] = e2f::radial_gate(d, P.cutoff);
                            cmax = fmaxf(cmax, s2[u]);
                        }
                    }
                    cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
                    cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
                    if (lane < 16) s_cmax[wave][lane] = cmax;
                    __syncthreads();
                    // ---- the group's largest logit per target, the same in all four waves
                    float gmax = s_cmax[0][tn];
#pragma unroll
                    for (int w = 1; w < NW; ++w) gmax = fmaxf(gmax, s_cmax[w][tn]);
                    if (m_ref == M_NONE) m_ref = fmaxf(gmax, M_NONE);   // first neighbours: the accumulator rows are still zero
                    const bool move = gmax > m_ref + M_STEP;
                    if (__builtin_expect(__ballot(move) != 0ull, 0)) {
                        const float f = move ? __builtin_amdgcn_exp2f(m_ref - gmax) : 1.0f;
                        m_ref = move ? gmax : m_ref;
                        z *= f;
                        // Rows of the accumulators are targets: T <- diag(f) T on the matrix cores in fp32.  Slice r
                        // pairs A_r[i][g] = f_i [i == 4g + r] with B_r[g][j] = T[4g + r][j], register r of lane (j, g).
                        float ar[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) ar[r] = tn == 4 * g + r ? f : 0.0f;
#pragma unroll
                        for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                            for (int x = 0; x < NS; ++x) {
                                f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    d = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[r], acc[mu][x][r], d, 0, 0, 0);
                                acc[mu][x] = d;
                            }
                    }
                    // ---- weights of this wave's chunk -> LDS
                    {
                        uint32_t wp[3][4];
#pragma unroll
                        for (int u = 0; u < 8; u += 2) {
                            float pg[2], rx[2], ry[2], rz[2];
#pragma unroll
                            for (int d = 0; d < 2; ++d) {
                                const float p = __builtin_amdgcn_exp2f(s2[u + d] - m_ref);
                                z += p;
                                pg[d] = p * gate[u + d];
                                const float4 pc = s_pos[(8 * cm + 4 * ((u + d) >> 2) + g) * 4 + ((u + d) & 3)];
                                rx[d] = pc.x - tp.x;
                                ry[d] = pc.y - tp.y;
                                rz[d] = pc.z - tp.z;
                            }
                            wp[0][u >> 1] = pack_bf16(pg[0] * rx[0], pg[1] * rx[1]);
                            wp[1][u >> 1] = pack_bf16(pg[0] * ry[0], pg[1] * ry[1]);
                            wp[2][u >> 1] = pack_bf16(pg[0] * rz[0], pg[1] * rz[1]);
                        }
#pragma unroll
                        for (int mu = 0; mu < 3; ++mu)
                            s_W[(wave * 3 + mu) * 64 + lane] = (u32x4){wp[mu][0], wp[mu][1], wp[mu][2], wp[mu][3]};
                    }
                    __syncthreads();
                    // ---- aggregate the chunks of the group into this wave's components
#pragma unroll
                    for (int cc = 0; cc < NW; ++cc) {
                        const int c = NW * G + cc;
                        if (c < nch) {
                            bf16x8 W[3];
#pragma unroll
                            for (int mu = 0; mu < 3; ++mu) W[mu] = __builtin_bit_cast(bf16x8, s_W[(cc * 3 + mu) * 64 + lane]);
                            const uint16_t *ba, *bb;   // the next chunk's rows replace each operand once it has been used
                            v_base(min(c + 1, nch - 1), ba, bb);
#pragma unroll
                            for (int p = 0; p < NP; ++p)
                                if (p < npair) {   // (wave-uniform)
                                    const bf16x8 b0 = vr.first(p), b1 = vr.second(p);
#pragma unroll
                                    for (int mu = 0; mu < 3; ++mu) acc[mu][1 + 2 * p] = mfma(W[mu], b0, acc[mu][1 + 2 * p]);
#pragma unroll
                                    for (int mu = 0; mu < 3; ++mu) acc[mu][2 + 2 * p] = mfma(W[mu], b1, acc[mu][2 + 2 * p]);
                                    vr.load_pair(p, ba, bb);
                                }
                            if (HAS_ODD && single) {   // (wave-uniform) the odd component last: see k_tile_heads
                                const bf16x8 bv = vr.single();
#pragma unroll
                                for (int mu = 0; mu < 3; ++mu) acc[mu][0] = mfma(W[mu], bv, acc[mu][0]);
                                vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);
                            }
                        }
                    }
                }
            }
        }
        a = b;
        ++pidx;
    }
    if constexpr (MODE == 1) {
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned lo = 0u, hi = 0u;
            for (int i = 0; i < 8; ++i) {
                lo |= (i < nt ? (unsigned)s_tpass[i] : 0u) << (4 * i);
                hi |= (8 + i < nt ? (unsigned)s_tpass[8 + i] : 0u) << (4 * i);
            }
            P.lists_hdr[tile] = make_int4(overflow ? -1 : out_cnt, (int)lo, (int)hi, 0);
        }
        if (overflow && !P.lists_only) {
            // (uniform) A crowded tile: its list does not fit the shared area, k_tile_heads will skip it.  This
            // workgroup runs the tile's heads itself, one after the other, building the lists per head.  The axis
            // operators of this launch may not be there yet (another workgroup forms them), so it forms its own
            // copy in the tile's list area, which stays unused.
            float* own_G = reinterpret_cast<float*>(P.lists_pos + (size_t)tile * LCAP * 4);
            static_assert((size_t)LCAP * 4 * sizeof(float4) >= (AXIS_PACKED_AT + AXIS_NNZ) * sizeof(float), "room for the operators");
            axis_ops<L>(P.cw, own_G, threadIdx.x, true);
            __threadfence_block();
            __syncthreads();
            TileParams Q = P;
            Q.G = own_G;
            for (int h = 0; h < P.H; ++h) {
                tile_item<L, NW, PBC, 0, CAP, NB>(Q, tile, h);
                __syncthreads();   // the next head reuses the shared arrays
            }
        }
        return;
    }

    // ---- epilogue: out = (1/z) sum_mu G_mu T_mu.  For one mu at a time the waves put their T_mu components into
    // LDS (the list and the weights are dead by then) and every wave forms the output components x_out = wave
    // (mod NW) from the non-zero entries of G_mu.  The code exists once per wave index, so that the components a
    // wave owns and the sparsity pattern are compile-time facts and each step is straight-line code.
    z += __shfl_xor(z, 16);
    z += __shfl_xor(z, 32);
    if (lane < 16) s_z[wave][lane] = z;
    auto finish = [&](auto wv_tag) {
        constexpr int WV = decltype(wv_tag)::value;
        constexpr int RO = (n - WV + NW - 1) / NW;                      // components WV, WV + NW, ...
        constexpr int X0 = WV * (n / NW) + (WV < n % NW ? WV : n % NW);  // this wave's accumulator components
        constexpr int NXW = n / NW + (WV < n % NW ? 1 : 0);
        f32x4 pr[RO];
#pragma unroll
        for (int i = 0; i < RO; ++i) pr[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mu = 0; mu < 3; ++mu) {
            __syncthreads();
#pragma unroll
            for (int x = 0; x < NXW; ++x) s_po[(X0 + x) * 64 + lane] = acc[mu][x + ((NXW & 1) ? 0 : 1)];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < RO; ++i) {
#pragma unroll
                for (int xi = 0; xi < n; ++xi)
                    if ((E2F_AXIS_NZ[mu][WV + NW * i] >> xi) & 1u)
                        pr[i] += s_G[AXIS_INDEX.v[mu][WV + NW * i][xi]] * s_po[xi * 64 + lane];
            }
        }
        f32x4 inv;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int tt = 4 * g + r;
            float zt = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) zt += s_z[w][tt];
            inv[r] = zt > 0.0f ? 1.0f / zt : 0.0f;
        }
        // rows of the output: one base pointer per target row, components C floats apart
        float* orp[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) orp[r] = P.out + (size_t)max(orow[r], 0) * n * P.C + head * 16 + tn;
        const size_t cstride = (size_t)P.C;
        if (nt == 16) {   // (uniform) every row exists: no per-row test
#pragma unroll
            for (int i = 0; i < RO; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) orp[r][(WV + NW * i) * cstride] = pr[i][r] * inv[r];
        } else {
#pragma unroll
            for (int i = 0; i < RO; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (orow[r] >= 0) orp[r][(WV + NW * i) * cstride] = pr[i][r] * inv[r];
        }
    };
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    if (wave_u == 0) finish(std::integral_constant<int, 0>{});
    if (wave_u == 1) finish(std::integral_constant<int, 1>{});
    if constexpr (NW > 2) {
        if (wave_u == 2) finish(std::integral_constant<int, 2>{});
        if (wave_u == 3) finish(std::integral_constant<int, 3>{});
    }
    if constexpr (NW > 4) {
        if (wave_u == 4) finish(std::integral_constant<int, 4>{});
        if (wave_u == 5) finish(std::integral_constant<int, 5>{});
        if (wave_u == 6) finish(std::integral_constant<int, 6>{});
        if (wave_u == 7) finish(std::integral_constant<int, 7>{});
    }
}

// The attention kernel for tiles whose candidate list the list kernel has left in memory (all but the rare crowded
// ones).  A workgroup of four waves owns one tile of 16 targets and `hpw` consecutive heads, which it runs one after
// the other: what belongs to the tile (the targets, their output rows, the candidate list with its slot positions,
// the axis operators) is fetched once, all of it requested before any of it is used, and stays in LDS for every head;
// what belongs to a head (its queries, its radial weights, the key and value rows of the first chunks) is requested
// while the head before it is in its epilogue.  The streaming loop and the epilogue are those of tile_item.
template <int L, bool CAP, int NB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_tile_heads(TileParams P) {
    constexpr int NW = 4, n = (L + 1) * (L + 1), NX = (n + NW - 1) / NW;
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    constexpr int LENT = LCAP + 8 * NW;   // the list, padded to whole groups of four chunks
    constexpr int W_BYTES = NW * 3 * 64 * 16, PO_BYTES = n * 64 * 16;
    __shared__ int s_ent[LENT];
    __shared__ unsigned long long s_mask[LENT];
    __shared__ float4 s_pos[LENT * 4];
    __shared__ __attribute__((aligned(16))) uint16_t s_q[16 * DKP];
    __shared__ float s_G[AXIS_NNZ];
    __shared__ float s_cmax[NW][16];
    __shared__ float s_z[NW][16];
    __shared__ int s_orow[16];
    // the weights while streaming; the same bytes hold one mu of all waves' accumulators in the epilogue
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[W_BYTES > PO_BYTES ? W_BYTES : PO_BYTES];
    u32x4* s_W = reinterpret_cast<u32x4*>(s_raw);
    f32x4* s_po = reinterpret_cast<f32x4*>(s_raw);
    static_assert(LCAP * 4 == 3 * 256 && LCAP <= 256 && 16 * (DKP / 8) <= 256 && AXIS_NNZ <= 256, "one request per thread");

    const int HG = P.H / P.hpw;
    int tile, hg;
    if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, HG, tile, hg)) return;   // whole workgroup
    const int head0 = hg * P.hpw;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tn = lane & 15, g = lane >> 4;
    // (components, accumulator slots and value rows of a wave as in tile_item)
    constexpr int NP = NX / 2, NS = 1 + 2 * NP;
    constexpr bool HAS_ODD = (NX & 1) || (n % NW != 0 && ((NX - 1) & 1));
    const int nxw = n / NW + (wave < n % NW ? 1 : 0);
    const int x0 = wave * (n / NW) + min(wave, n % NW);
    static_assert((n / NW) / 2 == NP, "every wave has NP pairs of components (a wave with one component more has it unpaired)");
    constexpr int npair = NP;
    const bool single = (nxw & 1) != 0;
    const int N = P.cv.N, H = P.H;
    const int t0 = tile * 16, nt = min(16, N - t0);
    const int tslot = min(t0 + tn, N - 1);

    // ---- everything the tile needs, requested together
    const int4 hd = P.lists_hdr[tile];
    const float4 tp = P.spos[tslot];
    const uint32_t capd = CAP ? P.cap_d2[tslot] : 0xffffffffu;
    const int capi = CAP ? P.cap_idx[tslot] : INT_MAX;
    const int orow_mine = tid < 16 ? (t0 + tid < N ? P.cv.perm[t0 + tid] : -1) : 0;   // output rows of the targets
    const float g_mine = tid < AXIS_NNZ ? P.G[AXIS_PACKED_AT + tid] : 0.0f;
    const int ent_mine = tid < LCAP ? P.lists_ent[(size_t)tile * LCAP + tid] : 0;
    const unsigned long long mask_mine = tid < LCAP ? P.lists_mask[(size_t)tile * LCAP + tid] : 0ull;
    float4 pos_mine[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) pos_mine[j] = P.lists_pos[(size_t)tile * LCAP * 4 + tid + 256 * j];
    // queries (16 targets x DKP binary16 of one head: one 16-byte piece per thread) and radial weights of a head
    auto fetch_q = [&](int head) -> u32x4 {
        const int tq = tid / (DKP / 8), f8 = tid % (DKP / 8);
        return tid < 16 * (DKP / 8)
                   ? *reinterpret_cast<const u32x4*>(P.q16 + ((size_t)min(t0 + tq, N - 1) * H + head) * DKP + 8 * f8)
                   : (u32x4){0u, 0u, 0u, 0u};
    };
    auto fetch_wb = [&](int head) -> float { return lane < P.B ? P.WbT[lane * H + head] : 0.0f; };
    u32x4 q_mine = fetch_q(head0);
    float wb_mine = fetch_wb(head0);

    const int cnt = hd.x;
    if (cnt < 0) return;   // (whole workgroup) a crowded tile: the list kernel has done it, with lists per head
    // ---- into LDS; what lies behind the list reads as groups without a valid slot, at a finite position
    if (tid < LCAP) {
        s_ent[tid] = tid < cnt ? ent_mine : 0;
        s_mask[tid] = tid < cnt ? mask_mine : 0ull;
    }
    if (tid < LENT - LCAP) {
        s_ent[LCAP + tid] = 0;
        s_mask[LCAP + tid] = 0ull;
    }
#pragma unroll
    for (int j = 0; j < 3; ++j) {   // (selected by value, component by component: the compiler would otherwise choose
        // between the addresses of two register arrays and move both into scratch memory)
        const bool in_list = ((tid + 256 * j) >> 2) < cnt;
        s_pos[tid + 256 * j] = make_float4(in_list ? pos_mine[j].x : tp.x, in_list ? pos_mine[j].y : tp.y,
                                           in_list ? pos_mine[j].z : tp.z, in_list ? pos_mine[j].w : tp.w);
    }
    if (tid < (LENT - LCAP) * 4) s_pos[LCAP * 4 + tid] = tp;
    if (tid < AXIS_NNZ) s_G[tid] = g_mine;
    if (tid < 16) s_orow[tid] = orow_mine;
    if (tid < 16 * (DKP / 8)) reinterpret_cast<u32x4*>(s_q)[tid] = q_mine;
    __syncthreads();

    const int nch = (cnt + 7) >> 3, ngr = (nch + NW - 1) / NW;
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * 1.44269504088896341f;
    const float c_g = -P.rbf_gamma * 1.44269504088896341f;
    const float rbf_mine = bias_coefficient<NB>(1.0f, lane, P.rbf_step, P.rbf_gamma);

    f16x8 kf[2][KS];
    VRows<NP> vr;
    auto load_K = [&](int c, int head) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
            const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, DKP, 8 * g);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[mt][ks] = *reinterpret_cast<const f16x8*>(P.k16 + off + 128 * ks);
        }
    };
    // v rows of this wave's components for the lane's two entries (k = 8g..8g+3 from entry g of the chunk, 8g+4..8g+7
    // from entry 4+g): the wave's single component, then its pairs (see e2f::v4_offset)
    auto v_base = [&](int c, int head, const uint16_t*& ba, const uint16_t*& bb) {
        const unsigned ea = (unsigned)s_ent[8 * c + g] >> 8, eb = (unsigned)s_ent[8 * c + 4 + g] >> 8;
        ba = P.v4 + (((size_t)ea * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
        bb = P.v4 + (((size_t)eb * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
    };
    auto first_rows = [&](int head) {   // the rows the streaming loop starts with
        if (nch > 0) {
            load_K(min(wave, nch - 1), head);
            const uint16_t *ba, *bb;
            v_base(0, head, ba, bb);
#pragma unroll
            for (int p = 0; p < NP; ++p)
                if (p < npair) vr.load_pair(p, ba, bb);
            if (HAS_ODD && single) vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);   // (in the order of their use)
        }
    };
    first_rows(head0);

    for (int hh = 0; hh < P.hpw; ++hh) {
        const int head = head0 + hh;
        // coefficients of this head's radial bias (bias_value)
        float cb[NB];
        {
            const float mine = wb_mine * rbf_mine;
#pragma unroll
            for (int b = 0; b < NB; ++b) cb[b] = read_lane(mine, b);
        }
        f32x4 acc[3][NS];
#pragma unroll
        for (int mu = 0; mu < 3; ++mu)
#pragma unroll
            for (int x = 0; x < NS; ++x) acc[mu][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
        constexpr float M_NONE = -1.0e30f;   // finite, so that a masked logit (-inf) gets the weight 2^-inf = 0
        float m_ref = M_NONE, z = 0.0f;

        for (int G = 0; G < ngr; ++G) {
            // ---- logits, pair geometry and cutoff mask of this wave's chunk
            const int cm = NW * G + wave;
            f32x4 S[2];
            {
                f16x8 qf[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const f16x8*>(s_q + tn * DKP + 32 * ks + 8 * g);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    S[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) S[mt] = mfma(kf[mt][ks], qf[ks], S[mt]);
                }
            }
            load_K(min(cm + NW, nch - 1), head);   // k rows of this wave's chunk in the next group
            float s2[8], gate[8];
            float cmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int ei = 8 * cm + 4 * mt + g;
                const unsigned mine4 = (unsigned)(s_mask[ei] >> (4 * tn));   // this target's four slots of the entry
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int u = 4 * mt + r;
                    const float4 pc = s_pos[ei * 4 + r];
                    const float d2 = e2f::dist2_exact(tp.x, tp.y, tp.z, pc.x, pc.y, pc.z);
                    // (bitwise on purpose: the eight candidates are evaluated side by side; the target itself is at
                    // distance zero, an image of it at a box length: neither passes)
                    const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f) &
                                    (!CAP || e2f::under_cap(d2, pc.w, capd, capi));
                    const float d = __builtin_amdgcn_sqrtf(d2);
                    float bias = bias_value<NB>(cb, d, d2, c_u, c_g, P.rbf_step);
                    // (evaluated for every candidate, not under its predicate: otherwise each of the eight
                    // candidates becomes a basic block of its own and their LDS reads are issued one by one)
                    asm("" : "+v"(bias));
                    s2[u] = ok ? S[mt][r] + bias : -INFINITY;
                    gate[u] = e2f::radial_gate(d, P.cutoff);
                    cmax = fmaxf(cmax, s2[u]);
                }
            }
            cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
            if (lane < 16) s_cmax[wave][lane] = cmax;
            __syncthreads();
            // ---- the group's largest logit per target, the same in all four waves
            float gmax = s_cmax[0][tn];
#pragma unroll
            for (int w = 1; w < NW; ++w) gmax = fmaxf(gmax, s_cmax[w][tn]);
            if (m_ref == M_NONE) m_ref = fmaxf(gmax, M_NONE);   // first neighbours: the accumulator rows are still zero
            const bool move = gmax > m_ref + M_STEP;
            if (__builtin_expect(__ballot(move) != 0ull, 0)) {
                const float f = move ? __builtin_amdgcn_exp2f(m_ref - gmax) : 1.0f;
                m_ref = move ? gmax : m_ref;
                z *= f;
                // Rows of the accumulators are targets: T <- diag(f) T on the matrix cores in fp32.  Slice r pairs
                // A_r[i][g] = f_i [i == 4g + r] with B_r[g][j] = T[4g + r][j], register r of lane (j, g).
                float ar[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) ar[r] = tn == 4 * g + r ? f : 0.0f;
#pragma unroll
                for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                    for (int x = 0; x < NS; ++x) {
                        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int r = 0; r < 4; ++r) d = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[r], acc[mu][x][r], d, 0, 0, 0);
                        acc[mu][x] = d;
                    }
            }
            // ---- weights of this wave's chunk -> LDS
            {
                uint32_t wp[3][4];
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    float pg[2], rx[2], ry[2], rz[2];
#pragma unroll
                    for (int d = 0; d < 2; ++d) {
                        const float p = __builtin_amdgcn_exp2f(s2[u + d] - m_ref);
                        z += p;
                        pg[d] = p * gate[u + d];
                        const float4 pc = s_pos[(8 * cm + 4 * ((u + d) >> 2) + g) * 4 + ((u + d) & 3)];
                        rx[d] = pc.x - tp.x;
                        ry[d] = pc.y - tp.y;
                        rz[d] = pc.z - tp.z;
                    }
                    wp[0][u >> 1] = pack_bf16(pg[0] * rx[0], pg[1] * rx[1]);
                    wp[1][u >> 1] = pack_bf16(pg[0] * ry[0], pg[1] * ry[1]);
                    wp[2][u >> 1] = pack_bf16(pg[0] * rz[0], pg[1] * rz[1]);
                }
#pragma unroll
                for (int mu = 0; mu < 3; ++mu)
                    s_W[(wave * 3 + mu) * 64 + lane] = (u32x4){wp[mu][0], wp[mu][1], wp[mu][2], wp[mu][3]};
            }
            __syncthreads();
            // ---- aggregate the chunks of the group into this wave's components
#pragma unroll
            for (int cc = 0; cc < NW; ++cc) {
                const int c = NW * G + cc;
                if (c < nch) {
                    bf16x8 W[3];
#pragma unroll
                    for (int mu = 0; mu < 3; ++mu) W[mu] = __builtin_bit_cast(bf16x8, s_W[(cc * 3 + mu) * 64 + lane]);
                    const uint16_t *ba, *bb;   // the next chunk's rows replace each operand once it has been used
                    v_base(min(c + 1, nch - 1), head, ba, bb);
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        if (p < npair) {   // (wave-uniform)
                            const bf16x8 b0 = vr.first(p), b1 = vr.second(p);
#pragma unroll
                            for (int mu = 0; mu < 3; ++mu) acc[mu][1 + 2 * p] = mfma(W[mu], b0, acc[mu][1 + 2 * p]);
#pragma unroll
                            for (int mu = 0; mu < 3; ++mu) acc[mu][2 + 2 * p] = mfma(W[mu], b1, acc[mu][2 + 2 * p]);
                            vr.load_pair(p, ba, bb);
                        }
                    // The wave with an odd component takes it last.  The waits on the pairs' rows are the same
                    // instructions for all waves, counted for the waves without the extra rows; with those rows
                    // requested first, the wave that has them waited at every chunk for rows it had just asked for.
                    if (HAS_ODD && single) {   // (wave-uniform)
                        const bf16x8 bv = vr.single();
#pragma unroll
                        for (int mu = 0; mu < 3; ++mu) acc[mu][0] = mfma(W[mu], bv, acc[mu][0]);
                        vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);
                    }
                }
            }
        }

        // ---- the next head's queries, radial weights and first rows are on their way during this head's epilogue
        const bool more = hh + 1 < P.hpw;
        if (more) {
            q_mine = fetch_q(head + 1);
            wb_mine = fetch_wb(head + 1);
            first_rows(head + 1);
        }
        // ---- epilogue: out = (1/z) sum_mu G_mu T_mu.  For one mu at a time the waves put their T_mu components into
        // LDS and every wave forms the output components x_out = wave (mod NW) from the non-zero entries of G_mu.  The
        // code exists once per wave index, so that a wave's components and the pattern are compile-time facts.
        z += __shfl_xor(z, 16);
        z += __shfl_xor(z, 32);
        if (lane < 16) s_z[wave][lane] = z;
        auto finish = [&](auto wv_tag) {
            constexpr int WV = decltype(wv_tag)::value;
            constexpr int RO = (n - WV + NW - 1) / NW;                      // components WV, WV + NW, ...
            constexpr int X0 = WV * (n / NW) + (WV < n % NW ? WV : n % NW);  // this wave's accumulator components
            constexpr int NXW = n / NW + (WV < n % NW ? 1 : 0);
            f32x4 pr[RO];
#pragma unroll
            for (int i = 0; i < RO; ++i) pr[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mu = 0; mu < 3; ++mu) {
                __syncthreads();
#pragma unroll
                for (int x = 0; x < NXW; ++x) s_po[(X0 + x) * 64 + lane] = acc[mu][x + ((NXW & 1) ? 0 : 1)];
                __syncthreads();
#pragma unroll
                for (int i = 0; i < RO; ++i) {
#pragma unroll
                    for (int xi = 0; xi < n; ++xi)
                        if ((E2F_AXIS_NZ[mu][WV + NW * i] >> xi) & 1u)
                            pr[i] += s_G[AXIS_INDEX.v[mu][WV + NW * i][xi]] * s_po[xi * 64 + lane];
                }
            }
            f32x4 inv;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int tt = 4 * g + r;
                float zt = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) zt += s_z[w][tt];
                inv[r] = zt > 0.0f ? 1.0f / zt : 0.0f;
            }
            // rows of the output: one base pointer per target row, components C floats apart
            int orow[4];
            float* orp[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                orow[r] = s_orow[4 * g + r];
                orp[r] = P.out + (size_t)max(orow[r], 0) * n * P.C + head * 16 + tn;
            }
            const size_t cstride = (size_t)P.C;
            if (nt == 16) {   // (uniform) every row exists: no per-row test
#pragma unroll
                for (int i = 0; i < RO; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r) orp[r][(WV + NW * i) * cstride] = pr[i][r] * inv[r];
            } else {
#pragma unroll
                for (int i = 0; i < RO; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (orow[r] >= 0) orp[r][(WV + NW * i) * cstride] = pr[i][r] * inv[r];
            }
        };
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        if (wave_u == 0) finish(std::integral_constant<int, 0>{});
        if (wave_u == 1) finish(std::integral_constant<int, 1>{});
        if (wave_u == 2) finish(std::integral_constant<int, 2>{});
        if (wave_u == 3) finish(std::integral_constant<int, 3>{});
        if (more) {
            // (every wave has left the streaming loop: the epilogue's barriers lie in between)
            if (tid < 16 * (DKP / 8)) reinterpret_cast<u32x4*>(s_q)[tid] = q_mine;
            __syncthreads();   // the new queries are in place; the partial outputs have been read
        }
    }
}

template <int L, int NW, bool PBC, int MODE, bool CAP, int NB>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(E2F_TILE_OCC(NW), E2F_TILE_OCC(NW)))) void k_tile(TileParams P) {
    int tile, head;
    if constexpr (MODE == 1) {
        if (blockIdx.x == 0) {   // (whole workgroup) the first workgroup forms the axis operators instead
            axis_ops<L>(P.cw, P.G_out, threadIdx.x, true);
            return;
        }
        tile = blockIdx.x - 1;
        head = 0;
    } else {
        if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, P.H, tile, head)) return;   // whole workgroup
    }
    tile_item<L, NW, PBC, MODE, CAP, NB>(P, tile, head);
}

// what: 1 the list kernel (with the axis operators), 2 the attention kernel reading the lists, 0 the attention kernel
// building its lists itself (after the axis-operator kernel)
template <int L>
void launch_L(const TileParams& P, const float* cw, float* G, int what, hipStream_t st) {
    const int grid = tile_grid(P.n_tiles, P.blk, P.H);
    // four waves per workgroup, two workgroups per CU: with eight waves the 128 registers left per wave do not
    // hold a wave's accumulators, value rows and key rows without spilling into the streaming loop
    const bool cap = P.cap_d2 != nullptr;
    // the radial bias is a polynomial of degree B - 1 with its coefficients in registers: instances for B <= 8 and B <= 16
    auto go = [&](auto pbc, auto capped) {
        constexpr bool PBC = decltype(pbc)::value, CAP = decltype(capped)::value;
        if (P.B > 8) {
            if (what == 1) k_tile<L, 4, PBC, 1, CAP, 16><<<P.n_tiles + 1, 256, 0, st>>>(P);
            else if (what == 2) k_tile_heads<L, CAP, 16><<<tile_grid(P.n_tiles, P.blk, P.H / P.hpw), 256, 0, st>>>(P);
            else {
                k_axis_ops<L><<<1, 128, 0, st>>>(cw, G, true);
                k_tile<L, 4, PBC, 0, CAP, 16><<<grid, 256, 0, st>>>(P);
            }
            return;
        }
        if (what == 1) {
            k_tile<L, 4, PBC, 1, CAP, 8><<<P.n_tiles + 1, 256, 0, st>>>(P);
        } else if (what == 2) {
            k_tile_heads<L, CAP, 8><<<tile_grid(P.n_tiles, P.blk, P.H / P.hpw), 256, 0, st>>>(P);
        } else {
            k_axis_ops<L><<<1, 128, 0, st>>>(cw, G, true);
            k_tile<L, 4, PBC, 0, CAP, 8><<<grid, 256, 0, st>>>(P);
        }
    };
    if (P.cv.periodic) cap ? go(std::true_type{}, std::true_type{}) : go(std::true_type{}, std::false_type{});
    else cap ? go(std::false_type{}, std::true_type{}) : go(std::false_type{}, std::false_type{});
}

}  // namespace

// packed: also the list of the pattern's entries behind the full form (G then holds 3 * 25 * 25 + 216 floats)
e2f_status e2f_launch_axis_ops(const e2f_ctx* ctx, const float* cw, float* G, hipStream_t st, bool packed) {
    switch (ctx->cfg.L_max) {
        case 1: k_axis_ops<1><<<1, 128, 0, st>>>(cw, G, packed); break;
        case 2: k_axis_ops<2><<<1, 128, 0, st>>>(cw, G, packed); break;
        case 3: k_axis_ops<3><<<1, 128, 0, st>>>(cw, G, packed); break;
        case 4: k_axis_ops<4><<<1, 128, 0, st>>>(cw, G, packed); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

bool e2f_tile_supported(const e2f_ctx* ctx) {
    const int C = ctx->cfg.C;
    return ctx->cfg.feat_dtype == E2F_BF16 && ctx->cfg.lf == 1 && ctx->Ch == 16 && ctx->cfg.L_max >= 1 &&
           ctx->cfg.B <= 16 && (C == 32 || C == 64 || C == 128 || C == 256);   // (a projection exists)
}

static e2f_status launch_tile(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const int32_t* table,
                              int table_K, float* out, int what, hipStream_t st, bool lists_only = false) {
    if (cv.N == 0) return E2F_OK;
    if (cv.N >= (1 << 26)) return E2F_ERR_UNSUPPORTED;   // a list entry keeps the slot group in 24 bits
    TileParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q16 = ws.q16; P.k16 = ws.k16; P.v4 = ws.v4; P.G = ws.G; P.WbT = ws.wbT;
    P.cap_d2 = ws.cap_d2; P.cap_idx = ws.cap_idx;
    P.out = out;
    P.lists_hdr = what == 0 ? nullptr : ws.lists_hdr;
    P.lists_ent = ws.lists_ent;
    P.lists_pos = ws.lists_pos;
    P.lists_mask = ws.lists_mask;
    P.table = table;
    P.table_K = table_K;
    P.cw = ws.cw;
    P.G_out = ws.G;
    P.lists_only = lists_only ? 1 : 0;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.n_tiles = (cv.N + 15) / 16; P.blk = tile_blk(P.n_tiles);
    // heads per workgroup of the attention kernel: up to four, as long as about eight rounds of workgroups are left
    // for the chip (measured: two and four heads are 2 % ahead of one at 100 000 atoms; at 20 000 atoms two heads are
    // 2 % ahead of four, at 10 000 one head is even with two or 1 % ahead)
    P.hpw = 1;
    while (P.hpw < 4 && P.H % (P.hpw * 2) == 0 && (long)P.n_tiles * P.H / (P.hpw * 2) >= 4096) P.hpw *= 2;
    P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    switch (ctx->cfg.L_max) {
        case 1: launch_L<1>(P, ws.cw, ws.G, what, st); break;
        case 2: launch_L<2>(P, ws.cw, ws.G, what, st); break;
        case 3: launch_L<3>(P, ws.cw, ws.G, what, st); break;
        case 4: launch_L<4>(P, ws.cw, ws.G, what, st); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

// With E2F_FLAG_TILE_LISTS_PER_HEAD in the configuration the attention kernel builds its lists per (tile, head)
// instead of reading the ones the list kernel leaves per tile (for A/B timing and tests).
e2f_status e2f_launch_tile(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const int32_t* table,
                           int table_K, float* out, hipStream_t st) {
    if (!ws.lists_hdr || (ctx->cfg.flags & E2F_FLAG_TILE_LISTS_PER_HEAD)) return launch_tile(ctx, cv, ws, table, table_K, out, 0, st);
    const e2f_status rc = launch_tile(ctx, cv, ws, table, table_K, out, 1, st);
    if (rc != E2F_OK) return rc;
    return launch_tile(ctx, cv, ws, table, table_K, out, 2, st);
}

e2f_status e2f_launch_tile_lists(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, hipStream_t st) {
    return launch_tile(ctx, cv, ws, nullptr, 0, nullptr, 1, st, true);
}
