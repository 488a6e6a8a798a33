// Fused on-the-fly equivariant attention (Sec. 3.4, Algorithm 1) with the pair geometry, the edge-frame
// rotation and the EAAS re-indexing (Sec. 3.3) evaluated inside the kernel.
//
// k_fused_valu: one wave per target atom, lanes over channels (CPL channels per lane).  The wave walks the
// target's 27-cell stencil 64 candidates at a time, keeps the slots that pass the cutoff predicate in an LDS
// list, and consumes the list in chunks of PB pairs:
//   lanes 0..PB-1   build one pair each: D(R_ij) blocks, radial bias per head, gate * |r|^lf   -> LDS
//   all lanes       logits of the chunk (q.k reduced over the lanes of a head), chunk maximum, one rescale
//                   of the running (mu, z, A) per chunk, then per pair: A += e^{s-mu} phi D^T P D v_j
// Nothing per pair is written to global memory; out_i = A/z is stored once, in the caller's atom order.
#include <limits.h>
#include <stdlib.h>

#include "e2f_device.h"

namespace {

struct FusedParams {
    E2fCellsView cv;
    const float4* spos;
    const float* q;
    const float* k;
    const void* v;
    const float* cw;
    const float* Wb;
    const uint32_t* cap_d2;   // neighbour cap thresholds per sorted slot, or null
    const int32_t* cap_idx;
    const int32_t* table;     // TABLE kernels: padded neighbour table [N][K] in the caller's atom order, -1 = empty
    int K;
    const int4* only_crowded; // or null; else the headers of the tile kernels' lists: only atoms of tiles with x < 0 are done
    float* out;
    int C, H, B, Ch;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

constexpr int PB = 16;    // pairs per chunk
constexpr int CAP = 192;  // capacity of the neighbour list in LDS

// TABLE: the neighbours come from the caller's padded table (the input form of Algorithm 1) instead of the cell walk;
// the pair geometry is still built from the positions.
template <int L, int LF, int CPL, typename VT, bool TABLE>
__global__ __launch_bounds__(64) void k_fused_valu(FusedParams P) {
    constexpr int n = (L + 1) * (L + 1);
    constexpr int DS = e2f::d_offset(L + 1);
    constexpr int DSP = (DS + 3) & ~3;
    __shared__ int s_list[CAP];
    __shared__ __attribute__((aligned(16))) float s_D[PB * DSP];
    __shared__ float s_bias[PB * E2F_MAX_H];
    __shared__ float s_wgt[PB];

    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N), lane = threadIdx.x;
    if (t < 0) return;  // padding block of the XCD map (whole wave)
    if (P.only_crowded && P.only_crowded[t >> 4].x >= 0) return;   // (whole wave) a tile kernel owns this atom
    const int C = P.C, H = P.H;
    const int nlanes = C / CPL;
    const bool active = lane < nlanes;
    const int c0 = active ? lane * CPL : 0;  // idle lanes shadow lane 0's loads and store nothing
    const int head = c0 / P.Ch;
    const int lanes_per_head = P.Ch / CPL;
    const float4 pi = P.spos[t];
    const uint32_t capd = P.cap_d2 ? P.cap_d2[t] : 0xffffffffu;
    const int capi = P.cap_idx ? P.cap_idx[t] : INT_MAX;

    float q[L + 1][CPL];
#pragma unroll
    for (int l = 0; l <= L; ++l)
#pragma unroll
        for (int u = 0; u < CPL; ++u) q[l][u] = P.q[((size_t)t * (L + 1) + l) * C + c0 + u];

    float A[n][CPL];
#pragma unroll
    for (int x = 0; x < n; ++x)
#pragma unroll
        for (int u = 0; u < CPL; ++u) A[x][u] = 0.0f;
    float mu = -INFINITY, z = 0.0f;

    // (the 18-run form also serves open boundaries: its extra runs are empty and every translation is zero)
    e2f::Stencil<true> st;
    st.init(P.cv, t);
    constexpr int RUN_SHIFT = 26;   // a list entry is slot | run << 26; the launcher checks N < 2^26

    int row = 0, base = st.lo[0];
    bool rows_done = false;
    const int32_t* trow = TABLE ? P.table + (size_t)P.cv.perm[t] * P.K : nullptr;
    int tb = 0;
    while (true) {
        // ---- fill the list
        int cnt = 0;
        while (TABLE && !rows_done && cnt + 64 <= CAP) {
            if (tb >= P.K) { rows_done = true; break; }
            const int aj = tb + lane < P.K ? trow[tb + lane] : -1;
            const int j = aj >= 0 ? P.cv.atom_slot[aj] : -1;
            bool ok = false;
            if (j >= 0 && j != t) {
                const float4 pj = P.spos[j];
                ok = e2f::is_neighbor(e2f::dist2_exact(pi.x, pi.y, pi.z, pj.x, pj.y, pj.z), P.rc2);
            }
            const unsigned long long mask = __ballot(ok);
            if (ok) s_list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = j;
            cnt += __popcll(mask);
            tb += 64;
        }
        while (!TABLE && !rows_done && cnt + 64 <= CAP) {
            if (base >= st.hi[row]) {
                ++row;
                if (row == 18) { rows_done = true; break; }
                base = st.lo[row];
                continue;
            }
            const int j = base + lane;
            bool ok = false;
            if (j < st.hi[row] && j != t) {
                const float4 pj = P.spos[j];
                const float d2 = e2f::dist2_exact(pi.x, pi.y, pi.z, pj.x + st.shift_x(row), pj.y + st.shift_y(row),
                                                  pj.z + st.shift_z(row));
                ok = e2f::is_neighbor(d2, P.rc2) && e2f::under_cap(d2, pj.w, capd, capi);
            }
            const unsigned long long mask = __ballot(ok);
            if (ok) s_list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = j | (row << RUN_SHIFT);
            cnt += __popcll(mask);
            base += 64;
        }
        __syncthreads();
        // ---- consume it
        for (int p0 = 0; p0 < cnt; p0 += PB) {
            const int np = min(PB, cnt - p0);
            if (lane < np) {
                const int e = s_list[p0 + lane], j = e & ((1 << RUN_SHIFT) - 1), run = e >> RUN_SHIFT;
                const float4 pj = P.spos[j];
                const float dx = (pj.x + st.shift_x(run)) - pi.x, dy = (pj.y + st.shift_y(run)) - pi.y;
                const float dz = (pj.z + st.shift_z(run)) - pi.z;
                const float d = sqrtf(dx * dx + dy * dy + dz * dz);
                if constexpr (LF != 0) e2f::align_D<L>(dx, dy, dz, d, s_D + lane * DSP);
                for (int hh = 0; hh < H; ++hh) {
                    float acc = 0.0f;
                    for (int b = 0; b < P.B; ++b) acc += P.Wb[hh * P.B + b] * e2f::radial_basis(d, b, P.rbf_step, P.rbf_gamma);
                    s_bias[lane * E2F_MAX_H + hh] = acc;
                }
                s_wgt[lane] = e2f::radial_gate(d, P.cutoff) * e2f::pow_lf<LF>(d);
            }
            __syncthreads();
            // logits of the chunk (Eq. kernel_score)
            float s_arr[PB];
            float cmax = -INFINITY;
#pragma unroll
            for (int p = 0; p < PB; ++p) {
                s_arr[p] = -INFINITY;
                if (p < np) {
                    const int j = s_list[p0 + p] & ((1 << RUN_SHIFT) - 1);
                    const float* kj = P.k + (size_t)j * (L + 1) * C + c0;
                    float dot = 0.0f;
#pragma unroll
                    for (int l = 0; l <= L; ++l)
#pragma unroll
                        for (int u = 0; u < CPL; ++u) dot += q[l][u] * kj[l * C + u];
                    for (int off = 1; off < lanes_per_head; off <<= 1) dot += __shfl_xor(dot, off);
                    s_arr[p] = dot * P.tau + s_bias[p * E2F_MAX_H + head];
                    cmax = fmaxf(cmax, s_arr[p]);
                }
            }
            // one rescale of the running state per chunk (the updates of mu, z and A in Algorithm 1, taken chunk-wise)
            const float mu_new = fmaxf(mu, cmax);
            const float scale = __expf(mu - mu_new);  // 0 on the first chunk (mu = -inf)
            z *= scale;
#pragma unroll
            for (int x = 0; x < n; ++x)
#pragma unroll
                for (int u = 0; u < CPL; ++u) A[x][u] *= scale;
            mu = mu_new;
#pragma unroll 1
            for (int p = 0; p < np; ++p) {
                // s_arr is indexed by a runtime p: select without dynamic register indexing
                float sp = s_arr[0];
#pragma unroll
                for (int x = 1; x < PB; ++x) sp = (p == x) ? s_arr[x] : sp;
                const float pe = __expf(sp - mu);
                z += pe;
                const float wgt = pe * s_wgt[p];
                const int j = s_list[p0 + p] & ((1 << RUN_SHIFT) - 1);
                const VT* vj = (const VT*)P.v + (size_t)j * n * C + c0;
                float vin[n][CPL];
#pragma unroll
                for (int x = 0; x < n; ++x)
#pragma unroll
                    for (int u = 0; u < CPL; ++u) vin[x][u] = e2f::load_as_float(vj + x * C + u);
                e2f::eaas_accumulate<L, LF, CPL>(vin, s_D + p * DSP, P.cw, wgt, A);
            }
            __syncthreads();
        }
        if (rows_done) break;
    }

    if (active) {
        const float inv = z > 0.0f ? 1.0f / z : 0.0f;
        float* o = P.out + (size_t)P.cv.perm[t] * n * C + c0;
#pragma unroll
        for (int x = 0; x < n; ++x)
#pragma unroll
            for (int u = 0; u < CPL; ++u) o[x * C + u] = A[x][u] * inv;
    }
}

template <int L, int LF, int CPL>
void launch_valu_dtype(const e2f_ctx* ctx, const FusedParams& P, hipStream_t st) {
    const int grid = e2f::xcd_grid(P.cv.N);
    if (P.table) {
        if (ctx->cfg.feat_dtype == E2F_BF16)
            k_fused_valu<L, LF, CPL, uint16_t, true><<<grid, 64, 0, st>>>(P);
        else
            k_fused_valu<L, LF, CPL, float, true><<<grid, 64, 0, st>>>(P);
    } else if (ctx->cfg.feat_dtype == E2F_BF16)
        k_fused_valu<L, LF, CPL, uint16_t, false><<<grid, 64, 0, st>>>(P);
    else
        k_fused_valu<L, LF, CPL, float, false><<<grid, 64, 0, st>>>(P);
}

template <int L, int LF>
bool launch_valu_cpl(const e2f_ctx* ctx, const FusedParams& P, hipStream_t st) {
    switch (ctx->cpl) {
        case 1: launch_valu_dtype<L, LF, 1>(ctx, P, st); return true;
        case 2: launch_valu_dtype<L, LF, 2>(ctx, P, st); return true;
        case 3: launch_valu_dtype<L, LF, 3>(ctx, P, st); return true;
        case 4: launch_valu_dtype<L, LF, 4>(ctx, P, st); return true;
    }
    return false;
}

template <int L>
bool launch_valu_lf(const e2f_ctx* ctx, const FusedParams& P, hipStream_t st) {
    switch (ctx->cfg.lf) {
        case 0: return launch_valu_cpl<L, 0>(ctx, P, st);
        case 1: return launch_valu_cpl<L, 1>(ctx, P, st);
        case 2: return launch_valu_cpl<L, 2>(ctx, P, st);
    }
    return false;
}

}  // namespace

static e2f_status launch_valu(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                              const int32_t* table, int32_t K, float* out, hipStream_t st, bool crowded_only = false) {
    if (cv.N == 0) return E2F_OK;
    if (cv.N >= (1 << 26)) return E2F_ERR_UNSUPPORTED;   // list entries carry the run in their top bits
    FusedParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = ws.v; P.cw = ws.cw; P.Wb = w->Wb; P.out = out;
    P.cap_d2 = ws.cap_d2; P.cap_idx = ws.cap_idx; P.table = table; P.K = K;
    P.only_crowded = crowded_only ? ws.lists_hdr : nullptr;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.Ch = ctx->Ch;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    bool ok = false;
    switch (ctx->cfg.L_max) {
        case 0: ok = launch_valu_lf<0>(ctx, P, st); break;
        case 1: ok = launch_valu_lf<1>(ctx, P, st); break;
        case 2: ok = launch_valu_lf<2>(ctx, P, st); break;
        case 3: ok = launch_valu_lf<3>(ctx, P, st); break;
        case 4: ok = launch_valu_lf<4>(ctx, P, st); break;
    }
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_fused(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                            float* out, hipStream_t st) {
    return launch_valu(ctx, cv, w, ws, nullptr, 0, out, st);
}

e2f_status e2f_launch_fused_crowded(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                    float* out, hipStream_t st) {
    return launch_valu(ctx, cv, w, ws, nullptr, 0, out, st, true);
}

e2f_status e2f_launch_fused_table(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                  const int32_t* table, int32_t K, float* out, hipStream_t st) {
    return launch_valu(ctx, cv, w, ws, table, K, out, st);
}
