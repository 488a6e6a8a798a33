// Fused on-the-fly attention with the non-linear pair feature in the logit (App. "Role of Non-linearity",
// Eqs. app-nonlin-fea and app-nonlin-alpha).  The reading built here: with Y^(l) the real harmonics of the unit pair
// vector, Q = W_Q1 h_i (the target's first query projection, all components) and V = W_V h_j,
//     a[l][c] = sum_m Q[l,m,c] Y^(l)_m ,   b[l][c] = sum_m V[l,m,c] Y^(l)_m          (invariants, degree by degree)
//     Fea     = sigma(a || b),  sigma(x) = x / (1 + e^-x)
//     s_ij,h  = tau sum_{l, c in h} q_i[l][c] k_j[l][c] (sigma(a[l][c]) + sigma(b[l][c])) + b_h(d_ij)
// and everything after the logit as in Algorithm 1 (softmax over the neighbours, gate outside, EAAS message).
//
// One workgroup per target atom, one thread per channel (one or more waves; every wave walks the stencil and reads the
// pair geometry that the first lanes of each wave build, identically), like the ALU form of the fused call.  The
// harmonics of the pair direction cost nothing extra: R_ij takes the pair direction to +z, so Y^(l)(r/|r|) is the
// m = 0 row of the block D^(l)(R_ij) that the message needs anyway.  The value row of a neighbour is read once and
// serves the feature and the message; the softmax is online per pair (Algorithm 1 as printed).
#include <limits.h>
#include <stdlib.h>

#include "e2f_device.h"

namespace {

struct NlParams {
    E2fCellsView cv;
    const float4* spos;
    const float* q;
    const float* k;
    const void* v;
    const void* q1;   // [N][n][C] sorted order, same type as v: W_Q1 h
    const float* cw;
    const float* Wb;
    float* out;
    int C, H, B, Ch;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

constexpr int PB = 16;    // pairs per chunk
constexpr int CAP = 192;  // capacity of the neighbour list in LDS

__device__ __forceinline__ float silu(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

template <int L, int LF, typename VT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_fused_nonlinear(NlParams P) {
    constexpr int CPL = 1;
    constexpr int n = (L + 1) * (L + 1);
    constexpr int DS = e2f::d_offset(L + 1);
    constexpr int DSP = (DS + 3) & ~3;
    __shared__ int s_list[CAP];
    __shared__ __attribute__((aligned(16))) float s_D[PB * DSP];
    __shared__ float s_bias[PB * E2F_MAX_H];
    __shared__ float s_wgt[PB];

    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N), lane = threadIdx.x & 63;
    if (t < 0) return;  // padding block of the XCD map (whole workgroup)
    const int C = P.C, H = P.H;
    const bool active = (int)threadIdx.x < C;
    const int c0 = active ? threadIdx.x : 0;  // idle lanes shadow channel 0's loads and store nothing
    const int head = c0 / P.Ch;
    const int lanes_per_head = P.Ch;
    const float4 pi = P.spos[t];

    float q[L + 1][CPL];
#pragma unroll
    for (int l = 0; l <= L; ++l)
#pragma unroll
        for (int u = 0; u < CPL; ++u) q[l][u] = P.q[((size_t)t * (L + 1) + l) * C + c0 + u];
    // the target's query components: in LDS (component-major), not in registers, where they would sit beside the
    // accumulators, the value row and its rotated copy
    extern __shared__ float s_q1[];   // [n][threads]
    const int nthreads = blockDim.x;
#pragma unroll
    for (int x = 0; x < n; ++x)
        s_q1[x * nthreads + threadIdx.x] = e2f::load_as_float((const VT*)P.q1 + ((size_t)t * n + x) * C + c0);

    float A[n][CPL];
#pragma unroll
    for (int x = 0; x < n; ++x)
#pragma unroll
        for (int u = 0; u < CPL; ++u) A[x][u] = 0.0f;
    float mu = -INFINITY, z = 0.0f;

    e2f::Stencil<true> st;   // (serves open boundaries too: the extra runs are empty, the translations zero)
    st.init(P.cv, t);
    constexpr int RUN_SHIFT = 26;   // a list entry is slot | run << 26; the launcher checks N < 2^26

    int row = 0, base = st.lo[0];
    bool rows_done = false;
    while (true) {
        // ---- fill the list
        int cnt = 0;
        while (!rows_done && cnt + 64 <= CAP) {
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
                ok = e2f::is_neighbor(d2, P.rc2);
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
                e2f::align_D<L>(dx, dy, dz, d, s_D + lane * DSP);   // also for LF = 0: the feature needs Y
                for (int hh = 0; hh < H; ++hh) {
                    float acc = 0.0f;
                    for (int b = 0; b < P.B; ++b) acc += P.Wb[hh * P.B + b] * e2f::radial_basis(d, b, P.rbf_step, P.rbf_gamma);
                    s_bias[lane * E2F_MAX_H + hh] = acc;
                }
                s_wgt[lane] = e2f::radial_gate(d, P.cutoff) * e2f::pow_lf<LF>(d);
            }
            __syncthreads();
#pragma unroll 1
            for (int p = 0; p < np; ++p) {
                const int j = s_list[p0 + p] & ((1 << RUN_SHIFT) - 1);
                const VT* vj = (const VT*)P.v + (size_t)j * n * C + c0;
                const float* kj = P.k + (size_t)j * (L + 1) * C + c0;
                const float* Dp = s_D + p * DSP;
                float vin[n][CPL];
#pragma unroll
                for (int x = 0; x < n; ++x)
#pragma unroll
                    for (int u = 0; u < CPL; ++u) vin[x][u] = e2f::load_as_float(vj + x * C + u);
                // logit with the pair feature: Y^(l)_m = D^(l)[m = 0][m]
                float dot = 0.0f;
#pragma unroll
                for (int l = 0; l <= L; ++l) {
                    float a[CPL], b[CPL];
#pragma unroll
                    for (int u = 0; u < CPL; ++u) a[u] = b[u] = 0.0f;
#pragma unroll
                    for (int m = 0; m < 2 * l + 1; ++m) {
                        const float y = Dp[e2f::d_offset(l) + l * (2 * l + 1) + m];
#pragma unroll
                        for (int u = 0; u < CPL; ++u) {
                            a[u] += s_q1[(l * l + m) * nthreads + threadIdx.x] * y;
                            b[u] += vin[l * l + m][u] * y;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < CPL; ++u) dot += q[l][u] * kj[l * C + u] * (silu(a[u]) + silu(b[u]));
                }
                for (int off = 1; off < lanes_per_head; off <<= 1) dot += __shfl_xor(dot, off);
                const float s = dot * P.tau + s_bias[p * E2F_MAX_H + head];
                // the recurrences of Algorithm 1
                const float mu_new = fmaxf(mu, s);
                const float scale = __expf(mu - mu_new);   // 0 for the first neighbour (mu = -inf)
                const float pe = __expf(s - mu_new);
                z = z * scale + pe;
#pragma unroll
                for (int x = 0; x < n; ++x)
#pragma unroll
                    for (int u = 0; u < CPL; ++u) A[x][u] *= scale;
                mu = mu_new;
                e2f::eaas_accumulate<L, LF, CPL>(vin, Dp, P.cw, pe * s_wgt[p], A);
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

template <int L, int LF>
bool launch_dtype(const e2f_ctx* ctx, const NlParams& P, hipStream_t st) {
    const int grid = e2f::xcd_grid(P.cv.N), threads = (P.C + 63) / 64 * 64;
    const size_t shm = (size_t)(L + 1) * (L + 1) * threads * sizeof(float);
    if (ctx->cfg.feat_dtype == E2F_BF16)
        k_fused_nonlinear<L, LF, uint16_t><<<grid, threads, shm, st>>>(P);
    else
        k_fused_nonlinear<L, LF, float><<<grid, threads, shm, st>>>(P);
    return true;
}

template <int L>
bool launch_lf(const e2f_ctx* ctx, const NlParams& P, hipStream_t st) {
    switch (ctx->cfg.lf) {
        case 0: return launch_dtype<L, 0>(ctx, P, st);
        case 1: return launch_dtype<L, 1>(ctx, P, st);
        case 2: return launch_dtype<L, 2>(ctx, P, st);
    }
    return false;
}

}  // namespace

// A head's channels sit in one wave (the logit is reduced by a butterfly over them); at most four waves per target.
bool e2f_nonlinear_supported(const e2f_ctx* ctx) {
    const int Ch = ctx->Ch;
    return ctx->cfg.C <= 256 && Ch <= 64 && (Ch & (Ch - 1)) == 0;
}

e2f_status e2f_launch_fused_nonlinear(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w,
                                      const E2fAttnWs& ws, const void* q1, float* out, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (cv.N >= (1 << 26)) return E2F_ERR_UNSUPPORTED;   // list entries carry the run in their top bits
    NlParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = ws.v; P.q1 = q1; P.cw = ws.cw; P.Wb = w->Wb; P.out = out;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.Ch = ctx->Ch;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    bool ok = false;
    switch (ctx->cfg.L_max) {
        case 0: ok = launch_lf<0>(ctx, P, st); break;
        case 1: ok = launch_lf<1>(ctx, P, st); break;
        case 2: ok = launch_lf<2>(ctx, P, st); break;
        case 3: ok = launch_lf<3>(ctx, P, st); break;
        case 4: ok = launch_lf<4>(ctx, P, st); break;
    }
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
