// Backward pass of the fused attention call for the degree-1 filter (the paper states the forward pass only,
// Algorithm 1; training and conservative forces F = -dE/dpos need its derivative).  As in the forward pass nothing
// per pair is written to memory: the pair quantities are recomputed from positions, q, k, v and two per-atom
// softmax statistics, and every atom's gradients are accumulated by the workgroup that owns the atom (no atomics,
// deterministic).  The message is linear in the pair vector for this filter, m_ij = sum_mu (r_ij)_mu G_mu v_j with
// the three axis operators G_mu = D(R_mu)^T P D(R_mu) of the tile kernel, which gives, per head, with g = dL/d out:
//     u_mu   = <g_i, G_mu v_j>                     w = sum_mu r_mu u_mu = <g_i, m_ij>
//     P_ij   = exp(s_ij - lse_i)                   alpha_ij = P_ij phi(d)
//     ds_ij  = P_ij (phi w - D_i),  D_i = <g_i, out_i>         (softmax with the gate outside, Eq. attn)
//     dq_i  += tau ds_ij k_j          dk_j += tau ds_ij q_i          dv_j += alpha_ij sum_mu r_mu G_mu^T g_i
//     dL/dr_ij = sum_heads [ alpha_ij u + (ds_ij b'(d) + P_ij w phi'(d)) r/d ],   dpos_j += dL/dr_ij,  dpos_i -= dL/dr_ij
// Three kernels, one workgroup per atom with one thread per channel: the softmax statistics (lse, D), the sums an
// atom owns as a target (dq, its share of dpos), and the sums it owns as a source (dk, dv, its share of dpos).  The
// last one walks the atom's own neighbours, which are exactly the targets that see it: the relation is symmetric
// (also under periodic boundaries, with opposite images), which is why a neighbour cap is not supported here.
#include <limits.h>

#include "e2f_axis_pattern.h"
#include "e2f_device.h"

namespace {

constexpr int BCAP = 128;   // neighbours per batch of the list

struct BwdParams {
    E2fCellsView cv;
    const float4* spos;   // sorted positions (folded on periodic axes), w = atom index
    const float* q;       // [N][L+1][C] sorted order
    const float* k;
    const void* v;        // [N][n][C] sorted order, feature dtype
    const float* G;       // [3][25][25] axis operators
    const float* Wb;      // [H][B]
    const float* out;     // forward result, caller's order
    const float* gout;    // dL/d out, caller's order
    float* lse;           // [N][H] sorted order: log of the softmax normaliser, reference included
    float* Dn;            // [N][H] sorted order: <g_i, out_i> per head
    float* gpos;          // [N][3] caller's order
    float* gq;            // [N][L+1][C] caller's order
    float* gk;
    float* gv;            // [N][n][C] caller's order
    int C, H, B, Ch;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

// Sum over the Ch threads of a head (Ch a power of two <= 64, heads aligned inside a wave).
__device__ __forceinline__ float head_sum(float x, int Ch) {
    for (int off = 1; off < Ch; off <<= 1) x += __shfl_xor(x, off);
    return x;
}

// The neighbours of slot t in batches: wave 0 walks the 18 stencil runs and packs (slot, image position) of the
// atoms inside the cutoff into LDS; every thread of the workgroup then reads the batch.
struct ListWalk {
    e2f::Stencil<true> st;
    int row, base;
    bool done;
    __device__ void init(const E2fCellsView& cv, int t) {
        st.init(cv, t);
        row = 0;
        base = st.lo[0];
        done = false;
    }
};

__device__ __forceinline__ int next_batch(const BwdParams& P, ListWalk& w, int t, const float4& pi, int* s_list,
                                          float4* s_pos, int* s_ctl) {
    __syncthreads();   // the previous batch has been consumed
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        int cnt = 0;
        while (!w.done && cnt + 64 <= BCAP) {
            if (w.base >= w.st.hi[w.row]) {
                ++w.row;
                if (w.row == 18) { w.done = true; break; }
                w.base = w.st.lo[w.row];
                continue;
            }
            const int j = w.base + lane;
            bool ok = false;
            float4 pj = pi;
            if (j < w.st.hi[w.row] && j != t) {
                pj = P.spos[j];
                pj.x += w.st.shift_x(w.row);
                pj.y += w.st.shift_y(w.row);
                pj.z += w.st.shift_z(w.row);
                ok = e2f::is_neighbor(e2f::dist2_exact(pi.x, pi.y, pi.z, pj.x, pj.y, pj.z), P.rc2);
            }
            const unsigned long long mask = __ballot(ok);
            const int at = cnt + __popcll(mask & ((1ull << lane) - 1ull));
            if (ok) {
                s_list[at] = j;
                s_pos[at] = pj;
            }
            cnt += __popcll(mask);
            w.base += 64;
        }
        if (lane == 0) {
            s_ctl[0] = cnt;
            s_ctl[1] = w.done ? 1 : 0;
        }
    }
    __syncthreads();
    return s_ctl[0];
}

// Radial bias of a head and its derivative with respect to the distance.
__device__ __forceinline__ void radial_bias(const BwdParams& P, int head, float d, float& b, float& db) {
    b = 0.0f;
    db = 0.0f;
    for (int i = 0; i < P.B; ++i) {
        const float x = d - (float)i * P.rbf_step;
        const float g = P.Wb[head * P.B + i] * __expf(-P.rbf_gamma * x * x);
        b += g;
        db += -2.0f * P.rbf_gamma * x * g;
    }
}

// u_mu = sum_{xo, xi} G_mu[xo][xi] A[xo] B[xi] over the non-zero pattern of the axis operators.
template <int L>
__device__ __forceinline__ void axis_bilinear(const float (&A)[(L + 1) * (L + 1)], const float (&B)[(L + 1) * (L + 1)],
                                              const float* s_G, float (&u)[3]) {
    constexpr int n = (L + 1) * (L + 1);
#pragma unroll
    for (int mu = 0; mu < 3; ++mu) {
        float acc = 0.0f;
#pragma unroll
        for (int xo = 0; xo < n; ++xo) {
            float inner = 0.0f;
#pragma unroll
            for (int xi = 0; xi < n; ++xi)
                if ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u) inner += s_G[(mu * E2F_MAX_N + xo) * E2F_MAX_N + xi] * B[xi];
            acc += A[xo] * inner;
        }
        u[mu] = acc;
    }
}

// ---- softmax statistics: lse_i = log sum_j exp(s_ij) and D_i = <g_i, out_i>, per head
template <int L>
__global__ __launch_bounds__(256) void k_bwd_stats(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP];
    __shared__ int s_ctl[2];
    const int t = blockIdx.x, C = P.C;
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    const float4 pi = P.spos[t];
    float qv[L + 1];
#pragma unroll
    for (int l = 0; l <= L; ++l) qv[l] = P.q[((size_t)t * (L + 1) + l) * C + c];
    float dsum = 0.0f;
    for (int x = 0; x < n; ++x) dsum += P.gout[((size_t)a * n + x) * C + c] * P.out[((size_t)a * n + x) * C + c];
    dsum = head_sum(dsum, P.Ch);
    float m = -INFINITY, z = 0.0f;
    ListWalk w;
    w.init(P.cv, t);
    while (true) {
        const int cnt = next_batch(P, w, t, pi, s_list, s_pos, s_ctl);
        for (int e = 0; e < cnt; ++e) {
            const int j = s_list[e];
            const float4 pj = s_pos[e];
            const float rx = pj.x - pi.x, ry = pj.y - pi.y, rz = pj.z - pi.z;
            const float d = sqrtf(rx * rx + ry * ry + rz * rz);
            float dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) dot += qv[l] * P.k[((size_t)j * (L + 1) + l) * C + c];
            dot = head_sum(dot, P.Ch);
            float b, db;
            radial_bias(P, head, d, b, db);
            const float s = dot * P.tau + b;
            const float mn = fmaxf(m, s);
            z = z * __expf(m - mn) + __expf(s - mn);
            m = mn;
        }
        if (s_ctl[1]) break;
    }
    if (live && c % P.Ch == 0) {
        P.lse[(size_t)t * P.H + head] = z > 0.0f ? m + logf(z) : 0.0f;
        P.Dn[(size_t)t * P.H + head] = dsum;
    }
}

// ---- what an atom owns as a target i: dq_i and -sum_j dL/dr_ij
template <int L, typename VT>
__global__ __launch_bounds__(256) void k_bwd_target(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP];
    __shared__ int s_ctl[2];
    __shared__ float s_G[3 * E2F_MAX_N * E2F_MAX_N];
    __shared__ float s_gp[E2F_MAX_H][3];
    const int t = blockIdx.x, C = P.C;
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    for (int i = threadIdx.x; i < 3 * E2F_MAX_N * E2F_MAX_N; i += blockDim.x) s_G[i] = P.G[i];
    const float4 pi = P.spos[t];
    float qv[L + 1], dq[L + 1], g[n];
#pragma unroll
    for (int l = 0; l <= L; ++l) {
        qv[l] = P.q[((size_t)t * (L + 1) + l) * C + c];
        dq[l] = 0.0f;
    }
#pragma unroll
    for (int x = 0; x < n; ++x) g[x] = P.gout[((size_t)a * n + x) * C + c];
    const float lse = P.lse[(size_t)t * P.H + head], Dn = P.Dn[(size_t)t * P.H + head];
    float gx = 0.0f, gy = 0.0f, gz = 0.0f;   // sum_j dL/dr_ij of this head
    ListWalk w;
    w.init(P.cv, t);
    while (true) {
        const int cnt = next_batch(P, w, t, pi, s_list, s_pos, s_ctl);   // (the first barrier also covers s_G)
        for (int e = 0; e < cnt; ++e) {
            const int j = s_list[e];
            const float4 pj = s_pos[e];
            const float rx = pj.x - pi.x, ry = pj.y - pi.y, rz = pj.z - pi.z;
            const float d = sqrtf(rx * rx + ry * ry + rz * rz);
            float kv[L + 1], dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) {
                kv[l] = P.k[((size_t)j * (L + 1) + l) * C + c];
                dot += qv[l] * kv[l];
            }
            float vj[n];
#pragma unroll
            for (int x = 0; x < n; ++x) vj[x] = e2f::load_as_float<VT>((const VT*)P.v + ((size_t)j * n + x) * C + c);
            float u[3];
            axis_bilinear<L>(g, vj, s_G, u);
            dot = head_sum(dot, P.Ch);
            u[0] = head_sum(u[0], P.Ch);
            u[1] = head_sum(u[1], P.Ch);
            u[2] = head_sum(u[2], P.Ch);
            float b, db;
            radial_bias(P, head, d, b, db);
            const float p = __expf(dot * P.tau + b - lse);
            const float phi = e2f::radial_gate(d, P.cutoff);
            const float dphi = -0.5f * 3.14159265358979f / P.cutoff * __sinf(3.14159265358979f * d / P.cutoff);
            const float wsum = rx * u[0] + ry * u[1] + rz * u[2];
            const float ds = p * (phi * wsum - Dn);
            const float alpha = p * phi;
            const float dd = (ds * db + p * wsum * dphi) / d;
#pragma unroll
            for (int l = 0; l <= L; ++l) dq[l] += P.tau * ds * kv[l];
            gx += alpha * u[0] + dd * rx;
            gy += alpha * u[1] + dd * ry;
            gz += alpha * u[2] + dd * rz;
        }
        if (s_ctl[1]) break;
    }
    if (live) {
#pragma unroll
        for (int l = 0; l <= L; ++l) P.gq[((size_t)a * (L + 1) + l) * C + c] = dq[l];
    }
    if (live && c % P.Ch == 0) {
        s_gp[head][0] = gx;
        s_gp[head][1] = gy;
        s_gp[head][2] = gz;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int c = threadIdx.x;
        float s = 0.0f;
        for (int hh = 0; hh < P.H; ++hh) s += s_gp[hh][c];
        P.gpos[(size_t)a * 3 + c] = -s;
    }
}

// ---- what an atom owns as a source j: dk_j, dv_j and +sum_i dL/dr_ij (added to the target kernel's share)
template <int L, typename VT>
__global__ __launch_bounds__(256) void k_bwd_source(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP];
    __shared__ int s_ctl[2];
    __shared__ float s_G[3 * E2F_MAX_N * E2F_MAX_N];
    __shared__ float s_gp[E2F_MAX_H][3];
    const int t = blockIdx.x, C = P.C;
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    for (int i = threadIdx.x; i < 3 * E2F_MAX_N * E2F_MAX_N; i += blockDim.x) s_G[i] = P.G[i];
    const float4 pj = P.spos[t];   // this atom is the source j of every pair below
    float kv[L + 1], dk[L + 1], vj[n], Y[3][n];
#pragma unroll
    for (int l = 0; l <= L; ++l) {
        kv[l] = P.k[((size_t)t * (L + 1) + l) * C + c];
        dk[l] = 0.0f;
    }
#pragma unroll
    for (int x = 0; x < n; ++x) {
        vj[x] = e2f::load_as_float<VT>((const VT*)P.v + ((size_t)t * n + x) * C + c);
        Y[0][x] = Y[1][x] = Y[2][x] = 0.0f;
    }
    float gx = 0.0f, gy = 0.0f, gz = 0.0f;   // sum_i dL/dr_ij of this head
    ListWalk w;
    w.init(P.cv, t);
    while (true) {
        const int cnt = next_batch(P, w, t, pj, s_list, s_pos, s_ctl);
        for (int e = 0; e < cnt; ++e) {
            const int i = s_list[e];           // the target, seen from j at its image s_pos[e]
            const float4 pim = s_pos[e];
            const int ai = __float_as_int(pim.w);
            const float rx = pj.x - pim.x, ry = pj.y - pim.y, rz = pj.z - pim.z;   // r_ij = pos_j - pos_i
            const float d = sqrtf(rx * rx + ry * ry + rz * rz);
            float qv[L + 1], dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) {
                qv[l] = P.q[((size_t)i * (L + 1) + l) * C + c];
                dot += qv[l] * kv[l];
            }
            float g[n];
#pragma unroll
            for (int x = 0; x < n; ++x) g[x] = P.gout[((size_t)ai * n + x) * C + c];
            float u[3];
            axis_bilinear<L>(g, vj, s_G, u);
            dot = head_sum(dot, P.Ch);
            u[0] = head_sum(u[0], P.Ch);
            u[1] = head_sum(u[1], P.Ch);
            u[2] = head_sum(u[2], P.Ch);
            float b, db;
            radial_bias(P, head, d, b, db);
            const float p = __expf(dot * P.tau + b - P.lse[(size_t)i * P.H + head]);
            const float phi = e2f::radial_gate(d, P.cutoff);
            const float dphi = -0.5f * 3.14159265358979f / P.cutoff * __sinf(3.14159265358979f * d / P.cutoff);
            const float wsum = rx * u[0] + ry * u[1] + rz * u[2];
            const float ds = p * (phi * wsum - P.Dn[(size_t)i * P.H + head]);
            const float alpha = p * phi;
            const float dd = (ds * db + p * wsum * dphi) / d;
#pragma unroll
            for (int l = 0; l <= L; ++l) dk[l] += P.tau * ds * qv[l];
            const float ax = alpha * rx, ay = alpha * ry, az = alpha * rz;
#pragma unroll
            for (int x = 0; x < n; ++x) {
                Y[0][x] += ax * g[x];
                Y[1][x] += ay * g[x];
                Y[2][x] += az * g[x];
            }
            gx += alpha * u[0] + dd * rx;
            gy += alpha * u[1] + dd * ry;
            gz += alpha * u[2] + dd * rz;
        }
        if (s_ctl[1]) break;
    }
    if (live) {
#pragma unroll
        for (int l = 0; l <= L; ++l) P.gk[((size_t)a * (L + 1) + l) * C + c] = dk[l];
    }
    // dv_j = sum_mu G_mu^T Y_mu
    float dv[n];
#pragma unroll
    for (int x = 0; x < n; ++x) dv[x] = 0.0f;
#pragma unroll
    for (int mu = 0; mu < 3; ++mu)
#pragma unroll
        for (int xo = 0; xo < n; ++xo)
#pragma unroll
            for (int xi = 0; xi < n; ++xi)
                if ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u) dv[xi] += s_G[(mu * E2F_MAX_N + xo) * E2F_MAX_N + xi] * Y[mu][xo];
    if (live) {
#pragma unroll
        for (int x = 0; x < n; ++x) P.gv[((size_t)a * n + x) * C + c] = dv[x];
    }
    if (live && c % P.Ch == 0) {
        s_gp[head][0] = gx;
        s_gp[head][1] = gy;
        s_gp[head][2] = gz;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int c = threadIdx.x;
        float s = 0.0f;
        for (int hh = 0; hh < P.H; ++hh) s += s_gp[hh][c];
        P.gpos[(size_t)a * 3 + c] += s;   // the target kernel wrote this atom's other share before
    }
}

template <int L>
void launch_L(const e2f_ctx* ctx, const BwdParams& P, hipStream_t st) {
    const int N = P.cv.N, C = P.C < 64 ? 64 : P.C;
    k_bwd_stats<L><<<N, C, 0, st>>>(P);
    if (ctx->cfg.feat_dtype == E2F_BF16) {
        k_bwd_target<L, uint16_t><<<N, C, 0, st>>>(P);
        k_bwd_source<L, uint16_t><<<N, C, 0, st>>>(P);
    } else {
        k_bwd_target<L, float><<<N, C, 0, st>>>(P);
        k_bwd_source<L, float><<<N, C, 0, st>>>(P);
    }
}

}  // namespace

bool e2f_backward_supported(const e2f_ctx* ctx) {
    const int Ch = ctx->Ch;
    return ctx->cfg.lf == 1 && ctx->cfg.L_max >= 1 && Ch <= 64 && (Ch & (Ch - 1)) == 0 && ctx->cfg.C <= 256;
}

e2f_status e2f_launch_backward(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                               const E2fBwdWs& bw, const float* out, const float* grad_out, float* grad_pos,
                               float* grad_q, float* grad_k, float* grad_v, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    BwdParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = ws.v; P.G = bw.G; P.Wb = w->Wb;
    P.out = out; P.gout = grad_out; P.lse = bw.lse; P.Dn = bw.Dn;
    P.gpos = grad_pos; P.gq = grad_q; P.gk = grad_k; P.gv = grad_v;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.Ch = ctx->Ch;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    e2f_status rc = e2f_launch_axis_ops(ctx, ws.cw, bw.G, st);
    if (rc != E2F_OK) return rc;
    switch (ctx->cfg.L_max) {
        case 1: launch_L<1>(ctx, P, st); break;
        case 2: launch_L<2>(ctx, P, st); break;
        case 3: launch_L<3>(ctx, P, st); break;
        case 4: launch_L<4>(ctx, P, st); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
