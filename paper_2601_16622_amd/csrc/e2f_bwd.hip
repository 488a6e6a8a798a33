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
constexpr int WP_BINS = 32;  // row length of the per-atom path-weight partials ((L_max + 1)^2 <= 25 used)
constexpr int WB_PER_THREAD = 8;   // radial basis functions per thread of a head in the dWb sums: B <= 8 * C/H

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
    // gradients of the attention's own weights (null unless asked for): per-atom partial sums, reduced afterwards
    const float* Gu;      // [3][25][25] axis operators with unit path weights
    float* pWb;           // [N][H][B]
    float* pwp;           // [N][WP_BINS], bin li * (L_max + 1) + lo
    // TL instances (the crowded tiles that the tile kernels of e2f_bwd_tile.hip leave out) read the tile layouts
    // instead of q, k, v, lse and Dn: q rows scaled by tau log2 e and k rows in binary16, value blocks, statistics
    // in base-2 units
    const uint16_t *q16, *k16, *v4;
    float2* stat4;            // [group of 4 slots][H][4] (lse, D)
    const int4* lists_hdr;    // per tile of 16 slots: x < 0 marks a crowded tile
    int C, H, B, Ch;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

constexpr float LOG2E = 1.44269504088896341f, LN2 = 0.69314718055994531f;

// Operand access in the plain layouts or (TL) in the layouts of the tile kernels (heads of 16 channels).
template <int L, bool TL>
__device__ __forceinline__ float load_q(const BwdParams& P, int t, int l, int c) {
    if constexpr (TL) {
        constexpr int DKP = ((L + 1) * 16 + 31) / 32 * 32;
        return (float)__builtin_bit_cast(_Float16, P.q16[((size_t)t * P.H + (c >> 4)) * DKP + l * 16 + (c & 15)]);
    } else {
        return P.q[((size_t)t * (L + 1) + l) * P.C + c];
    }
}
template <int L, bool TL>
__device__ __forceinline__ float load_k(const BwdParams& P, int j, int l, int c) {
    if constexpr (TL) {
        constexpr int DKP = ((L + 1) * 16 + 31) / 32 * 32;
        return (float)__builtin_bit_cast(_Float16, P.k16[e2f::k16_offset(j, P.H, c >> 4, DKP, l * 16 + (c & 15))]);
    } else {
        return P.k[((size_t)j * (L + 1) + l) * P.C + c];
    }
}
template <int L, typename VT, bool TL>
__device__ __forceinline__ float load_v(const BwdParams& P, int j, int x, int c) {
    constexpr int n = (L + 1) * (L + 1);
    if constexpr (TL)
        return e2f::bf16_bits_to_float(P.v4[((size_t)(j >> 2) * P.H + (c >> 4)) * n * 64 + e2f::v4_offset(n, x, c & 15) + (j & 3)]);
    else
        return e2f::load_as_float<VT>((const VT*)P.v + ((size_t)j * n + x) * P.C + c);
}
// Softmax weight P_ij from the dot product of the layout's q and k rows, the bias (natural units) and the statistic.
template <bool TL>
__device__ __forceinline__ float pair_prob(const BwdParams& P, float dot, float bias, float lse) {
    if constexpr (TL) return exp2f(dot + bias * LOG2E - lse);
    else return __expf(dot * P.tau + bias - lse);
}
template <bool TL>
__device__ __forceinline__ float load_lse(const BwdParams& P, int t, int head) {
    if constexpr (TL) return P.stat4[((size_t)(t >> 2) * P.H + head) * 4 + (t & 3)].x;
    else return P.lse[(size_t)t * P.H + head];
}
template <bool TL>
__device__ __forceinline__ float load_Dn(const BwdParams& P, int t, int head) {
    if constexpr (TL) return P.stat4[((size_t)(t >> 2) * P.H + head) * 4 + (t & 3)].y;
    else return P.Dn[(size_t)t * P.H + head];
}

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

// The workgroup then evaluates what depends on the distance alone, once per pair instead of once per channel:
// s_rad[e] = (phi, dphi/dd, d, -) and s_bias[e * H + h] = (b_h(d), db_h/dd).
__device__ __forceinline__ int next_batch(const BwdParams& P, ListWalk& w, int t, const float4& pi, int* s_list,
                                          float4* s_pos, float4* s_rad, float2* s_bias, int* s_ctl) {
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
    const int cnt = s_ctl[0];
    // what depends on the distance alone, spread over the whole workgroup: one (pair, head) item per thread and step
    for (int it = threadIdx.x; it < cnt * P.H; it += blockDim.x) {
        const int e = it / P.H, hh = it % P.H;
        const float4 pj = s_pos[e];
        const float rx = pj.x - pi.x, ry = pj.y - pi.y, rz = pj.z - pi.z;
        const float d = sqrtf(rx * rx + ry * ry + rz * rz);
        if (hh == 0) {
            const float arg = 3.14159265358979f * d / P.cutoff;   // in [0, pi]
            s_rad[e] = make_float4(0.5f * (1.0f + __cosf(arg)), -0.5f * 3.14159265358979f / P.cutoff * __sinf(arg), d, 0.0f);
        }
        float b = 0.0f, db = 0.0f;
        for (int i = 0; i < P.B; ++i) {
            const float x = d - (float)i * P.rbf_step;
            const float g = P.Wb[hh * P.B + i] * __expf(-P.rbf_gamma * x * x);
            b += g;
            db += -2.0f * P.rbf_gamma * x * g;
        }
        s_bias[it] = make_float2(b, db);
    }
    __syncthreads();
    return cnt;
}

// Node-level products with the axis operators, once per atom: T[mu] = G_mu^T a (TRANSPOSE) or G_mu a.
template <int L, bool TRANSPOSE>
__device__ __forceinline__ void axis_apply(const float (&a)[(L + 1) * (L + 1)], const float* s_G,
                                           float (&T)[3][(L + 1) * (L + 1)]) {
    constexpr int n = (L + 1) * (L + 1);
#pragma unroll
    for (int mu = 0; mu < 3; ++mu) {
#pragma unroll
        for (int x = 0; x < n; ++x) T[mu][x] = 0.0f;
#pragma unroll
        for (int xo = 0; xo < n; ++xo)
#pragma unroll
            for (int xi = 0; xi < n; ++xi)
                if ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u) {
                    const float gv = s_G[(mu * E2F_MAX_N + xo) * E2F_MAX_N + xi];
                    if (TRANSPOSE) T[mu][xi] += gv * a[xo];
                    else T[mu][xo] += gv * a[xi];
                }
    }
}

// ---- softmax statistics: lse_i = log sum_j exp(s_ij) and D_i = <g_i, out_i>, per head
template <int L, bool TL>
__global__ __launch_bounds__(256) void k_bwd_stats(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP], s_rad[BCAP];
    extern __shared__ float2 s_bias[];   // [BCAP][H]
    __shared__ int s_ctl[2];
    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N), C = P.C;
    if (t < 0) return;
    if (TL && P.lists_hdr[t >> 4].x >= 0) return;   // (whole workgroup) the tile kernels own this atom
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    const float4 pi = P.spos[t];
    float qv[L + 1];
#pragma unroll
    for (int l = 0; l <= L; ++l) qv[l] = load_q<L, TL>(P, t, l, c);
    float dsum = 0.0f;
    for (int x = 0; x < n; ++x) dsum += P.gout[((size_t)a * n + x) * C + c] * P.out[((size_t)a * n + x) * C + c];
    dsum = head_sum(dsum, P.Ch);
    float m = -INFINITY, z = 0.0f;
    ListWalk w;
    w.init(P.cv, t);
    while (true) {
        const int cnt = next_batch(P, w, t, pi, s_list, s_pos, s_rad, s_bias, s_ctl);
        for (int e = 0; e < cnt; ++e) {
            const int j = s_list[e];
            float dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) dot += qv[l] * load_k<L, TL>(P, j, l, c);
            dot = head_sum(dot, P.Ch);
            if constexpr (TL) {   // base-2 units, as the tile kernels keep them
                const float s = dot + s_bias[e * P.H + head].x * LOG2E;
                const float mn = fmaxf(m, s);
                z = z * exp2f(m - mn) + exp2f(s - mn);
                m = mn;
            } else {
                const float s = dot * P.tau + s_bias[e * P.H + head].x;
                const float mn = fmaxf(m, s);
                z = z * __expf(m - mn) + __expf(s - mn);
                m = mn;
            }
        }
        if (s_ctl[1]) break;
    }
    if (live && c % P.Ch == 0) {
        if constexpr (TL) {
            P.stat4[((size_t)(t >> 2) * P.H + head) * 4 + (t & 3)] = make_float2(z > 0.0f ? m + log2f(z) : 0.0f, dsum);
        } else {
            P.lse[(size_t)t * P.H + head] = z > 0.0f ? m + logf(z) : 0.0f;
            P.Dn[(size_t)t * P.H + head] = dsum;
        }
    }
}

// Degree of component x (index l*l + l + m).
__host__ __device__ constexpr int degree_of(int x) { return x >= 16 ? 4 : x >= 9 ? 3 : x >= 4 ? 2 : x >= 1 ? 1 : 0; }

// ---- what an atom owns as a target i: dq_i and -sum_j dL/dr_ij; with WGRAD also its partial sums of
//   dL/dWb[h][b] = sum_j ds_ij,h exp(-gamma (d_ij - mu_b)^2)
template <int L, typename VT, bool WGRAD, bool TL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void k_bwd_target(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP], s_rad[BCAP];
    extern __shared__ float2 s_bias[];   // [BCAP][H]
    __shared__ int s_ctl[2];
    __shared__ float s_G[3 * E2F_MAX_N * E2F_MAX_N];
    __shared__ float s_gp[E2F_MAX_H][3];
    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N), C = P.C;
    if (t < 0) return;
    if (TL && P.lists_hdr[t >> 4].x >= 0) return;   // (whole workgroup) the tile kernels own this atom
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    for (int i = threadIdx.x; i < 3 * E2F_MAX_N * E2F_MAX_N; i += blockDim.x) s_G[i] = P.G[i];
    const float4 pi = P.spos[t];
    float qv[L + 1], dq[L + 1], g[n];
#pragma unroll
    for (int l = 0; l <= L; ++l) {
        qv[l] = load_q<L, TL>(P, t, l, c);
        dq[l] = 0.0f;
    }
#pragma unroll
    for (int x = 0; x < n; ++x) g[x] = P.gout[((size_t)a * n + x) * C + c];
    const float lse = load_lse<TL>(P, t, head), Dn = load_Dn<TL>(P, t, head);
    float gx = 0.0f, gy = 0.0f, gz = 0.0f;   // sum_j dL/dr_ij of this head
    ListWalk w;
    w.init(P.cv, t);
    __syncthreads();
    float gt[3][n];   // G_mu^T g_i: u_mu = <g_i, G_mu v_j> = <gt_mu, v_j>
    axis_apply<L, true>(g, s_G, gt);
    float accWb[WGRAD ? WB_PER_THREAD : 1];
    if (WGRAD) {
#pragma unroll
        for (int i = 0; i < WB_PER_THREAD; ++i) accWb[i] = 0.0f;
    }
    while (true) {
        const int cnt = next_batch(P, w, t, pi, s_list, s_pos, s_rad, s_bias, s_ctl);
        for (int e = 0; e < cnt; ++e) {
            const int j = s_list[e];
            const float4 pj = s_pos[e];
            const float rx = pj.x - pi.x, ry = pj.y - pi.y, rz = pj.z - pi.z;
            const float4 rad = s_rad[e];
            const float2 bb = s_bias[e * P.H + head];
            float kv[L + 1], dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) {
                kv[l] = load_k<L, TL>(P, j, l, c);
                dot += qv[l] * kv[l];
            }
            float u[3] = {0.0f, 0.0f, 0.0f};
            dot = head_sum(dot, P.Ch);
            const float p = pair_prob<TL>(P, dot, bb.x, lse);
            const float phi = rad.x, dphi = rad.y;
#pragma unroll
            for (int x = 0; x < n; ++x) {
                const float vx = load_v<L, VT, TL>(P, j, x, c);
                u[0] += gt[0][x] * vx;
                u[1] += gt[1][x] * vx;
                u[2] += gt[2][x] * vx;
            }
            u[0] = head_sum(u[0], P.Ch);
            u[1] = head_sum(u[1], P.Ch);
            u[2] = head_sum(u[2], P.Ch);
            const float wsum = rx * u[0] + ry * u[1] + rz * u[2];
            const float ds = p * (phi * wsum - Dn);
            const float alpha = p * phi;
            const float dd = (ds * bb.y + p * wsum * dphi) / rad.z;
#pragma unroll
            for (int l = 0; l <= L; ++l) dq[l] += P.tau * ds * kv[l];
            if (WGRAD) {   // the head's threads share its basis functions: thread ci takes b = ci, ci + Ch, ...
#pragma unroll
                for (int i = 0; i < WB_PER_THREAD; ++i) {
                    const int b = c % P.Ch + i * P.Ch;
                    const float xb = rad.z - (float)b * P.rbf_step;
                    if (b < P.B) accWb[i] += ds * __expf(-P.rbf_gamma * xb * xb);
                }
            }
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
    if (WGRAD) {
        if (live) {
#pragma unroll
            for (int i = 0; i < WB_PER_THREAD; ++i) {
                const int b = c % P.Ch + i * P.Ch;
                if (b < P.B) P.pWb[((size_t)a * P.H + head) * P.B + b] = accWb[i];
            }
        }
    }
}

// Sum of the per-atom partials, one workgroup per output element, in a fixed order.
__global__ __launch_bounds__(256) void k_reduce_partials(const float* __restrict__ part, int N, int stride, int M,
                                                         float* __restrict__ out) {
    __shared__ float s_acc[256];
    const int m = blockIdx.x;
    float s = 0.0f;
    for (int a = threadIdx.x; a < N; a += 256) s += part[(size_t)a * stride + m];
    s_acc[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_acc[threadIdx.x] += s_acc[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0 && m < M) out[m] = s_acc[0];
}

// ---- what an atom owns as a source j: dk_j, dv_j and +sum_i dL/dr_ij (added to the target kernel's share); with
// WGRAD also its partial sums of the path-weight gradient.  The message is linear in the path weights,
// G_mu[xo][xi] = w_path[li(xi)][lo(xo)] Gu_mu[xo][xi] with the unit-weight operators Gu, so with the sums
// Y_mu = sum_i alpha_ij r_mu g_i that this kernel forms anyway
//   dL/dw_path[li][lo] = sum_j sum_mu sum_{xo in lo, xi in li} Y_mu[xo] Gu_mu[xo][xi] v_j[xi].
template <int L, typename VT, bool WGRAD, bool TL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_bwd_source(BwdParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[BCAP];
    __shared__ float4 s_pos[BCAP], s_rad[BCAP];
    extern __shared__ float2 s_bias[];   // [BCAP][H]
    __shared__ int s_ctl[2];
    __shared__ float s_G[3 * E2F_MAX_N * E2F_MAX_N];
    __shared__ float s_gp[E2F_MAX_H][3];
    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N), C = P.C;
    if (t < 0) return;
    if (TL && P.lists_hdr[t >> 4].x >= 0) return;   // (whole workgroup) the tile kernels own this atom
    const bool live = (int)threadIdx.x < C;        // workgroups have at least one full wave: the list walk needs it
    const int c = live ? threadIdx.x : 0, head = c / P.Ch;
    const int a = P.cv.perm[t];
    for (int i = threadIdx.x; i < 3 * E2F_MAX_N * E2F_MAX_N; i += blockDim.x) s_G[i] = P.G[i];
    const float4 pj = P.spos[t];   // this atom is the source j of every pair below
    float kv[L + 1], dk[L + 1], vj[n], Y[3][n];
#pragma unroll
    for (int l = 0; l <= L; ++l) {
        kv[l] = load_k<L, TL>(P, t, l, c);
        dk[l] = 0.0f;
    }
#pragma unroll
    for (int x = 0; x < n; ++x) {
        vj[x] = load_v<L, VT, TL>(P, t, x, c);
        Y[0][x] = Y[1][x] = Y[2][x] = 0.0f;
    }
    float gx = 0.0f, gy = 0.0f, gz = 0.0f;   // sum_i dL/dr_ij of this head
    ListWalk w;
    w.init(P.cv, t);
    __syncthreads();
    float Gv[3][n];   // G_mu v_j: u_mu = <g_i, G_mu v_j>
    axis_apply<L, false>(vj, s_G, Gv);
    while (true) {
        const int cnt = next_batch(P, w, t, pj, s_list, s_pos, s_rad, s_bias, s_ctl);
        for (int e = 0; e < cnt; ++e) {
            const int i = s_list[e];           // the target, seen from j at its image s_pos[e]
            const float4 pim = s_pos[e];
            const int ai = __float_as_int(pim.w);
            const float rx = pj.x - pim.x, ry = pj.y - pim.y, rz = pj.z - pim.z;   // r_ij = pos_j - pos_i
            const float4 rad = s_rad[e];
            const float2 bb = s_bias[e * P.H + head];
            float qv[L + 1], dot = 0.0f;
#pragma unroll
            for (int l = 0; l <= L; ++l) {
                qv[l] = load_q<L, TL>(P, i, l, c);
                dot += qv[l] * kv[l];
            }
            float g[n];
            float u[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int x = 0; x < n; ++x) {
                g[x] = P.gout[((size_t)ai * n + x) * C + c];
                u[0] += Gv[0][x] * g[x];
                u[1] += Gv[1][x] * g[x];
                u[2] += Gv[2][x] * g[x];
            }
            dot = head_sum(dot, P.Ch);
            u[0] = head_sum(u[0], P.Ch);
            u[1] = head_sum(u[1], P.Ch);
            u[2] = head_sum(u[2], P.Ch);
            const float p = pair_prob<TL>(P, dot, bb.x, load_lse<TL>(P, i, head));
            const float phi = rad.x, dphi = rad.y;
            const float wsum = rx * u[0] + ry * u[1] + rz * u[2];
            const float ds = p * (phi * wsum - load_Dn<TL>(P, i, head));
            const float alpha = p * phi;
            const float dd = (ds * bb.y + p * wsum * dphi) / rad.z;
#pragma unroll
            for (int l = 0; l <= L; ++l) dk[l] += (TL ? LN2 : P.tau) * ds * qv[l];   // (TL: the q rows carry tau log2 e)
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
    if (WGRAD) {
        // bins per thread, then summed over the channels in a fixed order
        __syncthreads();
        for (int i = threadIdx.x; i < 3 * E2F_MAX_N * E2F_MAX_N; i += blockDim.x) s_G[i] = P.Gu[i];
        __syncthreads();
        float bins[(L + 1) * (L + 1)], vr[n];   // (the value row is read again: keeping it through the loop costs registers)
#pragma unroll
        for (int i = 0; i < (L + 1) * (L + 1); ++i) bins[i] = 0.0f;
#pragma unroll
        for (int x = 0; x < n; ++x) vr[x] = load_v<L, VT, TL>(P, t, x, c);
#pragma unroll
        for (int mu = 0; mu < 3; ++mu)
#pragma unroll
            for (int xo = 0; xo < n; ++xo)
#pragma unroll
                for (int xi = 0; xi < n; ++xi)
                    if ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u)
                        bins[degree_of(xi) * (L + 1) + degree_of(xo)] +=
                            Y[mu][xo] * s_G[(mu * E2F_MAX_N + xo) * E2F_MAX_N + xi] * vr[xi];
        float* s_red = reinterpret_cast<float*>(s_bias);   // [(L+1)^2][C]: the list batches are done
        if (live) {
#pragma unroll
            for (int i = 0; i < (L + 1) * (L + 1); ++i) s_red[i * C + c] = bins[i];
        }
        __syncthreads();
        if ((int)threadIdx.x < WP_BINS) {
            float s = 0.0f;
            if ((int)threadIdx.x < (L + 1) * (L + 1))
                for (int cc = 0; cc < C; ++cc) s += s_red[threadIdx.x * C + cc];
            P.pwp[(size_t)a * WP_BINS + threadIdx.x] = s;
        }
    }
}

// ---- chain rule through the l-wise linear maps: dL/dh from dL/dq, dL/dk, dL/dv (all in the caller's atom order).
// With a1 = W_Q1 x, a2 = W_Q2 x for a row x = h[atom][l, m] and q[l] = sum_m a1 a2 (Eq. qk):
//     dx = W_Q1^T (dq[l] a2) + W_Q2^T (dq[l] a1) + the same with K + W_V^T dv[l, m].
// One workgroup per 8 atoms, one thread per channel: the thread forms its output channel of the four forward
// products (its own weight rows, the 8 rows x broadcast from LDS), then its input channel of the five transposed
// products (weight columns, coalesced across the workgroup).  Plain vector-ALU matrix work, fp32 accumulation.
template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&o)[8]);
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&o)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
template <>
__device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float (&o)[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    const uint32_t wv[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = __uint_as_float(wv[i] << 16);
        o[2 * i + 1] = __uint_as_float(wv[i] & 0xffff0000u);
    }
}

constexpr int PTA = 8;   // atoms per workgroup of the projection backward: every weight element read serves 8 rows

template <typename T>
__global__ __launch_bounds__(256) void k_bwd_project(const T* __restrict__ h, const T* __restrict__ WQ1,
                                                     const T* __restrict__ WQ2, const T* __restrict__ WK1,
                                                     const T* __restrict__ WK2, const T* __restrict__ WV,
                                                     const float* __restrict__ gq, const float* __restrict__ gk,
                                                     const float* __restrict__ gv, float* __restrict__ gh,
                                                     float* __restrict__ tbuf, int L, int C, int N) {
    extern __shared__ float4 sm4[];   // x[C][PTA], then t[5][C][PTA]
    float* s_x = reinterpret_cast<float*>(sm4);
    float* s_t = s_x + C * PTA;
    const int a0 = blockIdx.x * PTA, c = threadIdx.x, n = (L + 1) * (L + 1);
    int atom[PTA];
#pragma unroll
    for (int ta = 0; ta < PTA; ++ta) atom[ta] = min(a0 + ta, N - 1);   // a short last group repeats its last atom
    for (int l = 0; l <= L; ++l) {
        const size_t wo = (size_t)l * C * C;
        float dqv[PTA], dkv[PTA];
#pragma unroll
        for (int ta = 0; ta < PTA; ++ta) {
            dqv[ta] = gq[((size_t)atom[ta] * (L + 1) + l) * C + c];
            dkv[ta] = gk[((size_t)atom[ta] * (L + 1) + l) * C + c];
        }
        for (int m = 0; m < 2 * l + 1; ++m) {
            const int comp = l * l + m;
#pragma unroll
            for (int ta = 0; ta < PTA; ++ta) s_x[c * PTA + ta] = e2f::load_as_float<T>(h + ((size_t)atom[ta] * n + comp) * C + c);
            __syncthreads();
            float acc4[4][PTA];
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int ta = 0; ta < PTA; ++ta) acc4[k][ta] = 0.0f;
            for (int ci = 0; ci < C; ci += 8) {
                float w[4][8];
                load8<T>(WQ1 + wo + (size_t)c * C + ci, w[0]);
                load8<T>(WQ2 + wo + (size_t)c * C + ci, w[1]);
                load8<T>(WK1 + wo + (size_t)c * C + ci, w[2]);
                load8<T>(WK2 + wo + (size_t)c * C + ci, w[3]);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float4 xa = *reinterpret_cast<const float4*>(s_x + (ci + u) * PTA);
                    const float4 xb = *reinterpret_cast<const float4*>(s_x + (ci + u) * PTA + 4);
                    const float xs[PTA] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k)
#pragma unroll
                        for (int ta = 0; ta < PTA; ++ta) acc4[k][ta] += w[k][u] * xs[ta];
                }
            }
#pragma unroll
            for (int ta = 0; ta < PTA; ++ta) {
                s_t[(0 * C + c) * PTA + ta] = dqv[ta] * acc4[1][ta];
                s_t[(1 * C + c) * PTA + ta] = dqv[ta] * acc4[0][ta];
                s_t[(2 * C + c) * PTA + ta] = dkv[ta] * acc4[3][ta];
                s_t[(3 * C + c) * PTA + ta] = dkv[ta] * acc4[2][ta];
                s_t[(4 * C + c) * PTA + ta] = gv[((size_t)atom[ta] * n + comp) * C + c];
            }
            __syncthreads();
            if (tbuf) {   // the five row factors of the weight gradients: dW_k[l] = sum over rows of t_k (x) x
#pragma unroll
                for (int k = 0; k < 5; ++k)
#pragma unroll
                    for (int ta = 0; ta < PTA; ++ta)
                        if (a0 + ta < N)
                            tbuf[((size_t)k * N + a0 + ta) * n * C + (size_t)comp * C + c] = s_t[(k * C + c) * PTA + ta];
            }
            if (!gh) {   // (uniform) only the row factors were asked for
                __syncthreads();
                continue;
            }
            float dx[PTA];
#pragma unroll
            for (int ta = 0; ta < PTA; ++ta) dx[ta] = 0.0f;
            for (int co = 0; co < C; ++co) {
                const size_t wi = wo + (size_t)co * C + c;
                const float wk[5] = {e2f::load_as_float<T>(WQ1 + wi), e2f::load_as_float<T>(WQ2 + wi),
                                     e2f::load_as_float<T>(WK1 + wi), e2f::load_as_float<T>(WK2 + wi),
                                     e2f::load_as_float<T>(WV + wi)};
#pragma unroll
                for (int k = 0; k < 5; ++k) {
                    const float4 ta4 = *reinterpret_cast<const float4*>(s_t + (k * C + co) * PTA);
                    const float4 tb4 = *reinterpret_cast<const float4*>(s_t + (k * C + co) * PTA + 4);
                    dx[0] += wk[k] * ta4.x; dx[1] += wk[k] * ta4.y; dx[2] += wk[k] * ta4.z; dx[3] += wk[k] * ta4.w;
                    dx[4] += wk[k] * tb4.x; dx[5] += wk[k] * tb4.y; dx[6] += wk[k] * tb4.z; dx[7] += wk[k] * tb4.w;
                }
            }
#pragma unroll
            for (int ta = 0; ta < PTA; ++ta)
                if (a0 + ta < N) gh[((size_t)(a0 + ta) * n + comp) * C + c] = dx[ta];
            __syncthreads();
        }
    }
}

// ---- the same chain rule on the matrix cores, for bf16 features and C <= 128.  A workgroup owns one degree and a
// few consecutive tiles of 16 atoms and walks their (tile, order) slabs with one load of its weights; wave ct owns
// output channels 16 ct .. 16 ct + 15 of the forward products and the same input channels of the transposed ones.
// Both products are written with the channels as rows and the atoms as columns, (W x)^T = W X^T and
// dX^T = sum_k W_k^T T_k^T, so that the weights are the A operand (one 16-byte load per fragment, from W for the first
// and from the transposed copy WT for the second, kept in registers), a lane ends up with four consecutive channels
// of one atom (16-byte loads of dq, dk, dv and 16-byte stores of the result) and the row factors t_k cross the waves
// through LDS as [atom][channel] rows.  The feature rows of a slab are fetched once per workgroup and shared through
// LDS as well.  The factors are fp32; for the second product each is rounded to bf16, the counterpart of the forward
// pass rounding the projected values to bf16 (HL = 2 splits each into two bf16 instead, leading part and remainder,
// 16 significant bits together, at twice the LDS reads and matrix instructions of that product).
__global__ __launch_bounds__(256) void k_transpose_weights(const uint16_t* __restrict__ W0, const uint16_t* __restrict__ W1,
                                                           const uint16_t* __restrict__ W2, const uint16_t* __restrict__ W3,
                                                           const uint16_t* __restrict__ W4, int L1, int C,
                                                           uint16_t* __restrict__ WT) {
    // WT[k][l][ci][co] = W_k[l][co][ci]; one workgroup per (k, l, 16 x 16 tile)
    __shared__ uint16_t s[16][17];
    const int tiles = C / 16, t = blockIdx.x % (tiles * tiles), kl = blockIdx.x / (tiles * tiles);
    const int k = kl / L1, l = kl % L1, tr = t / tiles, tc = t % tiles;
    const uint16_t* W = k == 0 ? W0 : k == 1 ? W1 : k == 2 ? W2 : k == 3 ? W3 : W4;
    const int r = threadIdx.x >> 4, c = threadIdx.x & 15;
    s[r][c] = W[((size_t)l * C + 16 * tr + r) * C + 16 * tc + c];
    __syncthreads();
    WT[(((size_t)k * L1 + l) * C + 16 * tc + r) * C + 16 * tr + c] = s[c][r];
}

// Which workgroups take which degree: workgroups [first[d], first[d + 1]) own degree L - d (the highest degree, with
// the most slabs per tile, first) and tiles[d] consecutive tiles of 16 atoms each, so that every workgroup walks about
// the same number of (tile, order) slabs with one load of its weights.
constexpr int PROJECT_SLABS = 18;   // slabs a workgroup of k_bwd_project_mfma walks with one load of its weights
constexpr int PROJECT_SPLIT = 1;    // 1: the row factors as one bf16 each; 2: as two (leading part and remainder)
struct ProjectMap {
    int first[E2F_MAX_L + 2];
    int tiles[E2F_MAX_L + 1];
};

template <int C, int HL>
__global__ __launch_bounds__(64 * (C / 16)) void k_bwd_project_mfma(
    const uint16_t* __restrict__ h, const uint16_t* __restrict__ WQ1, const uint16_t* __restrict__ WQ2,
    const uint16_t* __restrict__ WK1, const uint16_t* __restrict__ WK2, const uint16_t* __restrict__ WT,
    const float* __restrict__ gq, const float* __restrict__ gk, const float* __restrict__ gv, float* __restrict__ gh,
    float* __restrict__ tbuf, int L, int N, ProjectMap map) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    constexpr int NS = C / 32, ROW = C + 8;   // LDS rows of 16 atoms, 16 bytes of padding against bank conflicts
    constexpr int PD = 3;                     // slabs in flight from memory
    // Two buffers each, used in turn.  In one pass of the loop a wave runs the second stage of slab s (reads s_T[s & 1]),
    // the first stage of slab s + 1 (reads s_X[(s + 1) & 1], writes s_T[(s + 1) & 1]) and stores the feature rows of
    // slab s + 2 (s_X[s & 1]): the two stages of consecutive slabs overlap inside a wave and one barrier per slab is enough.
    __shared__ __attribute__((aligned(16))) uint16_t s_T[2][5][HL][16][ROW];
    __shared__ __attribute__((aligned(16))) uint16_t s_X[2][16][ROW];
    // (the wave's index through readfirstlane, so that the compiler knows it to be the same in all lanes)
    const int tid = threadIdx.x, ct = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, i = lane & 15, g = lane >> 4;
    const int n_tiles = (N + 15) / 16, n = (L + 1) * (L + 1);
    int d = 0;
    while (d < L && (int)blockIdx.x >= map.first[d + 1]) ++d;
    const int l = L - d, nl = 2 * l + 1;
    const int tile0 = ((int)blockIdx.x - map.first[d]) * map.tiles[d];
    const int n_slabs = (min(n_tiles, tile0 + map.tiles[d]) - tile0) * nl;   // slab s: tile tile0 + s / nl, order s % nl
    if (n_slabs <= 0) return;
    const int ch0 = 16 * ct + 4 * g;   // the four channels this lane holds of its atom
    auto frag = [](const uint16_t* p) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(p)); };
    auto pack2 = [](float a, float b) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, bf16x2));
    };
    bf16x8 W1[4][NS], W2[5][NS];
    {
        const size_t row = ((size_t)l * C + 16 * ct + i) * C + 8 * g;
        const size_t lstride = (size_t)(L + 1) * C * C;
#pragma unroll
        for (int S = 0; S < NS; ++S) {
            W1[0][S] = frag(WQ1 + row + 32 * S);
            W1[1][S] = frag(WQ2 + row + 32 * S);
            W1[2][S] = frag(WK1 + row + 32 * S);
            W1[3][S] = frag(WK2 + row + 32 * S);
#pragma unroll
            for (int k = 0; k < 5; ++k) W2[k][S] = frag(WT + k * lstride + row + 32 * S);
        }
    }
    // What is read of a slab.  The feature rows of its 16 atoms, shared by the waves: thread tid fetches four channels
    // (xa, xc) of one row, which reach the waves through s_X.  dv for the lane's own atom and channels.  Both are
    // requested PD slabs before their use, in rings of registers indexed at compile time; dq and dk of a tile (lane's
    // atom and channels again) are requested when the tile before it starts.
    const int xa = tid / (C / 4), xc = 4 * (tid % (C / 4));
    // the four places where the sequence of slabs is walked (requests of x and of dv, first stage, second stage)
    // each keep (first atom of the tile, order); a cursor stays on the last slab once it gets there
    struct Cursor {
        int a0, m;
    };
    const int a_last = (tile0 + n_slabs / nl - 1) * 16;
    auto advance = [&](Cursor& c) {
        if (c.m + 1 < nl) {
            ++c.m;
        } else if (c.a0 < a_last) {
            c.m = 0;
            c.a0 += 16;
        }
    };
    Cursor cx = {tile0 * 16, 0}, cv = cx, cf = cx, co = cx;
    auto fetch_x = [&]() {
        const u32x2 v = *reinterpret_cast<const u32x2*>(h + ((size_t)min(cx.a0 + xa, N - 1) * n + l * l + cx.m) * C + xc);
        advance(cx);
        return v;
    };
    auto fetch_dv = [&]() {
        const f32x4 v = *reinterpret_cast<const f32x4*>(gv + ((size_t)min(cv.a0 + i, N - 1) * n + l * l + cv.m) * C + ch0);
        advance(cv);
        return v;
    };
    auto fetch_dqk = [&](int a0, f32x4& dq, f32x4& dk) {
        const size_t at = ((size_t)min(a0 + i, N - 1) * (L + 1) + l) * C + ch0;
        dq = *reinterpret_cast<const f32x4*>(gq + at);
        dk = *reinterpret_cast<const f32x4*>(gk + at);
    };
    auto store_x = [&](int s, u32x2 v) { *reinterpret_cast<u32x2*>(&s_X[s & 1][xa][xc]) = v; };
    f32x4 dq, dk, dq_next, dk_next;
    // first stage of slab s: the four forward products of the slab's rows, then the five row factors
    // t = (dq (WQ2 x), dq (WQ1 x), dk (WK2 x), dk (WK1 x), dv), to the workspace (fp32) and to LDS (bf16)
    auto factors = [&](int s, f32x4 dv, bool to_lds) {
        const int atom = cf.a0 + i, m = cf.m;
        const bool real = atom < N;
        if (m == 0) {   // (uniform) a new tile
            dq = dq_next;
            dk = dk_next;
            fetch_dqk(cf.a0 + 16, dq_next, dk_next);
        }
        advance(cf);
        f32x4 p[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = 0; S < NS; ++S) {
            const bf16x8 X = frag(&s_X[s & 1][i][32 * S + 8 * g]);
#pragma unroll
            for (int k = 0; k < 4; ++k) p[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(W1[k][S], X, p[k], 0, 0, 0);
        }
        // p[k][r] = (W_k x)[channel 16 ct + 4 g + r] of atom i
        f32x4 t[5];
        t[0] = dq * p[1];
        t[1] = dq * p[0];
        t[2] = dk * p[3];
        t[3] = dk * p[2];
        t[4] = dv;
        if (!real) {
#pragma unroll
            for (int k = 0; k < 5; ++k) t[k] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        if (tbuf && real) {   // the row factors of the weight gradients: dW_k[l] = sum over rows of t_k (x) x
            const size_t rowx = ((size_t)atom * n + l * l + m) * C;
#pragma unroll
            for (int k = 0; k < 5; ++k) *reinterpret_cast<f32x4*>(tbuf + (size_t)k * N * n * C + rowx + ch0) = t[k];
        }
        if (!to_lds) return;
        const int buf = s & 1;
#pragma unroll
        for (int k = 0; k < 5; ++k) {
            const u32x2 hi = {pack2(t[k][0], t[k][1]), pack2(t[k][2], t[k][3])};   // (round to nearest even)
            *reinterpret_cast<u32x2*>(&s_T[buf][k][0][i][ch0]) = hi;
            if constexpr (HL == 2) {   // the remainders: 16 significant bits together
                f32x4 rem;
#pragma unroll
                for (int r = 0; r < 4; ++r) rem[r] = t[k][r] - __builtin_bit_cast(float, (r & 1) ? (hi[r >> 1] & 0xffff0000u) : (hi[r >> 1] << 16));
                *reinterpret_cast<u32x2*>(&s_T[buf][k][HL - 1][i][ch0]) = (u32x2){pack2(rem[0], rem[1]), pack2(rem[2], rem[3])};
            }
        }
    };
    // ring slot of slab s: s % PD.  Before pass s of the loop the rings hold x of slabs s + 2 .. s + 4 and dv of
    // slabs s + 1 .. s + 3; s_X holds x of slabs s and s + 1 and s_T the factors of slab s.
    u32x2 xr[PD];
    f32x4 dvr[PD];
    fetch_dqk(tile0 * 16, dq_next, dk_next);
    store_x(0, fetch_x());
    store_x(1, fetch_x());
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        xr[(u + 2) % PD] = fetch_x();
        dvr[u] = fetch_dv();
    }
    __syncthreads();
    const bool lds = gh != nullptr;   // (uniform) without dL/dh only the row factors are asked for
    factors(0, dvr[0], lds);
    dvr[0] = fetch_dv();
    __syncthreads();
    // One pass of the loop, for slab s = s0 + u with ring slots known at compile time.  (LAST: a pass of the last,
    // partial group, which checks whether its slab and the next exist.  The passes of the full groups have no such
    // branches: the compiler places its waits on the loads by the least number of memory instructions on any path
    // from a request to its use, and a path that skips passes would make it wait for requests one pass old.)
    auto pass = [&](int s, int u, bool LAST) __attribute__((always_inline)) {
        // The first stage of the next slab and the second stage of this one are independent.
        auto first_stage = [&]() {
            // the feature rows of slab s + 2 have arrived: into the buffer that slab s used
            store_x(s + 2, xr[(u + 2) % PD]);
            xr[(u + 2) % PD] = fetch_x();
            if (!LAST || s + 1 < n_slabs) factors(s + 1, dvr[(u + 1) % PD], lds);
            dvr[(u + 1) % PD] = fetch_dv();
        };
        auto second_stage = [&]() {
            if (!lds) return;
            const int buf = s & 1;
            // (four partial sums: one accumulator would chain all the matrix instructions one after the other)
            f32x4 dp[4];   // (only dp[0] and dp[1] in use when HL == 1)
#pragma unroll
            for (int j = 0; j < 4; ++j) dp[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < 5; ++k)
#pragma unroll
                for (int S = 0; S < NS; ++S)
#pragma unroll
                    for (int hl = 0; hl < HL; ++hl) {
                        const int j = HL == 2 ? 2 * (S & 1) + hl : (k * NS + S) & 1;
                        dp[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(W2[k][S], frag(&s_T[buf][k][hl][i][32 * S + 8 * g]), dp[j], 0, 0, 0);
                    }
            const f32x4 dx = (dp[0] + dp[2]) + (dp[1] + dp[3]);
            // dx[r] = dL/dh[atom i][component][channel 16 ct + 4 g + r]
            const int atom = co.a0 + i;
            if (atom < N) *reinterpret_cast<f32x4*>(gh + ((size_t)atom * n + l * l + co.m) * C + ch0) = dx;
            advance(co);
        };
        first_stage();
        second_stage();
        __syncthreads();
    };
    int s0 = 0;
    for (; s0 + PD < n_slabs; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) pass(s0 + u, u, false);
    }
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (s0 + u < n_slabs) pass(s0 + u, u, true);   // (uniform)
}

// ---- gradients of the five projection matrices: dW_k[l][co][ci] = sum over atoms a and orders m of
// t_k[a][l, m][co] * h[a][l, m][ci], with the row factors t_k that k_bwd_project leaves in the workspace.  One
// workgroup per (chunk of atoms, degree, tile of 16 output channels), one thread per input channel; the factors of
// 16 rows at a time are staged in LDS and read from there by all threads at once.  Partial sums per chunk are
// added up afterwards in a fixed order.
constexpr int WG_SPLIT = 8;   // degree l is cut into WG_SPLIT * (2l+1) chunks of atoms: every workgroup gets N / WG_SPLIT rows
constexpr int WG_ROWS = 16;   // rows staged in LDS per step
template <typename T>
__global__ __launch_bounds__(256) void k_bwd_wgrad(const T* __restrict__ h, const float* __restrict__ tbuf, int L, int C,
                                                   int N, float* __restrict__ part) {
    __shared__ __attribute__((aligned(16))) float s_t[WG_ROWS][5][16];
    // slice s of the partial sums: degree l = floor(sqrt(s / WG_SPLIT)), chunk s - WG_SPLIT * l^2 of WG_SPLIT * (2l+1)
    const int slice = blockIdx.x, co0 = blockIdx.y * 16, ci = threadIdx.x;
    int l = 0;
    while (WG_SPLIT * (l + 1) * (l + 1) <= slice) ++l;
    const int n = (L + 1) * (L + 1), nl = 2 * l + 1;
    const int chunk = slice - WG_SPLIT * l * l, chunks = WG_SPLIT * nl;
    const int per = (N + chunks - 1) / chunks, a_lo = chunk * per, a_hi = min(N, a_lo + per);
    const int rows = max(a_hi - a_lo, 0) * nl;   // row r of the chunk: atom a_lo + r / nl, order r % nl
    const size_t kstride = (size_t)N * n * C;
    float acc[5][16];
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[k][j] = 0.0f;
    for (int r0 = 0; r0 < rows; r0 += WG_ROWS) {
        const int nr = min(WG_ROWS, rows - r0);
        __syncthreads();   // the previous rows have been consumed
        for (int e = threadIdx.x; e < nr * 80; e += blockDim.x) {
            const int rr = e / 80, k = (e % 80) / 16, jj = e % 16;
            const int r = r0 + rr;
            const size_t row = ((size_t)(a_lo + r / nl) * n + l * l + r % nl) * C;
            s_t[rr][k][jj] = tbuf[k * kstride + row + co0 + jj];
        }
        float x[WG_ROWS];
#pragma unroll
        for (int rr = 0; rr < WG_ROWS; ++rr) {
            const int r = r0 + min(rr, nr - 1);
            x[rr] = e2f::load_as_float<T>(h + ((size_t)(a_lo + r / nl) * n + l * l + r % nl) * C + ci);
        }
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < WG_ROWS; ++rr) {
            if (rr < nr) {
#pragma unroll
                for (int k = 0; k < 5; ++k)
#pragma unroll
                    for (int j4 = 0; j4 < 4; ++j4) {
                        const float4 tv = *reinterpret_cast<const float4*>(&s_t[rr][k][4 * j4]);
                        acc[k][4 * j4] += tv.x * x[rr];
                        acc[k][4 * j4 + 1] += tv.y * x[rr];
                        acc[k][4 * j4 + 2] += tv.z * x[rr];
                        acc[k][4 * j4 + 3] += tv.w * x[rr];
                    }
            }
        }
    }
    // part[slice][k][co][ci]
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) part[(((size_t)slice * 5 + k) * C + co0 + j) * C + ci] = acc[k][j];
}

// The same sums on the matrix cores for bf16 features: dW_k[co][ci] = sum_rows t_k[row][co] h[row][ci] is a product
// whose contraction runs over the rows (atoms x orders), the slow index of both arrays, so 32 rows at a time go through
// LDS in their own order (the factors split into two bf16, leading part and remainder, as in k_bwd_project_mfma) and
// a lane gathers the 8 rows of its column from there, two bytes at a time (writing them turned instead puts the 16
// lanes of a row into one bank).  A workgroup owns
// (slice of rows, 16 output channels) as above, its waves share the C input channels (C / 16 tiles over four waves);
// the rows of the next step are fetched while the products of this one run.
template <int C>
__global__ __launch_bounds__(256) void k_bwd_wgrad_mfma(const uint16_t* __restrict__ h, const float* __restrict__ tbuf, int L,
                                                        int N, float* __restrict__ part) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    constexpr int R = 32;                         // rows per step
    constexpr int PA = 5 * 16 + 2, PB = C + 2;    // row pitches in LDS (elements): an odd number of dwords, so that the
                                                  // four row groups of a gather fall into different banks
    constexpr int CT = C / 16, TPW = (CT + 3) / 4;   // input-channel tiles, tiles per wave
    constexpr int NTV = R * 80 / 256;             // factors per thread and step (32 rows x 5 k x 16 channels)
    constexpr int NHV = (R * C / 8 + 255) / 256;  // 16-byte pieces of the feature rows per thread and step
    __shared__ uint16_t s_A[2][R][PA];   // [leading part, remainder][row][k * 16 + co]
    __shared__ uint16_t s_B[R][PB];      // [row][ci]
    const int slice = blockIdx.x, co0 = blockIdx.y * 16, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
    int l = 0;
    while (WG_SPLIT * (l + 1) * (l + 1) <= slice) ++l;
    const int n = (L + 1) * (L + 1), nl = 2 * l + 1;
    const int chunk = slice - WG_SPLIT * l * l, chunks = WG_SPLIT * nl;
    const int per = (N + chunks - 1) / chunks, a_lo = chunk * per, a_hi = min(N, a_lo + per);
    const int rows = max(a_hi - a_lo, 0) * nl;   // row r of the chunk: atom a_lo + r / nl, order r % nl
    const size_t kstride = (size_t)N * n * C;
    auto row_offset = [&](int r) { return ((size_t)(a_lo + r / nl) * n + l * l + r % nl) * C; };
    f32x4 acc[5][TPW];
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int t = 0; t < TPW; ++t) acc[k][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float tv[NTV];
    u32x4 hv[NHV];
    auto fetch = [&](int r0) {   // element e of the factors: row e / 80, k (e % 80) / 16, channel e % 16
#pragma unroll
        for (int j = 0; j < NTV; ++j) {
            const int e = tid + 256 * j, rr = e / 80, k = (e % 80) / 16, jj = e % 16, r = r0 + rr;
            tv[j] = r < rows ? tbuf[k * kstride + row_offset(r) + co0 + jj] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < NHV; ++j) {
            const int e = tid + 256 * j, rr = e / (C / 8), c8 = e % (C / 8), r = r0 + rr;
            hv[j] = (rr < R && r < rows) ? *reinterpret_cast<const u32x4*>(h + row_offset(r) + 8 * c8) : (u32x4){0u, 0u, 0u, 0u};
        }
    };
    auto turn = [&]() {
#pragma unroll
        for (int j = 0; j < NTV; ++j) {
            const int e = tid + 256 * j, rr = e / 80, k = (e % 80) / 16, jj = e % 16;
            const uint16_t hi = e2f::float_to_bf16_bits(tv[j]);
            s_A[0][rr][k * 16 + jj] = hi;
            s_A[1][rr][k * 16 + jj] = e2f::float_to_bf16_bits(tv[j] - e2f::bf16_bits_to_float(hi));
        }
#pragma unroll
        for (int j = 0; j < NHV; ++j) {
            const int e = tid + 256 * j, rr = e / (C / 8), c8 = e % (C / 8);
            if (rr < R) {
#pragma unroll
                for (int q = 0; q < 4; ++q) *reinterpret_cast<uint32_t*>(&s_B[rr][8 * c8 + 2 * q]) = hv[j][q];
            }
        }
    };
    if (rows > 0) fetch(0);
    for (int r0 = 0; r0 < rows; r0 += R) {
        __syncthreads();   // the previous step's operands have been read
        turn();
        __syncthreads();
        if (r0 + R < rows) fetch(r0 + R);
        auto gather = [&](const uint16_t* col, int pitch) {   // rows 8g..8g+7 of one column
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                v[q] = (uint32_t)col[(8 * g + 2 * q) * pitch] | ((uint32_t)col[(8 * g + 2 * q + 1) * pitch] << 16);
            return __builtin_bit_cast(bf16x8, v);
        };
        bf16x8 A[2][5];
#pragma unroll
        for (int hl = 0; hl < 2; ++hl)
#pragma unroll
            for (int k = 0; k < 5; ++k) A[hl][k] = gather(&s_A[hl][0][k * 16 + i], PA);
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int ct = wave + 4 * t;
            if (ct < CT) {   // (wave-uniform)
                const bf16x8 Bv = gather(&s_B[0][16 * ct + i], PB);
#pragma unroll
                for (int k = 0; k < 5; ++k) {
                    acc[k][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[0][k], Bv, acc[k][t], 0, 0, 0);
                    acc[k][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[1][k], Bv, acc[k][t], 0, 0, 0);
                }
            }
        }
    }
    // part[slice][k][co][ci]: the result lane (i, g) holds rows co = 4g..4g+3 of column ci = i
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int ct = wave + 4 * t;
        if (ct < CT) {
#pragma unroll
            for (int k = 0; k < 5; ++k)
#pragma unroll
                for (int r = 0; r < 4; ++r) part[(((size_t)slice * 5 + k) * C + co0 + 4 * g + r) * C + 16 * ct + i] = acc[k][t][r];
        }
    }
}

// out[k][l][co][ci] = sum over the slices of degree l, in a fixed order.
__global__ void k_sum_chunks(const float* __restrict__ part, int L, int C, float* __restrict__ out) {
    const size_t CC = (size_t)C * C, M = (size_t)5 * (L + 1) * CC;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    const int k = (int)(i / ((L + 1) * CC)), l = (int)((i / CC) % (L + 1));
    const size_t e = i % CC;
    float s = 0.0f;
    for (int c = 0; c < WG_SPLIT * (2 * l + 1); ++c) s += part[((size_t)(WG_SPLIT * l * l + c) * 5 + k) * CC + e];
    out[i] = s;
}

template <int L, typename VT>
void launch_LV(const BwdParams& P, hipStream_t st) {
    const int N = P.cv.N, C = P.C < 64 ? 64 : P.C;
    const size_t shm = (size_t)BCAP * P.H * sizeof(float2);
    // with weight gradients the same bytes later hold the [(L+1)^2][C] channel sums of the path-weight bins
    const size_t shm_w = shm > (size_t)(L + 1) * (L + 1) * P.C * 4 ? shm : (size_t)(L + 1) * (L + 1) * P.C * 4;
    k_bwd_stats<L, false><<<e2f::xcd_grid(N), C, shm, st>>>(P);
    if (P.pWb) {
        k_bwd_target<L, VT, true, false><<<e2f::xcd_grid(N), C, shm, st>>>(P);
        k_bwd_source<L, VT, true, false><<<e2f::xcd_grid(N), C, shm_w, st>>>(P);
    } else {
        k_bwd_target<L, VT, false, false><<<e2f::xcd_grid(N), C, shm, st>>>(P);
        k_bwd_source<L, VT, false, false><<<e2f::xcd_grid(N), C, shm, st>>>(P);
    }
}

// The per-atom kernels over the tile layouts, for the atoms of crowded tiles only (every other workgroup leaves at
// once).  `what` 0: the statistics, which the tile kernels of the other tiles read too; 1: the pair kernels.
template <int L>
void launch_crowded(const BwdParams& P, int what, hipStream_t st) {
    const int N = P.cv.N, C = P.C < 64 ? 64 : P.C;
    const size_t shm = (size_t)BCAP * P.H * sizeof(float2);
    const size_t shm_w = shm > (size_t)(L + 1) * (L + 1) * P.C * 4 ? shm : (size_t)(L + 1) * (L + 1) * P.C * 4;
    if (what == 0) {
        k_bwd_stats<L, true><<<e2f::xcd_grid(N), C, shm, st>>>(P);
    } else if (P.pWb) {   // with the per-atom partial sums of the weight gradients
        k_bwd_target<L, uint16_t, true, true><<<e2f::xcd_grid(N), C, shm, st>>>(P);
        k_bwd_source<L, uint16_t, true, true><<<e2f::xcd_grid(N), C, shm_w, st>>>(P);
    } else {
        k_bwd_target<L, uint16_t, false, true><<<e2f::xcd_grid(N), C, shm, st>>>(P);
        k_bwd_source<L, uint16_t, false, true><<<e2f::xcd_grid(N), C, shm, st>>>(P);
    }
}

template <int L>
void launch_L(const e2f_ctx* ctx, const BwdParams& P, hipStream_t st) {
    if (ctx->cfg.feat_dtype == E2F_BF16) launch_LV<L, uint16_t>(P, st);
    else launch_LV<L, float>(P, st);
}

}  // namespace

bool e2f_backward_supported(const e2f_ctx* ctx) {
    const int Ch = ctx->Ch;
    return ctx->cfg.lf == 1 && ctx->cfg.L_max >= 1 && Ch <= 64 && (Ch & (Ch - 1)) == 0 && ctx->cfg.C <= 256;
}

e2f_status e2f_launch_backward(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                               const E2fBwdWs& bw, const float* out, const float* grad_out, float* grad_pos,
                               float* grad_q, float* grad_k, float* grad_v, const void* h, float* grad_h,
                               float* grad_Wb, float* grad_w_path, float* grad_W, const E2fBwdTileWs* tw,
                               hipStream_t st, bool lists_ready) {
    if (cv.N == 0) return E2F_OK;
    const bool wgrad = grad_Wb || grad_w_path;
    if (wgrad && ctx->cfg.B > WB_PER_THREAD * ctx->Ch) return E2F_ERR_UNSUPPORTED;
    if (tw && wgrad && !e2f_backward_tile_weight_gradients_supported(ctx)) return E2F_ERR_INVALID_ARG;
    BwdParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = ws.v; P.G = tw ? ws.G : bw.G; P.Wb = w->Wb;
    P.out = out; P.gout = grad_out; P.lse = bw.lse; P.Dn = bw.Dn;
    P.gpos = grad_pos; P.gq = grad_q; P.gk = grad_k; P.gv = grad_v;
    P.q16 = ws.q16; P.k16 = ws.k16; P.v4 = ws.v4;
    P.stat4 = tw ? reinterpret_cast<float2*>(tw->stat4) : nullptr;
    P.lists_hdr = ws.lists_hdr;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.Ch = ctx->Ch;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    P.Gu = nullptr; P.pWb = nullptr; P.pwp = nullptr;
    e2f_status rc;
    if (wgrad) {   // unit-weight path coefficients and axis operators (full form for the per-atom kernels, packed for the tile kernels)
        if ((rc = e2f_launch_unit_cw(ctx, bw.cw_unit, st)) != E2F_OK) return rc;
        if ((rc = e2f_launch_axis_ops(ctx, bw.cw_unit, bw.Gu, st)) != E2F_OK) return rc;
        if (tw && (rc = e2f_launch_axis_ops(ctx, bw.cw_unit, tw->Gu, st, true)) != E2F_OK) return rc;
        P.Gu = bw.Gu; P.pWb = bw.pWb; P.pwp = bw.pwp;
    }
    if (tw) {
        // pair work on the matrix cores, tile by tile; the atoms of crowded tiles (lists that do not fit) go through
        // the per-atom kernels, which read the same layouts and statistics
        if (!lists_ready && (rc = e2f_launch_tile_lists(ctx, cv, ws, st)) != E2F_OK) return rc;
        auto crowded = [&](int what) {
            switch (ctx->cfg.L_max) {
                case 1: launch_crowded<1>(P, what, st); break;
                case 2: launch_crowded<2>(P, what, st); break;
                case 3: launch_crowded<3>(P, what, st); break;
                default: launch_crowded<4>(P, what, st); break;
            }
        };
        crowded(0);
        if ((rc = e2f_launch_backward_tile(ctx, cv, ws, *tw, out, grad_out, grad_pos, grad_q, grad_k, grad_v, wgrad, st)) != E2F_OK)
            return rc;
        crowded(1);
        if (wgrad && (rc = e2f_launch_backward_tile_wsum(ctx, cv, ws, *tw, bw.pWb, bw.pwp, grad_Wb, grad_w_path, st)) != E2F_OK)
            return rc;
    }
    if (!tw && (rc = e2f_launch_axis_ops(ctx, ws.cw, bw.G, st)) != E2F_OK) return rc;
    if (!tw) switch (ctx->cfg.L_max) {
        case 1: launch_L<1>(ctx, P, st); break;
        case 2: launch_L<2>(ctx, P, st); break;
        case 3: launch_L<3>(ctx, P, st); break;
        case 4: launch_L<4>(ctx, P, st); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    if (wgrad && !tw) {
        const int L1 = ctx->cfg.L_max + 1, HB = ctx->cfg.H * ctx->cfg.B;
        if (grad_Wb) k_reduce_partials<<<HB, 256, 0, st>>>(bw.pWb, cv.N, HB, HB, grad_Wb);
        if (grad_w_path) k_reduce_partials<<<L1 * L1, 256, 0, st>>>(bw.pwp, cv.N, WP_BINS, L1 * L1, grad_w_path);
    }
    if (grad_h || grad_W) {
        const int C = P.C, L = ctx->cfg.L_max;
        const size_t shm = (size_t)6 * C * PTA * sizeof(float);
        const int groups = (cv.N + PTA - 1) / PTA;
        float* tbuf = grad_W ? bw.tbuf : nullptr;
        const dim3 wgrid(WG_SPLIT * (L + 1) * (L + 1), C / 16);
        const size_t M = (size_t)5 * (L + 1) * C * C;
        if (ctx->cfg.feat_dtype == E2F_BF16 && bw.wT && (C == 32 || C == 64 || C == 128)) {
            const int t16 = C / 16;
            k_transpose_weights<<<5 * (L + 1) * t16 * t16, 256, 0, st>>>(
                (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1, (const uint16_t*)w->WK2,
                (const uint16_t*)w->WV, L + 1, C, bw.wT);
            const int tiles = (cv.N + 15) / 16;
            // tiles per workgroup: about PROJECT_SLABS slabs each, whatever the degree
            ProjectMap map;
            map.first[0] = 0;
            for (int d = 0; d <= L; ++d) {
                const int nl = 2 * (L - d) + 1;
                map.tiles[d] = (PROJECT_SLABS + nl - 1) / nl;
                map.first[d + 1] = map.first[d] + (tiles + map.tiles[d] - 1) / map.tiles[d];
            }
#define E2F_BWD_PROJECT(CC)                                                                                            \
    k_bwd_project_mfma<CC, PROJECT_SPLIT><<<map.first[L + 1], 64 * (CC / 16), 0, st>>>(                                \
        (const uint16_t*)h, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,                 \
        (const uint16_t*)w->WK2, bw.wT, grad_q, grad_k, grad_v, grad_h, tbuf, L, cv.N, map)
            if (C == 32) E2F_BWD_PROJECT(32);
            else if (C == 64) E2F_BWD_PROJECT(64);
            else E2F_BWD_PROJECT(128);
#undef E2F_BWD_PROJECT
            if (grad_W) {
                if (C == 32) k_bwd_wgrad_mfma<32><<<wgrid, 256, 0, st>>>((const uint16_t*)h, tbuf, L, cv.N, bw.wpart);
                else if (C == 64) k_bwd_wgrad_mfma<64><<<wgrid, 256, 0, st>>>((const uint16_t*)h, tbuf, L, cv.N, bw.wpart);
                else k_bwd_wgrad_mfma<128><<<wgrid, 256, 0, st>>>((const uint16_t*)h, tbuf, L, cv.N, bw.wpart);
            }
        } else if (ctx->cfg.feat_dtype == E2F_BF16) {
            k_bwd_project<uint16_t><<<groups, C, shm, st>>>((const uint16_t*)h, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2,
                                                          (const uint16_t*)w->WK1, (const uint16_t*)w->WK2,
                                                          (const uint16_t*)w->WV, grad_q, grad_k, grad_v, grad_h, tbuf, L, C,
                                                          cv.N);
            if (grad_W) k_bwd_wgrad<uint16_t><<<wgrid, C, 0, st>>>((const uint16_t*)h, tbuf, L, C, cv.N, bw.wpart);
        } else {
            k_bwd_project<float><<<groups, C, shm, st>>>((const float*)h, (const float*)w->WQ1, (const float*)w->WQ2,
                                                       (const float*)w->WK1, (const float*)w->WK2, (const float*)w->WV,
                                                       grad_q, grad_k, grad_v, grad_h, tbuf, L, C, cv.N);
            if (grad_W) k_bwd_wgrad<float><<<wgrid, C, 0, st>>>((const float*)h, tbuf, L, C, cv.N, bw.wpart);
        }
        if (grad_W) k_sum_chunks<<<(unsigned)((M + 255) / 256), 256, 0, st>>>(bw.wpart, L, C, grad_W);
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
