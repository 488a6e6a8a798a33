// The paper's factorized node-centric pipeline for a degree-1 filter (Preliminaries, Eq. e2former_final with
// l = 1; Sec. 3.2 "Implementation of factorized message passing"; Sec. 3.4 Algorithm 1):
//
//   (i)   source term      h'_j = v_j (x) R^(1)(r_j - o)                        node level, EAAS with the frame of r_j - o
//   (ii)  aggregation      A1_i = sum_j alpha_ij h'_j ,  A0_i = sum_j alpha_ij v_j   Algorithm 1: scalar weights only
//   (iii) target coupling  m_i  = A1_i - A0_i (x) R^(1)(r_i - o)                 node level, binomial sign (-1)^(l-u)
//
// R^(1) is linear in its argument, so m_i equals sum_j alpha_ij v_j (x) R^(1)(r_j - r_i), the per-pair result.
// o is the centre of the atom's segment grid.  The Wigner rotations move from O(pairs) to O(atoms); the streaming
// kernel (ii) touches pairs only through the scalar alpha_ij, exactly as Algorithm 1 does, but gathers twice the
// rows per neighbour.  The two terms of (iii) cancel the dependence on o, so h' and the sums stay in fp32.
#include "e2f_device.h"

namespace {

constexpr int FPB = 16;  // atoms per wave in the node-level kernels
constexpr int FSC = 32;  // pairs per chunk in the streaming kernel
constexpr int FCAP = 320;

__device__ __forceinline__ float3 seg_origin(const E2fCellsView& cv, int slot) {
    const E2fSegGrid g = cv.grid[cv.sseg[slot]];
    return make_float3(g.ox + 0.5f * g.nx / g.ix, g.oy + 0.5f * g.ny / g.iy, g.oz + 0.5f * g.nz / g.iz);
}

// Node-level EAAS product with r = spos[slot] - o for FPB consecutive slots per wave.
//   TARGET = false: dst[slot] = src[slot] (x) R(r)                       (source term; src = v, dst = h')
//   TARGET = true : out[perm[slot]] = a1[slot] - a0[slot] (x) R(r)       (target coupling; src = A0, a1 = A1)
template <int L, int CPL, typename ST, bool TARGET>
__global__ __launch_bounds__(64) void k_fact_node(E2fCellsView cv, const float4* __restrict__ spos,
                                                  const ST* __restrict__ src, const float* __restrict__ a1,
                                                  const float* __restrict__ cw, int C, float* __restrict__ dst) {
    constexpr int n = (L + 1) * (L + 1);
    constexpr int DS = e2f::d_offset(L + 1), DSP = DS | 1;
    __shared__ float s_D[FPB * DSP];
    __shared__ float s_w[FPB];
    __shared__ float s_cw[n * E2F_NP];
    const int lane = threadIdx.x, t0 = blockIdx.x * FPB, nt = min(FPB, cv.N - t0);
    for (int x = lane; x < n * E2F_NP; x += 64) s_cw[x] = cw[x];
    if (lane < nt) {
        const float4 p = spos[t0 + lane];
        const float3 o = seg_origin(cv, t0 + lane);
        const float dx = p.x - o.x, dy = p.y - o.y, dz = p.z - o.z;
        const float d = sqrtf(dx * dx + dy * dy + dz * dz);
        const bool zero = !(d > 0.0f);
        s_w[lane] = d;
        e2f::align_D<L>(zero ? 0.0f : dx, zero ? 0.0f : dy, zero ? 1.0f : dz, zero ? 1.0f : d, s_D + lane * DSP);
    }
    __syncthreads();
    const bool active = lane * CPL < C;
    const int c0 = active ? lane * CPL : 0;
    for (int p = 0; p < nt; ++p) {
        const int slot = t0 + p;
        const ST* sp = src + (size_t)slot * n * C + c0;
        float v[n][CPL], acc[n][CPL];
#pragma unroll
        for (int x = 0; x < n; ++x)
#pragma unroll
            for (int u = 0; u < CPL; ++u) {
                v[x][u] = e2f::load_as_float(sp + x * C + u);
                acc[x][u] = 0.0f;
            }
        e2f::eaas_accumulate<L, 1, CPL>(v, s_D + p * DSP, s_cw, s_w[p], acc);
        if (active) {
            if constexpr (TARGET) {
                const float* ap = a1 + (size_t)slot * n * C + c0;
                float* op = dst + (size_t)cv.perm[slot] * n * C + c0;
#pragma unroll
                for (int x = 0; x < n; ++x)
#pragma unroll
                    for (int u = 0; u < CPL; ++u) op[x * C + u] = ap[x * C + u] - acc[x][u];
            } else {
                float* op = dst + (size_t)slot * n * C + c0;
#pragma unroll
                for (int x = 0; x < n; ++x)
#pragma unroll
                    for (int u = 0; u < CPL; ++u) op[x * C + u] = acc[x][u];
            }
        }
    }
}

struct StreamParams {
    E2fCellsView cv;
    const float4* spos;
    const float* q;
    const float* k;
    const void* v;     // [N][n][C] feature dtype
    const float* hp;   // [N][n][C] fp32 source terms
    const float* WbT;  // [B][H]
    float* a1;         // [N][n][C] fp32, sorted order
    float* a0;
    int C, H, B, Ch, halves;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

// Algorithm 1: one wave per (target atom, block of 64 channels), lanes = channels.
template <int L, typename VT>
__global__ __launch_bounds__(64) void k_fact_stream(StreamParams P) {
    constexpr int n = (L + 1) * (L + 1);
    __shared__ int s_list[FCAP];
    __shared__ float s_bias[FSC * E2F_MAX_H];
    __shared__ float s_gate[FSC];
    __shared__ float s_s[FSC * E2F_MAX_H];

    const int item = e2f::xcd_remap(blockIdx.x, P.cv.N * P.halves);
    if (item < 0) return;
    const int t = item / P.halves, hf = item % P.halves;
    const int lane = threadIdx.x, C = P.C, H = P.H;
    const bool active = hf * 64 + lane < C;
    const int c = active ? hf * 64 + lane : 0;
    const int head = c / P.Ch;
    const float4 pi = P.spos[t];

    float a1[n], a0[n];
#pragma unroll
    for (int x = 0; x < n; ++x) { a1[x] = 0.0f; a0[x] = 0.0f; }
    float mu = -INFINITY, z = 0.0f;

    int lo[9], pre[10];
    {
        int hi[9];
        e2f::stencil_rows(P.cv, t, lo, hi);
        pre[0] = 0;
#pragma unroll
        for (int r = 0; r < 9; ++r) pre[r + 1] = pre[r] + (hi[r] - lo[r]);
    }
    const int n_cand = pre[9];
    int cbase = 0;
    while (true) {
        int cnt = 0;
        while (cbase < n_cand && cnt + 256 <= FCAP) {
            int jj[4];
            float4 pj[4];
            int ln = lane;
            asm volatile("" : "+v"(ln));   // keeps (lane - pre[r]) from being hoisted into 36 registers
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int cc = cbase + 64 * u + ln;
                int j = -1;
#pragma unroll
                for (int r = 0; r < 9; ++r)
                    if (cc >= pre[r] && cc < pre[r + 1]) j = lo[r] + cc - pre[r];
                jj[u] = j;
                pj[u] = P.spos[j >= 0 ? j : t];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = jj[u] >= 0 && jj[u] != t &&
                                e2f::is_neighbor(e2f::dist2_exact(pi.x, pi.y, pi.z, pj[u].x, pj[u].y, pj[u].z), P.rc2);
                const unsigned long long mask = __ballot(ok);
                if (ok) s_list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = jj[u];
                cnt += __popcll(mask);
            }
            cbase += 256;
        }
        const bool done = cbase >= n_cand;
        __syncthreads();
        for (int p0 = 0; p0 < cnt; p0 += FSC) {
            const int np = min(FSC, cnt - p0);
            if (lane < np) {   // b(r_ij) per head and phi(r_ij): the only pair geometry Algorithm 1 needs
                const float4 pj = P.spos[s_list[p0 + lane]];
                const float dx = pj.x - pi.x, dy = pj.y - pi.y, dz = pj.z - pi.z;
                const float d = sqrtf(dx * dx + dy * dy + dz * dz);
                for (int hh = 0; hh < H; ++hh) s_bias[lane * E2F_MAX_H + hh] = 0.0f;
                for (int b = 0; b < P.B; ++b) {
                    const float gb = e2f::radial_basis(d, b, P.rbf_step, P.rbf_gamma);
                    for (int hh = 0; hh < H; ++hh) s_bias[lane * E2F_MAX_H + hh] += P.WbT[b * H + hh] * gb;
                }
                s_gate[lane] = e2f::radial_gate(d, P.cutoff);
            }
            __syncthreads();
            float q[L + 1];
#pragma unroll
            for (int l = 0; l <= L; ++l) q[l] = P.q[((size_t)t * (L + 1) + l) * C + c];
            float cmax = -INFINITY;
            for (int pb = 0; pb < np; pb += 8) {
                float kk[8][L + 1];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = s_list[p0 + min(pb + u, np - 1)];
#pragma unroll
                    for (int l = 0; l <= L; ++l) kk[u][l] = P.k[((size_t)j * (L + 1) + l) * C + c];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    float dot = 0.0f;
#pragma unroll
                    for (int l = 0; l <= L; ++l) dot += q[l] * kk[u][l];
                    for (int off = 1; off < P.Ch; off <<= 1) dot += __shfl_xor(dot, off);
                    if (pb + u < np) {
                        const float s = dot * P.tau + s_bias[(pb + u) * E2F_MAX_H + head];
                        cmax = fmaxf(cmax, s);
                        if ((lane & (P.Ch - 1)) == 0 && active) s_s[(pb + u) * E2F_MAX_H + head] = s;
                    }
                }
            }
            const float mu_new = fmaxf(mu, cmax);
            const float scale = __expf(mu - mu_new);
            z *= scale;
            mu = mu_new;
#pragma unroll
            for (int x = 0; x < n; ++x) { a1[x] *= scale; a0[x] *= scale; }
            __syncthreads();
            // A += e^{s-mu} phi [h'_j ; v_j]; the rows of pair p+1 are requested before pair p is accumulated
            auto load_rows = [&](int p, float (&r1)[n], float (&r0)[n]) {
                const int j = s_list[p0 + p];
                const float* hj = P.hp + (size_t)j * n * C + c;
                const VT* vj = (const VT*)P.v + (size_t)j * n * C + c;
#pragma unroll
                for (int x = 0; x < n; ++x) {
                    r1[x] = hj[x * C];
                    r0[x] = e2f::load_as_float(vj + x * C);
                }
            };
            float xa1[n], xa0[n], xb1[n], xb0[n];
            load_rows(0, xa1, xa0);
#pragma unroll 1
            for (int p = 0; p < np; p += 2) {
                load_rows(min(p + 1, np - 1), xb1, xb0);
                {
                    const float pe = __expf(s_s[p * E2F_MAX_H + head] - mu);
                    z += pe;
                    const float w = pe * s_gate[p];
#pragma unroll
                    for (int x = 0; x < n; ++x) { a1[x] += w * xa1[x]; a0[x] += w * xa0[x]; }
                }
                if (p + 1 < np) {
                    load_rows(min(p + 2, np - 1), xa1, xa0);
                    const float pe = __expf(s_s[(p + 1) * E2F_MAX_H + head] - mu);
                    z += pe;
                    const float w = pe * s_gate[p + 1];
#pragma unroll
                    for (int x = 0; x < n; ++x) { a1[x] += w * xb1[x]; a0[x] += w * xb0[x]; }
                }
            }
            __syncthreads();
        }
        if (done) break;
    }
    if (active) {
        const float inv = z > 0.0f ? 1.0f / z : 0.0f;
#pragma unroll
        for (int x = 0; x < n; ++x) {
            P.a1[((size_t)t * n + x) * C + c] = a1[x] * inv;
            P.a0[((size_t)t * n + x) * C + c] = a0[x] * inv;
        }
    }
}

template <int L, int CPL>
void launch_nodes(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const E2fFactWs& fw, bool target,
                  float* out, hipStream_t st) {
    const int blocks = (cv.N + FPB - 1) / FPB, C = ctx->cfg.C;
    if (target) {
        k_fact_node<L, CPL, float, true><<<blocks, 64, 0, st>>>(cv, ws.spos, fw.a0, fw.a1, ws.cw, C, out);
    } else if (ctx->cfg.feat_dtype == E2F_BF16) {
        k_fact_node<L, CPL, uint16_t, false><<<blocks, 64, 0, st>>>(cv, ws.spos, (const uint16_t*)ws.v, nullptr, ws.cw, C, fw.hp);
    } else {
        k_fact_node<L, CPL, float, false><<<blocks, 64, 0, st>>>(cv, ws.spos, (const float*)ws.v, nullptr, ws.cw, C, fw.hp);
    }
}

template <int L>
bool run_L(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const E2fFactWs& fw, float* out,
           hipStream_t st) {
    auto nodes = [&](bool target) {
        switch (ctx->cpl) {
            case 1: launch_nodes<L, 1>(ctx, cv, ws, fw, target, out, st); return true;
            case 2: launch_nodes<L, 2>(ctx, cv, ws, fw, target, out, st); return true;
            case 3: launch_nodes<L, 3>(ctx, cv, ws, fw, target, out, st); return true;
            case 4: launch_nodes<L, 4>(ctx, cv, ws, fw, target, out, st); return true;
        }
        return false;
    };
    if (!nodes(false)) return false;
    StreamParams P;
    P.cv = cv; P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = ws.v; P.hp = fw.hp; P.WbT = ws.wbT; P.a1 = fw.a1; P.a0 = fw.a0;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.Ch = ctx->Ch; P.halves = (ctx->cfg.C + 63) / 64;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    const int grid = e2f::xcd_grid(cv.N * P.halves);
    if (ctx->cfg.feat_dtype == E2F_BF16)
        k_fact_stream<L, uint16_t><<<grid, 64, 0, st>>>(P);
    else
        k_fact_stream<L, float><<<grid, 64, 0, st>>>(P);
    return nodes(true);
}

}  // namespace

bool e2f_factorized_supported(const e2f_ctx* ctx) {
    const int Ch = ctx->Ch;
    return ctx->cfg.lf == 1 && Ch <= 64 && (Ch & (Ch - 1)) == 0;
}

e2f_status e2f_launch_factorized(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, const E2fFactWs& fw,
                                 float* out, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    bool ok = false;
    switch (ctx->cfg.L_max) {
        case 1: ok = run_L<1>(ctx, cv, ws, fw, out, st); break;
        case 2: ok = run_L<2>(ctx, cv, ws, fw, out, st); break;
        case 3: ok = run_L<3>(ctx, cv, ws, fw, out, st); break;
        case 4: ok = run_L<4>(ctx, cv, ws, fw, out, st); break;
    }
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
