// Standalone EAAS tensor product (Sec. 3.3, Prop. EAAS): out[t] = h[t] (x) R^(lf)(r[t]), channel-wise, evaluated as
// rotate into the frame of r[t], re-index with P, rotate back.  This is the operation of the paper's tensor-product
// timing table ((128x0e+128x1e+128x2e) (x) (1x2e), 1k..32k products).  It is bound by HBM traffic: every element of
// h is read once and every element of out written once.
//
// One wave handles TPB consecutive products: lanes 0..TPB-1 build the Wigner blocks of one product each into LDS,
// then all lanes (lanes over channels, CPL channels per lane) run the products one after the other with coalesced
// loads and stores.
#include "e2f_device.h"

namespace {

constexpr int TPB = 16;

struct TpCoef {
    float c[E2F_MAX_N][E2F_NP];
};

template <int L, int LF, int CPL, typename T>
__global__ __launch_bounds__(64) void k_eaas_tp(const T* __restrict__ h, const float* __restrict__ r,
                                                const float* __restrict__ w_path, TpCoef tab, int C, int n_tp,
                                                float* __restrict__ out) {
    constexpr int n = (L + 1) * (L + 1);
    constexpr int DS = e2f::d_offset(L + 1);
    constexpr int DSP = DS | 1;
    __shared__ float s_D[TPB * DSP];
    __shared__ float s_w[TPB];
    __shared__ float s_cw[n * E2F_NP];
    const int lane = threadIdx.x, t0 = blockIdx.x * TPB, nt = min(TPB, n_tp - t0);
    for (int x = lane; x < n * E2F_NP; x += 64) {
        const int comp = x / E2F_NP, kk = x % E2F_NP;
        int lo = 0;
        while ((lo + 1) * (lo + 1) <= comp) ++lo;
        const int li = lo - LF + kk;
        s_cw[x] = (kk <= 2 * LF && li >= 0 && li <= L) ? w_path[li * (L + 1) + lo] * tab.c[comp][kk] : 0.0f;
    }
    if (lane < nt) {
        float dx = r[3 * (t0 + lane)], dy = r[3 * (t0 + lane) + 1], dz = r[3 * (t0 + lane) + 2];
        const float d = sqrtf(dx * dx + dy * dy + dz * dz);
        s_w[lane] = e2f::pow_lf<LF>(d);
        if constexpr (LF != 0) {
            const bool zero = !(d > 0.0f);   // r = 0: any frame will do, the weight |r|^lf is 0
            e2f::align_D<L>(zero ? 0.0f : dx, zero ? 0.0f : dy, zero ? 1.0f : dz, zero ? 1.0f : d, s_D + lane * DSP);
        }
    }
    __syncthreads();
    const bool active = lane * CPL < C;
    const int c0 = active ? lane * CPL : 0;
    for (int p = 0; p < nt; ++p) {
        const T* hp = h + (size_t)(t0 + p) * n * C + c0;
        float v[n][CPL], acc[n][CPL];
#pragma unroll
        for (int x = 0; x < n; ++x)
#pragma unroll
            for (int u = 0; u < CPL; ++u) {
                v[x][u] = e2f::load_as_float(hp + x * C + u);
                acc[x][u] = 0.0f;
            }
        e2f::eaas_accumulate<L, LF, CPL>(v, s_D + p * DSP, s_cw, s_w[p], acc);
        if (active) {
            float* op = out + (size_t)(t0 + p) * n * C + c0;
#pragma unroll
            for (int x = 0; x < n; ++x)
#pragma unroll
                for (int u = 0; u < CPL; ++u) op[x * C + u] = acc[x][u];
        }
    }
}

template <int L, int LF, int CPL>
void launch_dtype(const e2f_ctx* ctx, const void* h, const float* r, const float* w_path, const TpCoef& tab, int T,
                  float* out, hipStream_t st) {
    const int blocks = (T + TPB - 1) / TPB;
    if (ctx->cfg.feat_dtype == E2F_BF16)
        k_eaas_tp<L, LF, CPL, uint16_t><<<blocks, 64, 0, st>>>((const uint16_t*)h, r, w_path, tab, ctx->cfg.C, T, out);
    else
        k_eaas_tp<L, LF, CPL, float><<<blocks, 64, 0, st>>>((const float*)h, r, w_path, tab, ctx->cfg.C, T, out);
}

template <int L, int LF>
bool launch_cpl(const e2f_ctx* ctx, const void* h, const float* r, const float* w_path, const TpCoef& tab, int T,
                float* out, hipStream_t st) {
    switch (ctx->cpl) {
        case 1: launch_dtype<L, LF, 1>(ctx, h, r, w_path, tab, T, out, st); return true;
        case 2: launch_dtype<L, LF, 2>(ctx, h, r, w_path, tab, T, out, st); return true;
        case 3: launch_dtype<L, LF, 3>(ctx, h, r, w_path, tab, T, out, st); return true;
        case 4: launch_dtype<L, LF, 4>(ctx, h, r, w_path, tab, T, out, st); return true;
    }
    return false;
}

template <int L>
bool launch_lf(const e2f_ctx* ctx, const void* h, const float* r, const float* w_path, const TpCoef& tab, int T,
               float* out, hipStream_t st) {
    switch (ctx->cfg.lf) {
        case 0: return launch_cpl<L, 0>(ctx, h, r, w_path, tab, T, out, st);
        case 1: return launch_cpl<L, 1>(ctx, h, r, w_path, tab, T, out, st);
        case 2: return launch_cpl<L, 2>(ctx, h, r, w_path, tab, T, out, st);
    }
    return false;
}

}  // namespace

e2f_status e2f_launch_tensor_product(const e2f_ctx* ctx, const void* h, const float* r, const float* w_path, float* out,
                                     int32_t T, hipStream_t st) {
    if (T == 0) return E2F_OK;
    TpCoef tab;
    for (int x = 0; x < E2F_MAX_N; ++x)
        for (int k = 0; k < E2F_NP; ++k) tab.c[x][k] = ctx->coefP[x][k];
    bool ok = false;
    switch (ctx->cfg.L_max) {
        case 0: ok = launch_lf<0>(ctx, h, r, w_path, tab, T, out, st); break;
        case 1: ok = launch_lf<1>(ctx, h, r, w_path, tab, T, out, st); break;
        case 2: ok = launch_lf<2>(ctx, h, r, w_path, tab, T, out, st); break;
        case 3: ok = launch_lf<3>(ctx, h, r, w_path, tab, T, out, st); break;
        case 4: ok = launch_lf<4>(ctx, h, r, w_path, tab, T, out, st); break;
    }
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
