// Node-level stage: sorted positions, path-weighted P coefficients, and the l-wise projections
// Q1,Q2,K1,K2,V = W^(l) h^(l) with the invariant q,k of Eq. qk formed in the epilogue (Sec. 3.2).
//
// k_project_mfma: one wave owns 16 atoms (MFMA rows) of one degree l and a group of 16-wide output-channel
// tiles; for every order m it multiplies the 16 x C slab of h by W^T on the matrix cores and, for q and k,
// accumulates the element-wise product of the two projections over m, so Q1,Q2,K1,K2 never leave registers.
// k_project_simple is a plain one-thread-per-output version used by the materialized baseline.
#include "e2f_device.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct CoefTable {
    float c[E2F_MAX_N][3];
};

// spos[slot] = position of the atom in that slot; cw[comp][t] = P coefficient times its path weight.
__global__ void k_prepare(E2fCellsView cv, const float* __restrict__ pos, const float* __restrict__ w_path, int L,
                          int lf, CoefTable tab, float4* __restrict__ spos, float* __restrict__ cw,
                          const float* __restrict__ Wb, int H, int B, float* __restrict__ wbT) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < H * B) wbT[(t % B) * H + t / B] = Wb[t];
    if (t < cv.N) {
        const int a = cv.perm[t];
        spos[t] = make_float4(pos[3 * a], pos[3 * a + 1], pos[3 * a + 2], 0.0f);
    }
    const int n = (L + 1) * (L + 1);
    if (t < n * 3) {
        const int comp = t / 3, which = t % 3;
        int lo = 0;
        while ((lo + 1) * (lo + 1) <= comp) ++lo;
        const int li = (lf == 0) ? lo : lo + which - 1;
        float w = 0.0f;
        if (li >= 0 && li <= L && !(lf == 0 && which != 1)) w = w_path[li * (L + 1) + lo];
        cw[t] = w * tab.c[comp][which];
    }
}

template <typename T>
struct Frag;
// bf16: v_mfma_f32_16x16x32_bf16, lane (i = lane%16, g = lane/16) supplies A[i][32S + 8g + 0..7] and
// B[32S + 8g + 0..7][i]; one 16-byte load per fragment.
template <>
struct Frag<uint16_t> {
    static constexpr int KSTEP = 32;
    typedef bf16x8 type;
    __device__ static type load(const uint16_t* row, int S, int g) {
        return *reinterpret_cast<const type*>(row + 32 * S + 8 * g);
    }
    __device__ static f32x4 mma(type a, type b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};
// fp32: four v_mfma_f32_16x16x4_f32 per 16 channels; in step s lane (i,g) supplies A[i][16S + 4g + s] and
// B[16S + 4g + s][i], so each lane reads one float4 per 16 channels.
template <>
struct Frag<float> {
    static constexpr int KSTEP = 16;
    typedef f32x4 type;
    __device__ static type load(const float* row, int S, int g) {
        return *reinterpret_cast<const type*>(row + 16 * S + 4 * g);
    }
    __device__ static f32x4 mma(type a, type b, f32x4 c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
        return c;
    }
};

// C is the channel count (compile time so that fragments stay in registers), MG the number of orders m
// whose A fragments are held at once, CT the number of 16-wide output tiles per wave.
// TILED: store v for the MFMA attention kernel, bf16 [slot][head][tile][16 channels][16 tile rows] with the
// components in tile order (HI: l=4 rows 0..8, l=3 rows 9..15; LO: l=2 rows 0..4, l=1 rows 5..7, l=0 row 8,
// rows 9..15 zero), heads of 16 channels.
template <typename T, int C, int MG, int CT, bool TILED>
__global__ __launch_bounds__(64) void k_project_mfma(E2fCellsView cv, const T* __restrict__ h,
                                                     const T* __restrict__ WQ1, const T* __restrict__ WQ2,
                                                     const T* __restrict__ WK1, const T* __restrict__ WK2,
                                                     const T* __restrict__ WV, int L, float* __restrict__ q,
                                                     float* __restrict__ k, T* __restrict__ v) {
    typedef Frag<T> F;
    constexpr int NS = C / F::KSTEP;
    const int tile = blockIdx.x, l = blockIdx.y, cg = blockIdx.z;
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    const int N = cv.N, n = (L + 1) * (L + 1), nl = 2 * l + 1;
    const int slot_i = min(tile * 16 + i, N - 1);            // clamped rows are computed and not stored
    const T* hrow = h + ((size_t)cv.perm[slot_i] * n + l * l) * C;
    const size_t wrow = ((size_t)l * C + (cg * CT * 16 + i)) * C;  // row of W for output channel of tile 0

    f32x4 qacc[CT], kacc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        qacc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
        kacc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    for (int m0 = 0; m0 < nl; m0 += MG) {
        typename F::type A[MG][NS];
#pragma unroll
        for (int mm = 0; mm < MG; ++mm) {
            const int m = min(m0 + mm, nl - 1);
#pragma unroll
            for (int S = 0; S < NS; ++S) A[mm][S] = F::load(hrow + (size_t)m * C, S, g);
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const size_t wr = wrow + (size_t)ct * 16 * C;
            const int co = (cg * CT + ct) * 16 + i;
            // q and k: two projections each, multiplied element-wise and summed over m
#pragma unroll
            for (int which = 0; which < 2; ++which) {
                const T* W1 = which == 0 ? WQ1 : WK1;
                const T* W2 = which == 0 ? WQ2 : WK2;
                typename F::type B1[NS], B2[NS];
#pragma unroll
                for (int S = 0; S < NS; ++S) {
                    B1[S] = F::load(W1 + wr, S, g);
                    B2[S] = F::load(W2 + wr, S, g);
                }
                f32x4 acc = which == 0 ? qacc[ct] : kacc[ct];
#pragma unroll
                for (int mm = 0; mm < MG; ++mm) {
                    if (m0 + mm < nl) {
                        f32x4 p1 = {0.f, 0.f, 0.f, 0.f}, p2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int S = 0; S < NS; ++S) {
                            p1 = F::mma(A[mm][S], B1[S], p1);
                            p2 = F::mma(A[mm][S], B2[S], p2);
                        }
                        acc += p1 * p2;
                    }
                }
                if (which == 0) qacc[ct] = acc; else kacc[ct] = acc;
            }
            // v: stored per order
            typename F::type BV[NS];
#pragma unroll
            for (int S = 0; S < NS; ++S) BV[S] = F::load(WV + wr, S, g);
#pragma unroll
            for (int mm = 0; mm < MG; ++mm) {
                if (m0 + mm < nl) {
                    f32x4 p = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int S = 0; S < NS; ++S) p = F::mma(A[mm][S], BV[S], p);
                    // accumulator layout: lane (g, i) holds rows 4g + r, column i
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int slot = tile * 16 + 4 * g + r;
                        if (slot >= N) continue;
                        if constexpr (!TILED) {
                            e2f::store_from_float(v + ((size_t)slot * n + l * l + m0 + mm) * C + co, p[r]);
                        } else {
                            const int NT = L >= 3 ? 2 : 1, mi = m0 + mm;
                            const int TI = l >= 3 ? 0 : NT - 1;
                            const int pos = l == 4 ? mi : (l == 3 ? 9 + mi : (l == 2 ? mi : (l == 1 ? 5 + mi : 8)));
                            T* dst = v + ((((size_t)slot * (C / 16) + (co >> 4)) * NT + TI) * 16 + (co & 15)) * 16;
                            e2f::store_from_float(dst + pos, p[r]);
                            if (l == 0)
                                for (int z = 9; z < 16; ++z) e2f::store_from_float(dst + z, 0.0f);
                            if (l == 3 && L == 3 && mi == 0)
                                for (int z = 0; z < 9; ++z) e2f::store_from_float(dst + z, 0.0f);
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int co = (cg * CT + ct) * 16 + i;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int slot = tile * 16 + 4 * g + r;
            if (slot < N) {
                q[((size_t)slot * (L + 1) + l) * C + co] = qacc[ct][r];
                k[((size_t)slot * (L + 1) + l) * C + co] = kacc[ct][r];
            }
        }
    }
}

// Plain version: block = one sorted slot, thread = one output channel; fp32 outputs.
template <typename T>
__global__ void k_project_simple(E2fCellsView cv, const T* __restrict__ h, const T* __restrict__ WQ1,
                                 const T* __restrict__ WQ2, const T* __restrict__ WK1, const T* __restrict__ WK2,
                                 const T* __restrict__ WV, int L, int C, float* __restrict__ q, float* __restrict__ k,
                                 float* __restrict__ v) {
    extern __shared__ float s_h[];  // [n][C]
    const int slot = blockIdx.x, co = threadIdx.x, n = (L + 1) * (L + 1);
    const T* hrow = h + (size_t)cv.perm[slot] * n * C;
    for (int x = threadIdx.x; x < n * C; x += blockDim.x) s_h[x] = e2f::load_as_float(hrow + x);
    __syncthreads();
    for (int l = 0; l <= L; ++l) {
        const size_t wr = ((size_t)l * C + co) * C;
        float qs = 0.f, ks = 0.f;
        for (int m = 0; m < 2 * l + 1; ++m) {
            const float* x = s_h + (l * l + m) * C;
            float a1 = 0.f, a2 = 0.f, b1 = 0.f, b2 = 0.f, av = 0.f;
            for (int ci = 0; ci < C; ++ci) {
                const float hv = x[ci];
                a1 += e2f::load_as_float(WQ1 + wr + ci) * hv;
                a2 += e2f::load_as_float(WQ2 + wr + ci) * hv;
                b1 += e2f::load_as_float(WK1 + wr + ci) * hv;
                b2 += e2f::load_as_float(WK2 + wr + ci) * hv;
                av += e2f::load_as_float(WV + wr + ci) * hv;
            }
            qs += a1 * a2;
            ks += b1 * b2;
            v[((size_t)slot * n + l * l + m) * C + co] = av;
        }
        q[((size_t)slot * (L + 1) + l) * C + co] = qs;
        k[((size_t)slot * (L + 1) + l) * C + co] = ks;
    }
}

template <typename T, int C>
bool launch_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                 hipStream_t st, bool tiled) {
    if constexpr (C % Frag<T>::KSTEP != 0) {
        return false;
    } else {
        // orders m held in registers at once: bounded by the A fragments (C/KSTEP registers-quads per order)
        constexpr int MG = sizeof(T) == 2 ? (C <= 128 ? 9 : 4) : (C <= 64 ? 9 : (C <= 128 ? 5 : 2));
        constexpr int CT = (C / 16) % 4 == 0 ? 4 : ((C / 16) % 2 == 0 ? 2 : 1);
        const dim3 grid((cv.N + 15) / 16, ctx->cfg.L_max + 1, C / 16 / CT);
        if (tiled)
            k_project_mfma<T, C, MG, CT, true><<<grid, 64, 0, st>>>(cv, (const T*)h, (const T*)w->WQ1, (const T*)w->WQ2,
                                                                   (const T*)w->WK1, (const T*)w->WK2, (const T*)w->WV,
                                                                   ctx->cfg.L_max, ws.q, ws.k, (T*)ws.v);
        else
            k_project_mfma<T, C, MG, CT, false><<<grid, 64, 0, st>>>(cv, (const T*)h, (const T*)w->WQ1, (const T*)w->WQ2,
                                                                    (const T*)w->WK1, (const T*)w->WK2, (const T*)w->WV,
                                                                    ctx->cfg.L_max, ws.q, ws.k, (T*)ws.v);
        return true;
    }
}

template <typename T>
bool dispatch_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                   const E2fAttnWs& ws, hipStream_t st, bool tiled) {
    switch (ctx->cfg.C) {
        case 16: return launch_mfma<T, 16>(ctx, cv, h, w, ws, st, tiled);
        case 32: return launch_mfma<T, 32>(ctx, cv, h, w, ws, st, tiled);
        case 48: return launch_mfma<T, 48>(ctx, cv, h, w, ws, st, tiled);
        case 64: return launch_mfma<T, 64>(ctx, cv, h, w, ws, st, tiled);
        case 128: return launch_mfma<T, 128>(ctx, cv, h, w, ws, st, tiled);
        case 192: return launch_mfma<T, 192>(ctx, cv, h, w, ws, st, tiled);
        case 256: return launch_mfma<T, 256>(ctx, cv, h, w, ws, st, tiled);
    }
    return false;
}

}  // namespace

e2f_status e2f_launch_prepare(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, const e2f_weights* w,
                              const E2fAttnWs& ws, hipStream_t st) {
    CoefTable tab;
    for (int x = 0; x < E2F_MAX_N; ++x)
        for (int t = 0; t < 3; ++t) tab.c[x][t] = ctx->coefP[x][t];
    int work = cv.N > ctx->n * 3 ? cv.N : ctx->n * 3;
    if (ctx->cfg.H * ctx->cfg.B > work) work = ctx->cfg.H * ctx->cfg.B;
    k_prepare<<<(work + 255) / 256, 256, 0, st>>>(cv, pos, w->w_path, ctx->cfg.L_max, ctx->cfg.lf, tab, ws.spos, ws.cw,
                                                 w->Wb, ctx->cfg.H, ctx->cfg.B, ws.wbT);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_project_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                                   const E2fAttnWs& ws, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    const bool ok = ctx->cfg.feat_dtype == E2F_BF16 ? dispatch_mfma<uint16_t>(ctx, cv, h, w, ws, st, ctx->use_mfma_attn)
                                                    : dispatch_mfma<float>(ctx, cv, h, w, ws, st, false);
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_project_simple(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                                     float* q, float* k, float* v, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    const int L = ctx->cfg.L_max, C = ctx->cfg.C;
    const size_t shm = (size_t)ctx->n * C * sizeof(float);
    if (ctx->cfg.feat_dtype == E2F_BF16)
        k_project_simple<uint16_t><<<cv.N, C, shm, st>>>(cv, (const uint16_t*)h, (const uint16_t*)w->WQ1,
                                                         (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,
                                                         (const uint16_t*)w->WK2, (const uint16_t*)w->WV, L, C, q, k, v);
    else
        k_project_simple<float><<<cv.N, C, shm, st>>>(cv, (const float*)h, (const float*)w->WQ1, (const float*)w->WQ2,
                                                      (const float*)w->WK1, (const float*)w->WK2, (const float*)w->WV,
                                                      L, C, q, k, v);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
