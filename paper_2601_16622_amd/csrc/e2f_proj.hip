// Node-level stage: sorted positions, path-weighted P coefficients, and the l-wise projections
// Q1,Q2,K1,K2,V = W^(l) h^(l) with the invariant q,k of Eq. qk formed in the epilogue (Sec. 3.2).
//
// k_project_mfma: one wave owns 16 atoms (MFMA rows) of one degree l and a group of 16-wide output-channel
// tiles; for every order m it multiplies the 16 x C slab of h by W^T on the matrix cores and, for q and k,
// accumulates the element-wise product of the two projections over m, so Q1,Q2,K1,K2 never leave registers.
// k_project_simple is a plain one-thread-per-output version used by the materialized baseline.
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "e2f_device.h"

namespace {

// binary16 keeps |x| <= 65504: the invariants of Eq. qk are quadratic in the features, so un-normalised inputs can leave
// that range; they saturate instead of becoming infinite (an infinite logit would turn the softmax into NaN).  NaN stays.
__device__ __forceinline__ _Float16 to_f16_sat(float x) {
    return (_Float16)__builtin_amdgcn_fmed3f(x, -65504.0f, 65504.0f);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct CoefTable {
    float c[E2F_MAX_N][E2F_NP];
};

// spos[slot] = position of the atom in that slot (w carries its index in the caller's order); cw[comp][t] = P coefficient times its path weight.
__global__ void k_prepare(E2fCellsView cv, const float* __restrict__ pos, const float* __restrict__ w_path, int L,
                          int lf, CoefTable tab, float4* __restrict__ spos, float* __restrict__ cw,
                          const float* __restrict__ Wb, int H, int B, float* __restrict__ wbT) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < H * B) wbT[(t % B) * H + t / B] = Wb[t];
    if (t < cv.N) {
        const int a = cv.perm[t];
        float x = pos[3 * a], y = pos[3 * a + 1], z = pos[3 * a + 2];
        if (cv.periodic) {   // folded into the segment's box on its periodic axes
            const E2fSegGrid g = cv.grid[cv.sseg[t]];
            x = e2f::fold_coord(x, g.lx, g.rx);
            y = e2f::fold_coord(y, g.ly, g.ry);
            z = e2f::fold_coord(z, g.lz, g.rz);
        }
        spos[t] = make_float4(x, y, z, __int_as_float(a));   // w: the atom index
    }
    const int n = (L + 1) * (L + 1);
    if (t < n * E2F_NP) {
        const int comp = t / E2F_NP, kk = t % E2F_NP;
        int lo = 0;
        while ((lo + 1) * (lo + 1) <= comp) ++lo;
        const int li = lo - lf + kk;
        float w = 0.0f;
        if (kk <= 2 * lf && li >= 0 && li <= L) w = w_path[li * (L + 1) + lo];
        cw[t] = w * tab.c[comp][kk];
    }
}

// cw[comp][t] = P coefficient of the path into comp with every path weight one (w_path gradients).
__global__ void k_unit_cw(int L, int lf, CoefTable tab, float* __restrict__ cw) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    const int n = (L + 1) * (L + 1);
    if (t >= n * E2F_NP) return;
    const int comp = t / E2F_NP, kk = t % E2F_NP;
    int lo = 0;
    while ((lo + 1) * (lo + 1) <= comp) ++lo;
    const int li = lo - lf + kk;
    cw[t] = (kk <= 2 * lf && li >= 0 && li <= L) ? tab.c[comp][kk] : 0.0f;
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
// Stores cnt consecutive bf16 values val[0..cnt) at row[pos0..pos0+cnt): 4-byte stores wherever two neighbours
// share an aligned word, 2-byte stores at the ragged ends.  row is 4-byte aligned; pos0 and cnt are wave-uniform.
template <int MAXN>
__device__ __forceinline__ void store_run_bf16(uint16_t* row, int pos0, const float (&val)[MAXN], int cnt) {
    const int lead = pos0 & 1;
    if (lead && cnt > 0) row[pos0] = e2f::float_to_bf16_bits(val[0]);
#pragma unroll
    for (int k = 0; k + 1 < MAXN; ++k) {
        // pairs start at k = lead, lead + 2, ...
        if (((k - lead) & 1) == 0 && k >= lead && k + 1 < cnt) {
            const uint32_t w = (uint32_t)e2f::float_to_bf16_bits(val[k]) | ((uint32_t)e2f::float_to_bf16_bits(val[k + 1]) << 16);
            *reinterpret_cast<uint32_t*>(row + pos0 + k) = w;
        }
    }
#pragma unroll
    for (int k = 0; k < MAXN; ++k)
        if (k == cnt - 1 && k >= lead && ((k - lead) & 1) == 0) row[pos0 + k] = e2f::float_to_bf16_bits(val[k]);
}

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
            // v: one projection, stored per order (accumulator layout: lane (g, i) holds rows 4g + r, column i)
            typename F::type BV[NS];
#pragma unroll
            for (int S = 0; S < NS; ++S) BV[S] = F::load(WV + wr, S, g);
            f32x4 pv[MG];
#pragma unroll
            for (int mm = 0; mm < MG; ++mm) {
                pv[mm] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (m0 + mm < nl) {
#pragma unroll
                    for (int S = 0; S < NS; ++S) pv[mm] = F::mma(A[mm][S], BV[S], pv[mm]);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = tile * 16 + 4 * g + r;
                if (slot >= N) continue;
                if constexpr (!TILED) {
#pragma unroll
                    for (int mm = 0; mm < MG; ++mm)
                        if (m0 + mm < nl) e2f::store_from_float(v + ((size_t)slot * n + l * l + m0 + mm) * C + co, pv[mm][r]);
                } else {
                    const int NT = L >= 3 ? 2 : 1;
                    const int TI = l >= 3 ? 0 : NT - 1;
                    const int pos_l = l == 4 ? 0 : (l == 3 ? 9 : (l == 2 ? 0 : (l == 1 ? 5 : 8)));
                    uint16_t* row = reinterpret_cast<uint16_t*>(v) +
                                    ((((size_t)slot * (C / 16) + (co >> 4)) * NT + TI) * 16 + (co & 15)) * 16;
                    float val[MG];
#pragma unroll
                    for (int mm = 0; mm < MG; ++mm) val[mm] = pv[mm][r];
                    store_run_bf16<MG>(row, pos_l + m0, val, min(MG, nl - m0));
                    if (l == 0) {  // rows 9..15 of the LO tile are padding and must read as zero
                        const float zero[7] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        store_run_bf16<7>(row, 9, zero, 7);
                    }
                    if (l == 3 && L == 3 && m0 == 0) {  // without l = 4 the first nine HI rows are padding
                        const float zero[9] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        store_run_bf16<9>(row, 0, zero, 9);
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

// Weight-stationary variant for bf16 features (the fast path): a wave keeps the five 16 x C weight tiles of one
// degree l and one 16-channel output tile in registers as MFMA A operands and streams atoms through as B
// operands, 16 atoms x one order m at a time, with the next slab of h requested before the current one is used.
// Accumulator layout: lane (g, j) holds output channels 16*ct + 4g..4g+3 of atom j, so q and k go out as 16-byte
// stores and v as runs of consecutive orders.  All (l, channel tile) waves of one group of TPW atom tiles are
// dispatched back to back onto the same XCD, so that the partial rows they write (q, k rows are shared by the
// channel tiles, tiled v rows by two degrees) merge in that XCD's L2 before they reach memory, and the h rows
// they all read are fetched once.
template <int C, bool TILED>
__global__ __launch_bounds__(64) void k_project_ws(E2fCellsView cv, const uint16_t* __restrict__ h,
                                                   const uint16_t* __restrict__ WQ1, const uint16_t* __restrict__ WQ2,
                                                   const uint16_t* __restrict__ WK1, const uint16_t* __restrict__ WK2,
                                                   const uint16_t* __restrict__ WV, int L, int tpw,
                                                   float* __restrict__ q, float* __restrict__ k,
                                                   uint16_t* __restrict__ v) {
    typedef Frag<uint16_t> F;
    constexpr int NS = C / F::KSTEP;
    constexpr int NCT = C / 16;
    const int N = cv.N, n = (L + 1) * (L + 1);
    const int n_tiles = (N + 15) / 16;
    // block -> (XCD, position inside the XCD's queue) -> (group of atom tiles, degree, channel tile)
    const int per_group = (L + 1) * NCT;
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int group = (rest / per_group) * 8 + xcd, lc = rest % per_group;
    const int l = lc / NCT, ct = lc % NCT, nl = 2 * l + 1;
    const int lane = threadIdx.x, j = lane & 15, g = lane >> 4;
    const int tile0 = group * tpw, tile1 = min(tile0 + tpw, n_tiles);
    if (tile0 >= tile1) return;

    // stationary A operands: row (16 ct + j) of each weight matrix of degree l
    const size_t wrow = ((size_t)l * C + (ct * 16 + j)) * C;
    F::type Wf[5][NS];
#pragma unroll
    for (int S = 0; S < NS; ++S) {
        Wf[0][S] = F::load(WQ1 + wrow, S, g);
        Wf[1][S] = F::load(WQ2 + wrow, S, g);
        Wf[2][S] = F::load(WK1 + wrow, S, g);
        Wf[3][S] = F::load(WK2 + wrow, S, g);
        Wf[4][S] = F::load(WV + wrow, S, g);
    }

    auto load_x = [&](int tile, int m, F::type (&X)[NS]) {
        const int slot = min(tile * 16 + j, N - 1);  // clamped atoms are computed and not stored
        const uint16_t* row = h + ((size_t)cv.perm[slot] * n + l * l + m) * C;
#pragma unroll
        for (int S = 0; S < NS; ++S) X[S] = F::load(row, S, g);
    };

    // The weight tiles must have arrived before the streaming loads start: inside the loop the only loads in
    // flight are then the ring's own, in order, and the waits the compiler inserts leave PD-1 slabs outstanding
    // (with the weight loads still pending at loop entry every step would wait for everything).
    {
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int w = 0; w < 5; ++w)
#pragma unroll
            for (int S = 0; S < NS; ++S) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, Wf[w][S])));
    }
    // The (atom tile, order) steps of this wave form one sequence; PD slabs of h are in flight at any time
    // (memory latency is several steps long), in a ring of register buffers indexed at compile time.
    constexpr int PD = 4;
    const int n_steps = (tile1 - tile0) * nl;
    F::type X[PD][NS];
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        const int su = min(u, max(n_steps - 1, 0));
        load_x(tile0 + su / nl, su % nl, X[u]);
    }
    f32x4 qacc = {0.f, 0.f, 0.f, 0.f}, kacc = {0.f, 0.f, 0.f, 0.f};
    float vrun[4][2 * E2F_MAX_L + 1];
    // (full groups of PD steps without a check per step: the compiler sets its waits on the ring's loads by the fewest
    // memory instructions on any path from a request to its use, and a path that skips steps would make that one)
    auto step = [&](int st, int u) __attribute__((always_inline)) {
        const int tile = tile0 + st / nl, m = st % nl;
        const int slot = tile * 16 + j;
        // five independent accumulation chains, interleaved so that no MFMA waits for its predecessor
        f32x4 p[5];
#pragma unroll
        for (int w = 0; w < 5; ++w) p[w] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = 0; S < NS; ++S)
#pragma unroll
            for (int w = 0; w < 5; ++w) p[w] = F::mma(Wf[w][S], X[u][S], p[w]);
        // this buffer is free again: request the slab PD steps ahead (clamped to the last step)
        {
            const int sn = min(st + PD, n_steps - 1);
            load_x(tile0 + sn / nl, sn % nl, X[u]);
        }
        qacc += p[0] * p[1];
        kacc += p[2] * p[3];
        if constexpr (TILED) {
#pragma unroll
            for (int mm = 0; mm < 2 * E2F_MAX_L + 1; ++mm)
                if (mm == m) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) vrun[r][mm] = p[4][r];
                }
        } else if (slot < N) {
            uint16_t* dst = v + ((size_t)slot * n + l * l + m) * C + ct * 16 + 4 * g;
            const uint32_t w0 = (uint32_t)e2f::float_to_bf16_bits(p[4][0]) | ((uint32_t)e2f::float_to_bf16_bits(p[4][1]) << 16);
            const uint32_t w1 = (uint32_t)e2f::float_to_bf16_bits(p[4][2]) | ((uint32_t)e2f::float_to_bf16_bits(p[4][3]) << 16);
            *reinterpret_cast<uint2*>(dst) = make_uint2(w0, w1);
        }
        if (m == nl - 1) {  // last order of this atom tile: q, k (and the tiled v rows) go out
            if (slot < N) {
                *reinterpret_cast<f32x4*>(q + ((size_t)slot * (L + 1) + l) * C + ct * 16 + 4 * g) = qacc;
                *reinterpret_cast<f32x4*>(k + ((size_t)slot * (L + 1) + l) * C + ct * 16 + 4 * g) = kacc;
                if constexpr (TILED) {
                    const int NT = L >= 3 ? 2 : 1;
                    const int TI = l >= 3 ? 0 : NT - 1;
                    const int pos_l = l == 4 ? 0 : (l == 3 ? 9 : (l == 2 ? 0 : (l == 1 ? 5 : 8)));
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        uint16_t* row = v + ((((size_t)slot * NCT + ct) * NT + TI) * 16 + 4 * g + r) * 16;
                        store_run_bf16<2 * E2F_MAX_L + 1>(row, pos_l, vrun[r], nl);
                        if (l == 0) {
                            const float zero[7] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            store_run_bf16<7>(row, 9, zero, 7);
                        }
                        if (l == 3 && L == 3) {
                            const float zero[9] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                            store_run_bf16<9>(row, 0, zero, 9);
                        }
                    }
                }
            }
            qacc = (f32x4){0.f, 0.f, 0.f, 0.f};
            kacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    };
    int s0 = 0;
    for (; s0 + PD <= n_steps; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) step(s0 + u, u);
    }
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (s0 + u < n_steps) step(s0 + u, u);
}

// Weight-stationary projection for fp32 features (v_mfma_f32_16x16x4_f32), plain fp32 q, k, v.  The five fp32 weight
// tiles of one 16-channel output tile are 160 registers at 128 channels, so the work of an (atom tiles, degree) item
// is split between two kinds of waves: a QK wave keeps the four weight tiles of q and k for one output tile, a V wave
// the value weights of VT output tiles; both do 4 C / 16 chains of C / 4 matrix instructions per slab.  Each streams
// the slabs of h itself (PD in flight); the waves of one group of atom tiles go to one XCD, whose L2 serves the rows
// they share.  Block -> (XCD, group of atom tiles, degree, wave of the item) as in k_project_ws.
template <int C>
__global__ __launch_bounds__(64) void k_project_ws_f32(E2fCellsView cv, const float* __restrict__ h,
                                                       const float* __restrict__ WQ1, const float* __restrict__ WQ2,
                                                       const float* __restrict__ WK1, const float* __restrict__ WK2,
                                                       const float* __restrict__ WV, int L, int tpw,
                                                       float* __restrict__ q, float* __restrict__ k, float* __restrict__ v) {
    typedef Frag<float> F;
    constexpr int NS = C / F::KSTEP, NCT = C / 16, VT = 4, NVW = NCT / VT;   // V waves per item
    static_assert(NCT % VT == 0, "value waves take four output tiles each");
    const int N = cv.N, n = (L + 1) * (L + 1), n_tiles = (N + 15) / 16;
    const int per_group = (L + 1) * (NCT + NVW);
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int group = (rest / per_group) * 8 + xcd, lw = rest % per_group;
    const int l = lw / (NCT + NVW), wv = lw % (NCT + NVW), nl = 2 * l + 1;
    const bool value_wave = wv >= NCT;                 // (uniform)
    const int ct0 = value_wave ? (wv - NCT) * VT : wv;   // first output tile of this wave
    const int lane = threadIdx.x, j = lane & 15, g = lane >> 4;
    const int tile0 = group * tpw, tile1 = min(tile0 + tpw, n_tiles);
    if (tile0 >= tile1) return;
    // four stationary weight tiles: (WQ1, WQ2, WK1, WK2) of output tile ct0, or WV of output tiles ct0 .. ct0 + 3
    F::type Wf[4][NS];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float* W = value_wave ? WV : (t == 0 ? WQ1 : t == 1 ? WQ2 : t == 2 ? WK1 : WK2);
        const size_t wrow = ((size_t)l * C + ((ct0 + (value_wave ? t : 0)) * 16 + j)) * C;
#pragma unroll
        for (int S = 0; S < NS; ++S) Wf[t][S] = F::load(W + wrow, S, g);
    }
    auto load_x = [&](int tile, int m, F::type (&X)[NS]) {
        const int slot = min(tile * 16 + j, N - 1);  // clamped atoms are computed and not stored
        const float* row = h + ((size_t)cv.perm[slot] * n + l * l + m) * C;
#pragma unroll
        for (int S = 0; S < NS; ++S) X[S] = F::load(row, S, g);
    };
    {   // the weights have arrived before the stream starts: inside it only the ring's own loads are in flight
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int S = 0; S < NS; ++S) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, Wf[t][S])));
    }
    constexpr int PD = 2;
    const int n_steps = (tile1 - tile0) * nl;
    F::type X[PD][NS];
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        const int su = min(u, n_steps - 1);
        load_x(tile0 + su / nl, su % nl, X[u]);
    }
    f32x4 qacc = {0.f, 0.f, 0.f, 0.f}, kacc = {0.f, 0.f, 0.f, 0.f};
    // (full groups of PD steps without a check per step: the compiler sets its waits on the ring's loads by the fewest
    // memory instructions on any path from a request to its use, and a path that skips steps would make that one)
    auto step = [&](int st, int u) __attribute__((always_inline)) {
        const int tile = tile0 + st / nl, m = st % nl;
        const int slot = tile * 16 + j;
        // four independent chains, interleaved so that no matrix instruction waits for its predecessor
        f32x4 p[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) p[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = 0; S < NS; ++S)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    p[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(Wf[t][S][e], X[u][S][e], p[t], 0, 0, 0);
        {   // this buffer is free again: request the slab PD steps ahead (clamped to the last step)
            const int sn = min(st + PD, n_steps - 1);
            load_x(tile0 + sn / nl, sn % nl, X[u]);
        }
        // accumulator layout: lane (g, j) holds output channels 4g .. 4g + 3 of atom j
        if (value_wave) {
            if (slot < N) {
                float* dst = v + ((size_t)slot * n + l * l + m) * C + ct0 * 16 + 4 * g;
#pragma unroll
                for (int t = 0; t < 4; ++t) *reinterpret_cast<f32x4*>(dst + 16 * t) = p[t];
            }
        } else {
            qacc += p[0] * p[1];
            kacc += p[2] * p[3];
            if (m == nl - 1) {   // last order of this atom tile: q and k of the degree go out
                if (slot < N) {
                    *reinterpret_cast<f32x4*>(q + ((size_t)slot * (L + 1) + l) * C + ct0 * 16 + 4 * g) = qacc;
                    *reinterpret_cast<f32x4*>(k + ((size_t)slot * (L + 1) + l) * C + ct0 * 16 + 4 * g) = kacc;
                }
                qacc = (f32x4){0.f, 0.f, 0.f, 0.f};
                kacc = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    int s0 = 0;
    for (; s0 + PD <= n_steps; s0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) step(s0 + u, u);
    }
#pragma unroll
    for (int u = 0; u < PD; ++u)
        if (s0 + u < n_steps) step(s0 + u, u);
}

// Workgroup variant of the weight-stationary projection for the tiled v layout.  Global stores inside the
// streaming loop would share the wave's memory counter with the prefetched loads and force every wait to drain
// all of them, so nothing is stored while streaming: three waves split the degrees of one (32 atoms, 16
// channels) block between them (balanced by their number of orders), put q, k and the bf16 v tiles into LDS,
// and after a barrier the whole workgroup copies the finished block out with 16-byte, fully coalesced stores
// (every (atom, head) owns 1 KB of contiguous v).
constexpr int WG_TPW = 2;      // atom tiles (of 16) per workgroup
constexpr int WG_WAVES = 3;
struct WgRoles {
    int n_deg[WG_WAVES];
    int deg[WG_WAVES][E2F_MAX_L + 1];
};

// Outputs in the layout of the tile attention kernel (VL = 2): q and k per head in binary16, DKP = (L+1)*16
// features padded to a multiple of 32 (q times qscale), and v in groups of four consecutive slots,
// bf16 [slot/4][head][component][16 channels][4 slots]; rows beyond N read as zero.
struct WgGroupOut {
    uint16_t *q16, *k16, *v4;
    float qscale;
    int DKP;
};

template <int C, int VL>
__global__ __launch_bounds__(64 * WG_WAVES) void k_project_wg(E2fCellsView cv, const uint16_t* __restrict__ h,
                                                              const uint16_t* __restrict__ WQ1,
                                                              const uint16_t* __restrict__ WQ2,
                                                              const uint16_t* __restrict__ WK1,
                                                              const uint16_t* __restrict__ WK2,
                                                              const uint16_t* __restrict__ WV, int L, WgRoles roles,
                                                              float* __restrict__ q, float* __restrict__ k,
                                                              uint16_t* __restrict__ v, WgGroupOut go) {
    typedef Frag<uint16_t> F;
    constexpr int NS = C / F::KSTEP;
    constexpr int NCT = C / 16;
    constexpr int PD = 4;
    __shared__ __attribute__((aligned(16))) uint16_t s_v[WG_TPW * 16 * 2 * 256];          // [tile][atom][T][ch][pos]
    __shared__ __attribute__((aligned(16))) float s_q[WG_TPW * 16 * (E2F_MAX_L + 1) * 16];  // [tile][atom][l][ch]
    __shared__ __attribute__((aligned(16))) float s_k[WG_TPW * 16 * (E2F_MAX_L + 1) * 16];

    const int N = cv.N, n = (L + 1) * (L + 1), NT = L >= 3 ? 2 : 1;
    const int n_tiles = (N + 15) / 16;
    const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
    const int group = (rest / NCT) * 8 + xcd, ct = rest % NCT;
    const int tile0 = group * WG_TPW, tile1 = min(tile0 + WG_TPW, n_tiles);
    if (tile0 >= tile1) return;   // whole workgroup leaves together
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, j = lane & 15, g = lane >> 4;

    for (int x = tid; x < WG_TPW * 16 * 2 * 256 / 8; x += 64 * WG_WAVES)
        reinterpret_cast<uint4*>(s_v)[x] = make_uint4(0u, 0u, 0u, 0u);   // padding rows must read as zero
    // Atom index of this lane's row in every tile, fetched once: an index load inside the streaming loop would
    // have to be waited for, and waiting for the youngest load drains all the older ones.
    int atom_of[WG_TPW];
#pragma unroll
    for (int x = 0; x < WG_TPW; ++x) atom_of[x] = cv.perm[min((tile0 + x) * 16 + j, N - 1)];
    __syncthreads();

    for (int di = 0; di < roles.n_deg[wave]; ++di) {
        const int l = roles.deg[wave][di], nl = 2 * l + 1;
        const size_t wrow = ((size_t)l * C + (ct * 16 + j)) * C;
        F::type Wf[5][NS];
#pragma unroll
        for (int S = 0; S < NS; ++S) {
            Wf[0][S] = F::load(WQ1 + wrow, S, g);
            Wf[1][S] = F::load(WQ2 + wrow, S, g);
            Wf[2][S] = F::load(WK1 + wrow, S, g);
            Wf[3][S] = F::load(WK2 + wrow, S, g);
            Wf[4][S] = F::load(WV + wrow, S, g);
        }
        {   // the weight tiles must have arrived before the streaming loads start (see k_project_ws)
            typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int w = 0; w < 5; ++w)
#pragma unroll
                for (int S = 0; S < NS; ++S) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, Wf[w][S])));
        }
        const int n_steps = (tile1 - tile0) * nl;
        auto load_x = [&](int st, F::type (&X)[NS]) {
            const int lt = st / nl, m = st - lt * nl;
            int atom = atom_of[0];
#pragma unroll
            for (int x = 1; x < WG_TPW; ++x) atom = (lt == x) ? atom_of[x] : atom;
            const uint16_t* row = h + ((size_t)atom * n + l * l + m) * C;
#pragma unroll
            for (int S = 0; S < NS; ++S) X[S] = F::load(row, S, g);
        };
        F::type X[PD][NS];
#pragma unroll
        for (int u = 0; u < PD; ++u) load_x(min(u, n_steps - 1), X[u]);
        const int TI = l >= 3 ? 0 : NT - 1;
        const int pos_l = l == 4 ? 0 : (l == 3 ? 9 : (l == 2 ? 0 : (l == 1 ? 5 : 8)));
        f32x4 qacc = {0.f, 0.f, 0.f, 0.f}, kacc = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < n_steps; s0 += PD) {
#pragma unroll
            for (int u = 0; u < PD; ++u) {
                const int st = s0 + u;
                if (st < n_steps) {
                    const int lt = st / nl, m = st - lt * nl;   // local tile, order
                    f32x4 p[5];
#pragma unroll
                    for (int w = 0; w < 5; ++w) p[w] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int S = 0; S < NS; ++S)
#pragma unroll
                        for (int w = 0; w < 5; ++w) p[w] = F::mma(Wf[w][S], X[u][S], p[w]);
                    load_x(min(st + PD, n_steps - 1), X[u]);
                    qacc += p[0] * p[1];
                    kacc += p[2] * p[3];
                    // accumulator layout: lane (g, j) holds channels 4g..4g+3 of atom j
                    uint16_t* vrow = s_v + (((lt * 16 + j) * 2 + TI) * 16 + 4 * g) * 16 + pos_l + m;
#pragma unroll
                    for (int r = 0; r < 4; ++r) vrow[r * 16] = e2f::float_to_bf16_bits(p[4][r]);
                    if (m == nl - 1) {
                        *reinterpret_cast<f32x4*>(s_q + ((lt * 16 + j) * (E2F_MAX_L + 1) + l) * 16 + 4 * g) = qacc;
                        *reinterpret_cast<f32x4*>(s_k + ((lt * 16 + j) * (E2F_MAX_L + 1) + l) * 16 + 4 * g) = kacc;
                        qacc = (f32x4){0.f, 0.f, 0.f, 0.f};
                        kacc = (f32x4){0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
    }
    __syncthreads();
    // ---- copy out: v, 16 bytes per thread; every (atom, head = ct) block of NT*512 bytes is contiguous
    const int n_atoms = min(tile1 * 16, N) - tile0 * 16;
    if constexpr (VL == 2) {
        const int n_groups = (n_atoms + 3) >> 2;
        // v: 16-byte units of two channels, 8 bytes (four slots) per (group, component, channel)
        for (int x = tid; x < n_groups * n * 8; x += 64 * WG_WAVES) {
            const int gl = x / (n * 8), rem = x - gl * n * 8, comp = rem >> 3, ch = (rem & 7) * 2;
            int l = 0;
            while ((l + 1) * (l + 1) <= comp) ++l;
            const int m = comp - l * l;
            const int T = l >= 3 ? 0 : NT - 1;
            const int pos = (l == 4 ? 0 : (l == 3 ? 9 : (l == 2 ? 0 : (l == 1 ? 5 : 8)))) + m;
            uint16_t val[8];
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int a = 4 * gl + i;
                    val[4 * s2 + i] = a < n_atoms ? s_v[((a * 2 + T) * 16 + ch + s2) * 16 + pos] : (uint16_t)0;
                }
            uint2 pk0, pk1;   // the four slots of (comp, ch) and of (comp, ch + 1)
            pk0.x = val[0] | ((uint32_t)val[1] << 16);
            pk0.y = val[2] | ((uint32_t)val[3] << 16);
            pk1.x = val[4] | ((uint32_t)val[5] << 16);
            pk1.y = val[6] | ((uint32_t)val[7] << 16);
            uint16_t* blk = go.v4 + (((size_t)tile0 * 4 + gl) * NCT + ct) * n * 64;
            *reinterpret_cast<uint2*>(blk + e2f::v4_offset(n, comp, ch)) = pk0;
            *reinterpret_cast<uint2*>(blk + e2f::v4_offset(n, comp, ch + 1)) = pk1;
        }
        // q, k: 16-byte units of eight features (feature = l*16 + channel) in binary16
        const int u_per = go.DKP >> 3, DK = (L + 1) * 16;
        for (int x = tid; x < n_groups * 4 * u_per; x += 64 * WG_WAVES) {
            const int a = x / u_per, f0 = (x - a * u_per) * 8;
            const size_t slot = (size_t)tile0 * 16 + a;
            typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
            h16x8 qv, kv;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool real = a < n_atoms && f0 + i < DK;
                qv[i] = to_f16_sat(real ? s_q[a * (E2F_MAX_L + 1) * 16 + f0 + i] * go.qscale : 0.0f);
                kv[i] = to_f16_sat(real ? s_k[a * (E2F_MAX_L + 1) * 16 + f0 + i] : 0.0f);
            }
            const size_t dst = (slot * NCT + ct) * go.DKP + f0;
            *reinterpret_cast<h16x8*>(go.k16 + e2f::k16_offset(slot, NCT, ct, go.DKP, f0)) = kv;
            if (a < n_atoms) *reinterpret_cast<h16x8*>(go.q16 + dst) = qv;
        }
        return;
    }
    const int v_chunks = NT * 32;   // 16-byte chunks per atom
    for (int x = tid; x < n_atoms * v_chunks; x += 64 * WG_WAVES) {
        const int a = x / v_chunks, c16 = x - a * v_chunks;
        const int T = NT == 2 ? c16 / 32 : 0, inner = c16 % 32;
        const uint4 val = *reinterpret_cast<const uint4*>(s_v + ((a * 2 + T) * 256) + inner * 8);
        const size_t slot = (size_t)tile0 * 16 + a;
        *reinterpret_cast<uint4*>(v + ((slot * NCT + ct) * NT) * 256 + c16 * 8) = val;
    }
    // q and k: 64 contiguous bytes per (atom, degree)
    for (int x = tid; x < n_atoms * (L + 1) * 4; x += 64 * WG_WAVES) {
        const int a = x / ((L + 1) * 4), rem = x - a * (L + 1) * 4, l = rem >> 2, c4 = rem & 3;
        const size_t slot = (size_t)tile0 * 16 + a;
        const size_t dst = (slot * (L + 1) + l) * C + ct * 16 + c4 * 4;
        *reinterpret_cast<f32x4*>(q + dst) = *reinterpret_cast<const f32x4*>(s_q + (a * (E2F_MAX_L + 1) + l) * 16 + c4 * 4);
        *reinterpret_cast<f32x4*>(k + dst) = *reinterpret_cast<const f32x4*>(s_k + (a * (E2F_MAX_L + 1) + l) * 16 + c4 * 4);
    }
}

// Shared-slab projection for the layout of the tile attention kernel.  One workgroup owns (up to SH_TPW tiles of 16
// atoms, one degree l) and all output channels: wave ct holds the five 16 x C weight tiles of that degree for output
// channels 16 ct .. 16 ct + 15 as MFMA A operands (fetched once per workgroup); one more wave does nothing but fetch
// the next (atom tile, order) slab of h into LDS, where all the other waves read it as their B operand.  Every h row
// is fetched once (the per-channel-tile kernels above fetch it C/16 times) and a weight tile once per 64 atoms.  The
// fetching wave stores nothing and the computing waves load nothing inside the stream, so no wait ever covers a
// store and the outputs go straight from registers to memory: q and k of the degree after a tile's last order
// (binary16, 8 bytes per lane), v after a 16 x 16 transpose through a private 512-byte LDS patch (bf16, the four slots
// of a (component, channel) per lane).  Workgroups of the highest degree (most orders) are launched first.
constexpr int SH_TPW = 16;   // most tiles a workgroup takes; the launcher picks 4, 8 or 16 from the problem size
// CW: computing waves per workgroup.  C / 16 of them (all output channels in one workgroup) up to 128 channels; at 256
// channels a wave's five weight tiles are 160 registers, which leaves room for two waves per SIMD only, so a
// workgroup has four computing waves (64 output channels) and four workgroups share an (atom tiles, degree) item,
// each fetching its slabs itself; they are dispatched one after the other onto the same XCD, whose L2 serves the
// repeated rows.
template <int C, int CW = C / 16>
__global__ __launch_bounds__(64 * (CW + 1)) void k_project_sh(E2fCellsView cv, const uint16_t* __restrict__ h,
                                                                 const uint16_t* __restrict__ WQ1,
                                                                 const uint16_t* __restrict__ WQ2,
                                                                 const uint16_t* __restrict__ WK1,
                                                                 const uint16_t* __restrict__ WK2,
                                                                 const uint16_t* __restrict__ WV, int L, int n_groups,
                                                                 int tpw, WgGroupOut go) {
    typedef Frag<uint16_t> F;
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
    constexpr int NS = C / F::KSTEP, NCT = C / 16, ROW = C + 8, NLD = C / 32;   // NLD 16-byte loads per lane and slab
    constexpr int NCG = NCT / CW;   // workgroups per item
    static_assert(NCT % CW == 0, "whole groups of output tiles");
    __shared__ __attribute__((aligned(16))) uint16_t s_x[4][16 * ROW];   // slab st in buffer st mod 4
    __shared__ __attribute__((aligned(8))) uint16_t s_t[CW][256];
    __shared__ int s_vst[2 * E2F_MAX_L + 1];   // where the value rows of order m go (see below)
    __shared__ int s_atom[SH_TPW * 16];   // fetching wave: atom of every row of the workgroup's tiles
    const int N = cv.N, n = (L + 1) * (L + 1), n_tiles = (N + 15) / 16, N4 = (N + 3) / 4 * 4;
    int l, group, cg = 0;
    if constexpr (NCG == 1) {
        l = L - (int)blockIdx.x / n_groups;
        group = (int)blockIdx.x % n_groups;
    } else {   // per degree ceil(n_groups / 8) * 8 * NCG workgroups: block -> (XCD, group of atom tiles, channel group)
        const int per_deg = (n_groups + 7) / 8 * 8 * NCG, idx = (int)blockIdx.x % per_deg;
        l = L - (int)blockIdx.x / per_deg;
        group = ((idx >> 3) / NCG) * 8 + (idx & 7);
        cg = (idx >> 3) % NCG;
        if (group >= n_groups) return;   // whole workgroup
    }
    const int nl = 2 * l + 1;
    const int tile0 = group * tpw, nt = min(tpw, n_tiles - tile0);
    // (the wave's index through readfirstlane: the compiler then knows it, and the addresses built from it, to be the
    // same in all lanes and keeps them in scalar registers)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, j = lane & 15, g = lane >> 4;
    const int n_steps = nt * nl;   // step = local tile * nl + order
    // Where the value rows of component l*l + m go in the layout of e2f::v4_offset: (offset of channel 0) << 4 | number
    // of elements from one channel to the next (4 for a lone component, 8 inside a pair).
    if ((int)threadIdx.x < nl) {
        const int x = l * l + (int)threadIdx.x;
        s_vst[threadIdx.x] = (e2f::v4_offset(n, x, 0) << 4) | (e2f::v4_role(n, x) == 0 ? 4 : 8);
    }

    if (wave == CW) {
        // ---- the fetching wave: lane = (atom a of the tile, quarter of its row)
        // The atoms of the workgroup's tiles go through LDS: indexed by the local tile in registers they end up in
        // scratch memory, whose loads share the memory counter with the slab loads and are the youngest of them, so
        // that waiting for an atom index drained every slab in flight.
        const int a = lane >> 2, part = lane & 3;
        for (int x = part; x < SH_TPW; x += 4) s_atom[x * 16 + a] = cv.perm[min((tile0 + min(x, nt - 1)) * 16 + a, N - 1)];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        auto issue = [&](int st, u32x4 (&r)[NLD]) {
            st = min(st, n_steps - 1);
            const int lt = st / nl, m = st - lt * nl;
            const int atom = s_atom[lt * 16 + a];
            const uint16_t* row = h + ((size_t)atom * n + l * l + m) * C + part * (C / 4);
#pragma unroll
            for (int i = 0; i < NLD; ++i) r[i] = *reinterpret_cast<const u32x4*>(row + 8 * i);
        };
        auto put = [&](int buf, const u32x4 (&r)[NLD]) {
            uint16_t* d = s_x[buf] + a * ROW + part * (C / 4);
#pragma unroll
            for (int i = 0; i < NLD; ++i) *reinterpret_cast<u32x4*>(d + 8 * i) = r[i];
        };
        // The computing waves take two slabs per step (st, st + 1: two independent chains of matrix products, one
        // barrier).  Slabs st + 2 and st + 3 are written to LDS meanwhile (four buffers); slab k travels in r[k mod PD],
        // whose registers then take slab k + PD, so PD slabs are in flight at any time.
        constexpr int PD = 6;
        static_assert(PD % 2 == 0, "slabs are handed over in pairs");
        u32x4 r[PD][NLD];
#pragma unroll
        for (int u = 0; u < PD; ++u) issue(u, r[u]);
        put(0, r[0]);
        issue(PD, r[0]);
        put(1, r[1]);
        issue(PD + 1, r[1]);
        __syncthreads();
        // (the full groups of PD slabs without a check per pair: the compiler sets its waits on the loads by the
        // fewest memory instructions on any path from a request to its use, and a path that skips pairs would make
        // it wait for requests one pair old)
        auto pair = [&](int st, int u) __attribute__((always_inline)) {
            put((st + 2) & 3, r[(u + 2) % PD]);
            issue(st + 2 + PD, r[(u + 2) % PD]);
            put((st + 3) & 3, r[(u + 3) % PD]);
            issue(st + 3 + PD, r[(u + 3) % PD]);
            __syncthreads();
        };
        int s0 = 0;
        for (; s0 + PD <= n_steps; s0 += PD) {
#pragma unroll
            for (int u = 0; u < PD; u += 2) pair(s0 + u, u);
        }
#pragma unroll
        for (int u = 0; u < PD; u += 2)
            if (s0 + u < n_steps) pair(s0 + u, u);
        return;
    }

    // ---- the computing waves
    const int ct = cg * CW + wave;
    F::type Wf[5][NS];
    {   // weights of the degree; they must have arrived before the stream starts, so that inside it the wave's
        // memory counter only ever holds stores, which nothing waits for
        const size_t wrow = ((size_t)l * C + (ct * 16 + j)) * C;
#pragma unroll
        for (int S = 0; S < NS; ++S) {
            Wf[0][S] = F::load(WQ1 + wrow, S, g);
            Wf[1][S] = F::load(WQ2 + wrow, S, g);
            Wf[2][S] = F::load(WK1 + wrow, S, g);
            Wf[3][S] = F::load(WK2 + wrow, S, g);
            Wf[4][S] = F::load(WV + wrow, S, g);
        }
#pragma unroll
        for (int w = 0; w < 5; ++w)
#pragma unroll
            for (int S = 0; S < NS; ++S) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, Wf[w][S])));
    }
    f32x4 qacc = {0.f, 0.f, 0.f, 0.f}, kacc = {0.f, 0.f, 0.f, 0.f};
    const int DK = (L + 1) * 16;
    __syncthreads();
    // what follows the matrix products of one slab (local tile lt, order m)
    auto finish_slab = [&](int st, const f32x4 (&p)[5]) {
        const int lt = st / nl, m = st - lt * nl;
        qacc += p[0] * p[1];
        kacc += p[2] * p[3];
        // accumulator layout: lane (g, j) holds output channels 4g..4g+3 of atom j
        const int slot = (tile0 + lt) * 16 + j;
        {   // v: [channel][atom] patch, then one (channel, group of four slots) per lane
            const int vst = s_vst[m];   // (offset of channel 0) << 4 | elements between channels
            uint16_t* patch = s_t[wave];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                patch[(4 * g + r) * 16 + j] = slot < N ? e2f::float_to_bf16_bits(p[4][r]) : (uint16_t)0;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            const int ch = lane >> 2, G = lane & 3;
            const u32x2 unit = *reinterpret_cast<const u32x2*>(patch + ch * 16 + 4 * G);
            // the tile's part of the address is the same for the whole wave, the lane's part fits 32 bits
            uint16_t* tile_v = go.v4 + (size_t)(tile0 + lt) * 4 * NCT * n * 64;
            const unsigned lane_v = (unsigned)((G * NCT + ct) * n * 64 + (vst >> 4) + ch * (vst & 15));
            if (((tile0 + lt) * 4 + G) * 4 < N) *reinterpret_cast<u32x2*>(tile_v + lane_v) = unit;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
        }
        if (m == nl - 1) {   // last order of this tile: q and k of the degree go out
            h16x4 qv, kv;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                qv[r] = to_f16_sat(qacc[r] * go.qscale);
                kv[r] = to_f16_sat(slot < N ? kacc[r] : 0.0f);
            }
            // Addresses as (the tile's part, the same in all lanes) + (the lane's part, 32 bits), the lane's part
            // hidden from the optimizer: hoisted out of the loop as 64-bit addresses per lane they were spilled, and
            // a reload from scratch memory waits for every store in flight.
            const int KS = go.DKP >> 5;
            uint16_t* tile_q = go.q16 + (size_t)(tile0 + lt) * 16 * NCT * go.DKP;
            uint16_t* tile_k = go.k16 + (size_t)(tile0 + lt) * 4 * NCT * KS * 128;
            unsigned jj = (unsigned)j, g4 = 4u * (unsigned)g;
            asm volatile("" : "+v"(jj), "+v"(g4));
            auto lane_q = [&](unsigned f) { return (jj * NCT + ct) * go.DKP + f; };
            auto lane_k = [&](unsigned f) { return (((jj >> 2) * NCT + ct) * KS + (f >> 5)) * 128 + (jj & 3) * 32 + (f & 31); };
            if (slot < N) *reinterpret_cast<h16x4*>(tile_q + lane_q(l * 16 + g4)) = qv;
            if (slot < N4) *reinterpret_cast<h16x4*>(tile_k + lane_k(l * 16 + g4)) = kv;
            if (l == L && go.DKP > DK) {   // padding features read as zero
                const h16x4 zero = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
                if (slot < N) *reinterpret_cast<h16x4*>(tile_q + lane_q(DK + g4)) = zero;
                if (slot < N4) *reinterpret_cast<h16x4*>(tile_k + lane_k(DK + g4)) = zero;
            }
            qacc = (f32x4){0.f, 0.f, 0.f, 0.f};
            kacc = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    };
    for (int st = 0; st < n_steps; st += 2) {
        // two slabs per step: their products are independent chains, interleaved
        const uint16_t* xa = s_x[st & 3] + j * ROW;
        const uint16_t* xb = s_x[(st + 1) & 3] + j * ROW;   // (past the last slab: a copy of it, not used)
        f32x4 pa[5], pb[5];
#pragma unroll
        for (int w = 0; w < 5; ++w) pa[w] = pb[w] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int S = 0; S < NS; ++S) {
            const F::type Xa = F::load(xa, S, g), Xb = F::load(xb, S, g);
#pragma unroll
            for (int w = 0; w < 5; ++w) {
                pa[w] = F::mma(Wf[w][S], Xa, pa[w]);
                pb[w] = F::mma(Wf[w][S], Xb, pb[w]);
            }
        }
        finish_slab(st, pa);
        if (st + 1 < n_steps) finish_slab(st + 1, pb);
        __syncthreads();
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
        // few atoms: one channel tile per wave gives CT times the waves (each h slab is then fetched C/16 times)
        const int waves_ct = (cv.N + 15) / 16 * (ctx->cfg.L_max + 1) * (C / 16 / CT);
        auto go = [&](auto ct_tag) {
            constexpr int ct = decltype(ct_tag)::value;
            const dim3 grid((cv.N + 15) / 16, ctx->cfg.L_max + 1, C / 16 / ct);
            if (tiled)
                k_project_mfma<T, C, MG, ct, true><<<grid, 64, 0, st>>>(cv, (const T*)h, (const T*)w->WQ1, (const T*)w->WQ2,
                                                                       (const T*)w->WK1, (const T*)w->WK2, (const T*)w->WV,
                                                                       ctx->cfg.L_max, ws.q, ws.k, (T*)ws.v);
            else
                k_project_mfma<T, C, MG, ct, false><<<grid, 64, 0, st>>>(cv, (const T*)h, (const T*)w->WQ1, (const T*)w->WQ2,
                                                                        (const T*)w->WK1, (const T*)w->WK2, (const T*)w->WV,
                                                                        ctx->cfg.L_max, ws.q, ws.k, (T*)ws.v);
        };
        if (CT > 1 && waves_ct < 4096)
            go(std::integral_constant<int, 1>{});
        else
            go(std::integral_constant<int, CT>{});
        return true;
    }
}

template <int C>
bool launch_ws(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
               hipStream_t st, bool tiled) {
    if constexpr (C % 32 != 0 || C > 256) {
        return false;   // five stationary weight tiles must fit the register file
    } else {
        const int L = ctx->cfg.L_max, n_tiles = (cv.N + 15) / 16;
        const int tpw = 4;
        const int groups = (n_tiles + tpw - 1) / tpw;
        const int blocks = ((groups + 7) / 8) * (L + 1) * (C / 16) * 8;
        const uint16_t* hh = (const uint16_t*)h;
        if (tiled)
            k_project_ws<C, true><<<blocks, 64, 0, st>>>(cv, hh, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2,
                                                         (const uint16_t*)w->WK1, (const uint16_t*)w->WK2,
                                                         (const uint16_t*)w->WV, L, tpw, ws.q, ws.k, (uint16_t*)ws.v);
        else
            k_project_ws<C, false><<<blocks, 64, 0, st>>>(cv, hh, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2,
                                                          (const uint16_t*)w->WK1, (const uint16_t*)w->WK2,
                                                          (const uint16_t*)w->WV, L, tpw, ws.q, ws.k, (uint16_t*)ws.v);
        return true;
    }
}

template <int C>
bool launch_ws_f32(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                   hipStream_t st) {
    const int L = ctx->cfg.L_max, n_tiles = (cv.N + 15) / 16;
    // more tiles per wave fetch the weights less often; keep two rounds of waves for the chip (2048 fit at a time)
    const int per_group = (L + 1) * (C / 16 + C / 64);
    int tpw = 4;
    while (tpw > 1 && (n_tiles + tpw - 1) / tpw * per_group < 4096) tpw >>= 1;
    const int groups = (n_tiles + tpw - 1) / tpw;
    const int blocks = ((groups + 7) / 8) * per_group * 8;
    k_project_ws_f32<C><<<blocks, 64, 0, st>>>(cv, (const float*)h, (const float*)w->WQ1, (const float*)w->WQ2,
                                               (const float*)w->WK1, (const float*)w->WK2, (const float*)w->WV, L, tpw,
                                               ws.q, ws.k, (float*)ws.v);
    return true;
}
bool dispatch_ws_f32(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                     hipStream_t st) {
    // While the features fit the caches the per-tile kernel, which fetches its weights per wave, is a little faster
    // (0.29 against 0.33 ms at 6000 atoms, 128 channels, L = 4: 77 MB of features); beyond, it falls off (0.93
    // against 0.42 ms at 8000 atoms, 1.16 against 0.47 at 10 000).
    if ((long long)cv.N * ctx->n * ctx->cfg.C * 4 < (80ll << 20)) return false;
    switch (ctx->cfg.C) {
        case 64: return launch_ws_f32<64>(ctx, cv, h, w, ws, st);
        case 128: return launch_ws_f32<128>(ctx, cv, h, w, ws, st);
    }
    return false;
}

// 256 channels into the tile layouts: four workgroups of four computing waves per (atom tiles, degree).
bool launch_sh256(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                  hipStream_t st) {
    const int L = ctx->cfg.L_max, n_tiles = (cv.N + 15) / 16;
    WgGroupOut go;
    go.q16 = ws.q16; go.k16 = ws.k16; go.v4 = ws.v4;
    go.qscale = ctx->tau * 1.44269504088896341f;   // logits in base-2 units
    go.DKP = ((L + 1) * 16 + 31) / 32 * 32;
    int tpw = SH_TPW;
    while (tpw > 4 && (n_tiles + tpw - 1) / tpw * (L + 1) < 384) tpw >>= 1;
    const int n_groups = (n_tiles + tpw - 1) / tpw;
    k_project_sh<256, 4><<<(n_groups + 7) / 8 * 8 * 4 * (L + 1), 64 * 5, 0, st>>>(
        cv, (const uint16_t*)h, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,
        (const uint16_t*)w->WK2, (const uint16_t*)w->WV, L, n_groups, tpw, go);
    return true;
}

template <int C>
bool launch_wg(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
               hipStream_t st, int v_layout) {
    if constexpr (C % 32 != 0 || C > 128) {
        return false;
    } else {
        const int L = ctx->cfg.L_max, n_tiles = (cv.N + 15) / 16;
        // degrees, largest first, each to the wave with the least work so far
        WgRoles roles;
        int load[WG_WAVES];
        for (int wv = 0; wv < WG_WAVES; ++wv) { roles.n_deg[wv] = 0; load[wv] = 0; }
        for (int l = L; l >= 0; --l) {
            int best = 0;
            for (int wv = 1; wv < WG_WAVES; ++wv)
                if (load[wv] < load[best]) best = wv;
            roles.deg[best][roles.n_deg[best]++] = l;
            load[best] += 2 * l + 1;
        }
        const int groups = (n_tiles + WG_TPW - 1) / WG_TPW;
        const int blocks = ((groups + 7) / 8) * 8 * (C / 16);
        WgGroupOut go;
        go.q16 = ws.q16; go.k16 = ws.k16; go.v4 = ws.v4;
        go.qscale = ctx->tau * 1.44269504088896341f;   // logits in base-2 units
        go.DKP = ((L + 1) * 16 + 31) / 32 * 32;
        const bool use_sh = !(ctx->cfg.flags & E2F_FLAG_PROJECT_PER_CHANNEL_TILE);
        if (v_layout == 2 && use_sh) {
            // More tiles per workgroup fetch the weights less often and pay the start of a workgroup's stream less
            // often; keep a few workgroups per CU.  (Splitting the work into equal numbers of slabs per workgroup,
            // whatever the degree, measured slower at every size tried: 75 to 105 us against 70 at 10 000 atoms.)
            int tpw = SH_TPW;
            while (tpw > 4 && (n_tiles + tpw - 1) / tpw * (L + 1) < 384) tpw >>= 1;
            const int n_groups = (n_tiles + tpw - 1) / tpw;
            k_project_sh<C><<<n_groups * (L + 1), 64 * (C / 16 + 1), 0, st>>>(
                cv, (const uint16_t*)h, (const uint16_t*)w->WQ1, (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,
                (const uint16_t*)w->WK2, (const uint16_t*)w->WV, L, n_groups, tpw, go);
        } else if (v_layout == 2)
            k_project_wg<C, 2><<<blocks, 64 * WG_WAVES, 0, st>>>(cv, (const uint16_t*)h, (const uint16_t*)w->WQ1,
                                                                (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,
                                                                (const uint16_t*)w->WK2, (const uint16_t*)w->WV, L, roles,
                                                                ws.q, ws.k, (uint16_t*)ws.v, go);
        else
            k_project_wg<C, 1><<<blocks, 64 * WG_WAVES, 0, st>>>(cv, (const uint16_t*)h, (const uint16_t*)w->WQ1,
                                                                (const uint16_t*)w->WQ2, (const uint16_t*)w->WK1,
                                                                (const uint16_t*)w->WK2, (const uint16_t*)w->WV, L, roles,
                                                                ws.q, ws.k, (uint16_t*)ws.v, go);
        return true;
    }
}

bool dispatch_wg(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                 hipStream_t st, int v_layout) {
    switch (ctx->cfg.C) {
        case 32: return launch_wg<32>(ctx, cv, h, w, ws, st, v_layout);
        case 64: return launch_wg<64>(ctx, cv, h, w, ws, st, v_layout);
        case 128: return launch_wg<128>(ctx, cv, h, w, ws, st, v_layout);
    }
    return false;
}

bool dispatch_ws(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                 hipStream_t st, bool tiled) {
    switch (ctx->cfg.C) {
        case 32: return launch_ws<32>(ctx, cv, h, w, ws, st, tiled);
        case 64: return launch_ws<64>(ctx, cv, h, w, ws, st, tiled);
        case 128: return launch_ws<128>(ctx, cv, h, w, ws, st, tiled);
        case 256: return tiled ? false : launch_ws<256>(ctx, cv, h, w, ws, st, false);
    }
    return false;
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
        for (int t = 0; t < E2F_NP; ++t) tab.c[x][t] = ctx->coefP[x][t];
    int work = cv.N > ctx->n * E2F_NP ? cv.N : ctx->n * E2F_NP;
    if (ctx->cfg.H * ctx->cfg.B > work) work = ctx->cfg.H * ctx->cfg.B;
    k_prepare<<<(work + 255) / 256, 256, 0, st>>>(cv, pos, w->w_path, ctx->cfg.L_max, ctx->cfg.lf, tab, ws.spos, ws.cw,
                                                 w->Wb, ctx->cfg.H, ctx->cfg.B, ws.wbT);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_unit_cw(const e2f_ctx* ctx, float* cw, hipStream_t st) {
    CoefTable tab;
    for (int x = 0; x < E2F_MAX_N; ++x)
        for (int t = 0; t < E2F_NP; ++t) tab.c[x][t] = ctx->coefP[x][t];
    k_unit_cw<<<1, 256, 0, st>>>(ctx->cfg.L_max, ctx->cfg.lf, tab, cw);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

// q, k (fp32) and v (bf16) from the plain layouts into the tile kernel's: binary16 q rows scaled for base-2 logits, k rows
// grouped by four slots, value blocks (e2f::k16_offset, e2f::v4_offset); one workgroup per group of four sorted slots.
__global__ __launch_bounds__(256) void k_tile_relayout(int N, int L, int C, const float* __restrict__ q, const float* __restrict__ k,
                                                       const uint16_t* __restrict__ v, float qscale, uint16_t* __restrict__ q16,
                                                       uint16_t* __restrict__ k16, uint16_t* __restrict__ v4) {
    __shared__ int s_off[E2F_MAX_N];
    const int n = (L + 1) * (L + 1), H = C / 16, DK = (L + 1) * 16, DKP = (DK + 31) / 32 * 32, grp = blockIdx.x;
    if ((int)threadIdx.x < n) s_off[threadIdx.x] = e2f::v4_offset(n, threadIdx.x, 0) | (e2f::v4_role(n, threadIdx.x) == 0 ? 0 : 1 << 30);
    __syncthreads();
    for (int it = threadIdx.x; it < 4 * H * DKP; it += 256) {
        const int s = it / (H * DKP), head = (it / DKP) % H, f = it % DKP, slot = 4 * grp + s;
        const bool real = slot < N && f < DK;
        const size_t src = ((size_t)min(slot, N - 1) * (L + 1) + min(f >> 4, L)) * C + head * 16 + (f & 15);
        const _Float16 kv = to_f16_sat(real ? k[src] : 0.0f);
        k16[e2f::k16_offset(slot, H, head, DKP, f)] = __builtin_bit_cast(uint16_t, kv);
        if (slot < N) q16[((size_t)slot * H + head) * DKP + f] = __builtin_bit_cast(uint16_t, to_f16_sat(real ? q[src] * qscale : 0.0f));
    }
    for (int it = threadIdx.x; it < n * C; it += 256) {
        const int x = it / C, c = it % C, o = s_off[x];
        uint16_t b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int slot = 4 * grp + s;
            const uint16_t val = v[((size_t)min(slot, N - 1) * n + x) * C + c];
            b[s] = slot < N ? val : (uint16_t)0;
        }
        *reinterpret_cast<uint2*>(v4 + ((size_t)grp * H + (c >> 4)) * n * 64 + (o & 0xffffff) + (c & 15) * ((o >> 30) ? 8 : 4)) =
            make_uint2(b[0] | ((uint32_t)b[1] << 16), b[2] | ((uint32_t)b[3] << 16));
    }
}

e2f_status e2f_launch_project_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w,
                                   const E2fAttnWs& ws, int v_layout, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    bool ok;
    const bool tiled_v = v_layout == 1;
    if (v_layout == 2 && !e2f_tile_layouts_direct(ctx)) {
        // channel counts the tile-layout projection kernels are not built for: plain layouts, then a relayout
        if (ctx->cfg.feat_dtype != E2F_BF16 || !ws.q || !ws.k || !ws.v) return E2F_ERR_UNSUPPORTED;
        ok = dispatch_ws(ctx, cv, h, w, ws, st, false) || dispatch_mfma<uint16_t>(ctx, cv, h, w, ws, st, false);
        if (ok)
            k_tile_relayout<<<(cv.N + 3) / 4, 256, 0, st>>>(cv.N, ctx->cfg.L_max, ctx->cfg.C, ws.q, ws.k, (const uint16_t*)ws.v,
                                                         ctx->tau * 1.44269504088896341f, ws.q16, ws.k16, ws.v4);
    } else if (v_layout == 2)
        ok = ctx->cfg.feat_dtype == E2F_BF16 && (ctx->cfg.C == 256 ? launch_sh256(ctx, cv, h, w, ws, st) : dispatch_wg(ctx, cv, h, w, ws, st, 2));
    else if (ctx->cfg.feat_dtype == E2F_BF16)
        ok = (tiled_v && dispatch_wg(ctx, cv, h, w, ws, st, 1)) || dispatch_ws(ctx, cv, h, w, ws, st, tiled_v) ||
             dispatch_mfma<uint16_t>(ctx, cv, h, w, ws, st, tiled_v);
    else
        ok = dispatch_ws_f32(ctx, cv, h, w, ws, st) || dispatch_mfma<float>(ctx, cv, h, w, ws, st, false);
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
