// Fused on-the-fly equivariant attention on the matrix cores (bf16 operands, fp32 accumulation), for heads of
// 16 channels.  Same algorithm as k_fused_valu (Sec. 3.4, Algorithm 1 with the geometry and the EAAS steps of
// Sec. 3.3 inside the kernel); what changes is where the two block rotations and the re-indexing run.
//
// The (L+1)^2 components are split into two 16-row tiles, HI = {l=4 (9 rows), l=3 (7 rows)} and
// LO = {l=2 (5), l=1 (3), l=0 (1), 7 unused}; a 32-long contraction index k = 8g + r stands for HI row 4g+r
// (r < 4) or LO row 4g+r-4 (r >= 4).  With D1 the block-diagonal Wigner matrix of the aligning rotation and
// M = D1^T P (the re-indexing operator folded into the back rotation, path weights included), the message
// operator of a pair is G = M D1 = D^T P D.  Per pair, once, for every (input tile Tb, output tile To):
//
//   X[Tb][To] = D1c[Tb] . M[To]^T          4 x v_mfma_f32_16x16x32_bf16   (X[b][o] = G[o][b])
//
// whose accumulator layout (lane (g,o) holds rows b = 4g..4g+3 of column o) is exactly the A-operand layout of
// G[To] for the contraction over the 32 input rows, so G never leaves the lane: A[To] = bf16([X[HI][To]; X[LO][To]]).
// Then for every head (16 channels), with V the neighbour's value rows in tile order as the B operand:
//
//   A_i[To] += w * ( G[To] . V )            2 x v_mfma_f32_16x16x32_bf16 + 8 FMAs,  w = e^{s-mu} phi |r|^lf
//
// The running attention output A_i of Algorithm 1 is held in the lanes as 16x16 fp32 tiles per (head, tile).
//
// One wave per target atom.  Pairs are found as in k_fused_valu; per super-chunk of up to SC pairs, lanes =
// pairs compute the fp32 Wigner blocks, radial bias and gate into LDS (uniform code, no divergence).  Every
// lane then assembles its own A-operand fragments of D1 and M for one pair at a time from those blocks, using
// per-lane tables of LDS offsets and P coefficients built once at kernel start.

#include <limits.h>

#include "e2f_device.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

struct MfmaParams {
    E2fCellsView cv;
    const float4* spos;
    const float* q;
    const float* k;
    const uint16_t* vt;  // [slot][H][NT][16 channels][16 tile rows] bf16
    const float* cw;
    const float* WbT;  // [B][H]
    const uint32_t* cap_d2;   // neighbour cap thresholds per sorted slot, or null
    const int32_t* cap_idx;
    float* out;
    int B, lf;
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

constexpr int SC = 32;     // pairs per super-chunk
constexpr int CAPM = 320;  // capacity of the neighbour list in LDS (a fill step can add up to 256)

// Tile order of the components.  tile 0 = HI, tile 1 = LO.
__device__ __forceinline__ bool tile_row_to_lm(int tile, int row, int L, int& l, int& m) {
    if (tile == 0) {
        if (row < 9) { l = 4; m = row - 4; } else { l = 3; m = row - 12; }
    } else {
        if (row < 5) { l = 2; m = row - 2; } else if (row < 8) { l = 1; m = row - 6; } else if (row == 8) { l = 0; m = 0; } else return false;
    }
    return l <= L;
}

// Value held by a lane known at compile time, as a wave-uniform scalar (no LDS traffic, unlike __shfl).
__device__ __forceinline__ float read_lane(float x, int src_lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), src_lane));
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <int L, int H>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_fused_mfma(MfmaParams P) {
    constexpr int DS = e2f::d_offset(L + 1);
    constexpr int ZERO = DS;                          // slot that always holds 0
    constexpr int DST = (DS + 1) | 1;                 // odd stride: lanes = pairs write without bank conflicts
    constexpr bool HAS_HI = L >= 3;
    constexpr int NT = HAS_HI ? 2 : 1;
    constexpr int T0 = HAS_HI ? 0 : 1;                // first tile in use
    constexpr int C = 16 * H;
    __shared__ int s_list[CAPM];   // entries: slot | run << RUN_SHIFT
    // the target's 18 candidate runs (9 stencil rows, then their cells across a periodic x face): first slot,
    // candidates before the run, lattice translation
    __shared__ int s_rlo[32], s_rpre[32];
    __shared__ float4 s_rsh[32];
    constexpr int RUN_SHIFT = 26;    // the launcher checks N < 2^26
    __shared__ float s_D[SC * DST];
    __shared__ float s_bias[SC * H];
    __shared__ float s_wgt[SC];
    __shared__ float s_s[SC * H];
    __shared__ float s_cw[E2F_MAX_N * E2F_NP];

    const int t = e2f::xcd_remap(blockIdx.x, P.cv.N);
    if (t < 0) return;  // padding block of the XCD map (whole wave)
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    const float4 pi = P.spos[t];
    const uint32_t capd = P.cap_d2 ? P.cap_d2[t] : 0xffffffffu;
    const int capi = P.cap_idx ? P.cap_idx[t] : INT_MAX;
    for (int x = lane; x < (L + 1) * (L + 1) * E2F_NP; x += 64) s_cw[x] = P.cw[x];
    __syncthreads();

    // ---- per-lane fragment tables (constant for the whole kernel)
    // D1c fragment of input tile T: A[i = b][k], k <-> aligned row 4g+r of the same tile: D^l[a][b] if that row
    //   (l,a) and column i = (l,b) have the same degree.
    // M fragment of out tile T: B[k][j] = M[j][k], k = 8g+r <-> aligned row (r<4: HI row 4g+r, r>=4: LO row 4g+r-4)
    //   = (li,mi);  out row j = (lo,b):  M = D^lo[mo][b] * cw[(lo,mo)][kk]  with kk = li - lo + lf the path index;
    //   even kk: mo = mi, odd kk: mo = -mi (mi != 0).
    int offD1[NT][4], offM[NT][8];
    float cM[NT][8];
#pragma unroll
    for (int T = 0; T < NT; ++T) {
        const int tile = T0 + T;
        int li_, a_;
        const bool row_ok = tile_row_to_lm(tile, i, L, li_, a_);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int lr, a;
            const bool al_ok = tile_row_to_lm(tile, 4 * g + r, L, lr, a);
            offD1[T][r] = (row_ok && al_ok && lr == li_) ? e2f::d_offset(li_) + (a + li_) * (2 * li_ + 1) + (a_ + li_) : ZERO;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int ktile = HAS_HI ? (r < 4 ? 0 : 1) : 1;
            const int krow = 4 * g + (r & 3);
            int li, mi;
            const bool k_ok = (HAS_HI || r >= 4) && tile_row_to_lm(ktile, krow, L, li, mi);
            int off = ZERO;
            float coef = 0.0f;
            if (row_ok && k_ok) {
                const int lo = li_, b = a_;
                const int kk = li - lo + P.lf;   // path index: l_in = l_out - lf + kk
                if (kk >= 0 && kk <= 2 * P.lf && P.lf - li <= lo && !((kk & 1) && mi == 0)) {
                    const int mo = (kk & 1) ? -mi : mi;
                    if (mo <= lo && -mo <= lo) {
                        off = e2f::d_offset(lo) + (mo + lo) * (2 * lo + 1) + (b + lo);
                        coef = s_cw[(lo * lo + lo + mo) * E2F_NP + kk];
                    }
                }
            }
            offM[T][r] = off;
            cM[T][r] = coef;
        }
    }

    // ---- logits run with lanes over channels: lane <-> channels 2*lane, 2*lane+1; its head is lane/8
    const bool lg_active = lane < C / 2;
    const int c0 = lg_active ? 2 * lane : 0;
    const int head = c0 / 16;

    f32x4 acc[H][NT];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int T = 0; T < NT; ++T) acc[h][T] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float mu = -INFINITY, z = 0.0f;

    // The runs as one candidate range [0, n_cand): candidate c lies in the last run r with s_rpre[r] <= c.
    if (lane < 18) {
        int rlo, rhi;
        float4 sh;
        e2f::stencil_run(P.cv, t, lane, rlo, rhi, sh);
        int inc = rhi - rlo;   // -> inclusive scan over the runs
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) {
            const int up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        s_rlo[lane] = rlo;
        s_rsh[lane] = sh;
        s_rpre[lane + 1] = inc;
        if (lane == 0) s_rpre[0] = 0;
        if (lane < 13) s_rpre[19 + lane] = INT_MAX;   // stops of the search
    } else if (lane < 32) {
        s_rsh[lane] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    __syncthreads();
    const int n_cand = s_rpre[18];
    int cbase = 0;
    while (true) {
        // ---- fill the list: 4 x 64 candidates per step, their positions requested together
        int cnt = 0;
        while (cbase < n_cand && cnt + 256 <= CAPM) {
            int jj[4], run[4];
            float4 pj[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = cbase + 64 * u + lane;
                int r = 0;
#pragma unroll
                for (int step = 16; step >= 1; step >>= 1)
                    if (s_rpre[r + step] <= c) r += step;
                const int j = c < n_cand ? s_rlo[r] + c - s_rpre[r] : -1;
                jj[u] = j;
                run[u] = r;
                pj[u] = P.spos[j >= 0 ? j : t];
                const float4 sh = s_rsh[r & 31];   // the image this run sees (zero without periodic axes)
                pj[u].x += sh.x;
                pj[u].y += sh.y;
                pj[u].z += sh.z;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float d2 = e2f::dist2_exact(pi.x, pi.y, pi.z, pj[u].x, pj[u].y, pj[u].z);
                const bool ok = jj[u] >= 0 && jj[u] != t && e2f::is_neighbor(d2, P.rc2) &&
                                e2f::under_cap(d2, pj[u].w, capd, capi);
                const unsigned long long mask = __ballot(ok);
                if (ok) s_list[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = jj[u] | (run[u] << RUN_SHIFT);
                cnt += __popcll(mask);
            }
            cbase += 256;
        }
        const bool rows_done = cbase >= n_cand;
        __syncthreads();
        for (int p0 = 0; p0 < cnt; p0 += SC) {
            const int np = min(SC, cnt - p0);
            // ---- lanes = pairs: Wigner blocks (fp32), radial bias, gate
            if (lane < np) {
                const int e = s_list[p0 + lane], j = e & ((1 << RUN_SHIFT) - 1);
                const float4 pj = P.spos[j], sh = s_rsh[e >> RUN_SHIFT];
                const float dx = (pj.x + sh.x) - pi.x, dy = (pj.y + sh.y) - pi.y, dz = (pj.z + sh.z) - pi.z;
                const float d = sqrtf(dx * dx + dy * dy + dz * dz);
                e2f::align_D<L>(dx, dy, dz, d, s_D + lane * DST);
                s_D[lane * DST + ZERO] = 0.0f;
                float bias[H];
#pragma unroll
                for (int hh = 0; hh < H; ++hh) bias[hh] = 0.0f;
                for (int b = 0; b < P.B; ++b) {  // WbT is [B][H]: one uniform load per basis function
                    const float gb = e2f::radial_basis(d, b, P.rbf_step, P.rbf_gamma);
#pragma unroll
                    for (int hh = 0; hh < H; ++hh) bias[hh] += P.WbT[b * H + hh] * gb;
                }
#pragma unroll
                for (int hh = 0; hh < H; ++hh) s_bias[lane * H + hh] = bias[hh];
                s_wgt[lane] = e2f::radial_gate(d, P.cutoff) * (P.lf == 2 ? d * d : d);
            }
            __syncthreads();
            // ---- pass 1: logits of the super-chunk (Eq. kernel_score) and their maximum per head
            float cmax = -INFINITY;
            // the query row is re-read per super-chunk (cache hit) instead of living in registers across pass 2
            float q[L + 1][2];
#pragma unroll
            for (int l = 0; l <= L; ++l) {
                const float2 qq = *reinterpret_cast<const float2*>(P.q + ((size_t)t * (L + 1) + l) * C + c0);
                q[l][0] = qq.x;
                q[l][1] = qq.y;
            }
            for (int pb = 0; pb < np; pb += 8) {
                // all key rows of the batch are requested before the first one is used
                float2 kk[8][L + 1];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = s_list[p0 + min(pb + u, np - 1)] & ((1 << RUN_SHIFT) - 1);
                    const float* kj = P.k + (size_t)j * (L + 1) * C + c0;
#pragma unroll
                    for (int l = 0; l <= L; ++l) kk[u][l] = *reinterpret_cast<const float2*>(kj + l * C);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    float dot = 0.0f;
#pragma unroll
                    for (int l = 0; l <= L; ++l) dot += q[l][0] * kk[u][l].x + q[l][1] * kk[u][l].y;
                    dot += __shfl_xor(dot, 1);
                    dot += __shfl_xor(dot, 2);
                    dot += __shfl_xor(dot, 4);
                    if (pb + u < np) {
                        const float s = dot * P.tau + s_bias[(pb + u) * H + head];
                        cmax = fmaxf(cmax, s);
                        if ((lane & 7) == 0 && lg_active) s_s[(pb + u) * H + head] = s;
                    }
                }
            }
            // ---- one rescale of (mu, z, A) per super-chunk
            const float mu_new = fmaxf(mu, cmax);
            const float scale = __expf(mu - mu_new);
            z *= scale;
            mu = mu_new;
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float sc = read_lane(scale, 8 * h);
#pragma unroll
                for (int T = 0; T < NT; ++T) acc[h][T] *= sc;
            }
            __syncthreads();
            // ---- pass 2: per pair, assemble the fragments, then 4 MFMAs per head
            // Value rows live in one register set: as soon as head h of pair p has gone through its MFMAs, its
            // registers are refilled with head h of pair p+1, so every load has almost a whole pair of work to land.
            auto v_ptr = [&](int p) {
                const int j = s_list[p0 + p] & ((1 << RUN_SHIFT) - 1);
                return P.vt + (size_t)j * H * NT * 256 + i * 16 + 4 * g;
            };
            // The operator of one pair, G = D^T P D, as bf16 A operands per output tile.
            struct Frags {
                bf16x8 ga[NT];
                float wl;
            };
            auto assemble = [&](int p) {
                Frags f;
                const float pe = __expf(s_s[p * H + head] - mu);
                f.wl = pe * s_wgt[p];   // per lane: weight of this lane's head; pe is added to z when the pair is consumed
                const float* Dp = s_D + p * DST;
                bf16x8 d1c[NT], mf[NT];
#pragma unroll
                for (int T = 0; T < NT; ++T) {
                    const uint32_t u0 = pack_bf16(Dp[offD1[T][0]], Dp[offD1[T][1]]);
                    const uint32_t u1 = pack_bf16(Dp[offD1[T][2]], Dp[offD1[T][3]]);
                    // rows of the HI tile sit at r < 4 of the contraction index, rows of the LO tile at r >= 4
                    d1c[T] = (T0 + T == 0) ? __builtin_bit_cast(bf16x8, make_uint4(u0, u1, 0u, 0u))
                                           : __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, u0, u1));
                    const uint32_t m0 = pack_bf16(Dp[offM[T][0]] * cM[T][0], Dp[offM[T][1]] * cM[T][1]);
                    const uint32_t m1 = pack_bf16(Dp[offM[T][2]] * cM[T][2], Dp[offM[T][3]] * cM[T][3]);
                    const uint32_t m2 = pack_bf16(Dp[offM[T][4]] * cM[T][4], Dp[offM[T][5]] * cM[T][5]);
                    const uint32_t m3 = pack_bf16(Dp[offM[T][6]] * cM[T][6], Dp[offM[T][7]] * cM[T][7]);
                    mf[T] = __builtin_bit_cast(bf16x8, make_uint4(m0, m1, m2, m3));
                }
#pragma unroll
                for (int To = 0; To < NT; ++To) {
                    f32x4 x[2];
                    x[0] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    x[1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int Tb = 0; Tb < NT; ++Tb)
                        x[T0 + Tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(d1c[Tb], mf[To], (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                    f.ga[To] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(x[0][0], x[0][1]), pack_bf16(x[0][2], x[0][3]),
                                                                     pack_bf16(x[1][0], x[1][1]), pack_bf16(x[1][2], x[1][3])));
                }
                return f;
            };
            s16x4 vv[H][NT];
            {
                const uint16_t* v0 = v_ptr(0);
#pragma unroll
                for (int h = 0; h < H; ++h)
#pragma unroll
                    for (int T = 0; T < NT; ++T) vv[h][T] = *reinterpret_cast<const s16x4*>(v0 + (h * NT + T) * 256);
            }
            // Heads are software-pipelined: the MFMAs of head h+1 are issued before the accumulate FMAs of head h,
            // so that the matrix pipe and the vector ALU overlap inside one wave.
            auto head_mfma = [&](const Frags& f, int h, f32x4 (&tmp)[NT]) {
                uint2 vhi = make_uint2(0u, 0u), vlo;
                if constexpr (HAS_HI) {
                    vhi = __builtin_bit_cast(uint2, vv[h][0]);
                    vlo = __builtin_bit_cast(uint2, vv[h][1]);
                } else {
                    vlo = __builtin_bit_cast(uint2, vv[h][0]);
                }
                const bf16x8 bv = __builtin_bit_cast(bf16x8, make_uint4(vhi.x, vhi.y, vlo.x, vlo.y));
#pragma unroll
                for (int T = 0; T < NT; ++T)
                    tmp[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.ga[T], bv, (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
            };
            auto compute = [&](const Frags& f, const uint16_t* vnext) {
                f32x4 tmp[2][NT];
                head_mfma(f, 0, tmp[0]);
#pragma unroll
                for (int h = 0; h < H; ++h) {
                    if (h + 1 < H) head_mfma(f, h + 1, tmp[(h + 1) & 1]);
                    const float w = read_lane(f.wl, 8 * h);
#pragma unroll
                    for (int T = 0; T < NT; ++T) vv[h][T] = *reinterpret_cast<const s16x4*>(vnext + (h * NT + T) * 256);
#pragma unroll
                    for (int T = 0; T < NT; ++T) acc[h][T] += w * tmp[h & 1][T];
                }
            };
            Frags fa = assemble(0), fb;
#pragma unroll 1
            for (int p = 0; p < np; p += 2) {
                fb = assemble(min(p + 1, np - 1));
                z += __expf(s_s[p * H + head] - mu);
                compute(fa, v_ptr(min(p + 1, np - 1)));
                if (p + 1 < np) {
                    fa = assemble(min(p + 2, np - 1));
                    z += __expf(s_s[(p + 1) * H + head] - mu);
                    compute(fb, v_ptr(min(p + 2, np - 1)));
                }
            }
            __syncthreads();
        }
        if (rows_done) break;
    }

    // ---- out_i = A / z, caller's atom order; lane (g,i) holds tile rows 4g..4g+3 of channel 16h + i
    const float zinv = z > 0.0f ? 1.0f / z : 0.0f;
    float* o = P.out + (size_t)P.cv.perm[t] * (L + 1) * (L + 1) * C;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const float zi = read_lane(zinv, 8 * h);
#pragma unroll
        for (int T = 0; T < NT; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int l, m;
                if (tile_row_to_lm(T0 + T, 4 * g + r, L, l, m)) o[(l * l + l + m) * C + 16 * h + i] = acc[h][T][r] * zi;
            }
    }
}

template <int L>
bool launch_h(const e2f_ctx* ctx, const MfmaParams& P, hipStream_t st) {
    switch (ctx->cfg.H) {
        case 1: k_fused_mfma<L, 1><<<e2f::xcd_grid(P.cv.N), 64, 0, st>>>(P); return true;
        case 2: k_fused_mfma<L, 2><<<e2f::xcd_grid(P.cv.N), 64, 0, st>>>(P); return true;
        case 4: k_fused_mfma<L, 4><<<e2f::xcd_grid(P.cv.N), 64, 0, st>>>(P); return true;
        case 8: k_fused_mfma<L, 8><<<e2f::xcd_grid(P.cv.N), 64, 0, st>>>(P); return true;
    }
    return false;
}

}  // namespace

bool e2f_fused_mfma_supported(const e2f_ctx* ctx) {
    const int H = ctx->cfg.H;
    return ctx->cfg.feat_dtype == E2F_BF16 && (ctx->cfg.lf == 1 || ctx->cfg.lf == 2) && ctx->Ch == 16 && ctx->cfg.L_max >= 1 &&
           (H == 1 || H == 2 || H == 4 || H == 8);
}

e2f_status e2f_launch_fused_mfma(const e2f_ctx* ctx, const E2fCellsView& cv, const e2f_weights* w, const E2fAttnWs& ws,
                                 float* out, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (cv.N >= (1 << 26)) return E2F_ERR_UNSUPPORTED;   // list entries carry the run in their top bits
    MfmaParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.vt = (const uint16_t*)ws.v; P.cw = ws.cw; P.WbT = ws.wbT; P.out = out;
    P.cap_d2 = ws.cap_d2; P.cap_idx = ws.cap_idx;
    P.B = ctx->cfg.B;
    P.lf = ctx->cfg.lf;
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    bool ok = false;
    switch (ctx->cfg.L_max) {
        case 1: ok = launch_h<1>(ctx, P, st); break;
        case 2: ok = launch_h<2>(ctx, P, st); break;
        case 3: ok = launch_h<3>(ctx, P, st); break;
        case 4: ok = launch_h<4>(ctx, P, st); break;
    }
    if (!ok) return E2F_ERR_UNSUPPORTED;
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
