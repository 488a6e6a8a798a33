// Tile form of the fused attention for fp32 features (the paper's own precision; Sec. 3.4, Algorithm 1, with the linear
// factorization of the degree-1 filter as in e2f_tile.hip): the same algorithm as the bf16 tile kernel, with q, k, v,
// the softmax weights and every product in binary32 on the fp32 matrix instruction (16x16x4).
//     S^T = K Q^T          logits of 16 targets x 32 candidates
//     T_mu += W_mu V       W_mu[i][j] = e^{s_ij - m_i} phi(d_ij) (r_ij)_mu
//     out_i = (1/z_i) sum_mu G_mu T_i,mu
// A workgroup of eight waves owns (tile of 16 targets, head).  Candidate chunks are taken eight at a time: wave w
// scores chunk 8G + w (logits, pair geometry, softmax weights -> LDS), then every wave applies all eight chunks'
// weights to its own eighth of the components.  The candidate lists are those of the bf16 kernel (k_tile's list
// form); tiles whose list does not fit are left to the vector-ALU kernel.
// Register layout of v_mfma_f32_16x16x4_f32 (lane = 16 g + i): A operand: A[i][g]; B operand: B[g][i]; result:
// C[4g..4g+3][i].  The contraction index of a step is free to choose as long as both operands agree: the logits take
// feature g * DK/4 + s in step s (a lane reads DK/4 consecutive features of its row), the aggregation takes candidate
// (half mt, row 4g + r) in step (mt, r), which is where the logits' result registers already hold that pair's weight.
#include "e2f_tile_shared.h"

namespace {

struct TileF32Params {
    E2fCellsView cv;
    const float4* spos;
    const float *q, *k, *v;   // the projection's plain layouts in sorted order: q, k [N][L+1][C], v [N][n][C]
    float *qf;                // [N][H][DK] q scaled by tau log2 e, feature l * 16 + channel
    float *kf;                // [ceil(N/4)][H][4 slots][DK]
    float *vf;                // [ceil(N/4)][H][n][16 channels][4 slots]
    const float* G;           // axis operators, then their packed non-zeros
    const float* WbT;
    float* out;
    const int4* lists_hdr;
    const int* lists_ent;
    const float4* lists_pos;
    const unsigned long long* lists_mask;
    int C, H, B, n_tiles, blk;   // blk: tiles per XCD chunk (tile_blk)
    float qscale, rc2, cutoff, rbf_step, rbf_gamma;
};


__device__ __forceinline__ f32x4 mfma32(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// ---- q, k, v from the projection's plain layouts into the layouts above; one workgroup per group of four slots
template <int L>
__global__ __launch_bounds__(256) void k_f32_relayout(TileF32Params P) {
    constexpr int n = (L + 1) * (L + 1), DK = (L + 1) * 16;
    const int grp = blockIdx.x, N = P.cv.N, H = P.H, C = P.C;
    for (int it = threadIdx.x; it < 4 * H * DK; it += 256) {
        const int s = it / (H * DK), head = (it / DK) % H, f = it % DK, slot = 4 * grp + s;
        const size_t src = ((size_t)min(slot, N - 1) * (L + 1) + (f >> 4)) * C + head * 16 + (f & 15);
        const float kv = slot < N ? P.k[src] : 0.0f;
        P.kf[(((size_t)grp * H + head) * 4 + s) * DK + f] = kv;
        if (slot < N) P.qf[((size_t)slot * H + head) * DK + f] = P.q[src] * P.qscale;
    }
    for (int it = threadIdx.x; it < n * C; it += 256) {
        const int x = it / C, c = it % C;
        f32x4 four;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int slot = 4 * grp + s;
            const float val = P.v[((size_t)min(slot, N - 1) * n + x) * C + c];
            four[s] = slot < N ? val : 0.0f;
        }
        *reinterpret_cast<f32x4*>(P.vf + ((((size_t)grp * H + (c >> 4)) * n + x) * 16 + (c & 15)) * 4) = four;
    }
}

// NW waves per workgroup (4 or 8): chunks are taken NW at a time and the components are split NW ways.  With four
// waves two workgroups share a CU (one scores while the other's aggregation keeps the matrix cores busy); the key
// rows are then fetched at the start of the scoring step instead of a group ahead, which frees their registers.
template <int L, int NB, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_tile_f32(TileF32Params P) {
    constexpr int n = (L + 1) * (L + 1), NX = (n + NW - 1) / NW;
    constexpr int NT = 64 * NW;             // threads
    constexpr int LENT8 = LCAP + 8 * NW;    // the list in LDS, padded to whole groups of NW chunks
    constexpr bool K_AHEAD = NW >= 8;
    constexpr int DK = (L + 1) * 16, DQ = DK / 4, NQ = DQ / 4;   // a lane's share of a row: DQ floats in NQ pieces of 16 bytes
    constexpr int W_BYTES = NW * 3 * 2 * 64 * 16, PO_BYTES = n * 64 * 16;
    __shared__ int s_ent[LENT8];
    __shared__ unsigned long long s_mask[LENT8];
    __shared__ float4 s_pos[LENT8 * 4];
    __shared__ __attribute__((aligned(16))) float s_q[16 * DK];
    __shared__ float s_G[AXIS_NNZ];
    __shared__ float s_cmax[NW][16];
    __shared__ float s_z[NW][16];
    __shared__ int s_orow[16];
    // the weights while streaming; the same bytes hold one mu of all waves' accumulators in the epilogue
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[W_BYTES > PO_BYTES ? W_BYTES : PO_BYTES];
    f32x4* s_W = reinterpret_cast<f32x4*>(s_raw);   // [chunk of the group][mu][half][lane]
    f32x4* s_po = reinterpret_cast<f32x4*>(s_raw);
    static_assert(LCAP <= NT && 16 * DK / 4 <= 2 * NT && AXIS_NNZ <= NT, "one request per thread (two for the queries)");
    constexpr int NPOS = (LENT8 * 4 + NT - 1) / NT;   // slot positions per thread

    int tile, head;
    if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, P.H, tile, head)) return;   // whole workgroup
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tn = lane & 15, g = lane >> 4;
    // components [x0, x0 + nxw) belong to this wave: n / NW each, the first n % NW waves one more
    const int nxw = n / NW + (wave < n % NW ? 1 : 0);
    const int x0 = wave * (n / NW) + min(wave, n % NW);
    const int N = P.cv.N, H = P.H;
    const int t0 = tile * 16, nt = min(16, N - t0);
    const int tslot = min(t0 + tn, N - 1);

    // ---- everything the tile needs, requested together
    const int4 hd = P.lists_hdr[tile];
    const float4 tp = P.spos[tslot];
    const int orow_mine = tid < 16 ? (t0 + tid < N ? P.cv.perm[t0 + tid] : -1) : 0;
    const float g_mine = tid < AXIS_NNZ ? P.G[AXIS_PACKED_AT + tid] : 0.0f;
    const int ent_mine = tid < LCAP ? P.lists_ent[(size_t)tile * LCAP + tid] : 0;
    const unsigned long long mask_mine = tid < LCAP ? P.lists_mask[(size_t)tile * LCAP + tid] : 0ull;
    float4 pos_mine[NPOS];
#pragma unroll
    for (int j = 0; j < NPOS; ++j)
        pos_mine[j] = tid + NT * j < LCAP * 4 ? P.lists_pos[(size_t)tile * LCAP * 4 + tid + NT * j] : tp;
    f32x4 q_mine[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int u = tid + NT * j;
        q_mine[j] = u < 16 * DK / 4
                        ? *reinterpret_cast<const f32x4*>(P.qf + ((size_t)min(t0 + u / (DK / 4), N - 1) * H + head) * DK + 4 * (u % (DK / 4)))
                        : (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const float wb_mine = lane < P.B ? P.WbT[lane * H + head] : 0.0f;

    const int cnt = hd.x;
    if (cnt < 0) return;   // (whole workgroup) a crowded tile: left to the vector-ALU kernel
    if (tid < LCAP) {
        s_ent[tid] = tid < cnt ? ent_mine : 0;
        s_mask[tid] = tid < cnt ? mask_mine : 0ull;
    }
    if (tid < LENT8 - LCAP) {
        s_ent[LCAP + tid] = 0;
        s_mask[LCAP + tid] = 0ull;
    }
#pragma unroll
    for (int j = 0; j < NPOS; ++j) {   // (selected by value, component by component)
        const int at = tid + NT * j;
        const bool in_list = (at >> 2) < cnt;
        if (at < LENT8 * 4)
            s_pos[at] = make_float4(in_list ? pos_mine[j].x : tp.x, in_list ? pos_mine[j].y : tp.y,
                                    in_list ? pos_mine[j].z : tp.z, in_list ? pos_mine[j].w : tp.w);
    }
    if (tid < AXIS_NNZ) s_G[tid] = g_mine;
    if (tid < 16) s_orow[tid] = orow_mine;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (tid + NT * j < 16 * DK / 4) reinterpret_cast<f32x4*>(s_q)[tid + NT * j] = q_mine[j];
    __syncthreads();

    const int nch = (cnt + 7) >> 3, ngr = (nch + NW - 1) / NW;
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * 1.44269504088896341f;
    const float c_g = -P.rbf_gamma * 1.44269504088896341f;
    float cb[NB];
    {
        const float mine = bias_coefficient<NB>(wb_mine, lane, P.rbf_step, P.rbf_gamma);
#pragma unroll
        for (int b = 0; b < NB; ++b) cb[b] = read_lane(mine, b);
    }

    f32x4 kr[2][NQ];   // this lane's share of the key rows of its two candidates (one per half)
    auto load_K = [&](int c) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
            const float* row = P.kf + ((((size_t)((unsigned)e >> 8)) * H + head) * 4 + (tn & 3)) * DK + g * DQ;
#pragma unroll
            for (int j = 0; j < NQ; ++j) kr[mt][j] = *reinterpret_cast<const f32x4*>(row + 4 * j);
        }
    };
    // value rows of this wave's components: for half mt the four slots of list entry 8c + 4mt + g, channel tn
    f32x4 vr[NX][2];
    auto load_V = [&](int c, int xi) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const unsigned e = (unsigned)s_ent[8 * c + 4 * mt + g] >> 8;
            vr[xi][mt] = *reinterpret_cast<const f32x4*>(P.vf + ((((size_t)e * H + head) * n + x0 + xi) * 16 + tn) * 4);
        }
    };
    if (nch > 0) {
        if (K_AHEAD) load_K(min(wave, nch - 1));
#pragma unroll
        for (int xi = 0; xi < NX; ++xi)
            if (xi < nxw) load_V(0, xi);
    }

    f32x4 acc[3][NX];
#pragma unroll
    for (int mu = 0; mu < 3; ++mu)
#pragma unroll
        for (int x = 0; x < NX; ++x) acc[mu][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    constexpr float M_NONE = -1.0e30f;   // finite, so that a masked logit (-inf) gets the weight 2^-inf = 0
    float m_ref = M_NONE, z = 0.0f;

    for (int G = 0; G < ngr; ++G) {
        // ---- logits, pair geometry and cutoff mask of this wave's chunk
        const int cm = NW * G + wave;
        if (!K_AHEAD) load_K(min(cm, nch - 1));
        f32x4 S[2];
        {
            f32x4 qr[NQ];
#pragma unroll
            for (int j = 0; j < NQ; ++j) qr[j] = *reinterpret_cast<const f32x4*>(s_q + tn * DK + g * DQ + 4 * j);
            // (four partial sums, so that consecutive matrix instructions go to different accumulators)
            f32x4 Sp[2][2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) Sp[mt][0] = Sp[mt][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NQ; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) Sp[mt][e & 1] = mfma32(kr[mt][j][e], qr[j][e], Sp[mt][e & 1]);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) S[mt] = Sp[mt][0] + Sp[mt][1];
        }
        if (K_AHEAD) load_K(min(cm + NW, nch - 1));
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
                // (bitwise on purpose; the target itself is at distance zero, an image of it at a box length)
                const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f);
                const float d = __builtin_amdgcn_sqrtf(d2);
                float bias = bias_value<NB>(cb, d, d2, c_u, c_g, P.rbf_step);
                asm("" : "+v"(bias));   // (evaluated for every candidate: one basic block)
                s2[u] = ok ? S[mt][r] + bias : -INFINITY;
                gate[u] = e2f::radial_gate(d, P.cutoff);
                cmax = fmaxf(cmax, s2[u]);
            }
        }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
        if (lane < 16) s_cmax[wave][lane] = cmax;
        __syncthreads();
        // ---- the group's largest logit per target, the same in all waves
        float gmax = s_cmax[0][tn];
#pragma unroll
        for (int w = 1; w < NW; ++w) gmax = fmaxf(gmax, s_cmax[w][tn]);
        if (m_ref == M_NONE) m_ref = fmaxf(gmax, M_NONE);   // first neighbours: the accumulator rows are still zero
        const bool move = gmax > m_ref + M_STEP;
        if (__builtin_expect(__ballot(move) != 0ull, 0)) {
            const float f = move ? __builtin_amdgcn_exp2f(m_ref - gmax) : 1.0f;
            m_ref = move ? gmax : m_ref;
            z *= f;
            // rows of the accumulators are targets: T <- diag(f) T, slice r pairs A_r[i][g] = f_i [i == 4g + r] with
            // B_r[g][j] = T[4g + r][j]
            float ar[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) ar[r] = tn == 4 * g + r ? f : 0.0f;
#pragma unroll
            for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                for (int x = 0; x < NX; ++x) {
                    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int r = 0; r < 4; ++r) d = mfma32(ar[r], acc[mu][x][r], d);
                    acc[mu][x] = d;
                }
        }
        // ---- weights of this wave's chunk -> LDS
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f32x4 wx, wy, wz;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int u = 4 * mt + r;
                const float p = __builtin_amdgcn_exp2f(s2[u] - m_ref);
                z += p;
                const float pg = p * gate[u];
                const float4 pc = s_pos[(8 * cm + 4 * mt + g) * 4 + r];
                wx[r] = pg * (pc.x - tp.x);
                wy[r] = pg * (pc.y - tp.y);
                wz[r] = pg * (pc.z - tp.z);
            }
            s_W[((wave * 3 + 0) * 2 + mt) * 64 + lane] = wx;
            s_W[((wave * 3 + 1) * 2 + mt) * 64 + lane] = wy;
            s_W[((wave * 3 + 2) * 2 + mt) * 64 + lane] = wz;
        }
        __syncthreads();
        // ---- aggregate the chunks of the group into this wave's components
#pragma unroll 1
        for (int cc = 0; cc < NW; ++cc) {
            const int c = NW * G + cc;
            if (c < nch) {
                f32x4 W[3][2];
#pragma unroll
                for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) W[mu][mt] = s_W[((cc * 3 + mu) * 2 + mt) * 64 + lane];
                const int cnext = min(c + 1, nch - 1);
                // (steps outermost: consecutive matrix instructions go to different accumulators)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int xi = 0; xi < NX; ++xi)
                            if (xi < nxw) {   // (wave-uniform)
#pragma unroll
                                for (int mu = 0; mu < 3; ++mu) acc[mu][xi] = mfma32(W[mu][mt][r], vr[xi][mt][r], acc[mu][xi]);
                            }
#pragma unroll
                for (int xi = 0; xi < NX; ++xi)
                    if (xi < nxw) load_V(cnext, xi);   // the next chunk's rows replace the operands
            }
        }
    }

    // ---- epilogue: out = (1/z) sum_mu G_mu T_mu.  For one mu at a time the waves put their T_mu components into LDS
    // and every wave forms the output components x_out = wave (mod NW) from the non-zero entries of G_mu.  The code
    // exists once per wave index, so that a wave's components and the pattern are compile-time facts.
    z += __shfl_xor(z, 16);
    z += __shfl_xor(z, 32);
    if (lane < 16) s_z[wave][lane] = z;
    auto finish = [&](auto wv_tag) {
        constexpr int WV = decltype(wv_tag)::value;
        constexpr int RO = WV < n ? (n - WV + NW - 1) / NW : 0;           // components WV, WV + NW, ...
        constexpr int X0 = WV * (n / NW) + (WV < n % NW ? WV : n % NW);   // this wave's accumulator components
        constexpr int NXW = n / NW + (WV < n % NW ? 1 : 0);
        f32x4 pr[RO > 0 ? RO : 1];
#pragma unroll
        for (int i = 0; i < RO; ++i) pr[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mu = 0; mu < 3; ++mu) {
            __syncthreads();
#pragma unroll
            for (int x = 0; x < NXW; ++x) s_po[(X0 + x) * 64 + lane] = acc[mu][x];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < RO; ++i) {
#pragma unroll
                for (int xi = 0; xi < n; ++xi)
                    if ((E2F_AXIS_NZ[mu][WV + NW * i] >> xi) & 1u)
                        pr[i] += s_G[AXIS_INDEX.v[mu][WV + NW * i][xi]] * s_po[xi * 64 + lane];
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int tt = 4 * g + r, row = s_orow[tt];
            float zt = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) zt += s_z[w][tt];
            const float inv = zt > 0.0f ? 1.0f / zt : 0.0f;
            if (row >= 0) {
                float* orp = P.out + (size_t)row * n * P.C + head * 16 + tn;
#pragma unroll
                for (int i = 0; i < RO; ++i) orp[(size_t)(WV + NW * i) * P.C] = pr[i][r] * inv;
            }
        }
    };
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    if (wave_u == 0) finish(std::integral_constant<int, 0>{});
    if (wave_u == 1) finish(std::integral_constant<int, 1>{});
    if (wave_u == 2) finish(std::integral_constant<int, 2>{});
    if (wave_u == 3) finish(std::integral_constant<int, 3>{});
    if constexpr (NW > 4) {
        if (wave_u == 4) finish(std::integral_constant<int, 4>{});
        if (wave_u == 5) finish(std::integral_constant<int, 5>{});
        if (wave_u == 6) finish(std::integral_constant<int, 6>{});
        if (wave_u == 7) finish(std::integral_constant<int, 7>{});
    }
    (void)nt;
}

template <int L>
void launch_L(const TileF32Params& P, hipStream_t st) {
    const int grid = tile_grid(P.n_tiles, P.blk, P.H);
    k_f32_relayout<L><<<(P.cv.N + 3) / 4, 256, 0, st>>>(P);
#ifndef E2F_F32_NW
#define E2F_F32_NW 4
#endif
    if (P.B > 8) k_tile_f32<L, 16, E2F_F32_NW><<<grid, 64 * E2F_F32_NW, 0, st>>>(P);
    else k_tile_f32<L, 8, E2F_F32_NW><<<grid, 64 * E2F_F32_NW, 0, st>>>(P);
}

}  // namespace

bool e2f_tile_f32_supported(const e2f_ctx* ctx) {
    const int C = ctx->cfg.C;
    return ctx->cfg.feat_dtype == E2F_F32 && ctx->cfg.lf == 1 && ctx->Ch == 16 && ctx->cfg.L_max >= 1 &&
           ctx->cfg.B <= 16 && C % 16 == 0 && C <= 256;
}

// The fp32 tile kernel for every tile whose candidate list fits; q, k, v in the plain layouts and the candidate lists
// (e2f_launch_tile_lists) must be in `ws`.  Crowded tiles are left untouched: the caller runs the vector-ALU kernel
// for them.
e2f_status e2f_launch_tile_f32(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws, float* out, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    TileF32Params P;
    P.cv = cv;
    P.spos = ws.spos; P.q = ws.q; P.k = ws.k; P.v = static_cast<const float*>(ws.v);
    P.qf = ws.qf; P.kf = ws.kf; P.vf = ws.vf; P.G = ws.G; P.WbT = ws.wbT; P.out = out;
    P.lists_hdr = ws.lists_hdr; P.lists_ent = ws.lists_ent; P.lists_pos = ws.lists_pos; P.lists_mask = ws.lists_mask;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.n_tiles = (cv.N + 15) / 16; P.blk = tile_blk(P.n_tiles);
    P.qscale = ctx->tau * 1.44269504088896341f;   // logits in base-2 units
    P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    switch (ctx->cfg.L_max) {
        case 1: launch_L<1>(P, st); break;
        case 2: launch_L<2>(P, st); break;
        case 3: launch_L<3>(P, st); break;
        case 4: launch_L<4>(P, st); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
