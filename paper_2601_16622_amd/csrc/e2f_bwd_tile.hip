// Backward pass of the fused attention call for the degree-1 filter on the matrix cores, in the tile form of the
// forward pass (e2f_tile.hip): tiles of 16 atoms against chunks of 32 candidate atoms taken from the tile's candidate
// list.  With g = dL/d out and the three axis operators G_mu (message m_ij = sum_mu (r_ij)_mu G_mu v_j), per head
//     u_mu   = <g_i, G_mu v_j>                     w = sum_mu r_mu u_mu
//     P_ij   = 2^(s_ij - lse_i)                    alpha_ij = P_ij phi(d)           (logits in base-2 units)
//     ds_ij  = P_ij (phi w - D_i),  D_i = <g_i, out_i>
//     dq_i  += tau ds_ij k_j          dk_j += tau ds_ij q_i          dv_j += alpha_ij sum_mu r_mu G_mu^T g_i
//     dL/dr_ij = sum_heads [ alpha_ij u + (ds_ij b'(d) + P_ij w phi'(d)) r/d ],   dpos_j += dL/dr_ij,  dpos_i -= dL/dr_ij
// (the paper states the forward pass only, Algorithm 1; this is its derivative with the neighbour sets held fixed).
// Nothing per pair is written to memory and every atom's sums are formed by the workgroup that owns its tile (no
// atomics, deterministic).  The neighbour relation is symmetric (under periodic boundaries with opposite images), so
// one candidate list per tile serves the atom as a target (its neighbours j) and as a source (the targets i that see
// it).  Four kernels share the list:
//   k_bwd_tile_stats    lse_i and D_i per (atom, head): the logits S^T = K Q^T of the forward pass, nothing else
//   k_bwd_tile_pairs    <target side>  dq_i and the atom's share -sum_j dL/dr_ij:  U^T_mu = V (G_mu^T g)^T over the 400
//                       (component, channel) elements of a head, then dQ += dS K
//                       <source side>  dk_j and +sum_i dL/dr_ij:  the same kernel with the roles exchanged,
//                       U^T_mu = g (G_mu v)^T, dK += dS^T Q
//   k_bwd_tile_dv       dv_j = sum_mu G_mu^T Y_mu with Y_mu += W_mu g, W_mu[j][i] = alpha_ij (r_ij)_mu: the forward
//                       kernel's aggregation with dL/d out in place of the value rows and no running softmax
// Operand layouts: a contraction over (component, channel) wants 8 consecutive such elements of one atom per lane
// (rows in the k16 layout, e2f::k16_offset, with 13 steps of 32 elements), a contraction over candidates wants the four
// slots of a group per lane (the v4 layout); the relayout kernels below write what the forward pass does not keep.
#include "e2f_tile_shared.h"

namespace {

struct BwdTileParams {
    E2fCellsView cv;
    const float4* spos;
    const uint16_t *q16, *k16, *v4;   // the forward pass's layouts: q rows (scaled by tau log2 e), k rows grouped, value blocks
    uint16_t *q16g;                   // q rows in the grouped layout of k16
    uint16_t *q4, *k4;                // [group][H][KS][16 features][2 feature tiles][4 slots] bf16
    uint16_t *vrow, *grow;            // [group][H][VS steps][4 slots][32] bf16 rows of v and of dL/d out
    uint16_t *g4;                     // dL/d out in the layout of v4
    const float* G;                   // axis operators, then their packed non-zeros
    const float* WbT;
    const float *out, *gout;          // caller's order
    float2* stat4;                    // [group][H][4 slots] (lse in base-2 units, D)
    float* gp_part;                   // [2 sides][head groups][N sorted slots][3]
    // gradients of the attention's own weights (kernels with WGR): partial sums per tile, and the axis operators
    // with unit path weights (full form, then packed)
    float* pWb_t;                     // [tiles][H][B]
    float* pwp_t;                     // [tiles][head groups][32], bin li * (L_max + 1) + lo
    const float* Gu;
    float *gq, *gk, *gv, *gpos;       // caller's order
    const int4* lists_hdr;
    const int* lists_ent;
    const float4* lists_pos;
    const unsigned long long* lists_mask;
    int C, H, B, n_tiles, hpw, blk;   // blk: tiles per XCD chunk (tile_blk)
    float tau, rc2, cutoff, rbf_step, rbf_gamma;
};

constexpr int LENT = LCAP + 32;   // the list in LDS, padded to whole groups of four chunks
// Degree of component x (index l*l + l + m).
constexpr int e2f_degree_of(int x) { return x >= 16 ? 4 : x >= 9 ? 3 : x >= 4 ? 2 : x >= 1 ? 1 : 0; }
// The non-zero entries of the axis operators grouped by (mu, l_in, l_out): entry = x_out | x_in << 8 | position in the
// packed list << 16; start[mu][5 l_in + l_out] .. start[mu][5 l_in + l_out + 1] are the entries of one group.
struct PathTable {
    uint32_t ent[AXIS_NNZ];
    int16_t start[3][26];
    constexpr PathTable() : ent(), start() {
        int count = 0;
        for (int mu = 0; mu < 3; ++mu) {
            for (int bin = 0; bin < 25; ++bin) {
                start[mu][bin] = (int16_t)count;
                for (int xo = 0; xo < E2F_MAX_N; ++xo)
                    for (int xi = 0; xi < E2F_MAX_N; ++xi)
                        if (e2f_degree_of(xi) == bin / 5 && e2f_degree_of(xo) == bin % 5 && ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u))
                            ent[count++] = (uint32_t)xo | ((uint32_t)xi << 8) | ((uint32_t)AXIS_INDEX.v[mu][xo][xi] << 16);
            }
            start[mu][25] = (int16_t)count;
        }
    }
};
__device__ constexpr PathTable PATH_TABLE{};
constexpr float LOG2E = 1.44269504088896341f, LN2 = 0.69314718055994531f;

// ---- relayout: q rows -> grouped layout, q and k -> four slots of a feature per lane (bf16)
// One workgroup per group of four sorted slots, thread = (head, feature).
template <int L>
__global__ __launch_bounds__(256) void k_bwd_relayout_qk(BwdTileParams P) {
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    const int grp = blockIdx.x, N = P.cv.N, H = P.H;
    for (int it = threadIdx.x; it < H * DKP; it += 256) {
        const int head = it / DKP, f = it % DKP;
        uint16_t qv[4], kv[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int slot = 4 * grp + s;
            qv[s] = slot < N ? P.q16[((size_t)slot * H + head) * DKP + f] : (uint16_t)0;
            kv[s] = P.k16[e2f::k16_offset(slot, H, head, DKP, f)];   // (zero behind the last atom)
            P.q16g[e2f::k16_offset(slot, H, head, DKP, f)] = qv[s];
        }
        const size_t o4 = (((size_t)grp * H + head) * KS + (f >> 5)) * 128 + (f & 15) * 8 + ((f >> 4) & 1) * 4;
        uint16_t qb[4], kb[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            qb[s] = e2f::float_to_bf16_bits((float)__builtin_bit_cast(_Float16, qv[s]));
            kb[s] = e2f::float_to_bf16_bits((float)__builtin_bit_cast(_Float16, kv[s]));
        }
        *reinterpret_cast<u32x2*>(P.q4 + o4) = (u32x2){qb[0] | ((uint32_t)qb[1] << 16), qb[2] | ((uint32_t)qb[3] << 16)};
        *reinterpret_cast<u32x2*>(P.k4 + o4) = (u32x2){kb[0] | ((uint32_t)kb[1] << 16), kb[2] | ((uint32_t)kb[3] << 16)};
    }
}

// ---- relayout: value blocks (four slots of a (component, channel) together) -> rows of (component, channel)
// One workgroup per group of four sorted slots, thread = (head, component, 8 channels): 16-byte stores.
template <int L>
__global__ __launch_bounds__(256) void k_bwd_relayout_v(BwdTileParams P) {
    constexpr int n = (L + 1) * (L + 1), VK = n * 16, VS = (VK + 31) / 32, VKP = VS * 32;
    __shared__ int s_off[n];
    if ((int)threadIdx.x < n) s_off[threadIdx.x] = e2f::v4_offset(n, threadIdx.x, 0) | (e2f::v4_role(n, threadIdx.x) == 0 ? 0 : 1 << 30);
    __syncthreads();
    const int grp = blockIdx.x, H = P.H;
    for (int it = threadIdx.x; it < H * (VKP / 8); it += 256) {
        const int head = it / (VKP / 8), kk = (it % (VKP / 8)) * 8;
        u32x2 four[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) four[j] = (u32x2){0u, 0u};
        if (kk < VK) {
            const int x = kk >> 4, ch = kk & 15, o = s_off[x];
            const uint16_t* src = P.v4 + ((size_t)grp * H + head) * n * 64 + (o & 0xffffff) + ch * ((o >> 30) ? 8 : 4);
#pragma unroll
            for (int j = 0; j < 8; ++j) four[j] = *reinterpret_cast<const u32x2*>(src + j * ((o >> 30) ? 8 : 4));
        }
        const size_t base = e2f::k16_offset(4 * (size_t)grp, H, head, VKP, kk);
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = sl < 2 ? four[2 * j][0] : four[2 * j][1], hi = sl < 2 ? four[2 * j + 1][0] : four[2 * j + 1][1];
                w[j] = (sl & 1) ? (lo >> 16) | (hi & 0xffff0000u) : (lo & 0xffffu) | (hi << 16);
            }
            *reinterpret_cast<u32x4*>(P.vrow + base + 32 * sl) = (u32x4){w[0], w[1], w[2], w[3]};
        }
    }
}

// ---- relayout: dL/d out (caller's order, fp32) -> bf16 rows and bf16 value-block layout in sorted order
// One workgroup per group of four sorted slots, thread = (component, 8 channels).
template <int L>
__global__ __launch_bounds__(256) void k_bwd_relayout_g(BwdTileParams P) {
    constexpr int n = (L + 1) * (L + 1), VK = n * 16, VS = (VK + 31) / 32, VKP = VS * 32;
    __shared__ int s_off[n];
    if ((int)threadIdx.x < n) s_off[threadIdx.x] = e2f::v4_offset(n, threadIdx.x, 0) | (e2f::v4_role(n, threadIdx.x) == 0 ? 0 : 1 << 30);
    __syncthreads();
    const int grp = blockIdx.x, H = P.H, C = P.C, N = P.cv.N;
    int atom[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) atom[s] = 4 * grp + s < N ? P.cv.perm[4 * grp + s] : -1;
    for (int it = threadIdx.x; it < n * (C / 8); it += 256) {
        const int x = it / (C / 8), c = (it % (C / 8)) * 8, head = c >> 4, ch = c & 15;
        float v[4][8];   // (rows of absent atoms as zeros)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const float* src = P.gout + ((size_t)max(atom[s], 0) * n + x) * C + c;
            const f32x4 lo = *reinterpret_cast<const f32x4*>(src), hi = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[s][j] = atom[s] >= 0 ? lo[j] : 0.0f;
                v[s][4 + j] = atom[s] >= 0 ? hi[j] : 0.0f;
            }
        }
        const int o = s_off[x], cs = (o >> 30) ? 8 : 4;
        uint16_t* d4 = P.g4 + ((size_t)grp * H + head) * n * 64 + (o & 0xffffff) + ch * cs;
#pragma unroll
        for (int j = 0; j < 8; ++j)   // the four slots of a channel side by side
            *reinterpret_cast<u32x2*>(d4 + j * cs) = (u32x2){pack_bf16(v[0][j], v[1][j]), pack_bf16(v[2][j], v[3][j])};
        const size_t base = e2f::k16_offset(4 * (size_t)grp, H, head, VKP, x * 16 + ch);
#pragma unroll
        for (int s = 0; s < 4; ++s)   // eight channels of a slot side by side
            *reinterpret_cast<u32x4*>(P.grow + base + 32 * s) = (u32x4){pack_bf16(v[s][0], v[s][1]), pack_bf16(v[s][2], v[s][3]),
                                                                       pack_bf16(v[s][4], v[s][5]), pack_bf16(v[s][6], v[s][7])};
    }
    if (VK < VKP) {   // the rows' padding must be finite: it meets zeros of the other operand
        for (int it = threadIdx.x; it < H * 4 * (VKP - VK); it += 256) {
            const int head = it / (4 * (VKP - VK)), s = (it / (VKP - VK)) % 4, kk = VK + it % (VKP - VK);
            P.grow[e2f::k16_offset(4 * (size_t)grp + s, H, head, VKP, kk)] = 0;
        }
    }
}

// The tile's candidate list (entries, pair masks, slot positions) into LDS; what lies behind the list reads as groups
// without a valid slot, at the position `tp`.  Returns the number of entries, or -1 for a crowded tile whose list was
// not written (whole workgroup).  Ends with a barrier.
__device__ __forceinline__ int load_list(const BwdTileParams& P, int tile, int tid, const float4& tp, int* s_ent,
                                         unsigned long long* s_mask, float4* s_pos) {
    static_assert(LCAP * 4 == 3 * 256 && LCAP <= 256, "one request per thread");
    const int4 hd = P.lists_hdr[tile];
    const int ent_mine = tid < LCAP ? P.lists_ent[(size_t)tile * LCAP + tid] : 0;
    const unsigned long long mask_mine = tid < LCAP ? P.lists_mask[(size_t)tile * LCAP + tid] : 0ull;
    float4 pos_mine[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) pos_mine[j] = P.lists_pos[(size_t)tile * LCAP * 4 + tid + 256 * j];
    const int cnt = hd.x;
    if (cnt < 0) return -1;
    if (tid < LCAP) {
        s_ent[tid] = tid < cnt ? ent_mine : 0;
        s_mask[tid] = tid < cnt ? mask_mine : 0ull;
    }
    if (tid < LENT - LCAP) {
        s_ent[LCAP + tid] = 0;
        s_mask[LCAP + tid] = 0ull;
    }
#pragma unroll
    for (int j = 0; j < 3; ++j) {   // (selected by value: a select between two register arrays would move both to scratch)
        const bool in_list = ((tid + 256 * j) >> 2) < cnt;
        s_pos[tid + 256 * j] = make_float4(in_list ? pos_mine[j].x : tp.x, in_list ? pos_mine[j].y : tp.y,
                                           in_list ? pos_mine[j].z : tp.z, in_list ? pos_mine[j].w : tp.w);
    }
    if (tid < (LENT - LCAP) * 4) s_pos[LCAP * 4 + tid] = tp;
    __syncthreads();
    return cnt;
}

// Coefficients of a head's radial bias (bias_value): `mine` is Wb[h][lane] for lane < B, else 0.
template <int NB>
__device__ __forceinline__ void bias_coefficients(const BwdTileParams& P, int lane, float mine, float (&cb)[NB]) {
    const float t = bias_coefficient<NB>(mine, lane, P.rbf_step, P.rbf_gamma);
#pragma unroll
    for (int b = 0; b < NB; ++b) cb[b] = read_lane(t, b);
}

// ---- softmax statistics: lse_i (base-2 units, reference included) and D_i = <g_i, out_i>, per head
template <int L, int NB>
__global__ __launch_bounds__(256) void k_bwd_tile_stats(BwdTileParams P) {
    constexpr int NW = 4, n = (L + 1) * (L + 1);
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    static_assert(16 * (DKP / 8) <= 256, "one request per thread");
    __shared__ int s_ent[LENT];
    __shared__ unsigned long long s_mask[LENT];
    __shared__ float4 s_pos[LENT * 4];
    __shared__ __attribute__((aligned(16))) uint16_t s_q[16 * DKP];
    __shared__ float s_m[NW][16], s_zz[NW][16], s_D[16];
    const int HG = P.H / P.hpw;
    int tile, hg;
    if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, HG, tile, hg)) return;   // whole workgroup
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tn = lane & 15, g = lane >> 4;
    const int N = P.cv.N, H = P.H, C = P.C;
    const int t0 = tile * 16, tslot = min(t0 + tn, N - 1);
    const float4 tp = P.spos[tslot];
    const int cnt = load_list(P, tile, tid, tp, s_ent, s_mask, s_pos);
    if (cnt < 0) return;   // (whole workgroup) a crowded tile: done by the per-atom kernels
    const int nch = (cnt + 7) >> 3;
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * LOG2E, c_g = -P.rbf_gamma * LOG2E;
    // the atom whose D this thread helps to form: thread = (tile atom, channel of the head)
    const int dt = tid >> 4, dch = tid & 15;
    const int datom = t0 + dt < N ? P.cv.perm[t0 + dt] : -1;
    for (int hh = 0; hh < P.hpw; ++hh) {
        const int head = hg * P.hpw + hh;
        if (tid < 16 * (DKP / 8)) {
            const int tq = tid / (DKP / 8), f8 = tid % (DKP / 8);
            reinterpret_cast<u32x4*>(s_q)[tid] =
                *reinterpret_cast<const u32x4*>(P.q16 + ((size_t)min(t0 + tq, N - 1) * H + head) * DKP + 8 * f8);
        }
        float cb[NB];
        bias_coefficients(P, lane, lane < P.B ? P.WbT[lane * H + head] : 0.0f, cb);
        // <g, out> of this thread's (atom, channel): requested here, summed after the streaming loop
        float dg[n], dout[n];
#pragma unroll
        for (int x = 0; x < n; ++x) {
            const size_t o = ((size_t)max(datom, 0) * n + x) * C + head * 16 + dch;
            dg[x] = P.gout[o];
            dout[x] = P.out[o];
        }
        f16x8 kf[2][KS];
        auto load_K = [&](int c) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
                const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, DKP, 8 * g);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf[mt][ks] = *reinterpret_cast<const f16x8*>(P.k16 + off + 128 * ks);
            }
        };
        if (wave < nch) load_K(wave);
        __syncthreads();   // s_q is in place
        constexpr float M_NONE = -1.0e30f;
        float m = M_NONE, z = 0.0f;
        for (int c = wave; c < nch; c += NW) {
            f32x4 S[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                S[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    S[mt] = mfma(kf[mt][ks], *reinterpret_cast<const f16x8*>(s_q + tn * DKP + 32 * ks + 8 * g), S[mt]);
            }
            load_K(min(c + NW, nch - 1));
            float s2[8], cmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int ei = 8 * c + 4 * mt + g;
                const unsigned mine4 = (unsigned)(s_mask[ei] >> (4 * tn));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float4 pc = s_pos[ei * 4 + r];
                    const float d2 = e2f::dist2_exact(tp.x, tp.y, tp.z, pc.x, pc.y, pc.z);
                    const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f);
                    const float d = __builtin_amdgcn_sqrtf(d2);
                    float bias = bias_value<NB>(cb, d, d2, c_u, c_g, P.rbf_step);
                    asm("" : "+v"(bias));
                    s2[4 * mt + r] = ok ? S[mt][r] + bias : -INFINITY;
                    cmax = fmaxf(cmax, s2[4 * mt + r]);
                }
            }
            const float mn = fmaxf(m, cmax);
            z *= __builtin_amdgcn_exp2f(m - mn);
#pragma unroll
            for (int u = 0; u < 8; ++u) z += __builtin_amdgcn_exp2f(s2[u] - mn);
            m = mn;
        }
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
            const float mo = __shfl_xor(m, off), zo = __shfl_xor(z, off), mn = fmaxf(m, mo);
            z = z * __builtin_amdgcn_exp2f(m - mn) + zo * __builtin_amdgcn_exp2f(mo - mn);
            m = mn;
        }
        if (lane < 16) {
            s_m[wave][lane] = m;
            s_zz[wave][lane] = z;
        }
        {
            float dsum = 0.0f;
#pragma unroll
            for (int x = 0; x < n; ++x) dsum += dg[x] * dout[x];
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) dsum += __shfl_xor(dsum, off);
            if (dch == 0) s_D[dt] = datom >= 0 ? dsum : 0.0f;
        }
        __syncthreads();
        if (tid < 16 && t0 + tid < N) {
            float mm = s_m[0][tid], zz = s_zz[0][tid];
#pragma unroll
            for (int w = 1; w < NW; ++w) {
                const float mo = s_m[w][tid], zo = s_zz[w][tid], mn = fmaxf(mm, mo);
                zz = zz * __builtin_amdgcn_exp2f(mm - mn) + zo * __builtin_amdgcn_exp2f(mo - mn);
                mm = mn;
            }
            const int slot = t0 + tid;
            P.stat4[((size_t)(slot >> 2) * H + head) * 4 + (slot & 3)] = make_float2(zz > 0.0f ? mm + __log2f(zz) : 0.0f, s_D[tid]);
        }
        __syncthreads();   // the next head reuses s_q, s_D and the partials
    }
}

// ---- pair kernel.  SRC = false: the tile's atoms are targets i, candidates are their neighbours j; it forms dq_i and
// -sum_j dL/dr_ij.  SRC = true: the tile's atoms are sources j, candidates are the targets i that see them; it forms
// dk_j and +sum_i dL/dr_ij.  A workgroup owns (tile, hpw heads); its four waves take the tile's chunks in turn and
// never wait for each other inside a head.  Per chunk a wave computes
//   S^T   = Rc Rt^T        logits: candidate rows Rc (k, or q) against the tile's rows Rt (q, or k) from LDS
//   U^T_mu = Xc Xt_mu^T    Xc the candidates' rows of v (or of dL/d out), Xt_mu = G_mu^T g (or G_mu v) of the tile's
//                          atoms, formed once per head into LDS as B operands
//   dT   += dS Y4          dS in the logits' register layout is the A operand; Y4 the candidates' k (or q) with the four
//                          slots of a group per lane
// and the per-pair scalars in between, one tile atom per lane against 8 candidates.
// WGR (target side, B <= 8): also the tile's partial sums of dL/dWb[h][b] = sum_ij ds_ij exp(-gamma (d_ij - b step)^2).
template <int L, bool SRC, int NB, bool WGR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_bwd_tile_pairs(BwdTileParams P) {
    static_assert(!WGR || (!SRC && NB <= 8), "the sums over the radial basis are formed on the target side, in the form for B <= 8");
    constexpr int NW = 4, n = (L + 1) * (L + 1);
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    constexpr int VK = n * 16, VS = (VK + 31) / 32, VKP = VS * 32;
    constexpr int VP = (VS + 2) / 3;   // the value rows are fetched in three phases of at most VP steps
    constexpr int NT = L + 1;          // feature tiles of 16 in dq / dk
    constexpr int GX_BYTES = 3 * VS * 64 * 16, RED_BYTES = NW * NT * 64 * 16;
    static_assert(16 * (DKP / 8) <= 256, "one request per thread");
    __shared__ int s_ent[LENT];
    __shared__ unsigned long long s_mask[LENT];
    __shared__ float4 s_pos[LENT * 4];
    __shared__ __attribute__((aligned(16))) uint16_t s_rows[16 * DKP];
    __shared__ float s_gp[NW][16][3];
    __shared__ float s_wb[NW][8];
    __shared__ float s_G[AXIS_NNZ];
    // the tile side of U as B operands [mu][step][lane]; at the end of a head the same bytes hold the waves' dq tiles
    __shared__ __attribute__((aligned(16))) unsigned char s_big[GX_BYTES > RED_BYTES ? GX_BYTES : RED_BYTES];
    u32x4* s_GX = reinterpret_cast<u32x4*>(s_big);
    uint16_t* s_GX16 = reinterpret_cast<uint16_t*>(s_big);
    f32x4* s_red = reinterpret_cast<f32x4*>(s_big);

    const int HG = P.H / P.hpw;
    int tile, hg;
    if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, HG, tile, hg)) return;   // whole workgroup
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tn = lane & 15, g = lane >> 4;
    const int N = P.cv.N, H = P.H, C = P.C;
    const int t0 = tile * 16, tslot = min(t0 + tn, N - 1);
    const float4 tp = P.spos[tslot];
    const float* __restrict__ Gp = P.G + AXIS_PACKED_AT;
    const float g_mine = tid < AXIS_NNZ ? Gp[tid] : 0.0f;
    const int cnt = load_list(P, tile, tid, tp, s_ent, s_mask, s_pos);
    if (cnt < 0) return;   // (whole workgroup) a crowded tile: done by the per-atom kernels
    if (tid < AXIS_NNZ) s_G[tid] = g_mine;
    __syncthreads();
    const int nch = (cnt + 7) >> 3;
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * LOG2E, c_g = -P.rbf_gamma * LOG2E;
    const float rev = 0.5f / P.cutoff, dphi_scale = -0.5f * 3.14159265358979f / P.cutoff;
    // candidate rows of the logits, of U and of the dq product
    const uint16_t* rowsK = SRC ? P.q16g : P.k16;
    const uint16_t* rowsV = SRC ? P.grow : P.vrow;
    const uint16_t* rows4 = SRC ? P.q4 : P.k4;
    // prologue roles: thread = (tile atom, channel of the head)
    const int pt = tid >> 4, pch = tid & 15, pslot = t0 + pt;
    const int patom = pslot < N ? P.cv.perm[pslot] : -1;
    float gp_acc = 0.0f;   // threads 0..47: (tile atom, axis) sums over this workgroup's heads

    for (int hh = 0; hh < P.hpw; ++hh) {
        const int head = hg * P.hpw + hh;
        // ---- the first chunk's rows are requested before the head's set-up, which hides their latency
        f16x8 kf[2][KS];
        bf16x8 X[2][VP];
        auto load_K = [&](int c) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
                const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, DKP, 8 * g);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf[mt][ks] = *reinterpret_cast<const f16x8*>(rowsK + off + 128 * ks);
            }
        };
        auto load_X = [&](int c, int first, int count) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
                const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, VKP, 8 * g);
#pragma unroll
                for (int s = 0; s < VP; ++s)
                    if (s < count) X[mt][s] = *reinterpret_cast<const bf16x8*>(rowsV + off + 128 * (first + s));
            }
        };
        if (wave < nch) {
            load_K(wave);
            load_X(wave, 0, VP);
        }
        // ---- the tile's rows of the logits -> LDS
        if (tid < 16 * (DKP / 8)) {
            const int tq = tid / (DKP / 8), f8 = tid % (DKP / 8), slot = min(t0 + tq, N - 1);
            reinterpret_cast<u32x4*>(s_rows)[tid] =
                SRC ? *reinterpret_cast<const u32x4*>(P.k16 + e2f::k16_offset(slot, H, head, DKP, 8 * f8))
                    : *reinterpret_cast<const u32x4*>(P.q16 + ((size_t)slot * H + head) * DKP + 8 * f8);
        }
        // ---- the tile side of U: G_mu^T g_i (targets) or G_mu v_j (sources), bf16, as B operands
        {
            float in[n], o[3][n];
#pragma unroll
            for (int x = 0; x < n; ++x) {
                // (loaded from a clamped row and then selected: a load per branch keeps 25 addresses alive)
                if (SRC)
                    in[x] = e2f::bf16_bits_to_float(P.v4[((size_t)(min(pslot, N - 1) >> 2) * H + head) * n * 64 +
                                                         e2f::v4_offset(n, x, pch) + (min(pslot, N - 1) & 3)]);
                else
                    in[x] = P.gout[((size_t)max(patom, 0) * n + x) * C + head * 16 + pch];
                in[x] = pslot < N ? in[x] : 0.0f;
            }
#pragma unroll
            for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                for (int x = 0; x < n; ++x) o[mu][x] = 0.0f;
#pragma unroll
            for (int mu = 0; mu < 3; ++mu)
#pragma unroll
                for (int xo = 0; xo < n; ++xo)
#pragma unroll
                    for (int xi = 0; xi < n; ++xi)
                        if ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u) {
                            const float gv = s_G[AXIS_INDEX.v[mu][xo][xi]];
                            if (SRC) o[mu][xo] += gv * in[xi];
                            else o[mu][xi] += gv * in[xo];
                        }
#pragma unroll
            for (int mu = 0; mu < 3; ++mu) {
#pragma unroll
                for (int x = 0; x < n; ++x) {
                    const int kk = x * 16 + pch;
                    s_GX16[((mu * VS + (kk >> 5)) * 64 + ((kk & 31) >> 3) * 16 + pt) * 8 + (kk & 7)] = e2f::float_to_bf16_bits(o[mu][x]);
                }
                if (VK < VKP) {
                    const int kk = VK + pch;
                    s_GX16[((mu * VS + (kk >> 5)) * 64 + ((kk & 31) >> 3) * 16 + pt) * 8 + (kk & 7)] = 0;
                }
            }
        }
        float cb[NB];
        bias_coefficients(P, lane, lane < P.B ? P.WbT[lane * H + head] : 0.0f, cb);
        // the tile atom's own statistics (targets); sources read those of the candidates per chunk
        const float2 st_mine = P.stat4[((size_t)(tslot >> 2) * H + head) * 4 + (tslot & 3)];
        __syncthreads();

        f32x4 dacc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) dacc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        float gx = 0.0f, gy = 0.0f, gz = 0.0f;
        float wbacc[WGR ? NB : 1];   // per lane: sum over its pairs of ds e^{-gamma d^2} u^b (the factor of b comes at the end)
        if constexpr (WGR) {
#pragma unroll
            for (int b = 0; b < NB; ++b) wbacc[b] = 0.0f;
        }

        for (int c = wave; c < nch; c += NW) {
            const int cn = min(c + NW, nch - 1);
            // candidates' statistics (sources) and their rows for the dq product
            float4 st[2][2];
            if (SRC) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    const unsigned grp = (unsigned)s_ent[8 * c + 4 * mt + g] >> 8;
                    const float4* sp = reinterpret_cast<const float4*>(P.stat4 + ((size_t)grp * H + head) * 4);
                    st[mt][0] = sp[0];
                    st[mt][1] = sp[1];
                }
            }
            // ---- logits
            f32x4 S[2];
            {
                f16x8 qf[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const f16x8*>(s_rows + tn * DKP + 32 * ks + 8 * g);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    S[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) S[mt] = mfma(kf[mt][ks], qf[ks], S[mt]);
                }
            }
            // ---- U in three phases of steps; the rows of the next phase are fetched while the per-pair scalars of
            // this one are worked out
            f32x4 U[3][2];
#pragma unroll
            for (int mu = 0; mu < 3; ++mu) U[mu][0] = U[mu][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
            // (the tile side's operands are the same for every chunk; read through an index the compiler cannot
            // follow they stay in LDS instead of being held, and spilled, across the loop)
            int gx_lane = lane;
            asm volatile("" : "+v"(gx_lane));
            auto u_phase = [&](int first, int count) {
#pragma unroll
                for (int s = 0; s < VP; ++s)
                    if (s < count) {
#pragma unroll
                        for (int mu = 0; mu < 3; ++mu) {
                            const bf16x8 b = __builtin_bit_cast(bf16x8, s_GX[(mu * VS + first + s) * 64 + gx_lane]);
                            U[mu][0] = mfma(X[0][s], b, U[mu][0]);
                            U[mu][1] = mfma(X[1][s], b, U[mu][1]);
                        }
                    }
            };
            // what depends on the pair's distance and logit alone: P_ij, the gate and the bias's derivative
            float p[8], phi[8], db[8];
            auto scalars = [&](int mt) {
                const int ei = 8 * c + 4 * mt + g;
                const unsigned mine4 = (unsigned)(s_mask[ei] >> (4 * tn));
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int u = 4 * mt + r;
                    const float4 pc = s_pos[ei * 4 + r];
                    const float d2 = e2f::dist2_exact(tp.x, tp.y, tp.z, pc.x, pc.y, pc.z);
                    const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f);
                    const float d = __builtin_amdgcn_sqrtf(d2);
                    float bias, dbias;   // the bias in base-2 units, its derivative in natural units
                    bias_value_grad<NB>(cb, d, d2, c_u, c_g, P.rbf_step, P.rbf_gamma, bias, dbias);
                    asm("" : "+v"(bias), "+v"(dbias));   // (evaluated for every candidate: one basic block)
                    const float lse = SRC ? (r == 0 ? st[mt][0].x : r == 1 ? st[mt][0].z : r == 2 ? st[mt][1].x : st[mt][1].z) : st_mine.x;
                    p[u] = ok ? __builtin_amdgcn_exp2f(S[mt][r] + bias - lse) : 0.0f;
                    db[u] = ok ? dbias : 0.0f;
                    phi[u] = 0.5f + 0.5f * __builtin_amdgcn_cosf(d * rev);
                }
            };
            u_phase(0, VP);
            load_X(c, VP, min(VP, VS - VP));
            scalars(0);
            u_phase(VP, min(VP, VS - VP));
            load_X(c, 2 * VP, VS - 2 * VP);
            scalars(1);
            u_phase(2 * VP, VS - 2 * VP);
            // the candidates' k (q) rows, four slots of a group per lane, for the dq (dk) product; requested before the
            // next chunk's rows, so that waiting for them (loads complete in order) does not wait for those
            VRows<KS> y4;
            {
                const unsigned ea = (unsigned)s_ent[8 * c + g] >> 8, eb = (unsigned)s_ent[8 * c + 4 + g] >> 8;
                const uint16_t* ba = rows4 + ((size_t)ea * H + head) * KS * 128 + tn * 8;
                const uint16_t* bb = rows4 + ((size_t)eb * H + head) * KS * 128 + tn * 8;
#pragma unroll
                for (int pp = 0; pp < KS; ++pp) y4.load_pair(pp, ba, bb);
            }
            load_X(cn, 0, VP);
            load_K(cn);
            // ---- ds and the position gradient
            float ds[8];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int ei = 8 * c + 4 * mt + g;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int u = 4 * mt + r;
                    const float4 pc = s_pos[ei * 4 + r];
                    // r_ij = pos_j - pos_i: candidate minus tile atom for targets, the reverse for sources
                    const float rx = SRC ? tp.x - pc.x : pc.x - tp.x, ry = SRC ? tp.y - pc.y : pc.y - tp.y,
                                rz = SRC ? tp.z - pc.z : pc.z - tp.z;
                    const float d2 = rx * rx + ry * ry + rz * rz;
                    const float rd = p[u] > 0.0f ? __builtin_amdgcn_rsqf(d2) : 0.0f;
                    const float u0 = U[0][mt][r], u1 = U[1][mt][r], u2 = U[2][mt][r];
                    const float w = rx * u0 + ry * u1 + rz * u2;
                    const float Dn = SRC ? (r == 0 ? st[mt][0].y : r == 1 ? st[mt][0].w : r == 2 ? st[mt][1].y : st[mt][1].w) : st_mine.y;
                    // (selected: the statistics of slots behind the last atom are never written)
                    ds[u] = p[u] > 0.0f ? p[u] * (phi[u] * w - Dn) : 0.0f;
                    const float alpha = p[u] * phi[u];
                    // phi' = -(pi / 2 r_c) sin(pi d / r_c), and sin = 2 sqrt(phi (1 - phi)) on [0, r_c]
                    const float dphi = 2.0f * dphi_scale * __builtin_amdgcn_sqrtf(fmaxf(phi[u] * (1.0f - phi[u]), 0.0f));
                    const float dd = (ds[u] * db[u] + p[u] * w * dphi) * rd;
                    gx += alpha * u0 + dd * rx;
                    gy += alpha * u1 + dd * ry;
                    gz += alpha * u2 + dd * rz;
                    if constexpr (WGR) {
                        // exp(-gamma (d - b step)^2) = e^{-gamma d^2} u^b e^{-gamma (b step)^2}, u = e^{2 gamma step d}
                        float t = ds[u] * __builtin_amdgcn_exp2f(c_g * d2);
                        const float uu = __builtin_amdgcn_exp2f(c_u * (d2 * rd));
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            wbacc[b] += t;
                            t *= uu;
                        }
                    }
                }
            }
            // ---- dq (dk) += dS Y4
            {
                const bf16x8 A = __builtin_bit_cast(bf16x8, (u32x4){pack_bf16(ds[0], ds[1]), pack_bf16(ds[2], ds[3]),
                                                                    pack_bf16(ds[4], ds[5]), pack_bf16(ds[6], ds[7])});
#pragma unroll
                for (int t = 0; t < NT; ++t) dacc[t] = mfma(A, (t & 1) ? y4.second(t >> 1) : y4.first(t >> 1), dacc[t]);
            }
        }
        // ---- the waves' partial sums together: dq (dk) rows of the tile's atoms, caller's order
        gx += __shfl_xor(gx, 16); gx += __shfl_xor(gx, 32);
        gy += __shfl_xor(gy, 16); gy += __shfl_xor(gy, 32);
        gz += __shfl_xor(gz, 16); gz += __shfl_xor(gz, 32);
        __syncthreads();   // every wave has left the loop: s_GX is free
        if (lane < 16) {
            s_gp[wave][lane][0] = gx;
            s_gp[wave][lane][1] = gy;
            s_gp[wave][lane][2] = gz;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) s_red[(wave * NT + t) * 64 + lane] = dacc[t];
        __syncthreads();
        if (tid < 48) {
            const int t = tid / 3, ax = tid % 3;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += s_gp[w][t][ax];
            gp_acc += s;
        }
        if constexpr (WGR) {   // the tile's sums over the radial basis: lanes, then waves, in a fixed order
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float v = wbacc[b];
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) v += __shfl_xor(v, off);
                if (lane == 0) s_wb[wave][b] = v;
            }
        }
        {
            const float scale = SRC ? LN2 : P.tau;   // q rows carry tau log2 e; k rows are plain
            float* dst = SRC ? P.gk : P.gq;
            for (int it = tid; it < NT * 64; it += 256) {
                const int t = it >> 6, ln = it & 63;
                f32x4 s = s_red[t * 64 + ln];
#pragma unroll
                for (int w = 1; w < NW; ++w) s += s_red[(w * NT + t) * 64 + ln];
                const int fch = ln & 15, gg = ln >> 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int slot = t0 + 4 * gg + r;
                    if (slot < N) dst[((size_t)P.cv.perm[slot] * (L + 1) + t) * C + head * 16 + fch] = s[r] * scale;
                }
            }
        }
        __syncthreads();   // the next head rewrites s_rows, s_GX and the partials
        if constexpr (WGR) {
            if (tid < P.B) {
                const float bs = (float)tid * P.rbf_step;
                P.pWb_t[((size_t)tile * H + head) * P.B + tid] =
                    (s_wb[0][tid] + s_wb[1][tid] + s_wb[2][tid] + s_wb[3][tid]) * __expf(-P.rbf_gamma * bs * bs);
            }
        }
    }
    if (tid < 48 && t0 + tid / 3 < N)
        P.gp_part[(((size_t)(SRC ? 1 : 0) * HG + hg) * N + t0 + tid / 3) * 3 + tid % 3] = SRC ? gp_acc : -gp_acc;
}

// ---- dv_j = sum_mu G_mu^T Y_mu,  Y_mu[j] = sum_i alpha_ij (r_ij)_mu g_i: the aggregation of the forward kernel with the
// tile's atoms as sources j, the candidates as the targets i that see them, dL/d out in place of the value rows and
// the softmax weights from the stored statistics.  The waves score a chunk each and share the weights through LDS (two
// buffers, one barrier per group of four chunks); every wave aggregates all four chunks into its quarter of the
// components.
// WGR: also the tile's partial sums of the path-weight gradient.  The message is linear in the path weights,
// G_mu[xo][xi] = w_path[li(xi)][lo(xo)] Gu_mu[xo][xi] with the unit-weight operators Gu, so
//   dL/dw_path[li][lo] = sum_j sum_mu sum_{xo in lo, xi in li} Y_mu[j][xo] Gu_mu[xo][xi] v_j[xi],
// formed in the epilogue from the Y_mu that are in LDS there anyway.
template <int L, int NB, bool WGR>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_bwd_tile_dv(BwdTileParams P) {
    constexpr int NW = 4, n = (L + 1) * (L + 1), NX = (n + NW - 1) / NW;
    constexpr int DK = (L + 1) * 16, KS = (DK + 31) / 32, DKP = KS * 32;
    constexpr int W_BYTES = 2 * NW * 3 * 64 * 16, PO_BYTES = n * 64 * 16;
    static_assert(16 * (DKP / 8) <= 256, "one request per thread");
    __shared__ int s_ent[LENT];
    __shared__ unsigned long long s_mask[LENT];
    __shared__ float4 s_pos[LENT * 4];
    __shared__ __attribute__((aligned(16))) uint16_t s_rows[16 * DKP];
    __shared__ float s_G[AXIS_NNZ];
    __shared__ float s_Gu[WGR ? AXIS_NNZ : 1];
    __shared__ float s_bins[NW][32];
    __shared__ __attribute__((aligned(16))) f32x4 s_vt[WGR ? n * 64 : 1];   // value rows of the tile's atoms, [component][lane]
    __shared__ uint32_t s_tab[WGR ? AXIS_NNZ : 1];   // PATH_TABLE in LDS (a dependent read from memory per entry otherwise)
    __shared__ int16_t s_tstart[WGR ? 3 * 26 : 1];
    __shared__ int s_orow[16];
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[W_BYTES > PO_BYTES ? W_BYTES : PO_BYTES];
    u32x4* s_W = reinterpret_cast<u32x4*>(s_raw);
    f32x4* s_po = reinterpret_cast<f32x4*>(s_raw);

    const int HG = P.H / P.hpw;
    int tile, hg;
    if (!tile_xcd_remap(blockIdx.x, P.n_tiles, P.blk, HG, tile, hg)) return;   // whole workgroup
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, tn = lane & 15, g = lane >> 4;
    constexpr int NP = NX / 2, NS = 1 + 2 * NP;
    constexpr bool HAS_ODD = (NX & 1) || (n % NW != 0 && ((NX - 1) & 1));
    const int nxw = n / NW + (wave < n % NW ? 1 : 0);
    const int x0 = wave * (n / NW) + min(wave, n % NW);
    static_assert((n / NW) / 2 == NP, "every wave has NP pairs of components (a wave with one component more has it unpaired)");
    constexpr int npair = NP;
    const bool single = (nxw & 1) != 0;
    const int N = P.cv.N, H = P.H;
    const int t0 = tile * 16, nt = min(16, N - t0), tslot = min(t0 + tn, N - 1);
    const float4 tp = P.spos[tslot];
    const int orow_mine = tid < 16 ? (t0 + tid < N ? P.cv.perm[t0 + tid] : -1) : 0;
    const float g_mine = tid < AXIS_NNZ ? P.G[AXIS_PACKED_AT + tid] : 0.0f;
    const float gu_mine = WGR && tid < AXIS_NNZ ? P.Gu[AXIS_PACKED_AT + tid] : 0.0f;
    const int cnt = load_list(P, tile, tid, tp, s_ent, s_mask, s_pos);
    if (cnt < 0) return;   // (whole workgroup) a crowded tile: done by the per-atom kernels
    if (tid < AXIS_NNZ) s_G[tid] = g_mine;
    if (WGR && tid < AXIS_NNZ) {
        s_Gu[tid] = gu_mine;
        s_tab[tid] = PATH_TABLE.ent[tid];
        if (tid < 3 * 26) s_tstart[tid] = PATH_TABLE.start[tid / 26][tid % 26];
    }
    if (tid < 16) s_orow[tid] = orow_mine;
    if (WGR && tid < NW * 32) (&s_bins[0][0])[tid] = 0.0f;   // the waves' bins li * (L + 1) + lo, over this workgroup's heads
    const int nch = (cnt + 7) >> 3, ngr = (nch + NW - 1) / NW;
    const float c_u = 2.0f * P.rbf_gamma * P.rbf_step * LOG2E, c_g = -P.rbf_gamma * LOG2E;

    f16x8 kf[2][KS];
    VRows<NP> vr;
    auto load_K = [&](int c, int head) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int e = s_ent[8 * c + 4 * mt + (tn >> 2)];
            const size_t off = e2f::k16_offset(4 * (size_t)((unsigned)e >> 8) + (tn & 3), H, head, DKP, 8 * g);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[mt][ks] = *reinterpret_cast<const f16x8*>(P.q16g + off + 128 * ks);
        }
    };
    auto v_base = [&](int c, int head, const uint16_t*& ba, const uint16_t*& bb) {
        const unsigned ea = (unsigned)s_ent[8 * c + g] >> 8, eb = (unsigned)s_ent[8 * c + 4 + g] >> 8;
        ba = P.g4 + (((size_t)ea * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
        bb = P.g4 + (((size_t)eb * H + head) * n + x0) * 64 + (single ? 64 : 0) + tn * 8;
    };

    for (int hh = 0; hh < P.hpw; ++hh) {
        const int head = hg * P.hpw + hh;
        if (tid < 16 * (DKP / 8)) {   // the tile's k rows
            const int tq = tid / (DKP / 8), f8 = tid % (DKP / 8);
            reinterpret_cast<u32x4*>(s_rows)[tid] =
                *reinterpret_cast<const u32x4*>(P.k16 + e2f::k16_offset(min(t0 + tq, N - 1), H, head, DKP, 8 * f8));
        }
        float cb[NB];
        bias_coefficients(P, lane, lane < P.B ? P.WbT[lane * H + head] : 0.0f, cb);
        if (nch > 0) {
            load_K(min(wave, nch - 1), head);
            const uint16_t *ba, *bb;
            v_base(0, head, ba, bb);
#pragma unroll
            for (int p = 0; p < NP; ++p)
                if (p < npair) vr.load_pair(p, ba, bb);
            if (HAS_ODD && single) vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);
        }
        f32x4 acc[3][NS];
#pragma unroll
        for (int mu = 0; mu < 3; ++mu)
#pragma unroll
            for (int x = 0; x < NS; ++x) acc[mu][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
        __syncthreads();   // s_rows (and, for the first head, s_G and s_orow) are in place

        for (int G = 0; G < ngr; ++G) {
            const int cm = NW * G + wave;
            // the candidates' lse: the four slots of the lane's two entries
            float4 st[2][2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const unsigned grp = (unsigned)s_ent[8 * cm + 4 * mt + g] >> 8;
                const float4* sp = reinterpret_cast<const float4*>(P.stat4 + ((size_t)grp * H + head) * 4);
                st[mt][0] = sp[0];
                st[mt][1] = sp[1];
            }
            f32x4 S[2];
            {
                f16x8 qf[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const f16x8*>(s_rows + tn * DKP + 32 * ks + 8 * g);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    S[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) S[mt] = mfma(kf[mt][ks], qf[ks], S[mt]);
                }
            }
            load_K(min(cm + NW, nch - 1), head);
            {
                uint32_t wp[3][4];
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    float pg[2], rx[2], ry[2], rz[2];
#pragma unroll
                    for (int dd = 0; dd < 2; ++dd) {
                        const int uu_ = u + dd, mt = uu_ >> 2, r = uu_ & 3, ei = 8 * cm + 4 * mt + g;
                        const unsigned mine4 = (unsigned)(s_mask[ei] >> (4 * tn));
                        const float4 pc = s_pos[ei * 4 + r];
                        const float d2 = e2f::dist2_exact(tp.x, tp.y, tp.z, pc.x, pc.y, pc.z);
                        const bool ok = (((mine4 >> r) & 1u) != 0u) & (d2 < P.rc2) & (d2 > 0.0f);
                        const float d = __builtin_amdgcn_sqrtf(d2);
                        float bias = bias_value<NB>(cb, d, d2, c_u, c_g, P.rbf_step);
                        asm("" : "+v"(bias));
                        const float lse = r == 0 ? st[mt][0].x : r == 1 ? st[mt][0].z : r == 2 ? st[mt][1].x : st[mt][1].z;
                        const float p = ok ? __builtin_amdgcn_exp2f(S[mt][r] + bias - lse) : 0.0f;
                        pg[dd] = p * e2f::radial_gate(d, P.cutoff);
                        rx[dd] = tp.x - pc.x;   // r_ij = pos_j - pos_i with j the tile's atom
                        ry[dd] = tp.y - pc.y;
                        rz[dd] = tp.z - pc.z;
                    }
                    wp[0][u >> 1] = pack_bf16(pg[0] * rx[0], pg[1] * rx[1]);
                    wp[1][u >> 1] = pack_bf16(pg[0] * ry[0], pg[1] * ry[1]);
                    wp[2][u >> 1] = pack_bf16(pg[0] * rz[0], pg[1] * rz[1]);
                }
#pragma unroll
                for (int mu = 0; mu < 3; ++mu)
                    s_W[(((G & 1) * NW + wave) * 3 + mu) * 64 + lane] = (u32x4){wp[mu][0], wp[mu][1], wp[mu][2], wp[mu][3]};
            }
            __syncthreads();
#pragma unroll
            for (int cc = 0; cc < NW; ++cc) {
                const int c = NW * G + cc;
                if (c < nch) {
                    bf16x8 W[3];
#pragma unroll
                    for (int mu = 0; mu < 3; ++mu) W[mu] = __builtin_bit_cast(bf16x8, s_W[(((G & 1) * NW + cc) * 3 + mu) * 64 + lane]);
                    const uint16_t *ba, *bb;
                    v_base(min(c + 1, nch - 1), head, ba, bb);
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        if (p < npair) {   // (wave-uniform)
                            const bf16x8 b0 = vr.first(p), b1 = vr.second(p);
#pragma unroll
                            for (int mu = 0; mu < 3; ++mu) acc[mu][1 + 2 * p] = mfma(W[mu], b0, acc[mu][1 + 2 * p]);
#pragma unroll
                            for (int mu = 0; mu < 3; ++mu) acc[mu][2 + 2 * p] = mfma(W[mu], b1, acc[mu][2 + 2 * p]);
                            vr.load_pair(p, ba, bb);
                        }
                    if (HAS_ODD && single) {   // (wave-uniform) the odd component last: see k_tile_heads
                        const bf16x8 bv = vr.single();
#pragma unroll
                        for (int mu = 0; mu < 3; ++mu) acc[mu][0] = mfma(W[mu], bv, acc[mu][0]);
                        vr.load_single(ba - 64 - tn * 4, bb - 64 - tn * 4);
                    }
                }
            }
        }
        // ---- epilogue: dv = sum_mu G_mu^T Y_mu.  For one mu at a time the waves put their Y_mu components into LDS and
        // every wave forms the components x_in = wave (mod NW) from the non-zero entries of G_mu.
        auto finish = [&](auto wv_tag) {
            constexpr int WV = decltype(wv_tag)::value;
            constexpr int RO = (n - WV + NW - 1) / NW;
            constexpr int X0 = WV * (n / NW) + (WV < n % NW ? WV : n % NW);
            constexpr int NXW = n / NW + (WV < n % NW ? 1 : 0);
            f32x4 pr[RO];
#pragma unroll
            for (int i = 0; i < RO; ++i) pr[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mu = 0; mu < 3; ++mu) {
                __syncthreads();
#pragma unroll
                for (int x = 0; x < NXW; ++x) s_po[(X0 + x) * 64 + lane] = acc[mu][x + ((NXW & 1) ? 0 : 1)];
                __syncthreads();
#pragma unroll
                for (int i = 0; i < RO; ++i) {
#pragma unroll
                    for (int xo = 0; xo < n; ++xo)
                        if ((E2F_AXIS_NZ[mu][xo] >> (WV + NW * i)) & 1u) {   // (one statement; braces kept for the diff)
                            pr[i] += s_G[AXIS_INDEX.v[mu][xo][WV + NW * i]] * s_po[xo * 64 + lane];
                        }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = s_orow[4 * g + r];
                if (row >= 0) {
                    float* orp = P.gv + (size_t)row * n * P.C + head * 16 + tn;
#pragma unroll
                    for (int i = 0; i < RO; ++i) orp[(size_t)(WV + NW * i) * P.C] = pr[i][r];
                }
            }
        };
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        if (wave_u == 0) finish(std::integral_constant<int, 0>{});
        if (wave_u == 1) finish(std::integral_constant<int, 1>{});
        if (wave_u == 2) finish(std::integral_constant<int, 2>{});
        if (wave_u == 3) finish(std::integral_constant<int, 3>{});
        if constexpr (WGR) {
            // ---- path-weight bins of this head: sum over the tile's atoms j (rows 4g..4g+3 of a lane), channels (lanes)
            // and the entries (x_out, x_in) of a group (mu, l_in, l_out) of Y_mu[x_out] Gu_mu[x_out][x_in] v_j[x_in].  A
            // loop over a table rather than straight-line code: the Y_mu go through LDS once more, one mu at a time.
            {
                const size_t grp = min((size_t)(t0 >> 2) + g, (size_t)(N - 1) >> 2);
                for (int x = wave; x < n; x += NW) {
                    const u32x2 four = *reinterpret_cast<const u32x2*>(P.v4 + (grp * H + head) * n * 64 + e2f::v4_offset(n, x, tn));
                    s_vt[x * 64 + lane] = (f32x4){__uint_as_float(four[0] << 16), __uint_as_float(four[0] & 0xffff0000u),
                                                  __uint_as_float(four[1] << 16), __uint_as_float(four[1] & 0xffff0000u)};
                }
            }
#pragma unroll
            for (int mu = 0; mu < 3; ++mu) {
                __syncthreads();
#pragma unroll
                for (int sl = 0; sl < NS; ++sl) {   // accumulator slot sl holds component x0 + sl (odd count) or x0 + sl - 1
                    const int xl = sl - (single ? 0 : 1);
                    if (xl >= 0 && xl < nxw) s_po[(x0 + xl) * 64 + lane] = acc[mu][sl];
                }
                __syncthreads();
                for (int bin = wave; bin < 25; bin += NW) {
                    const int li = bin / 5, lo = bin % 5;
                    const int e0 = s_tstart[mu * 26 + bin], e1 = s_tstart[mu * 26 + bin + 1];
                    if (li > L || lo > L || e0 == e1) continue;   // (wave-uniform)
                    float sum = 0.0f;
#pragma unroll 4
                    for (int e = e0; e < e1; ++e) {
                        const uint32_t en = s_tab[e];
                        const f32x4 y = s_po[(en & 0xffu) * 64 + lane], v = s_vt[((en >> 8) & 0xffu) * 64 + lane];
                        sum += s_Gu[en >> 16] * (y[0] * v[0] + y[1] * v[1] + y[2] * v[2] + y[3] * v[3]);
                    }
#pragma unroll
                    for (int off = 1; off < 64; off <<= 1) sum += __shfl_xor(sum, off);
                    if (lane == 0) s_bins[wave][li * (L + 1) + lo] += sum;
                }
            }
        }
        __syncthreads();   // the next head rewrites s_rows and the weight buffers
    }
    if constexpr (WGR) {   // the tile's bins: the waves' sums in a fixed order (the last head's barrier lies in between)
        if (tid < 32)
            P.pwp_t[((size_t)tile * HG + hg) * 32 + tid] =
                tid < (L + 1) * (L + 1) ? s_bins[0][tid] + s_bins[1][tid] + s_bins[2][tid] + s_bins[3][tid] : 0.0f;
    }
    (void)nt;
}

// Sums of the weight-gradient partials in a fixed order: one workgroup per output element m, over the tiles whose
// list fitted (rows_per_tile rows each) and over the atoms of the crowded tiles (per-atom kernels' rows).
__global__ __launch_bounds__(256) void k_bwd_wsum(E2fCellsView cv, const int4* __restrict__ hdr, const float* __restrict__ tile_part,
                                                  int rows_per_tile, int tile_stride, const float* __restrict__ atom_part,
                                                  int atom_stride, int n_tiles, int M, float* __restrict__ out) {
    __shared__ float s_acc[256];
    const int m = blockIdx.x, N = cv.N;
    float s = 0.0f;
    for (int t = threadIdx.x; t < n_tiles; t += 256) {
        if (hdr[t].x >= 0) {
            for (int r = 0; r < rows_per_tile; ++r) s += tile_part[((size_t)t * rows_per_tile + r) * tile_stride + m];
        } else {
            for (int slot = 16 * t; slot < min(16 * t + 16, N); ++slot) s += atom_part[(size_t)cv.perm[slot] * atom_stride + m];
        }
    }
    s_acc[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_acc[threadIdx.x] += s_acc[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0 && m < M) out[m] = s_acc[0];
}

// gpos[atom] = sum of the partial sums of both sides and all head groups, in a fixed order
__global__ __launch_bounds__(256) void k_bwd_gpos_reduce(E2fCellsView cv, const float* __restrict__ part, int parts,
                                                         const int4* __restrict__ hdr, float* __restrict__ gpos) {
    const int i = blockIdx.x * 256 + threadIdx.x, N = cv.N;
    if (i >= N * 3) return;
    const int slot = i / 3, ax = i % 3;
    if (hdr[slot >> 4].x < 0) return;   // a crowded tile: written by the per-atom kernels
    float s = 0.0f;
    for (int p = 0; p < parts; ++p) s += part[((size_t)p * N + slot) * 3 + ax];
    gpos[(size_t)cv.perm[slot] * 3 + ax] = s;
}

template <int L>
void launch_L(const BwdTileParams& P, bool wgrad, hipStream_t st) {
    const int N = P.cv.N, groups = (N + 3) / 4, HG = P.H / P.hpw;
    const int grid = tile_grid(P.n_tiles, P.blk, HG);
    // the statistics kernel, whose workgroups are short, runs faster on small XCD chunks (0.099 against 0.110 ms at
    // 10 000 atoms with 20 tiles per chunk instead of 79)
    BwdTileParams Ps = P;
    Ps.blk = P.blk < TILE_BLK_MANY ? P.blk : TILE_BLK_MANY;
    const int grid_s = tile_grid(P.n_tiles, Ps.blk, HG);
    k_bwd_relayout_qk<L><<<groups, 256, 0, st>>>(P);
    k_bwd_relayout_v<L><<<groups, 256, 0, st>>>(P);
    k_bwd_relayout_g<L><<<groups, 256, 0, st>>>(P);
    if (P.B > 8) {   // (the radial bias polynomial has its coefficients in registers: instances for B <= 8 and B <= 16)
        k_bwd_tile_stats<L, 16><<<grid_s, 256, 0, st>>>(Ps);
        k_bwd_tile_pairs<L, false, 16, false><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_pairs<L, true, 16, false><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_dv<L, 16, false><<<grid, 256, 0, st>>>(P);
    } else if (wgrad) {
        k_bwd_tile_stats<L, 8><<<grid_s, 256, 0, st>>>(Ps);
        k_bwd_tile_pairs<L, false, 8, true><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_pairs<L, true, 8, false><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_dv<L, 8, true><<<grid, 256, 0, st>>>(P);
    } else {
        k_bwd_tile_stats<L, 8><<<grid_s, 256, 0, st>>>(Ps);
        k_bwd_tile_pairs<L, false, 8, false><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_pairs<L, true, 8, false><<<grid, 256, 0, st>>>(P);
        k_bwd_tile_dv<L, 8, false><<<grid, 256, 0, st>>>(P);
    }
    k_bwd_gpos_reduce<<<(N * 3 + 255) / 256, 256, 0, st>>>(P.cv, P.gp_part, 2 * HG, P.lists_hdr, P.gpos);
}

}  // namespace

// Heads per workgroup of the tile kernels above: up to four, as long as about eight rounds of workgroups are left for the
// chip (a head's set-up is not shared between heads here, so fewer, longer workgroups only pay in the tail: measured
// 1.5 % behind with two heads per workgroup at 10 000 atoms).
static int e2f_bwd_tile_heads_per_workgroup(int n_tiles, int H) {
    int hpw = 1;
    while (hpw < 4 && H % (hpw * 2) == 0 && (long)n_tiles * H / (hpw * 2) >= 4096) hpw *= 2;
    return hpw;
}

E2fBwdTileWs e2f_bwd_tile_ws_layout(const e2f_ctx* ctx, int32_t N, void* ws, size_t offset) {
    E2fBwdTileWs T;
    size_t off = offset;
    auto take = [&](size_t bytes) {
        char* p = ws ? static_cast<char*>(ws) + off : nullptr;
        off += e2f_align_up(bytes);
        return p;
    };
    const size_t H = ctx->cfg.H, n = ctx->n, groups = ((size_t)N + 3) / 4;
    const size_t DKP = ((size_t)(ctx->cfg.L_max + 1) * 16 + 31) / 32 * 32, VKP = (n * 16 + 31) / 32 * 32;
    T.q16g = (uint16_t*)take(groups * 4 * H * DKP * 2);
    T.q4 = (uint16_t*)take(groups * 4 * H * DKP * 2);
    T.k4 = (uint16_t*)take(groups * 4 * H * DKP * 2);
    T.vrow = (uint16_t*)take(groups * 4 * H * VKP * 2);
    T.grow = (uint16_t*)take(groups * 4 * H * VKP * 2);
    T.g4 = (uint16_t*)take(groups * H * n * 64 * 2);
    T.stat4 = (float*)take(groups * 4 * H * 8);
    T.gp_part = (float*)take((size_t)2 * H * N * 3 * 4);
    const size_t n_tiles = ((size_t)N + 15) / 16;
    T.pWb_t = (float*)take(n_tiles * H * ctx->cfg.B * 4);
    T.pwp_t = (float*)take(n_tiles * H * 32 * 4);
    T.Gu = (float*)take((size_t)(3 * E2F_MAX_N * E2F_MAX_N + 256) * 4);
    T.bytes = off;
    return T;
}

// The tile kernels of the backward pass for every tile whose candidate list fits; the lists (and the axis operators)
// must have been written by e2f_launch_tile_lists, q16 / k16 / v4 by the projection in the tile layout.
bool e2f_backward_tile_weight_gradients_supported(const e2f_ctx* ctx) { return ctx->cfg.B <= 8; }

// wgrad: also the per-tile partial sums of dL/dWb and dL/dw_path (tw.Gu must hold the unit-weight axis operators).
e2f_status e2f_launch_backward_tile(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws,
                                    const E2fBwdTileWs& tw, const float* out, const float* grad_out, float* grad_pos,
                                    float* grad_q, float* grad_k, float* grad_v, bool wgrad, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (wgrad && !e2f_backward_tile_weight_gradients_supported(ctx)) return E2F_ERR_UNSUPPORTED;
    BwdTileParams P;
    P.cv = cv;
    P.spos = ws.spos; P.q16 = ws.q16; P.k16 = ws.k16; P.v4 = ws.v4; P.G = ws.G; P.WbT = ws.wbT;
    P.q16g = tw.q16g; P.q4 = tw.q4; P.k4 = tw.k4; P.vrow = tw.vrow; P.grow = tw.grow; P.g4 = tw.g4;
    P.stat4 = reinterpret_cast<float2*>(tw.stat4); P.gp_part = tw.gp_part;
    P.pWb_t = tw.pWb_t; P.pwp_t = tw.pwp_t; P.Gu = tw.Gu;
    P.out = out; P.gout = grad_out; P.gq = grad_q; P.gk = grad_k; P.gv = grad_v; P.gpos = grad_pos;
    P.lists_hdr = ws.lists_hdr; P.lists_ent = ws.lists_ent; P.lists_pos = ws.lists_pos; P.lists_mask = ws.lists_mask;
    P.C = ctx->cfg.C; P.H = ctx->cfg.H; P.B = ctx->cfg.B; P.n_tiles = (cv.N + 15) / 16; P.blk = tile_blk(P.n_tiles);
    P.hpw = e2f_bwd_tile_heads_per_workgroup(P.n_tiles, P.H);
    P.tau = ctx->tau; P.rc2 = ctx->rc2; P.cutoff = ctx->cfg.cutoff; P.rbf_step = ctx->rbf_step; P.rbf_gamma = ctx->rbf_gamma;
    switch (ctx->cfg.L_max) {
        case 1: launch_L<1>(P, wgrad, st); break;
        case 2: launch_L<2>(P, wgrad, st); break;
        case 3: launch_L<3>(P, wgrad, st); break;
        case 4: launch_L<4>(P, wgrad, st); break;
        default: return E2F_ERR_UNSUPPORTED;
    }
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

// Sums of the partials that the tile kernels (per tile) and the per-atom kernels (atoms of crowded tiles) leave.
e2f_status e2f_launch_backward_tile_wsum(const e2f_ctx* ctx, const E2fCellsView& cv, const E2fAttnWs& ws,
                                         const E2fBwdTileWs& tw, const float* atom_pWb, const float* atom_pwp,
                                         float* grad_Wb, float* grad_w_path, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    const int n_tiles = (cv.N + 15) / 16, HB = ctx->cfg.H * ctx->cfg.B, L1 = ctx->cfg.L_max + 1;
    const int hpw = e2f_bwd_tile_heads_per_workgroup(n_tiles, ctx->cfg.H);
    if (grad_Wb) k_bwd_wsum<<<HB, 256, 0, st>>>(cv, ws.lists_hdr, tw.pWb_t, 1, HB, atom_pWb, HB, n_tiles, HB, grad_Wb);
    if (grad_w_path)
        k_bwd_wsum<<<L1 * L1, 256, 0, st>>>(cv, ws.lists_hdr, tw.pwp_t, ctx->cfg.H / hpw, 32, atom_pwp, 32, n_tiles, L1 * L1, grad_w_path);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
