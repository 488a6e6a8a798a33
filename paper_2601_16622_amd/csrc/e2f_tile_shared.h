// Shared by the tile kernels of the forward pass (e2f_tile.hip) and of the backward pass (e2f_bwd_tile.hip): vector
// types, matrix-core wrappers, the value-row registers of a chunk, the XCD-aware workgroup map and the packed index
// of the axis operators' non-zero pattern.
#pragma once
#include <limits.h>

#include <type_traits>

#include "e2f_axis_pattern.h"
#include "e2f_device.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int CAPG = 256;      // candidate groups (of four slots) held in LDS per batch
constexpr int LCAP = E2F_TILE_LCAP;   // entries of a precomputed list; longer lists are built in the kernel
static_assert(LCAP <= CAPG, "a precomputed list must fit the list area in LDS");
// Consecutive tiles whose (tile, head) items form one XCD chunk, head-major: the tiles are cut into 8 k chunks of equal
// size, so that every XCD gets k chunks.  The larger the chunk, the smaller the share of candidate rows that its
// neighbours on other XCDs fetch as well (L2 fills of the attention kernel at 10 000 atoms: 613 MB with chunks of 16
// tiles, 508 with 27, 467 with 40, 407 with 79, at the same kernel time; a chunk of about 80 tiles reads about 4 MB of
// rows per head, the size of an XCD's L2): up to 640 tiles every XCD gets one chunk.  Beyond that size the XCDs run
// several chunks one after the other and finish at different times, and small chunks are faster (100 000 atoms:
// 2.36 ms with chunks of 79 tiles, 2.30 with 40, 2.28 with 20): chunks of at most 20 tiles there.
constexpr int TILE_BLK_ONE = 80, TILE_BLK_MANY = 20;
inline int tile_blk(int n_tiles) {
    const int cap = n_tiles <= 8 * TILE_BLK_ONE ? TILE_BLK_ONE : TILE_BLK_MANY;
    const int k = (n_tiles + 8 * cap - 1) / (8 * cap);
    const int blk = (n_tiles + 8 * k - 1) / (8 * (k > 0 ? k : 1));
    return blk > 0 ? blk : 1;
}
// workgroups of a launch over (tile, head group) items in that order
inline int tile_grid(int n_tiles, int blk, int HG) { return ((n_tiles + blk - 1) / blk + 7) / 8 * 8 * blk * HG; }
#ifndef E2F_TILE_OCC
#define E2F_TILE_OCC(NW) ((NW) / 2)
#endif
constexpr float M_STEP = 20.0f; // the softmax reference moves when a logit exceeds it by this much (base-2 units)

// Registers for the value rows of one chunk: the wave's single component (8 bytes per entry) and NP pairs of
// components (16 bytes per entry), for the lane's two list entries a and b.
template <int NP>
struct VRows {
    u32x2 sa, sb;
    u32x4 pa[NP > 0 ? NP : 1], pb[NP > 0 ? NP : 1];
    __device__ __forceinline__ void load_single(const uint16_t* a, const uint16_t* b) {
        sa = *reinterpret_cast<const u32x2*>(a);
        sb = *reinterpret_cast<const u32x2*>(b);
    }
    // a, b: the first pair's 16 bytes of this lane's channel; pairs are 128 elements apart
    __device__ __forceinline__ void load_pair(int p, const uint16_t* a, const uint16_t* b) {
        pa[p] = *reinterpret_cast<const u32x4*>(a + p * 128);
        pb[p] = *reinterpret_cast<const u32x4*>(b + p * 128);
    }
    // B operands (32 candidates x 16 channels; this lane: 8 candidates of its channel)
    __device__ __forceinline__ bf16x8 single() const {
        return __builtin_bit_cast(bf16x8, (u32x4){sa[0], sa[1], sb[0], sb[1]});
    }
    __device__ __forceinline__ bf16x8 first(int p) const {
        return __builtin_bit_cast(bf16x8, (u32x4){pa[p][0], pa[p][1], pb[p][0], pb[p][1]});
    }
    __device__ __forceinline__ bf16x8 second(int p) const {
        return __builtin_bit_cast(bf16x8, (u32x4){pa[p][2], pa[p][3], pb[p][2], pb[p][3]});
    }
};

__device__ __forceinline__ float read_lane(float x, int src_lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), src_lane));
}
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma(f16x8 a, f16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Radial bias of a head, b(d) = sum_b Wb[b] exp(-gamma (d - b step)^2), in base-2 units, evaluated per pair from NB
// coefficients that every lane holds (uniform).  Up to 8 basis functions: a polynomial in u = e^{2 gamma step d},
//     b(d) = e^{-gamma d^2} sum_b cb[b] u^b ,       cb[b] = Wb[b] e^{-gamma (b step)^2} log2 e .
// Up to 16: u^15 would leave the range of binary32, so the same expansion is taken around the middle basis function
// m = NB/2, x = d - m step:  b(d) = e^{-gamma x^2} ( sum_{b >= m} cb[b] t^(b-m) + sum_{b < m} cb[b] t^-(m-b) ) with
// t = e^{2 gamma step x} and cb[b] = Wb[b] e^{-gamma ((b-m) step)^2} log2 e; every power stays below e^60.
template <int NB>
__device__ __forceinline__ float bias_coefficient(float wb, int b, float step, float gamma) {
    const float bs = (float)(b - (NB > 8 ? NB / 2 : 0)) * step;
    return wb * __expf(-gamma * bs * bs) * 1.44269504088896341f;
}
// c_u = 2 gamma step log2 e, c_g = -gamma log2 e
template <int NB>
__device__ __forceinline__ float bias_value(const float (&cb)[NB], float d, float d2, float c_u, float c_g, float step) {
    if constexpr (NB <= 8) {
        const float uu = __builtin_amdgcn_exp2f(c_u * d);
        float poly = cb[NB - 1];
#pragma unroll
        for (int bb = NB - 2; bb >= 0; --bb) poly = poly * uu + cb[bb];
        return __builtin_amdgcn_exp2f(c_g * d2) * poly;
    } else {
        constexpr int M = NB / 2;
        const float x = d - (float)M * step;
        const float t = __builtin_amdgcn_exp2f(c_u * x), ti = __builtin_amdgcn_exp2f(-c_u * x);
        float hi = cb[NB - 1], lo = cb[0];
#pragma unroll
        for (int bb = NB - 2; bb >= M; --bb) hi = hi * t + cb[bb];
#pragma unroll
        for (int bb = 1; bb < M; ++bb) lo = lo * ti + cb[bb];
        return __builtin_amdgcn_exp2f(c_g * x * x) * (hi + lo * ti);
    }
}
// The bias (base-2 units) and its derivative with respect to d in natural units.
template <int NB>
__device__ __forceinline__ void bias_value_grad(const float (&cb)[NB], float d, float d2, float c_u, float c_g, float step,
                                                float gamma, float& bias, float& dbias) {
    constexpr float LN2 = 0.69314718055994531f;
    if constexpr (NB <= 8) {
        const float uu = __builtin_amdgcn_exp2f(c_u * d), E = __builtin_amdgcn_exp2f(c_g * d2);
        float poly = cb[NB - 1], dpoly = 0.0f;   // the polynomial and its derivative in u
#pragma unroll
        for (int bb = NB - 2; bb >= 0; --bb) {
            dpoly = dpoly * uu + poly;
            poly = poly * uu + cb[bb];
        }
        bias = E * poly;
        // 2 gamma (step e^{-gamma d^2} u poly'(u) - d b) ln 2
        dbias = 2.0f * gamma * (step * E * uu * dpoly - d * bias) * LN2;
    } else {
        constexpr int M = NB / 2;
        const float x = d - (float)M * step;
        const float t = __builtin_amdgcn_exp2f(c_u * x), ti = __builtin_amdgcn_exp2f(-c_u * x), E = __builtin_amdgcn_exp2f(c_g * x * x);
        float hi = cb[NB - 1], dhi = 0.0f, lo = cb[0], dlo = 0.0f;
#pragma unroll
        for (int bb = NB - 2; bb >= M; --bb) {
            dhi = dhi * t + hi;
            hi = hi * t + cb[bb];
        }
#pragma unroll
        for (int bb = 1; bb < M; ++bb) {
            dlo = dlo * ti + lo;
            lo = lo * ti + cb[bb];
        }
        // with Lo(ti) = ti lo(ti):  t d/dt of the bracket = t hi'(t) - ti Lo'(ti) = t hi' - ti (lo + ti lo')
        const float low = lo * ti;
        bias = E * (hi + low);
        dbias = 2.0f * gamma * (step * E * (t * dhi - low - ti * ti * dlo) - x * bias) * LN2;
    }
}

// The candidate list in LDS is private to a wave, whose LDS operations complete in order: ordering them in the
// instruction stream is all that is needed, no workgroup barrier.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}
// Workgroups are dealt to the 8 XCDs round-robin, each XCD with its own L2.  A chunk of blk consecutive tiles
// (neighbours in space) goes to one XCD and is run head by head, so that the workgroups resident on an XCD at any
// time read the k and v rows of one head over one region.
__device__ __forceinline__ bool tile_xcd_remap(int bid, int n_tiles, int blk, int H, int& tile, int& head) {
    const int xcd = bid & 7, idx = bid >> 3, per = blk * H;
    const int chunk = (idx / per) * 8 + xcd, within = idx % per;
    head = within / blk;
    tile = chunk * blk + within % blk;
    return tile < n_tiles;
}

// Position of every entry of the non-zero pattern in a packed list of the 216 (order: mu, x_out, x_in); the epilogue
// of the attention kernel reads the operators from that list (0.9 KB per workgroup instead of 7.5 KB).
struct AxisIndex {
    int16_t v[3][E2F_MAX_N][E2F_MAX_N];
    int count;
    constexpr AxisIndex() : v(), count(0) {
        for (int mu = 0; mu < 3; ++mu)
            for (int xo = 0; xo < E2F_MAX_N; ++xo)
                for (int xi = 0; xi < E2F_MAX_N; ++xi) v[mu][xo][xi] = ((E2F_AXIS_NZ[mu][xo] >> xi) & 1u) ? (int16_t)count++ : (int16_t)-1;
    }
};
constexpr AxisIndex AXIS_INDEX{};
constexpr int AXIS_NNZ = AXIS_INDEX.count;
static_assert(AXIS_NNZ == 216, "the pattern of the degree-1 axis operators at L_max = 4");
constexpr int AXIS_PACKED_AT = 3 * E2F_MAX_N * E2F_MAX_N;   // the packed list follows the full operators

}  // namespace
