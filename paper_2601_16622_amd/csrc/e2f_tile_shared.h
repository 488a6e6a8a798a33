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
#ifndef E2F_TILE_BLK
#define E2F_TILE_BLK 16
#endif
constexpr int TILE_BLK = E2F_TILE_BLK;   // consecutive tiles whose (tile, head) items form one XCD chunk, head-major
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

// The candidate list in LDS is private to a wave, whose LDS operations complete in order: ordering them in the
// instruction stream is all that is needed, no workgroup barrier.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}
// Workgroups are dealt to the 8 XCDs round-robin, each XCD with its own L2.  A chunk of TILE_BLK consecutive tiles
// (neighbours in space) goes to one XCD and is run head by head, so that the workgroups resident on an XCD at any
// time read the k and v rows of one head over one small region.
__device__ __forceinline__ bool tile_xcd_remap(int bid, int n_tiles, int H, int& tile, int& head) {
    const int xcd = bid & 7, idx = bid >> 3, per = TILE_BLK * H;
    const int chunk = (idx / per) * 8 + xcd, within = idx % per;
    head = within / TILE_BLK;
    tile = chunk * TILE_BLK + within % TILE_BLK;
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
