// Device-side building blocks: cutoff predicate, stencil walk over the cell list, pair geometry,
// Wigner matrices of the edge-aligning rotation, and the EAAS message for a lane's channels.
#pragma once
#include <hip/hip_runtime.h>

#include "e2f_internal.h"
#include "e2f_wigner_gen.h"

namespace e2f {

// Offset of the degree-l block in a packed array of (2l+1)x(2l+1) matrices: sum_{l'<l} (2l'+1)^2.
__host__ __device__ constexpr int d_offset(int l) { return l * (4 * l * l - 1) / 3; }

// Squared distance exactly as the neighbour predicate defines it: every operation rounded to binary32,
// no fused multiply-add, order (dx*dx + dy*dy) + dz*dz.
__device__ __forceinline__ float dist2_exact(float xi, float yi, float zi, float xj, float yj, float zj) {
#pragma clang fp contract(off)
    float dx = xj - xi;
    float dy = yj - yi;
    float dz = zj - zi;
    float xx = dx * dx;
    float yy = dy * dy;
    float zz = dz * dz;
    float s = xx + yy;
    return s + zz;
}

__device__ __forceinline__ bool is_neighbor(float d2, float rc2) { return d2 < rc2 && d2 > 0.0f; }

// Neighbour cap (the max_neighbors setting of the paper's model table): with a cap K, atom j counts for target i
// only if the pair's key (bits of d^2, atom index of j) is not above the target's threshold key, the K-th smallest
// key among its neighbours inside the cutoff (nearest first, ties to the lower atom index).  Without a cap the
// threshold is (0xffffffff, INT_MAX), above every key.  `w` is the w component of a sorted position: the atom index.
__device__ __forceinline__ bool under_cap(float d2, float w, uint32_t cap_d2, int cap_idx) {
    const uint32_t b = __float_as_uint(d2);
    // (bitwise on purpose: callers evaluate several candidates side by side and must stay in one basic block)
    return (b < cap_d2) | ((b == cap_d2) & (__float_as_int(w) <= cap_idx));
}

// Coordinate folded into a periodic box of length len (inv = 1/len rounded to binary32), every operation rounded
// to binary32: q = floor(x inv), w = x - len q, then one correction step into [0, len).  len == 0: open axis.
__device__ __forceinline__ float fold_coord(float x, float len, float inv) {
#pragma clang fp contract(off)
    if (!(len > 0.0f)) return x;
    const float q = floorf(x * inv);
    const float t = len * q;
    float w = x - t;
    if (w < 0.0f) w = w + len;
    if (w >= len) w = w - len;
    return w;
}

// Runs of sorted slots that hold a target's candidates: without periodic axes the 27-cell stencil as 9 rows
// (cells along x are adjacent in the sorted order); with them 18 runs, where run 9 + r is the cell of row r
// that lies across a periodic x face (empty if the target's cell does not touch one).  Rows outside an open
// grid come back empty.  Candidates of run r are seen at their position plus shift(r), a lattice translation.
template <bool PBC>
struct Stencil {
    static constexpr int NR = PBC ? 18 : 9;
    int lo[NR], hi[NR];
    float sxe, sy[3], sz[3];   // translations: of the extra runs along x, of the rows per y and z offset

    __device__ __forceinline__ void init(const E2fCellsView& cv, int slot) {
        const E2fSegGrid g = cv.grid[cv.sseg[slot]];
        const int local = cv.scell[slot] - g.base;
        const int cx = local % g.nx;
        const int cy = (local / g.nx) % g.ny;
        const int cz = local / (g.nx * g.ny);
        const int x0 = max(cx - 1, 0), x1 = min(cx + 1, g.nx - 1);
        int xe = -1;   // the cell across the x face
        sxe = 0.0f;
        if (PBC && g.lx > 0.0f) {
            if (cx == 0) { xe = g.nx - 1; sxe = -g.lx; }
            else if (cx == g.nx - 1) { xe = 0; sxe = g.lx; }
        }
#pragma unroll
        for (int d = 0; d < 3; ++d) { sy[d] = 0.0f; sz[d] = 0.0f; }
#pragma unroll
        for (int r = 0; r < 9; ++r) {
            int y = cy + (r % 3) - 1, z = cz + (r / 3) - 1;
            if (PBC && g.ly > 0.0f) {
                if (y < 0) { y += g.ny; sy[r % 3] = -g.ly; }
                else if (y >= g.ny) { y -= g.ny; sy[r % 3] = g.ly; }
            }
            if (PBC && g.lz > 0.0f) {
                if (z < 0) { z += g.nz; sz[r / 3] = -g.lz; }
                else if (z >= g.nz) { z -= g.nz; sz[r / 3] = g.lz; }
            }
            const bool inside = y >= 0 && y < g.ny && z >= 0 && z < g.nz;
            const int row = g.base + (z * g.ny + y) * g.nx;
            lo[r] = inside ? cv.cell_start[row + x0] : 0;
            hi[r] = inside ? cv.cell_start[row + x1 + 1] : 0;
            if (PBC) {
                lo[9 + r] = inside && xe >= 0 ? cv.cell_start[row + xe] : 0;
                hi[9 + r] = inside && xe >= 0 ? cv.cell_start[row + xe + 1] : 0;
            }
        }
    }
    __device__ __forceinline__ float shift_x(int r) const { return PBC && r >= 9 ? sxe : 0.0f; }
    __device__ __forceinline__ float shift_y(int r) const { return PBC ? sy[(r % 9) % 3] : 0.0f; }
    __device__ __forceinline__ float shift_z(int r) const { return PBC ? sz[(r % 9) / 3] : 0.0f; }
};

// Run r of the 18-run stencil on its own (for kernels that keep the runs in a table, one lane per run):
// first and last sorted slot and the lattice translation of its candidates.
__device__ __forceinline__ void stencil_run(const E2fCellsView& cv, int slot, int r, int& lo, int& hi, float4& sh) {
    const E2fSegGrid g = cv.grid[cv.sseg[slot]];
    const int local = cv.scell[slot] - g.base;
    const int cx = local % g.nx, rr = r % 9;
    int y = (local / g.nx) % g.ny + (rr % 3) - 1, z = local / (g.nx * g.ny) + (rr / 3) - 1;
    sh = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (g.ly > 0.0f) {
        if (y < 0) { y += g.ny; sh.y = -g.ly; }
        else if (y >= g.ny) { y -= g.ny; sh.y = g.ly; }
    }
    if (g.lz > 0.0f) {
        if (z < 0) { z += g.nz; sh.z = -g.lz; }
        else if (z >= g.nz) { z -= g.nz; sh.z = g.lz; }
    }
    bool have = y >= 0 && y < g.ny && z >= 0 && z < g.nz;
    int x_first = max(cx - 1, 0), x_last = min(cx + 1, g.nx - 1);
    if (r >= 9) {   // the cell across a periodic x face
        have = have && g.lx > 0.0f && (cx == 0 || cx == g.nx - 1);
        x_first = x_last = cx == 0 ? g.nx - 1 : 0;
        sh.x = cx == 0 ? -g.lx : g.lx;
    }
    const int row = g.base + (z * g.ny + y) * g.nx;
    lo = have ? cv.cell_start[row + x_first] : 0;
    hi = have ? cv.cell_start[row + x_last + 1] : 0;
}

// The open-boundary stencil as plain arrays.
__device__ __forceinline__ void stencil_rows(const E2fCellsView& cv, int slot, int (&lo)[9], int (&hi)[9]) {
    Stencil<false> s;
    s.init(cv, slot);
#pragma unroll
    for (int r = 0; r < 9; ++r) {
        lo[r] = s.lo[r];
        hi[r] = s.hi[r];
    }
}

// Workgroups are dealt to the 8 XCDs round-robin and every XCD has its own L2.  Work items (targets in cell
// order) are cut into chunks of XCD_CHUNK consecutive items and chunk c goes to XCD c % 8: an XCD works on
// contiguous stretches, so the neighbour rows its waves share stay in its L2, while every XCD still sees all
// regions of the system (boundary cells carry fewer pairs than interior ones).  Returns -1 for padding blocks;
// launch xcd_grid(n) blocks.
constexpr int XCD_CHUNK = 128;
__host__ __device__ inline int xcd_grid(int n) {
    const int chunks = (n + XCD_CHUNK - 1) / XCD_CHUNK;
    return ((chunks + 7) / 8) * 8 * XCD_CHUNK;
}
__device__ __forceinline__ int xcd_remap(int bid, int n) {
    const int xcd = bid & 7, idx = bid >> 3;
    const int t = ((idx / XCD_CHUNK) * 8 + xcd) * XCD_CHUNK + idx % XCD_CHUNK;
    return t < n ? t : -1;
}

template <int l>
__device__ __forceinline__ void delta_align(const float* c, const float* s, float* d) {
    if constexpr (l == 0) e2f_delta_align_l0(c, s, d);
    if constexpr (l == 1) e2f_delta_align_l1(c, s, d);
    if constexpr (l == 2) e2f_delta_align_l2(c, s, d);
    if constexpr (l == 3) e2f_delta_align_l3(c, s, d);
    if constexpr (l == 4) e2f_delta_align_l4(c, s, d);
}

// Degree-l block of D(R), R = Ry(-theta) Rz(-phi) (the rotation taking r/|r| to +z; Sec. 3.3), in the
// real basis with Y(R x) = D(R) Y(x):  D = Delta(-theta) Z(-phi), Delta from the generated series and Z
// the rotation of each (m,-m) pair by m*phi.  ck/sk = cos/sin(k theta), cm/sm = cos/sin(m phi).
// D may point into LDS: every entry is written once, as soon as it is known, so that the blocks never
// have to be held in registers together.
template <int l>
__device__ __forceinline__ void align_block(const float* ck, const float* sk, const float* cm, const float* sm, float* D) {
    constexpr int n = 2 * l + 1;
    float dl[n * n];
    delta_align<l>(ck, sk, dl);
#pragma unroll
    for (int a = 0; a <= l; ++a) {  // cosine-type rows
        D[(a + l) * n + l] = dl[(a + l) * n + l];
#pragma unroll
        for (int m = 1; m <= l; ++m) {
            D[(a + l) * n + l + m] = dl[(a + l) * n + l + m] * cm[m];
            D[(a + l) * n + l - m] = dl[(a + l) * n + l + m] * sm[m];
        }
    }
#pragma unroll
    for (int a = 1; a <= l; ++a) {  // sine-type rows
        D[(l - a) * n + l] = 0.0f;
#pragma unroll
        for (int m = 1; m <= l; ++m) {
            D[(l - a) * n + l + m] = -dl[(l - a) * n + l - m] * sm[m];
            D[(l - a) * n + l - m] = dl[(l - a) * n + l - m] * cm[m];
        }
    }
}

template <int L, int l = 0>
__device__ __forceinline__ void align_all_blocks(const float* ck, const float* sk, const float* cm, const float* sm,
                                                 float* D) {
    align_block<l>(ck, sk, cm, sm, D + d_offset(l));
    if constexpr (l < L) align_all_blocks<L, l + 1>(ck, sk, cm, sm, D);
}

// All blocks l = 0..L of D(R_ij) for the pair vector (dx,dy,dz) of length d > 0, packed at d_offset(l).
template <int L>
__device__ __forceinline__ void align_D(float dx, float dy, float dz, float d, float* D) {
    // hardware reciprocal and square root (1 ulp): the angles only feed rotation matrices
    const float inv = __builtin_amdgcn_rcpf(d);
    const float rho = __builtin_amdgcn_sqrtf(dx * dx + dy * dy);
    const float ct = dz * inv, st = rho * inv;
    float cp = 1.0f, sp = 0.0f;
    if (rho > 0.0f) {
        const float ir = __builtin_amdgcn_rcpf(rho);
        cp = dx * ir;
        sp = dy * ir;
    }
    float ck[E2F_MAX_L + 1], sk[E2F_MAX_L + 1], cm[E2F_MAX_L + 1], sm[E2F_MAX_L + 1];
    ck[0] = 1.0f; sk[0] = 0.0f; cm[0] = 1.0f; sm[0] = 0.0f;
#pragma unroll
    for (int k = 1; k <= L; ++k) {
        ck[k] = ck[k - 1] * ct - sk[k - 1] * st;
        sk[k] = sk[k - 1] * ct + ck[k - 1] * st;
        cm[k] = cm[k - 1] * cp - sm[k - 1] * sp;
        sm[k] = sm[k - 1] * cp + cm[k - 1] * sp;
    }
    align_all_blocks<L>(ck, sk, cm, sm, D);
}

// Radial pieces of Eq. attn: gate phi(d) and the Gaussian basis value g_b(d).
// phi(d) = (1 + cos(pi d / cutoff)) / 2.  The hardware cosine takes its argument in revolutions, so the argument is
// d times 1/(2 cutoff), a factor that does not depend on the pair (no division per pair).
__device__ __forceinline__ float radial_gate(float d, float cutoff) {
    return 0.5f + 0.5f * __builtin_amdgcn_cosf(d * (0.5f / cutoff));
}
__device__ __forceinline__ float radial_basis(float d, int b, float step, float gamma) {
    const float t = d - (float)b * step;
    return __expf(-gamma * t * t);
}

// Key rows of the tile attention kernel (binary16, DKP = 32 KS features per head, zero-padded): per (group of four
// slots, head) a block [KS][4 slots][32 features], so that the 16 lanes that fetch one 32-feature step of a group's
// four rows read 256 contiguous bytes.  Returns the offset, in elements, of (slot, head, feature f).
__host__ __device__ __forceinline__ size_t k16_offset(size_t slot, int H, int head, int DKP, int f) {
    return (((slot >> 2) * H + head) * (DKP >> 5) + (f >> 5)) * 128 + (slot & 3) * 32 + (f & 31);
}

// Value rows of the tile attention kernel: per (group of four slots, head) a block of n * 64 bf16.  The n components are
// split among the four waves of a workgroup (n / 4 each, the first n % 4 waves one more, contiguous ranges); inside a
// wave's range an odd first component stands alone as [16 channels][4 slots] and the others go in pairs as
// [16 channels][2 components][4 slots], so that a lane fetches the four slots of two components with one 16-byte
// load (a vector memory instruction costs the same whether it moves 8 or 16 bytes per lane).  Returns the offset, in
// bf16 elements, of (component x, channel ch, first slot) inside the block.
__host__ __device__ __forceinline__ int v4_offset(int n, int x, int ch) {
    const int q = n / 4, rem = n % 4;
    int w = 0, x0 = 0, nxw = q + (rem > 0 ? 1 : 0);
    while (x >= x0 + nxw) {
        x0 += nxw;
        ++w;
        nxw = q + (w < rem ? 1 : 0);
    }
    const int odd = nxw & 1;
    int local = x - x0;
    if (odd && local == 0) return x0 * 64 + ch * 4;
    local -= odd;
    return x0 * 64 + odd * 64 + (local >> 1) * 128 + ch * 8 + (local & 1) * 4;
}
// 0: component x stands alone in that layout, 1: it is the first of a pair, 2: the second.
__host__ __device__ __forceinline__ int v4_role(int n, int x) {
    const int q = n / 4, rem = n % 4;
    int w = 0, x0 = 0, nxw = q + (rem > 0 ? 1 : 0);
    while (x >= x0 + nxw) {
        x0 += nxw;
        ++w;
        nxw = q + (w < rem ? 1 : 0);
    }
    const int odd = nxw & 1, local = x - x0;
    if (odd && local == 0) return 0;
    return 1 + ((local - odd) & 1);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ float load_as_float(const T* p);
template <>
__device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_as_float<uint16_t>(const uint16_t* p) { return bf16_bits_to_float(*p); }

template <typename T>
__device__ __forceinline__ void store_from_float(T* p, float x);
template <>
__device__ __forceinline__ void store_from_float<float>(float* p, float x) { *p = x; }
template <>
__device__ __forceinline__ void store_from_float<uint16_t>(uint16_t* p, float x) { *p = float_to_bf16_bits(x); }

// EAAS message for NC channels held by one thread, accumulated into acc (Prop. EAAS, Sec. 3.3):
//   acc[lo] += D^T ( wgt * P( D v ) ),  P from cw[comp * E2F_NP + k] (path weights included), where k selects the
//   input degree l_in = l_out - LF + k; even k reads the same order m, odd k reads order -m (and m = 0 drops out).
// Dp points at the packed blocks of D(R_ij); `wgt` already contains |r|^LF and the attention weight.
// LF = 0 needs no rotation (P is the identity on each degree).
template <int L, int LF, int NC, typename DPtr>
__device__ __forceinline__ void eaas_accumulate(const float (&v)[(L + 1) * (L + 1)][NC], DPtr Dp, const float* cw,
                                                float wgt, float (&acc)[(L + 1) * (L + 1)][NC]) {
    constexpr int n = (L + 1) * (L + 1);
    if constexpr (LF == 0) {
#pragma unroll
        for (int x = 0; x < n; ++x) {
            const float f = wgt * cw[x * E2F_NP];
#pragma unroll
            for (int u = 0; u < NC; ++u) acc[x][u] += f * v[x][u];
        }
    } else {
        float vt[n][NC];
#pragma unroll
        for (int l = 0; l <= L; ++l) {
            const int nl = 2 * l + 1, base = l * l, off = d_offset(l);
#pragma unroll
            for (int a = 0; a < nl; ++a) {
#pragma unroll
                for (int u = 0; u < NC; ++u) vt[base + a][u] = 0.0f;
#pragma unroll
                for (int b = 0; b < nl; ++b) {
                    if (a < l && b == l) continue;  // sine-type rows have no m = 0 column
                    const float dab = Dp[off + a * nl + b];
#pragma unroll
                    for (int u = 0; u < NC; ++u) vt[base + a][u] += dab * v[base + b][u];
                }
            }
        }
#pragma unroll
        for (int lo = 0; lo <= L; ++lo) {
            const int nl = 2 * lo + 1, base = lo * lo, off = d_offset(lo);
            float y[2 * L + 1][NC];
#pragma unroll
            for (int a = 0; a < nl; ++a) {
                const int m = a - lo, am = m < 0 ? -m : m;
#pragma unroll
                for (int u = 0; u < NC; ++u) y[a][u] = 0.0f;
#pragma unroll
                for (int k = 0; k <= 2 * LF; ++k) {
                    const int li = lo - LF + k;
                    if (li < 0 || li > L || LF - li > lo || am > li) continue;  // no such path / order
                    if ((k & 1) && m == 0) continue;
                    const int ms = (k & 1) ? -m : m;
                    const float c = cw[(base + a) * E2F_NP + k];
#pragma unroll
                    for (int u = 0; u < NC; ++u) y[a][u] += c * vt[li * li + li + ms][u];
                }
#pragma unroll
                for (int u = 0; u < NC; ++u) y[a][u] *= wgt;
            }
#pragma unroll
            for (int a = 0; a < nl; ++a) {
#pragma unroll
                for (int b = 0; b < nl; ++b) {
                    if (a < lo && b == lo) continue;
                    const float dab = Dp[off + a * nl + b];
#pragma unroll
                    for (int u = 0; u < NC; ++u) acc[base + b][u] += dab * y[a][u];
                }
            }
        }
    }
}

// |r|^LF
template <int LF>
__device__ __forceinline__ float pow_lf(float d) {
    if constexpr (LF == 0) return 1.0f;
    if constexpr (LF == 1) return d;
    return d * d;
}

}  // namespace e2f
