// GPU cell lists: per-segment bounding boxes, grids of edge >= cutoff, a deterministic counting sort of the
// atoms by (segment, cell, atom index), and the neighbour-set test kernels that walk the result.
#include <limits.h>

#include "e2f_device.h"

namespace {

__device__ __forceinline__ int float_to_ordered(float f) {
    int i = __float_as_int(f);
    return i >= 0 ? i : i ^ 0x7fffffff;
}
__device__ __forceinline__ float ordered_to_float(int i) { return __int_as_float(i >= 0 ? i : i ^ 0x7fffffff); }

__global__ void k_cells_init(int32_t* bbox, int S, int32_t* cell_start, int32_t* cell_fill, int max_cells) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < S * 6) bbox[i] = (i % 6 < 3) ? INT_MAX : INT_MIN;
    if (i <= max_cells) cell_start[i] = 0;
    if (i < max_cells) cell_fill[i] = 0;
}

// Segment of every atom (binary search in the offsets) and the segment bounding boxes.
__global__ void k_cells_bbox(const float* __restrict__ pos, const int32_t* __restrict__ seg_offsets, int N, int S,
                             int32_t* __restrict__ atom_seg, int32_t* __restrict__ bbox) {
    const int a = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = a < N;
    int s = 0;
    float x = 0.f, y = 0.f, z = 0.f;
    if (live) {
        int lo = 0, hi = S;  // largest s with seg_offsets[s] <= a
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (seg_offsets[mid] <= a) lo = mid; else hi = mid;
        }
        s = lo;
        atom_seg[a] = s;
        x = pos[3 * a]; y = pos[3 * a + 1]; z = pos[3 * a + 2];
    }
    // One set of atomics per workgroup when all of it sits in one segment (the common case: few, large segments),
    // else one per wave that does, else one per atom.
    __shared__ float s_box[16][6];
    __shared__ int s_seg[16];
    const int s0 = __shfl(s, 0), wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
    const bool uniform = __all(live && s == s0);
    float mnx = x, mny = y, mnz = z, mxx = x, mxy = y, mxz = z;
    if (uniform) {
        for (int off = 32; off > 0; off >>= 1) {
            mnx = fminf(mnx, __shfl_xor(mnx, off)); mny = fminf(mny, __shfl_xor(mny, off));
            mnz = fminf(mnz, __shfl_xor(mnz, off)); mxx = fmaxf(mxx, __shfl_xor(mxx, off));
            mxy = fmaxf(mxy, __shfl_xor(mxy, off)); mxz = fmaxf(mxz, __shfl_xor(mxz, off));
        }
    }
    if ((threadIdx.x & 63) == 0) {
        s_seg[wave] = uniform ? s0 : -1;
        s_box[wave][0] = mnx; s_box[wave][1] = mny; s_box[wave][2] = mnz;
        s_box[wave][3] = mxx; s_box[wave][4] = mxy; s_box[wave][5] = mxz;
    }
    __syncthreads();
    bool block_uniform = s_seg[0] >= 0;
    for (int w = 1; w < n_waves; ++w) block_uniform = block_uniform && s_seg[w] == s_seg[0];
    if (block_uniform) {
        if (threadIdx.x < 6) {
            float v = s_box[0][threadIdx.x];
            for (int w = 1; w < n_waves; ++w) v = threadIdx.x < 3 ? fminf(v, s_box[w][threadIdx.x]) : fmaxf(v, s_box[w][threadIdx.x]);
            if (threadIdx.x < 3)
                atomicMin(&bbox[s_seg[0] * 6 + threadIdx.x], float_to_ordered(v));
            else
                atomicMax(&bbox[s_seg[0] * 6 + threadIdx.x], float_to_ordered(v));
        }
    } else if (uniform) {
        if ((threadIdx.x & 63) == 0) {
            atomicMin(&bbox[s * 6 + 0], float_to_ordered(mnx)); atomicMin(&bbox[s * 6 + 1], float_to_ordered(mny));
            atomicMin(&bbox[s * 6 + 2], float_to_ordered(mnz)); atomicMax(&bbox[s * 6 + 3], float_to_ordered(mxx));
            atomicMax(&bbox[s * 6 + 4], float_to_ordered(mxy)); atomicMax(&bbox[s * 6 + 5], float_to_ordered(mxz));
        }
    } else if (live) {
        atomicMin(&bbox[s * 6 + 0], float_to_ordered(x)); atomicMin(&bbox[s * 6 + 1], float_to_ordered(y));
        atomicMin(&bbox[s * 6 + 2], float_to_ordered(z)); atomicMax(&bbox[s * 6 + 3], float_to_ordered(x));
        atomicMax(&bbox[s * 6 + 4], float_to_ordered(y)); atomicMax(&bbox[s * 6 + 5], float_to_ordered(z));
    }
}

// One block: grid of every segment (edge doubled until the segment stays within its cell budget of
// 27 + 2 * atoms, so the total never exceeds the workspace), then an exclusive scan of the cell counts.
// A periodic axis (box length > 0) gets floor(length / edge) >= 3 cells that tile the box exactly, origin 0.
__global__ void k_cells_grid(const int32_t* __restrict__ bbox, const int32_t* __restrict__ seg_offsets, int S,
                             float edge0, const float* __restrict__ box, E2fSegGrid* __restrict__ grid) {
    __shared__ int s_part[1024];
    __shared__ int s_carry;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int s0 = 0; s0 < S; s0 += blockDim.x) {
        const int s = s0 + threadIdx.x;
        int cells = 0;
        E2fSegGrid g = {0.f, 0.f, 0.f, 1.f, 1.f, 1.f, 1, 1, 1, 0, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (s < S) {
            const int ns = seg_offsets[s + 1] - seg_offsets[s];
            cells = 1;  // an empty segment keeps one empty cell
            // box: [S][6], lengths (0 = open axis) and their reciprocals as the host rounded them
            const float lx = box ? box[6 * s] : 0.0f, ly = box ? box[6 * s + 1] : 0.0f, lz = box ? box[6 * s + 2] : 0.0f;
            g.lx = lx; g.ly = ly; g.lz = lz;
            g.rx = box ? box[6 * s + 3] : 0.0f;
            g.ry = box ? box[6 * s + 4] : 0.0f;
            g.rz = box ? box[6 * s + 5] : 0.0f;
            if (ns > 0) {
                const float mnx = ordered_to_float(bbox[s * 6 + 0]), mny = ordered_to_float(bbox[s * 6 + 1]);
                const float mnz = ordered_to_float(bbox[s * 6 + 2]), mxx = ordered_to_float(bbox[s * 6 + 3]);
                const float mxy = ordered_to_float(bbox[s * 6 + 4]), mxz = ordered_to_float(bbox[s * 6 + 5]);
                const long long budget = 27ll + 2ll * ns;
                float edge = edge0;
                long long nx = 1, ny = 1, nz = 1;
                bool fits = false;
                auto cells_along = [&](float len, float extent) -> long long {
                    const long long whole = (long long)floorf((len > 0.0f ? len : extent) / edge);
                    return len > 0.0f ? (whole > 3 ? whole : 3) : whole + 1;   // (27 cells always fit the budget)
                };
                for (int it = 0; it < 200 && !fits; ++it) {  // bounded: edge overflows to inf long before
                    nx = cells_along(lx, mxx - mnx);
                    ny = cells_along(ly, mxy - mny);
                    nz = cells_along(lz, mxz - mnz);
                    fits = nx >= 1 && ny >= 1 && nz >= 1 && nx <= budget && ny <= budget && nz <= budget &&
                           nx * ny * nz <= budget;
                    if (!fits) edge *= 2.0f;
                }
                if (!fits) {  // non-finite coordinates: one cell holds the whole segment
                    nx = ny = nz = 1;
                    edge = edge0;
                }
                g.ox = lx > 0.0f ? 0.0f : mnx;
                g.oy = ly > 0.0f ? 0.0f : mny;
                g.oz = lz > 0.0f ? 0.0f : mnz;
                g.ix = lx > 0.0f ? (float)nx / lx : 1.0f / edge;
                g.iy = ly > 0.0f ? (float)ny / ly : 1.0f / edge;
                g.iz = lz > 0.0f ? (float)nz / lz : 1.0f / edge;
                g.nx = (int)nx; g.ny = (int)ny; g.nz = (int)nz;
                cells = (int)(nx * ny * nz);
            }
        }
        // block-wide exclusive scan of `cells`
        s_part[threadIdx.x] = cells;
        __syncthreads();
        for (int off = 1; off < (int)blockDim.x; off <<= 1) {
            int v = (threadIdx.x >= (unsigned)off) ? s_part[threadIdx.x - off] : 0;
            __syncthreads();
            s_part[threadIdx.x] += v;
            __syncthreads();
        }
        const int incl = s_part[threadIdx.x];
        const int carry = s_carry;
        if (s < S) {
            g.base = carry + incl - cells;
            grid[s] = g;
        }
        __syncthreads();
        if (threadIdx.x == blockDim.x - 1) s_carry = carry + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) grid[S].base = s_carry;   // cells in use: what the scan of the counts has to cover
}

__global__ void k_cells_assign(const float* __restrict__ pos, const int32_t* __restrict__ atom_seg,
                               const E2fSegGrid* __restrict__ grid, int N, int32_t* __restrict__ atom_cell,
                               int32_t* __restrict__ atom_sub, int32_t* __restrict__ cell_count /* = cell_start + 1 */) {
    const int a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= N) return;
    const E2fSegGrid g = grid[atom_seg[a]];
    const float fx = (e2f::fold_coord(pos[3 * a], g.lx, g.rx) - g.ox) * g.ix;
    const float fy = (e2f::fold_coord(pos[3 * a + 1], g.ly, g.ry) - g.oy) * g.iy;
    const float fz = (e2f::fold_coord(pos[3 * a + 2], g.lz, g.rz) - g.oz) * g.iz;
    int cx = (int)floorf(fx), cy = (int)floorf(fy), cz = (int)floorf(fz);
    cx = min(max(cx, 0), g.nx - 1); cy = min(max(cy, 0), g.ny - 1); cz = min(max(cz, 0), g.nz - 1);
    const int c = g.base + (cz * g.ny + cy) * g.nx + cx;
    atom_cell[a] = c;
    // Order inside the cell: Morton index over 4x4x4 sub-cells, so that atoms that are consecutive in the sorted
    // order (the 16-atom target tiles and the 4-slot candidate groups of the attention kernels) are close in space.
    const int sx = min(max((int)((fx - (float)cx) * 4.0f), 0), 3), sy = min(max((int)((fy - (float)cy) * 4.0f), 0), 3);
    const int sz = min(max((int)((fz - (float)cz) * 4.0f), 0), 3);
    auto spread = [](int v) { return (v & 1) | ((v & 2) << 2); };   // bit 0 -> 0, bit 1 -> 3
    atom_sub[a] = spread(sx) | (spread(sy) << 1) | (spread(sz) << 2);
    atomicAdd(&cell_count[c], 1);
}

// One block: in-place inclusive scan of data[0..n) (data[0] is 0, data[c+1] the count of cell c), which turns
// the counts into first-slot offsets.  Every thread sums one contiguous chunk, the chunk sums are scanned across
// the block, and a second sweep writes the running totals.
__global__ void k_cells_scan(int32_t* __restrict__ data, const E2fSegGrid* __restrict__ grid, int S) {
    __shared__ int s_part[1024];
    const int n = grid[S].base + 1;   // cells in use + 1; the counts beyond are zero and never read
    const int chunk = (n + (int)blockDim.x - 1) / (int)blockDim.x;
    const int b = min((int)threadIdx.x * chunk, n), e = min(b + chunk, n);
    int sum = 0;
    for (int i = b; i < e; ++i) sum += data[i];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < (int)blockDim.x; off <<= 1) {
        const int v = (threadIdx.x >= (unsigned)off) ? s_part[threadIdx.x - off] : 0;
        __syncthreads();
        s_part[threadIdx.x] += v;
        __syncthreads();
    }
    int run = s_part[threadIdx.x] - sum;
    for (int i = b; i < e; ++i) {
        run += data[i];
        data[i] = run;
    }
}

__global__ void k_cells_scatter(const int32_t* __restrict__ atom_cell, const int32_t* __restrict__ cell_start, int N,
                                int32_t* __restrict__ cell_fill, int32_t* __restrict__ tmp_slot) {
    const int a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= N) return;
    const int c = atom_cell[a];
    tmp_slot[cell_start[c] + atomicAdd(&cell_fill[c], 1)] = a;
}

// The scatter above fills each cell in arrival order; ranking every atom among its cell mates by (sub-cell, atom
// index) makes the final order independent of that.
__global__ void k_cells_rank(const int32_t* __restrict__ tmp_slot, const int32_t* __restrict__ atom_cell,
                             const int32_t* __restrict__ atom_sub, const int32_t* __restrict__ atom_seg, const int32_t* __restrict__ cell_start, int N,
                             const E2fSegGrid* __restrict__ grid, int32_t* __restrict__ perm,
                             int32_t* __restrict__ scell, int32_t* __restrict__ sseg, int32_t* __restrict__ atom_slot,
                             int4* __restrict__ sinfo) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= N) return;
    const int a = tmp_slot[t];
    const int c = atom_cell[a];
    const int b = cell_start[c], e = cell_start[c + 1];
    const int sa = atom_sub[a];
    int rank = 0;
    for (int u = b; u < e; ++u) {
        const int o = tmp_slot[u], so = atom_sub[o];
        rank += (so < sa || (so == sa && o < a)) ? 1 : 0;
    }
    perm[b + rank] = a;
    scell[b + rank] = c;
    sseg[b + rank] = atom_seg[a];
    atom_slot[a] = b + rank;
    const E2fSegGrid g = grid[atom_seg[a]];
    const int local = c - g.base;
    sinfo[2 * (b + rank)] = make_int4(atom_seg[a], local % g.nx, (local / g.nx) % g.ny, local / (g.nx * g.ny));
    sinfo[2 * (b + rank) + 1] = make_int4(g.nx, g.ny, g.nz, g.base);
}

// One wave per target: walk the 27-cell stencil 64 candidates at a time.
// Position of an atom as the predicate sees it: folded into the segment's box on periodic axes.
template <bool PBC>
__device__ __forceinline__ void atom_position(const float* __restrict__ pos, int atom, const E2fSegGrid& g, float& x,
                                              float& y, float& z) {
    x = pos[3 * atom];
    y = pos[3 * atom + 1];
    z = pos[3 * atom + 2];
    if (PBC) {
        x = e2f::fold_coord(x, g.lx, g.rx);
        y = e2f::fold_coord(y, g.ly, g.ry);
        z = e2f::fold_coord(z, g.lz, g.rz);
    }
}

template <bool LIST, bool PBC>
__global__ __launch_bounds__(64) void k_neighbors(E2fCellsView cv, const float* __restrict__ pos, float rc2,
                                                  int32_t* __restrict__ degree, const int64_t* __restrict__ offsets,
                                                  int32_t* __restrict__ idx) {
    const int t = blockIdx.x, lane = threadIdx.x;
    const int ai = cv.perm[t];
    const E2fSegGrid g = cv.grid[cv.sseg[t]];
    float xi, yi, zi;
    atom_position<PBC>(pos, ai, g, xi, yi, zi);
    e2f::Stencil<PBC> st;
    st.init(cv, t);
    int cnt = 0;
    const int64_t out0 = LIST ? offsets[ai] : 0;
    for (int r = 0; r < e2f::Stencil<PBC>::NR; ++r)
        for (int base = st.lo[r]; base < st.hi[r]; base += 64) {
            const int j = base + lane;
            bool ok = false;
            int aj = 0;
            if (j < st.hi[r] && j != t) {
                aj = cv.perm[j];
                float xj, yj, zj;
                atom_position<PBC>(pos, aj, g, xj, yj, zj);
                ok = e2f::is_neighbor(e2f::dist2_exact(xi, yi, zi, xj + st.shift_x(r), yj + st.shift_y(r),
                                                       zj + st.shift_z(r)), rc2);
            }
            const unsigned long long mask = __ballot(ok);
            if (LIST && ok) idx[out0 + cnt + __popcll(mask & ((1ull << lane) - 1ull))] = aj;
            cnt += __popcll(mask);
        }
    if (!LIST && lane == 0) degree[ai] = cnt;
}

// Neighbour cap: one wave per target finds the K-th smallest key (bits of d^2, atom index) among the target's
// neighbours inside the cutoff by an 8-bit radix select over the 64-bit keys (a 256-bin histogram in LDS per digit;
// the keys are kept in LDS after one stencil walk, or, beyond 512 neighbours, the stencil is walked once per digit,
// so there is no limit on their number), then writes the threshold key and / or the
// table row of the selected atoms (in cell order, -1 padded).  Keys are unique, so exactly min(K, degree) atoms pass.
template <bool PBC>
__global__ __launch_bounds__(64) void k_select_neighbors(E2fCellsView cv, const float* __restrict__ pos, float rc2,
                                                         int K, uint32_t* __restrict__ cap_d2,
                                                         int32_t* __restrict__ cap_idx, int32_t* __restrict__ table,
                                                         int32_t* __restrict__ count) {
    __shared__ int s_hist[256];
    const int t = blockIdx.x, lane = threadIdx.x;
    const int ai = cv.perm[t];
    const E2fSegGrid g = cv.grid[cv.sseg[t]];
    float xi, yi, zi;
    atom_position<PBC>(pos, ai, g, xi, yi, zi);
    e2f::Stencil<PBC> st;
    st.init(cv, t);
    // walk(f): f(ok, key, atom) for every candidate of this lane, all lanes in step
    auto walk = [&](auto&& f) {
        for (int r = 0; r < e2f::Stencil<PBC>::NR; ++r)
            for (int base = st.lo[r]; base < st.hi[r]; base += 64) {
                const int j = base + lane;
                bool ok = false;
                int aj = 0;
                unsigned long long key = ~0ull;
                if (j < st.hi[r] && j != t) {
                    aj = cv.perm[j];
                    float xj, yj, zj;
                    atom_position<PBC>(pos, aj, g, xj, yj, zj);
                    const float d2 = e2f::dist2_exact(xi, yi, zi, xj + st.shift_x(r), yj + st.shift_y(r),
                                                      zj + st.shift_z(r));
                    ok = e2f::is_neighbor(d2, rc2);
                    key = ((unsigned long long)__float_as_uint(d2) << 32) | (unsigned int)aj;
                }
                f(ok, key, aj);
            }
    };
    // first walk: count the neighbours and keep their keys in LDS while they fit (they do in any physical system)
    constexpr int KEEP = 512;
    __shared__ unsigned long long s_key[KEEP];
    int total = 0;
    walk([&](bool ok, unsigned long long key, int) {
        const unsigned long long mask = __ballot(ok);
        const int at = total + __popcll(mask & ((1ull << lane) - 1ull));
        if (ok && at < KEEP) s_key[at] = key;
        total += __popcll(mask);
    });
    __syncthreads();
    const bool in_lds = total <= KEEP;
    // keys(f): f(ok, key) over all neighbour keys, from LDS or by walking the stencil again
    auto keys = [&](auto&& f) {
        if (in_lds) {
            for (int base = 0; base < total; base += 64) {
                const bool ok = base + lane < total;
                f(ok, ok ? s_key[base + lane] : ~0ull);
            }
        } else {
            walk([&](bool ok, unsigned long long key, int) { f(ok, key); });
        }
    };
    unsigned long long thr = ~0ull;   // no cap needed: every neighbour passes
    if (total > K) {
        unsigned long long prefix = 0ull;
        int want = K;   // rank (1-based) of the key looked for among the keys that share the prefix
        for (int shift = 56; shift >= 0; shift -= 8) {
            for (int b = lane; b < 256; b += 64) s_hist[b] = 0;
            __syncthreads();
            keys([&](bool ok, unsigned long long key) {
                const bool same = shift == 56 || (key >> (shift + 8)) == (prefix >> (shift + 8));
                if (ok && same) atomicAdd(&s_hist[(int)((key >> shift) & 255ull)], 1);
            });
            __syncthreads();
            // lane l owns bins 4l..4l+3; find the bin where the running count reaches `want`
            const int h0 = s_hist[4 * lane], h1 = s_hist[4 * lane + 1], h2 = s_hist[4 * lane + 2], h3 = s_hist[4 * lane + 3];
            int incl = h0 + h1 + h2 + h3;
            for (int off = 1; off < 64; off <<= 1) {
                const int v = __shfl_up(incl, off);
                if (lane >= off) incl += v;
            }
            const int before = incl - (h0 + h1 + h2 + h3);
            const bool mine = before < want && want <= incl;
            int bin = 0, below = 0;
            if (mine) {
                int c = before;
                if (want <= c + h0) { bin = 4 * lane; below = c; }
                else if (want <= c + h0 + h1) { bin = 4 * lane + 1; below = c + h0; }
                else if (want <= c + h0 + h1 + h2) { bin = 4 * lane + 2; below = c + h0 + h1; }
                else { bin = 4 * lane + 3; below = c + h0 + h1 + h2; }
            }
            const int src = __ffsll((long long)__ballot(mine)) - 1;   // exactly one lane
            bin = __shfl(bin, src);
            below = __shfl(below, src);
            prefix |= (unsigned long long)bin << shift;
            want -= below;
            __syncthreads();
        }
        thr = prefix;
    }
    if (lane == 0) {
        if (cap_d2) cap_d2[t] = (uint32_t)(thr >> 32);
        if (cap_idx) cap_idx[t] = (thr == ~0ull) ? INT_MAX : (int32_t)(thr & 0xffffffffull);
        if (count) count[ai] = total < K ? total : K;
    }
    if (table) {
        int32_t* row = table + (size_t)ai * K;
        int n_out = 0;
        walk([&](bool ok, unsigned long long key, int aj) {
            const bool take = ok && key <= thr;
            const unsigned long long mask = __ballot(take);
            if (take) row[n_out + __popcll(mask & ((1ull << lane) - 1ull))] = aj;
            n_out += __popcll(mask);
        });
        for (int x = n_out + lane; x < K; x += 64) row[x] = -1;
    }
}

}  // namespace

e2f_status e2f_launch_build_cells(const e2f_ctx* ctx, e2f_cells* c, const float* pos, const int32_t* seg_offsets,
                                  hipStream_t st) {
    const int N = c->view.N, S = c->view.S;
    if (N == 0) return E2F_OK;
    const int tb = 256;
    int32_t* cell_start = const_cast<int32_t*>(c->view.cell_start);
    const int n_init = c->max_cells + 1 > S * 6 ? c->max_cells + 1 : S * 6;
    k_cells_init<<<(n_init + tb - 1) / tb, tb, 0, st>>>(c->bbox, S, cell_start, c->cell_fill, c->max_cells);
    k_cells_bbox<<<(N + 1023) / 1024, 1024, 0, st>>>(pos, seg_offsets, N, S, c->atom_seg, c->bbox);
    // edge a hair above the cutoff: the binary32 predicate can accept a pair whose exact |dx| exceeds the
    // cutoff by rounding, and cell coordinates carry rounding of their own
    k_cells_grid<<<1, 1024, 0, st>>>(c->bbox, seg_offsets, S, e2f_cell_edge(ctx->cfg.cutoff),
                                     c->view.periodic ? c->box : nullptr, const_cast<E2fSegGrid*>(c->view.grid));
    k_cells_assign<<<(N + tb - 1) / tb, tb, 0, st>>>(pos, c->atom_seg, c->view.grid, N, c->atom_cell, c->atom_sub, cell_start + 1);
    k_cells_scan<<<1, 1024, 0, st>>>(cell_start, c->view.grid, S);
    k_cells_scatter<<<(N + tb - 1) / tb, tb, 0, st>>>(c->atom_cell, cell_start, N, c->cell_fill, c->tmp_slot);
    k_cells_rank<<<(N + tb - 1) / tb, tb, 0, st>>>(c->tmp_slot, c->atom_cell, c->atom_sub, c->atom_seg, cell_start, N,
                                                  c->view.grid, const_cast<int32_t*>(c->view.perm),
                                                  const_cast<int32_t*>(c->view.scell),
                                                  const_cast<int32_t*>(c->view.sseg),
                                                  const_cast<int32_t*>(c->view.atom_slot),
                                                  const_cast<int4*>(c->view.sinfo));
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_count_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, int32_t* degree,
                                      hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (cv.periodic) k_neighbors<false, true><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, degree, nullptr, nullptr);
    else k_neighbors<false, false><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, degree, nullptr, nullptr);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_list_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos,
                                     const int64_t* offsets, int32_t* idx, hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (cv.periodic) k_neighbors<true, true><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, nullptr, offsets, idx);
    else k_neighbors<true, false><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, nullptr, offsets, idx);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}

e2f_status e2f_launch_select_neighbors(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, int32_t K,
                                       uint32_t* cap_d2, int32_t* cap_idx, int32_t* table, int32_t* count,
                                       hipStream_t st) {
    if (cv.N == 0) return E2F_OK;
    if (cv.periodic) k_select_neighbors<true><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, K, cap_d2, cap_idx, table, count);
    else k_select_neighbors<false><<<cv.N, 64, 0, st>>>(cv, pos, ctx->rc2, K, cap_d2, cap_idx, table, count);
    E2F_HIP_CHECK(hipGetLastError());
    return E2F_OK;
}
