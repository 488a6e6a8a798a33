// Edge-centric baseline: the same operator computed the way the paper's "materialize per edge" comparison
// does (App. A; Table triton-role): build the edge list, write per-edge tensors to device memory (pair
// geometry, rotation matrices, gathered keys, scores, attention weights, messages) with one simple kernel
// per stage, then reduce per atom.  Used only to compare latency and memory with the fused kernel; it
// allocates O(E) memory and synchronises with the host.
#include "e2f_device.h"

namespace {

struct EdgeBuffers {
    int32_t* src;   // [E] target slot
    int32_t* dst;   // [E] neighbour slot
    float4* geo;    // [E] dx, dy, dz, d
    float* D;       // [E][DSP] blocks of D(R_ij)
    float* kg;      // [E][(L+1) C] gathered keys
    float* score;   // [E][H]
    float* alpha;   // [E][H]
    float* msg;     // [E][n][C]
};

__global__ __launch_bounds__(64) void k_edge_walk(E2fCellsView cv, const float4* __restrict__ spos, float rc2,
                                                  int32_t* __restrict__ degree, const int64_t* __restrict__ eoff,
                                                  int32_t* __restrict__ src, int32_t* __restrict__ dst) {
    const int t = blockIdx.x, lane = threadIdx.x;
    const float4 pi = spos[t];
    int lo[9], hi[9];
    e2f::stencil_rows(cv, t, lo, hi);
    int cnt = 0;
    const int64_t e0 = eoff ? eoff[t] : 0;
    for (int r = 0; r < 9; ++r)
        for (int base = lo[r]; base < hi[r]; base += 64) {
            const int j = base + lane;
            bool ok = false;
            if (j < hi[r] && j != t) {
                const float4 pj = spos[j];
                ok = e2f::is_neighbor(e2f::dist2_exact(pi.x, pi.y, pi.z, pj.x, pj.y, pj.z), rc2);
            }
            const unsigned long long mask = __ballot(ok);
            if (eoff && ok) {
                const int64_t e = e0 + cnt + __popcll(mask & ((1ull << lane) - 1ull));
                src[e] = t;
                dst[e] = j;
            }
            cnt += __popcll(mask);
        }
    if (!eoff && lane == 0) degree[t] = cnt;
}

// One block: eoff[0] = 0, eoff[t+1] = sum of degree[0..t].
__global__ void k_scan_degree(const int32_t* __restrict__ degree, int N, int64_t* __restrict__ eoff) {
    __shared__ long long s_part[1024];
    __shared__ long long s_carry;
    if (threadIdx.x == 0) { s_carry = 0; eoff[0] = 0; }
    __syncthreads();
    for (int i0 = 0; i0 < N; i0 += blockDim.x) {
        const int i = i0 + threadIdx.x;
        s_part[threadIdx.x] = (i < N) ? degree[i] : 0;
        __syncthreads();
        for (int off = 1; off < (int)blockDim.x; off <<= 1) {
            long long v = (threadIdx.x >= (unsigned)off) ? s_part[threadIdx.x - off] : 0;
            __syncthreads();
            s_part[threadIdx.x] += v;
            __syncthreads();
        }
        const long long incl = s_part[threadIdx.x], carry = s_carry;
        if (i < N) eoff[i + 1] = carry + incl;
        __syncthreads();
        if (threadIdx.x == blockDim.x - 1) s_carry = carry + incl;
        __syncthreads();
    }
}

template <int L, int LF>
__global__ void k_edge_geometry(int64_t E, const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                const float4* __restrict__ spos, const float* __restrict__ Wb, int H, int B,
                                float cutoff, float rbf_step, float rbf_gamma, float4* __restrict__ geo,
                                float* __restrict__ D, float* __restrict__ score, float* __restrict__ alpha) {
    constexpr int DS = e2f::d_offset(L + 1), DSP = (DS + 3) & ~3;
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const float4 pi = spos[src[e]], pj = spos[dst[e]];
    const float dx = pj.x - pi.x, dy = pj.y - pi.y, dz = pj.z - pi.z;
    const float d = sqrtf(dx * dx + dy * dy + dz * dz);
    geo[e] = make_float4(dx, dy, dz, d);
    if constexpr (LF != 0) {
        float Dl[DS];
        e2f::align_D<L>(dx, dy, dz, d, Dl);
#pragma unroll
        for (int x = 0; x < DS; ++x) D[e * DSP + x] = Dl[x];
    }
    const float wgt = e2f::radial_gate(d, cutoff) * e2f::pow_lf<LF>(d);
    for (int hh = 0; hh < H; ++hh) {
        float acc = 0.0f;
        for (int b = 0; b < B; ++b) acc += Wb[hh * B + b] * e2f::radial_basis(d, b, rbf_step, rbf_gamma);
        score[e * H + hh] = acc;   // bias for now; the q.k term is added by k_edge_score
        alpha[e * H + hh] = wgt;   // gate for now; multiplied by the softmax weight later
    }
}

__global__ void k_edge_gather_k(int64_t E, const int32_t* __restrict__ dst, const float* __restrict__ k, int row,
                                float* __restrict__ kg) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E * row) return;
    const int64_t e = i / row;
    kg[i] = k[(size_t)dst[e] * row + (i - e * row)];
}

__global__ void k_edge_score(int64_t E, const int32_t* __restrict__ src, const float* __restrict__ q,
                             const float* __restrict__ kg, int L, int C, int H, int Ch, float tau,
                             float* __restrict__ score) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E * H) return;
    const int64_t e = i / H;
    const int hh = (int)(i - e * H);
    const float* qi = q + (size_t)src[e] * (L + 1) * C;
    const float* ke = kg + (size_t)e * (L + 1) * C;
    float dot = 0.0f;
    for (int l = 0; l <= L; ++l)
        for (int c = hh * Ch; c < (hh + 1) * Ch; ++c) dot += qi[l * C + c] * ke[l * C + c];
    score[i] += tau * dot;
}

// alpha = softmax over the edges of a target, times the gate already stored in alpha (Eq. attn).
__global__ void k_edge_softmax(int N, int H, const int64_t* __restrict__ eoff, const float* __restrict__ score,
                               float* __restrict__ alpha) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N * H) return;
    const int t = i / H, hh = i % H;
    const int64_t e0 = eoff[t], e1 = eoff[t + 1];
    float mx = -INFINITY, z = 0.0f;
    for (int64_t e = e0; e < e1; ++e) mx = fmaxf(mx, score[e * H + hh]);
    for (int64_t e = e0; e < e1; ++e) z += __expf(score[e * H + hh] - mx);
    for (int64_t e = e0; e < e1; ++e) alpha[e * H + hh] *= __expf(score[e * H + hh] - mx) / z;
}

template <int L, int LF>
__global__ void k_edge_message(int64_t E, const int32_t* __restrict__ dst, const float* __restrict__ v,
                               const float* __restrict__ D, const float* __restrict__ cw, int C,
                               float* __restrict__ msg) {
    constexpr int n = (L + 1) * (L + 1);
    constexpr int DS = e2f::d_offset(L + 1), DSP = (DS + 3) & ~3;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= E * C) return;
    const int64_t e = i / C;
    const int c = (int)(i - e * C);
    const float* vj = v + (size_t)dst[e] * n * C + c;
    float vin[n][1], acc[n][1];
#pragma unroll
    for (int x = 0; x < n; ++x) {
        vin[x][0] = vj[x * C];
        acc[x][0] = 0.0f;
    }
    e2f::eaas_accumulate<L, LF, 1>(vin, D + e * DSP, cw, 1.0f, acc);
#pragma unroll
    for (int x = 0; x < n; ++x) msg[((size_t)e * n + x) * C + c] = acc[x][0];
}

__global__ void k_edge_reduce(E2fCellsView cv, const int64_t* __restrict__ eoff, const float* __restrict__ alpha,
                              const float* __restrict__ msg, int n, int C, int H, int Ch, float* __restrict__ out) {
    const int t = blockIdx.x;
    const int64_t e0 = eoff[t], e1 = eoff[t + 1];
    float* o = out + (size_t)cv.perm[t] * n * C;
    for (int x = threadIdx.x; x < n * C; x += blockDim.x) {
        const int hh = (x % C) / Ch;
        float acc = 0.0f;
        for (int64_t e = e0; e < e1; ++e) acc += alpha[e * H + hh] * msg[(size_t)e * n * C + x];
        o[x] = acc;
    }
}

template <int L, int LF>
e2f_status run(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
               float* out, hipStream_t st, size_t* edges_out, size_t* peak_bytes_out, hipEvent_t* ev) {
    const int N = cv.N, C = ctx->cfg.C, H = ctx->cfg.H, n = ctx->n;
    constexpr int DS = e2f::d_offset(L + 1), DSP = (DS + 3) & ~3;
    const int row = (L + 1) * C;
    // node-level buffers of the baseline: fp32 q, k, v, degrees and edge offsets
    const size_t node_bytes = e2f_align_up((size_t)N * row * 4) * 2 + e2f_align_up((size_t)N * n * C * 4) +
                              e2f_align_up((size_t)N * 4) + e2f_align_up((size_t)(N + 1) * 8);
    char* node = nullptr;
    if (hipMalloc((void**)&node, node_bytes) != hipSuccess) return E2F_ERR_OOM;
    char* p = node;
    float* q = (float*)p; p += e2f_align_up((size_t)N * row * 4);
    float* k = (float*)p; p += e2f_align_up((size_t)N * row * 4);
    float* v = (float*)p; p += e2f_align_up((size_t)N * n * C * 4);
    int32_t* degree = (int32_t*)p; p += e2f_align_up((size_t)N * 4);
    int64_t* eoff = (int64_t*)p;

    // with profiling on: stage 0 = node-level kernels, stage 1 = host synchronisation and allocation of the edge
    // tensors, stage 2 = the edge kernels
    if (ev) (void)hipEventRecord(ev[0], st);
    e2f_status rc = e2f_launch_project_simple(ctx, cv, h, w, q, k, v, st);
    if (rc != E2F_OK) { (void)hipFree(node); return rc; }
    k_edge_walk<<<N, 64, 0, st>>>(cv, ws.spos, ctx->rc2, degree, nullptr, nullptr, nullptr);
    k_scan_degree<<<1, 1024, 0, st>>>(degree, N, eoff);
    if (ev) (void)hipEventRecord(ev[1], st);
    int64_t E = 0;
    if (hipMemcpyAsync(&E, eoff + N, sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipFree(node);
        return E2F_ERR_HIP;
    }
    if (edges_out) *edges_out = (size_t)E;

    const size_t Ea = E > 0 ? (size_t)E : 1;
    const size_t sizes[8] = {Ea * 4, Ea * 4, Ea * 16, Ea * DSP * 4, Ea * row * 4, Ea * H * 4, Ea * H * 4,
                             Ea * (size_t)n * C * 4};
    size_t edge_bytes = 0;
    for (size_t s : sizes) edge_bytes += e2f_align_up(s);
    char* edge = nullptr;
    if (hipMalloc((void**)&edge, edge_bytes) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(node);
        return E2F_ERR_OOM;
    }
    if (peak_bytes_out) *peak_bytes_out = node_bytes + edge_bytes;
    EdgeBuffers eb;
    p = edge;
    eb.src = (int32_t*)p; p += e2f_align_up(sizes[0]);
    eb.dst = (int32_t*)p; p += e2f_align_up(sizes[1]);
    eb.geo = (float4*)p; p += e2f_align_up(sizes[2]);
    eb.D = (float*)p; p += e2f_align_up(sizes[3]);
    eb.kg = (float*)p; p += e2f_align_up(sizes[4]);
    eb.score = (float*)p; p += e2f_align_up(sizes[5]);
    eb.alpha = (float*)p; p += e2f_align_up(sizes[6]);
    eb.msg = (float*)p;

    const int tb = 256;
    if (ev) (void)hipEventRecord(ev[2], st);
    if (E > 0) {
        k_edge_walk<<<N, 64, 0, st>>>(cv, ws.spos, ctx->rc2, nullptr, eoff, eb.src, eb.dst);
        k_edge_geometry<L, LF><<<(unsigned)((E + tb - 1) / tb), tb, 0, st>>>(
            E, eb.src, eb.dst, ws.spos, w->Wb, H, ctx->cfg.B, ctx->cfg.cutoff, ctx->rbf_step, ctx->rbf_gamma, eb.geo,
            eb.D, eb.score, eb.alpha);
        k_edge_gather_k<<<(unsigned)((E * row + tb - 1) / tb), tb, 0, st>>>(E, eb.dst, k, row, eb.kg);
        k_edge_score<<<(unsigned)((E * H + tb - 1) / tb), tb, 0, st>>>(E, eb.src, q, eb.kg, L, C, H, ctx->Ch, ctx->tau,
                                                                      eb.score);
        k_edge_softmax<<<(N * H + tb - 1) / tb, tb, 0, st>>>(N, H, eoff, eb.score, eb.alpha);
        k_edge_message<L, LF><<<(unsigned)((E * C + tb - 1) / tb), tb, 0, st>>>(E, eb.dst, v, eb.D, ws.cw, C, eb.msg);
    }
    k_edge_reduce<<<N, 256, 0, st>>>(cv, eoff, eb.alpha, eb.msg, n, C, H, ctx->Ch, out);
    if (ev) (void)hipEventRecord(ev[3], st);
    hipError_t err = hipGetLastError();
    if (err == hipSuccess) err = hipStreamSynchronize(st);
    (void)hipFree(edge);
    (void)hipFree(node);
    return err == hipSuccess ? E2F_OK : E2F_ERR_HIP;
}

template <int L>
e2f_status run_lf(const e2f_ctx* ctx, const E2fCellsView& cv, const void* h, const e2f_weights* w, const E2fAttnWs& ws,
                  float* out, hipStream_t st, size_t* edges_out, size_t* peak_bytes_out, hipEvent_t* ev) {
    switch (ctx->cfg.lf) {
        case 0: return run<L, 0>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 1: return run<L, 1>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 2: return run<L, 2>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
    }
    return E2F_ERR_UNSUPPORTED;
}

}  // namespace

e2f_status e2f_run_materialized(const e2f_ctx* ctx, const E2fCellsView& cv, const float* pos, const void* h,
                                const e2f_weights* w, const E2fAttnWs& ws, float* out, hipStream_t st,
                                size_t* edges_out, size_t* peak_bytes_out, hipEvent_t* ev) {
    if (edges_out) *edges_out = 0;
    if (peak_bytes_out) *peak_bytes_out = 0;
    if (cv.N == 0) return E2F_OK;
    e2f_status rc = e2f_launch_prepare(ctx, cv, pos, w, ws, st);
    if (rc != E2F_OK) return rc;
    switch (ctx->cfg.L_max) {
        case 0: return run_lf<0>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 1: return run_lf<1>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 2: return run_lf<2>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 3: return run_lf<3>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
        case 4: return run_lf<4>(ctx, cv, h, w, ws, out, st, edges_out, peak_bytes_out, ev);
    }
    return E2F_ERR_UNSUPPORTED;
}
