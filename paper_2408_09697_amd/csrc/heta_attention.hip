// Graph attention as the relation-specific aggregation (R-GAT, Section 2.1 of the paper: one GAT
// module per mono-relation subgraph, outputs summed over the relations and activated by ReLU).
// The module is the attention layer of the GAT paper (Velickovic et al. 2018, Eqs. 1-4, multi-head
// concatenation) on a bipartite relation with K heads of width F:
//
//     s_e[k]     = LeakyReLU(el[u_e, k] + er[v_e, k])
//     alpha_e[k] = exp(s_e[k]) / sum_{e' into v_e} exp(s_e'[k])
//     o[v, kF+f] = sum_{e into v} alpha_e[k] z[u_e, kF+f]
//
// el = <z_u[k,:], a[k,:]> and er = <h_v, q[k,:]> are row scores computed by attn_score_kernel.
//
// Split of the work: everything that touches only scalars per edge (logits, softmax statistics, the
// weights alpha, their LeakyReLU-gated form) runs in "row sweep" kernels over the schedule-ordered
// adjacency and leaves one weight per (edge slot, head) in a workspace; everything that moves feature
// rows is then the ordinary segmented gather-reduce with those weights (aggregate_slot_weighted), so
// the hub-chunk / long-row / equal-degree-batch scheduling is shared with the R-GCN aggregation.
//
// Backward, for upstream gradient g = dL/do, with dot[v,k] = <g[v,k,:], o[v,k,:]>:
//     dz[u]     = sum_{e out of u} alpha_e g[v_e]                           (CSC gather, weights alpha)
//     gate_e    = alpha_e * LeakyReLU'(el + er)
//     der[v,k]  = sum_{e into v} gate_e (<g[v], z[u_e]>_k - dot[v,k])
//               = <g[v], sum_e gate_e z[u_e]>_k - dot[v,k] sum_e gate_e      (CSR gather, weights gate)
//     del[u,k]  = <z[u], sum_{e out of u} gate_e g[v_e]>_k - sum_e gate_e dot[v_e,k]   (CSC gather, weights gate)
// i.e. the per-edge dot products of the softmax backward collapse, by linearity, into weighted
// aggregations followed by one per-row, per-head dot product.  No atomics anywhere.
#include <algorithm>

#include "heta_internal.h"

namespace heta {

namespace {

using bf16_t = uint16_t;
constexpr int kMaxHeads = 16;
constexpr int kShortDegAttn = 32; // same split as the aggregation: below, one thread per (row, head)

__device__ __forceinline__ float lrelu(float x, float slope) { return x > 0.f ? x : slope * x; }

// ---- row sweeps ------------------------------------------------------------------------------------------
// One sweep visits every edge slot of a schedule once per phase and touches only scalars: the neighbour's
// id, KT consecutive heads of its score (one vector load), and the per-slot weights it writes.
//   rows of fewer than 32 edges: one thread per row; 32..511 edges: one wavefront per row;
//   hub rows (>= 512 edges): one wavefront per 256-edge chunk writes partial statistics, a second kernel
//   combines a row's chunks in chunk order, and (forward only) a third writes the weights.
enum SweepOp { SWEEP_FWD = 0, SWEEP_BWD_CSR = 1, SWEEP_BWD_CSC = 2 };
enum Phase { PH_MAX = 0, PH_SUM = 1, PH_ALPHA = 2, PH_BWD_DST = 3, PH_BWD_SRC = 4 };

struct SweepParams {
    const int64_t *sptr;
    const int32_t *sidx;
    const int32_t *perm;
    const HubChunk *hub_chunks;
    const int64_t *hub_chunk_ptr;
    int64_t n_hub_rows, n_hub_chunks;
    int64_t q0, q1;       // schedule positions of this launch
    int K;
    float slope;
    const float *row_a;   // [rows][K]  score half of the row side (er for the CSR, el for the CSC)
    const float *nbr_a;   // [nbrs][K]  score half of the neighbour side
    float *smax, *sinv;   // [dst][K]   softmax shift and 1/denominator: written by FWD (nullable), read by the others
    const float *dot;     // [dst][K]   <g, o> per head (backward)
    float *alpha;         // [E][K] by edge slot (FWD, BWD_CSC)
    float *gate;          // [E][K] by edge slot: alpha * LeakyReLU' (BWD_SRC; BWD_DST if non-null), or alpha on the
                          // edges with a positive logit (FWD, if non-null)
    float dot_shift;      // BWD_CSR: corr = dot * (sum of gates - dot_shift)
    float *corr;          // [rows][K]  the scalar term subtracted from the row's score gradient (BWD_*)
    const float *nbr_pack; // BWD_CSC: [dst][4][K] = the destination's er, smax, sinv, dot side by side (one cache line
                          // per neighbour instead of four gathers)
    float *part;          // hub chunks: [n_hub_chunks][K][2] partial statistics
    float *hub_stat;      // hub rows (FWD): [n_hub_rows][K][2] = shift, 1/denominator
};

template <int KT> __device__ __forceinline__ void loadk(const float *p, float *v);
template <> __device__ __forceinline__ void loadk<1>(const float *p, float *v) { v[0] = *p; }
template <> __device__ __forceinline__ void loadk<2>(const float *p, float *v)
{
    const float2 t = *reinterpret_cast<const float2 *>(p);
    v[0] = t.x; v[1] = t.y;
}
template <> __device__ __forceinline__ void loadk<4>(const float *p, float *v)
{
    const float4 t = *reinterpret_cast<const float4 *>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <int KT> __device__ __forceinline__ void storek(float *p, const float *v);
template <> __device__ __forceinline__ void storek<1>(float *p, const float *v) { *p = v[0]; }
template <> __device__ __forceinline__ void storek<2>(float *p, const float *v) { *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]); }
template <> __device__ __forceinline__ void storek<4>(float *p, const float *v)
{
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// One edge slot e, heads k0 .. k0+KT-1.  ar: the row's score half; m, inv: shift and 1/denominator of the
// row (unused by PH_MAX and PH_BWD_SRC, which reads the neighbour's); acc: running max or sum.
template <int KT, int PH>
__device__ __forceinline__ void visit(const SweepParams &p, int64_t e, int k0, const float *ar, const float *m,
                                      const float *inv, float *acc)
{
    const int64_t id = p.sidx[e];
    float x[KT];
    float mv[KT], iv[KT], dv[KT];
    if (PH == PH_BWD_SRC) {
        const float *pk = p.nbr_pack + id * 4 * p.K + k0;
        loadk<KT>(pk, x);
        loadk<KT>(pk + p.K, mv);
        loadk<KT>(pk + 2 * p.K, iv);
        loadk<KT>(pk + 3 * p.K, dv);
    } else {
        loadk<KT>(p.nbr_a + id * p.K + k0, x);
    }
    float a[KT], gt[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        x[k] += ar[k];
        const float sc = lrelu(x[k], p.slope);
        if (PH == PH_MAX) {
            acc[k] = fmaxf(acc[k], sc);
        } else if (PH == PH_SUM) {
            acc[k] += expf(sc - m[k]);
        } else if (PH == PH_ALPHA) {
            a[k] = expf(sc - m[k]) * inv[k];
            gt[k] = x[k] > 0.f ? a[k] : 0.f; // the weight restricted to edges with a positive logit
        } else if (PH == PH_BWD_DST) {
            gt[k] = expf(sc - m[k]) * inv[k] * (x[k] > 0.f ? 1.f : p.slope);
            acc[k] += gt[k];
        } else {
            a[k] = expf(sc - mv[k]) * iv[k];
            gt[k] = a[k] * (x[k] > 0.f ? 1.f : p.slope);
            acc[k] = fmaf(gt[k], dv[k], acc[k]);
        }
    }
    if (PH == PH_ALPHA || PH == PH_BWD_SRC) storek<KT>(p.alpha + e * p.K + k0, a);
    if (PH == PH_BWD_SRC || ((PH == PH_ALPHA || PH == PH_BWD_DST) && p.gate)) storek<KT>(p.gate + e * p.K + k0, gt);
}

template <int W, int KT, int PH>
__device__ __forceinline__ void sweep_range(const SweepParams &p, int64_t e0, int64_t e1, int lane, int k0, const float *ar,
                                            const float *m, const float *inv, float *acc)
{
#pragma unroll 4
    for (int64_t e = e0 + lane; e < e1; e += W) visit<KT, PH>(p, e, k0, ar, m, inv, acc);
}

template <int KT> __device__ __forceinline__ void wave_sum(float *v)
{
#pragma unroll
    for (int k = 0; k < KT; ++k)
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v[k] += __shfl_xor(v[k], off, 64);
}
template <int KT> __device__ __forceinline__ void wave_max(float *v)
{
#pragma unroll
    for (int k = 0; k < KT; ++k)
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v[k] = fmaxf(v[k], __shfl_xor(v[k], off, 64));
}

// rows below the hub threshold: W = 1 (one thread per row) or W = 64 (one wavefront per row)
template <int W, int KT, int OP>
__global__ void __launch_bounds__(256) attn_rows_kernel(SweepParams p)
{
    const int lane = W == 1 ? 0 : (threadIdx.x & 63);
    const int64_t q = p.q0 + (W == 1 ? static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x
                                     : static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6));
    if (q >= p.q1) return; // uniform per wavefront when W = 64
    const int k0 = blockIdx.y * KT;
    const int64_t row = p.perm[q];
    const int64_t e0 = p.sptr[q], e1 = p.sptr[q + 1];
    float ar[KT], acc[KT], m[KT], inv[KT];
    loadk<KT>(p.row_a + row * p.K + k0, ar);
    if (OP == SWEEP_FWD && W == 1 && e1 - e0 <= 4 && e1 > e0) {
        // up to four edges (most rows of a power-law graph): the logits stay in registers, one pass
        const int n = static_cast<int>(e1 - e0);
        float sc[4][KT];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < n) {
                loadk<KT>(p.nbr_a + static_cast<int64_t>(p.sidx[e0 + j]) * p.K + k0, sc[j]);
#pragma unroll
                for (int k = 0; k < KT; ++k) sc[j][k] = lrelu(sc[j][k] + ar[k], p.slope);
            } else {
#pragma unroll
                for (int k = 0; k < KT; ++k) sc[j][k] = -INFINITY;
            }
        }
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            m[k] = fmaxf(fmaxf(sc[0][k], sc[1][k]), fmaxf(sc[2][k], sc[3][k]));
            float den = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) den += j < n ? expf(sc[j][k] - m[k]) : 0.f; // same order as the general path
            inv[k] = 1.f / den;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < n) {
                float a[KT], gt[KT];
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    a[k] = expf(sc[j][k] - m[k]) * inv[k];
                    gt[k] = sc[j][k] > 0.f ? a[k] : 0.f; // LeakyReLU keeps the sign of the logit
                }
                storek<KT>(p.alpha + (e0 + j) * p.K + k0, a);
                if (p.gate) storek<KT>(p.gate + (e0 + j) * p.K + k0, gt);
            }
        }
        if (p.smax) {
            storek<KT>(p.smax + row * p.K + k0, m);
            storek<KT>(p.sinv + row * p.K + k0, inv);
        }
    } else if (OP == SWEEP_FWD) {
#pragma unroll
        for (int k = 0; k < KT; ++k) m[k] = -INFINITY;
        sweep_range<W, KT, PH_MAX>(p, e0, e1, lane, k0, ar, nullptr, nullptr, m);
        if (W == 64) wave_max<KT>(m);
#pragma unroll
        for (int k = 0; k < KT; ++k) acc[k] = 0.f;
        sweep_range<W, KT, PH_SUM>(p, e0, e1, lane, k0, ar, m, nullptr, acc);
        if (W == 64) wave_sum<KT>(acc);
        const bool empty = e1 == e0;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            inv[k] = empty ? 0.f : 1.f / acc[k];
            if (empty) m[k] = 0.f;
        }
        sweep_range<W, KT, PH_ALPHA>(p, e0, e1, lane, k0, ar, m, inv, nullptr);
        if (lane == 0 && p.smax) {
            storek<KT>(p.smax + row * p.K + k0, m);
            storek<KT>(p.sinv + row * p.K + k0, inv);
        }
    } else {
#pragma unroll
        for (int k = 0; k < KT; ++k) acc[k] = 0.f;
        if (OP == SWEEP_BWD_CSR) {
            loadk<KT>(p.smax + row * p.K + k0, m);
            loadk<KT>(p.sinv + row * p.K + k0, inv);
            sweep_range<W, KT, PH_BWD_DST>(p, e0, e1, lane, k0, ar, m, inv, acc);
        } else {
            sweep_range<W, KT, PH_BWD_SRC>(p, e0, e1, lane, k0, ar, nullptr, nullptr, acc);
        }
        if (W == 64) wave_sum<KT>(acc);
        if (lane == 0) {
            if (OP == SWEEP_BWD_CSR) {
                float d[KT];
                loadk<KT>(p.dot + row * p.K + k0, d);
#pragma unroll
                for (int k = 0; k < KT; ++k) acc[k] = (acc[k] - p.dot_shift) * d[k];
            }
            storek<KT>(p.corr + row * p.K + k0, acc);
        }
    }
}

// hub row of chunk w: the h with hub_chunk_ptr[h] <= w < hub_chunk_ptr[h + 1]
__device__ __forceinline__ int64_t hub_of_chunk(const SweepParams &p, int64_t w)
{
    int64_t lo = 0, hi = p.n_hub_rows; // invariant: ptr[lo] <= w < ptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (p.hub_chunk_ptr[mid] <= w) lo = mid;
        else hi = mid;
    }
    return lo;
}

// hub chunks, first kernel: partial statistics of one chunk (and the backward's weights)
template <int KT, int OP>
__global__ void __launch_bounds__(256) attn_hub_partial_kernel(SweepParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (w >= p.n_hub_chunks) return; // uniform per wavefront
    const int k0 = blockIdx.y * KT;
    const HubChunk c = p.hub_chunks[w];
    const int64_t row = p.perm[hub_of_chunk(p, w)];
    const int64_t e0 = c.e0, e1 = c.e0 + c.len;
    float ar[KT], acc[KT], m[KT], inv[KT];
    loadk<KT>(p.row_a + row * p.K + k0, ar);
    float *out = p.part + (w * p.K + k0) * 2;
    if (OP == SWEEP_FWD) {
#pragma unroll
        for (int k = 0; k < KT; ++k) m[k] = -INFINITY;
        sweep_range<64, KT, PH_MAX>(p, e0, e1, lane, k0, ar, nullptr, nullptr, m);
        wave_max<KT>(m);
#pragma unroll
        for (int k = 0; k < KT; ++k) acc[k] = 0.f;
        sweep_range<64, KT, PH_SUM>(p, e0, e1, lane, k0, ar, m, nullptr, acc);
        wave_sum<KT>(acc);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                out[2 * k] = m[k];
                out[2 * k + 1] = acc[k];
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < KT; ++k) acc[k] = 0.f;
        if (OP == SWEEP_BWD_CSR) {
            loadk<KT>(p.smax + row * p.K + k0, m);
            loadk<KT>(p.sinv + row * p.K + k0, inv);
            sweep_range<64, KT, PH_BWD_DST>(p, e0, e1, lane, k0, ar, m, inv, acc);
        } else {
            sweep_range<64, KT, PH_BWD_SRC>(p, e0, e1, lane, k0, ar, nullptr, nullptr, acc);
        }
        wave_sum<KT>(acc);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < KT; ++k) out[2 * k] = acc[k];
        }
    }
}

// hub rows, second kernel: one wavefront per (hub row, head) combines the row's chunks in chunk order
template <int OP>
__global__ void __launch_bounds__(256) attn_hub_combine_kernel(SweepParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t h = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (h >= p.n_hub_rows) return;
    const int k = blockIdx.y;
    const int64_t row = p.perm[h];
    const int64_t s0 = p.hub_chunk_ptr[h], s1 = p.hub_chunk_ptr[h + 1];
    if (OP == SWEEP_FWD) {
        float m = -INFINITY;
        for (int64_t s = s0 + lane; s < s1; s += 64) m = fmaxf(m, p.part[(s * p.K + k) * 2]);
        wave_max<1>(&m);
        float den = 0.f;
        for (int64_t s = s0 + lane; s < s1; s += 64) den += p.part[(s * p.K + k) * 2 + 1] * expf(p.part[(s * p.K + k) * 2] - m);
        wave_sum<1>(&den);
        if (lane == 0) {
            const float inv = 1.f / den; // a hub row has edges
            p.hub_stat[(h * p.K + k) * 2] = m;
            p.hub_stat[(h * p.K + k) * 2 + 1] = inv;
            if (p.smax) {
                p.smax[row * p.K + k] = m;
                p.sinv[row * p.K + k] = inv;
            }
        }
    } else {
        float a = 0.f;
        for (int64_t s = s0 + lane; s < s1; s += 64) a += p.part[(s * p.K + k) * 2];
        wave_sum<1>(&a);
        if (lane == 0) p.corr[row * p.K + k] = OP == SWEEP_BWD_CSR ? (a - p.dot_shift) * p.dot[row * p.K + k] : a;
    }
}

// hub chunks, third kernel (forward): the weights, from the combined statistics
template <int KT>
__global__ void __launch_bounds__(256) attn_hub_alpha_kernel(SweepParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (w >= p.n_hub_chunks) return;
    const int k0 = blockIdx.y * KT;
    const HubChunk c = p.hub_chunks[w];
    const int64_t h = hub_of_chunk(p, w);
    const int64_t row = p.perm[h];
    float ar[KT], m[KT], inv[KT];
    loadk<KT>(p.row_a + row * p.K + k0, ar);
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        m[k] = p.hub_stat[(h * p.K + k0 + k) * 2];
        inv[k] = p.hub_stat[(h * p.K + k0 + k) * 2 + 1];
    }
    sweep_range<64, KT, PH_ALPHA>(p, c.e0, c.e0 + c.len, lane, k0, ar, m, inv, nullptr);
}

// pack[v][0..3][K] = er[v], smax[v], sinv[v], dot[v]
__global__ void __launch_bounds__(256) attn_pack_kernel(const float *er, const float *smax, const float *sinv, const float *dot,
                                                        int64_t n, int K, float *pack)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= n * K) return;
    const int64_t v = t / K;
    const int k = static_cast<int>(t - v * K);
    float *o = pack + v * 4 * K + k;
    o[0] = er[t];
    o[K] = smax[t];
    o[2 * K] = sinv[t];
    o[3 * K] = dot[t];
}

inline size_t hub_scratch_bytes(const Schedule &s, int K)
{
    return static_cast<size_t>(s.n_hub_chunks + s.n_hub_rows) * K * 2 * sizeof(float);
}

template <int KT, int OP>
heta_status launch_sweeps_kt(const Schedule &s, SweepParams p, hipStream_t st)
{
    const int64_t n_long_or_hub = s.rows_with_deg_ge[kShortDegAttn];
    const unsigned gy = p.K / KT;
    if (s.n_hub_rows > 0) {
        const unsigned cb = (unsigned)((s.n_hub_chunks + 3) / 4), rb = (unsigned)((s.n_hub_rows + 3) / 4);
        hipLaunchKernelGGL((attn_hub_partial_kernel<KT, OP>), dim3(cb, gy), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_hub_partial_kernel");
        hipLaunchKernelGGL((attn_hub_combine_kernel<OP>), dim3(rb, p.K), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_hub_combine_kernel");
        if (OP == SWEEP_FWD) {
            hipLaunchKernelGGL((attn_hub_alpha_kernel<KT>), dim3(cb, gy), dim3(256), 0, st, p);
            HETA_LAUNCH_CHECK("attn_hub_alpha_kernel");
        }
    }
    if (n_long_or_hub > s.n_hub_rows) {
        p.q0 = s.n_hub_rows;
        p.q1 = n_long_or_hub;
        hipLaunchKernelGGL((attn_rows_kernel<64, KT, OP>), dim3((unsigned)((p.q1 - p.q0 + 3) / 4), gy), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_rows_kernel");
    }
    if (s.n_rows > n_long_or_hub) {
        p.q0 = n_long_or_hub;
        p.q1 = s.n_rows;
        hipLaunchKernelGGL((attn_rows_kernel<1, KT, OP>), dim3((unsigned)((p.q1 - p.q0 + 255) / 256), gy), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_rows_kernel");
    }
    return HETA_OK;
}

// `hub_scratch`: hub_scratch_bytes(s, K) bytes of device memory for the hub rows' partial statistics
template <int OP>
heta_status launch_sweeps(const Schedule &s, SweepParams p, float *hub_scratch, hipStream_t st, const char *name)
{
    if (s.n_rows == 0) return HETA_OK;
    p.sptr = s.d_sptr;
    p.sidx = s.d_sidx;
    p.perm = s.d_perm;
    p.hub_chunks = s.d_hub_chunks;
    p.hub_chunk_ptr = s.d_hub_chunk_ptr;
    p.n_hub_rows = s.n_hub_rows;
    p.n_hub_chunks = s.n_hub_chunks;
    p.part = hub_scratch;
    p.hub_stat = hub_scratch + s.n_hub_chunks * p.K * 2;
    // Algorithmic bytes: per edge one 4-byte id, per edge and head the neighbour's 4-byte terms and the
    // 4-byte weights written; per row its offsets and per-head terms.
    const double per_edge = 4.0 + p.K * (OP == SWEEP_BWD_CSC ? 24.0 : 8.0);
    ProfScope prof(name, st, per_edge * static_cast<double>(s.n_edges) + static_cast<double>(s.n_rows) * (12.0 + 12.0 * p.K), 0);
    // KT consecutive heads per thread need 4*KT-byte aligned score rows
    const uintptr_t all = reinterpret_cast<uintptr_t>(p.row_a) | reinterpret_cast<uintptr_t>(p.nbr_a) |
                          reinterpret_cast<uintptr_t>(p.smax) | reinterpret_cast<uintptr_t>(p.sinv) |
                          reinterpret_cast<uintptr_t>(p.dot) | reinterpret_cast<uintptr_t>(p.nbr_pack) | reinterpret_cast<uintptr_t>(p.alpha) |
                          reinterpret_cast<uintptr_t>(p.gate) | reinterpret_cast<uintptr_t>(p.corr);
    if (p.K % 4 == 0 && all % 16 == 0) return launch_sweeps_kt<4, OP>(s, p, st);
    if (p.K % 2 == 0 && all % 8 == 0) return launch_sweeps_kt<2, OP>(s, p, st);
    return launch_sweeps_kt<1, OP>(s, p, st);
}

// ---- per-row, per-head dot products -------------------------------------------------------------------
// out[i, k] = sum_j x[i, j] y_k[j] - corr[i, k], one wavefront per row.
//   per_head = 1: j runs over head k's columns [kF, (k+1)F); y is a second matrix (ld_y > 0) or one
//                 row shared by every i (ld_y = 0: the attention vector a, laid out [K][F] = [d]).
//   per_head = 0: j runs over all d columns and y_k = y + k*d (a [K][d] matrix shared by every row).
struct DotParams {
    const void *x;
    int64_t ld_x;
    const void *y;
    int64_t ld_y;
    int64_t n;
    int d, K, F, per_head;
    float scale;          // out = scale * <x, y> - corr
    const float *corr;
    float *out;
    // optional second operand with rows of its own (per_head only): out2 = scale2 * <x, y2>, in the same pass over x
    const void *y2;
    float scale2;
    float *out2;
};

template <typename T> __device__ __forceinline__ float ld1(const T *p);
template <> __device__ __forceinline__ float ld1<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld1<bf16_t>(const bf16_t *p) { return __uint_as_float(static_cast<uint32_t>(*p) << 16); }

template <typename T, int EPC> __device__ __forceinline__ void ldv(const T *p, float *f);
template <> __device__ __forceinline__ void ldv<float, 4>(const float *p, float *f)
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
}
template <> __device__ __forceinline__ void ldv<float, 1>(const float *p, float *f) { f[0] = *p; }
template <> __device__ __forceinline__ void ldv<bf16_t, 4>(const bf16_t *p, float *f)
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}
template <> __device__ __forceinline__ void ldv<bf16_t, 1>(const bf16_t *p, float *f) { f[0] = ld1(p); }

template <typename TX, typename TY, int EPC>
__global__ void __launch_bounds__(256) attn_rowdot_kernel(DotParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (i >= p.n) return; // uniform per wavefront
    const TX *x = static_cast<const TX *>(p.x) + i * p.ld_x;
    const TY *y = static_cast<const TY *>(p.y) + i * p.ld_y;
    float res = 0.f;
    for (int k = 0; k < p.K; ++k) {
        const int j0 = p.per_head ? k * p.F : 0, j1 = p.per_head ? (k + 1) * p.F : p.d;
        const TY *yk = p.per_head ? y : y + static_cast<int64_t>(k) * p.d;
        float part = 0.f;
        for (int j = j0 + lane * EPC; j < j1; j += 64 * EPC) {
            float a[EPC], b[EPC];
            ldv<TX, EPC>(x + j, a);
            ldv<TY, EPC>(yk + j, b);
#pragma unroll
            for (int t = 0; t < EPC; ++t) part = fmaf(a[t], b[t], part);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        if (lane == k) res = part;
    }
    if (lane < p.K) p.out[i * p.K + lane] = p.scale * res - (p.corr ? p.corr[i * p.K + lane] : 0.f);
}

// Fast path: a row's 16-byte chunks are spread over a group of L lanes (L a power of two, T chunks per
// lane), 64 / L rows per wavefront, every chunk loaded once; the per-head sums are segmented cross-lane
// reductions.  Needs 4-element chunks that do not straddle heads and, per head, a power-of-two number of
// chunks (cph); a head then lies inside one t (cph <= L) or covers whole t's (cph a multiple of L).
template <typename TX, typename TY, int T, int R>
__global__ void __launch_bounds__(256) attn_rowdot_fast_kernel(DotParams p, int L, int cph)
{
    const int lane = threadIdx.x & 63;
    const int G = 64 / L, g = lane / L, l = lane % L;
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * R * G + g; // rows first, first + G, ...
    const int n_chunks = p.d / 4;
    float xv[R][T][4];
    bool live[R];
    // every load of the wavefront's R row groups is issued before the first use
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int64_t i = first + static_cast<int64_t>(r) * G;
        live[r] = i < p.n;
        const TX *x = static_cast<const TX *>(p.x) + (live[r] ? i : 0) * p.ld_x;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int c = l + L * t;
            if (live[r] && c < n_chunks) ldv<TX, 4>(x + 4 * c, xv[r][t]);
            else xv[r][t][0] = xv[r][t][1] = xv[r][t][2] = xv[r][t][3] = 0.f;
        }
    }
    if (p.per_head) {
      for (int pass = 0; pass < (p.y2 ? 2 : 1); ++pass) { // uniform: the second operand's rows against the same x registers
        const void *yp = pass ? p.y2 : p.y;
        float *outp = pass ? p.out2 : p.out;
        const float scl = pass ? p.scale2 : p.scale;
        const float *corrp = pass ? nullptr : p.corr;
        float part[R][T];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t i = first + static_cast<int64_t>(r) * G;
            const TY *y = static_cast<const TY *>(yp) + (live[r] ? i : 0) * p.ld_y;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int c = l + L * t;
                float yv[4] = {0.f, 0.f, 0.f, 0.f};
                if (live[r] && c < n_chunks) ldv<TY, 4>(y + 4 * c, yv);
                part[r][t] = xv[r][t][0] * yv[0] + xv[r][t][1] * yv[1] + xv[r][t][2] * yv[2] + xv[r][t][3] * yv[3];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t i = first + static_cast<int64_t>(r) * G;
            if (cph <= L) {
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    for (int off = cph >> 1; off > 0; off >>= 1) part[r][t] += __shfl_xor(part[r][t], off, 64);
                    const int c = l + L * t;
                    if (live[r] && c < n_chunks && (l & (cph - 1)) == 0) {
                        const int k = c / cph;
                        outp[i * p.K + k] = scl * part[r][t] - (corrp ? corrp[i * p.K + k] : 0.f);
                    }
                }
            } else {
                const int m = cph / L; // t's per head
                float acc = 0.f;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    acc += part[r][t];
                    if ((t + 1) % m == 0) {
                        for (int off = L >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
                        const int k = t / m;
                        if (live[r] && l == 0 && k < p.K) outp[i * p.K + k] = scl * acc - (corrp ? corrp[i * p.K + k] : 0.f);
                        acc = 0.f;
                    }
                }
            }
        }
      }
    } else {
        // y_k = p.y + k d is shared by every row (ld_y = 0): one load per k serves the R rows
        for (int k = 0; k < p.K; ++k) {
            const TY *yk = static_cast<const TY *>(p.y) + static_cast<int64_t>(k) * p.d;
            float yv[T][4];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int c = l + L * t;
                if (c < n_chunks) ldv<TY, 4>(yk + 4 * c, yv[t]);
                else yv[t][0] = yv[t][1] = yv[t][2] = yv[t][3] = 0.f;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int64_t i = first + static_cast<int64_t>(r) * G;
                float acc = 0.f;
#pragma unroll
                for (int t = 0; t < T; ++t)
                    acc += xv[r][t][0] * yv[t][0] + xv[r][t][1] * yv[t][1] + xv[r][t][2] * yv[t][2] + xv[r][t][3] * yv[t][3];
                for (int off = L >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
                if (live[r] && l == 0) p.out[i * p.K + k] = p.scale * acc - (p.corr ? p.corr[i * p.K + k] : 0.f);
            }
        }
    }
}

// a[i] -= b[i]
__global__ void __launch_bounds__(256) attn_sub_kernel(float *a, const float *b, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) a[i] -= b[i];
}

template <typename TX, typename TY>
heta_status launch_rowdot_t(const DotParams &p, hipStream_t st)
{
    if (p.n == 0) return HETA_OK;
    const size_t sx = sizeof(TX), sy = sizeof(TY);
    if (p.y2) { // only the one-pass kernel takes a second operand: anything else runs as two launches
        const int nc = p.d / 4, cph2 = p.F / 4;
        int L2 = 1;
        while (L2 < nc && L2 < 64) L2 <<= 1;
        const int T2 = (nc + L2 - 1) / L2;
        const bool one_pass = p.per_head && p.ld_y && (reinterpret_cast<uintptr_t>(p.x) % (4 * sx) == 0) && (p.ld_x % 4 == 0) &&
                              (reinterpret_cast<uintptr_t>(p.y) % (4 * sy) == 0) && (reinterpret_cast<uintptr_t>(p.y2) % (4 * sy) == 0) &&
                              (p.ld_y % 4 == 0) && (p.d % 4 == 0) && (p.F % 4 == 0) && T2 <= 4 && cph2 > 0 &&
                              (cph2 & (cph2 - 1)) == 0 && (cph2 <= L2 || T2 % (cph2 / L2) == 0);
        if (!one_pass) {
            DotParams a = p, b = p;
            a.y2 = nullptr;
            b.y = p.y2;
            b.y2 = nullptr;
            b.scale = p.scale2;
            b.corr = nullptr;
            b.out = p.out2;
            heta_status e = launch_rowdot_t<TX, TY>(a, st);
            return e != HETA_OK ? e : launch_rowdot_t<TX, TY>(b, st);
        }
    }
    const bool vec = (reinterpret_cast<uintptr_t>(p.x) % (4 * sx) == 0) && (p.ld_x % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(p.y) % (4 * sy) == 0) && (p.ld_y % 4 == 0) && (p.d % 4 == 0) &&
                     (p.F % 4 == 0);
    const int64_t blocks = (p.n + 3) / 4;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "attention: too many rows");
    const double bytes = static_cast<double>(p.n) * (p.d * (sx + (p.ld_y ? sy : 0) + (p.y2 ? sy : 0)) + 4.0 * p.K * ((p.corr ? 2 : 1) + (p.y2 ? 1 : 0)));
    ProfScope prof("attn_rowdot_kernel", st, bytes, 0);
    if (vec) {
        const int n_chunks = p.d / 4;
        int L = 1;
        while (L < n_chunks && L < 64) L <<= 1;
        const int T = (n_chunks + L - 1) / L;
        const int cph = p.F / 4;
        const bool pow2 = (cph & (cph - 1)) == 0;
        if (T <= 4 && (!p.per_head || (pow2 && (cph <= L || T % (cph / L) == 0)))) {
            const int R = T == 1 ? 4 : (T == 2 ? 2 : 1); // row groups per wavefront, all loads in flight together
            const int64_t rows_per_block = static_cast<int64_t>(4) * R * (64 / L);
            const dim3 grid((unsigned)((p.n + rows_per_block - 1) / rows_per_block));
            switch (T) {
            case 1: hipLaunchKernelGGL((attn_rowdot_fast_kernel<TX, TY, 1, 4>), grid, dim3(256), 0, st, p, L, cph); break;
            case 2: hipLaunchKernelGGL((attn_rowdot_fast_kernel<TX, TY, 2, 2>), grid, dim3(256), 0, st, p, L, cph); break;
            case 3: hipLaunchKernelGGL((attn_rowdot_fast_kernel<TX, TY, 3, 1>), grid, dim3(256), 0, st, p, L, cph); break;
            default: hipLaunchKernelGGL((attn_rowdot_fast_kernel<TX, TY, 4, 1>), grid, dim3(256), 0, st, p, L, cph); break;
            }
        } else {
            hipLaunchKernelGGL((attn_rowdot_kernel<TX, TY, 4>), dim3((unsigned)blocks), dim3(256), 0, st, p);
        }
    } else {
        hipLaunchKernelGGL((attn_rowdot_kernel<TX, TY, 1>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    }
    HETA_LAUNCH_CHECK("attn_rowdot_kernel");
    return HETA_OK;
}

heta_status launch_rowdot(const DotParams &p, heta_dtype x_dt, heta_dtype y_dt, hipStream_t st)
{
    if (x_dt == HETA_F32) return y_dt == HETA_F32 ? launch_rowdot_t<float, float>(p, st) : launch_rowdot_t<float, bf16_t>(p, st);
    return y_dt == HETA_F32 ? launch_rowdot_t<bf16_t, float>(p, st) : launch_rowdot_t<bf16_t, bf16_t>(p, st);
}

// ---- backward of the scores -------------------------------------------------------------------------
// dx[i, j] = beta dx[i, j] + sum_k ds[i, k] y_k[j]   (per_head: only k = j / F, y_k[j] = vec[j])
__global__ void __launch_bounds__(256) attn_score_bwd_input_kernel(const float *ds, const float *vec, int64_t n, int d,
                                                                   int K, int F, int per_head, float *dx, int64_t ld_dx,
                                                                   float beta)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / d;
    const int j = static_cast<int>(t % d);
    if (i >= n) return;
    float v = 0.f;
    if (per_head) {
        v = ds[i * K + j / F] * vec[j];
    } else {
        for (int k = 0; k < K; ++k) v = fmaf(ds[i * K + k], vec[static_cast<int64_t>(k) * d + j], v);
    }
    float *o = dx + i * ld_dx + j;
    *o = beta != 0.f ? *o + v : v;
}

// the same, four columns per thread (rows 16-byte aligned, heads a multiple of four columns wide)
__global__ void __launch_bounds__(256) attn_score_bwd_input_vec_kernel(const float *ds, const float *vec, int64_t n, int d,
                                                                       int K, int F, int per_head, float *dx,
                                                                       int64_t ld_dx, float beta)
{
    const int d4 = d / 4;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / d4;
    const int j = static_cast<int>(t - i * d4) * 4;
    if (i >= n) return;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (per_head) {
        const float s = ds[i * K + j / F];
        const float4 w = *reinterpret_cast<const float4 *>(vec + j);
        v = make_float4(s * w.x, s * w.y, s * w.z, s * w.w);
    } else {
        for (int k = 0; k < K; ++k) {
            const float s = ds[i * K + k];
            const float4 w = *reinterpret_cast<const float4 *>(vec + static_cast<int64_t>(k) * d + j);
            v.x = fmaf(s, w.x, v.x); v.y = fmaf(s, w.y, v.y); v.z = fmaf(s, w.z, v.z); v.w = fmaf(s, w.w, v.w);
        }
    }
    float4 *o = reinterpret_cast<float4 *>(dx + i * ld_dx + j);
    if (beta != 0.f) {
        const float4 old = *o;
        v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
    }
    *o = v;
}

// dvec_k[j] = sum_i ds[i, k] x[i, j]: stage 1, one workgroup per (slab of rows, 256 columns), partial sums
// to part[slab][k][j] (per_head: part[slab][j], only k = j / F); stage 2 adds the slabs in order.
constexpr int kSlabRows = 512;
template <typename T>
__global__ void __launch_bounds__(256) attn_score_bwd_param_kernel(const T *x, int64_t ld_x, const float *ds, int64_t n,
                                                                   int d, int K, int F, int per_head, float *part)
{
    const int j = blockIdx.y * 256 + threadIdx.x;
    const int64_t slab = blockIdx.x;
    const int64_t i0 = slab * kSlabRows, i1 = min(n, i0 + kSlabRows);
    if (j >= d) return;
    const int nk = per_head ? 1 : K;
    float acc[kMaxHeads];
#pragma unroll
    for (int k = 0; k < kMaxHeads; ++k) acc[k] = 0.f;
    const int kh = per_head ? j / F : 0;
    for (int64_t i = i0; i < i1; ++i) {
        const float xv = ld1(x + i * ld_x + j);
        if (per_head) {
            acc[0] = fmaf(ds[i * K + kh], xv, acc[0]);
        } else {
#pragma unroll
            for (int k = 0; k < kMaxHeads; ++k)
                if (k < K) acc[k] = fmaf(ds[i * K + k], xv, acc[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < kMaxHeads; ++k)
        if (k < nk) part[(slab * nk + k) * d + j] = acc[k];
}

// the same, four columns per lane and four row groups per workgroup (rows 16 / 8-byte aligned, heads a
// multiple of four columns wide); the row groups are added in order through LDS
// KH = 0: per head (one accumulator per column); KH > 0: every head uses the whole row, K <= KH accumulators per column
template <typename T, int KH>
__global__ void __launch_bounds__(256) attn_score_bwd_param_vec_kernel(const T *x, int64_t ld_x, const float *ds, int64_t n,
                                                                       int d, int K, int F, float *part)
{
    constexpr int NA = KH == 0 ? 1 : KH;
    __shared__ float4 red[4][64];
    const int lane = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int j = (blockIdx.y * 64 + lane) * 4;
    const int64_t slab = blockIdx.x;
    const int64_t i0 = slab * kSlabRows, i1 = min(n, i0 + kSlabRows);
    const bool live = j < d;
    const int nk = KH == 0 ? 1 : K;
    const int kh = KH == 0 && live ? j / F : 0;
    float acc[NA][4];
#pragma unroll
    for (int k = 0; k < NA; ++k) acc[k][0] = acc[k][1] = acc[k][2] = acc[k][3] = 0.f;
    if (live) {
        constexpr int U = KH > 4 ? 4 : 8; // rows in flight per row group
        for (int64_t ib = i0 + rg; ib < i1; ib += 4 * U) {
            float xv[U][4], sv[U][NA];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t i = ib + 4 * u;
                if (i < i1) {
                    ldv<T, 4>(x + i * ld_x + j, xv[u]);
                    if (KH == 0) {
                        sv[u][0] = ds[i * K + kh];
                    } else {
#pragma unroll
                        for (int k = 0; k < NA; ++k) sv[u][k] = k < K ? ds[i * K + k] : 0.f;
                    }
                } else {
                    xv[u][0] = xv[u][1] = xv[u][2] = xv[u][3] = 0.f;
#pragma unroll
                    for (int k = 0; k < NA; ++k) sv[u][k] = 0.f;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < NA; ++k)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[k][c] = fmaf(sv[u][k], xv[u][c], acc[k][c]);
        }
    }
#pragma unroll
    for (int k = 0; k < NA; ++k) {
        if (k < nk) { // uniform
            red[rg][lane] = make_float4(acc[k][0], acc[k][1], acc[k][2], acc[k][3]);
            __syncthreads();
            if (rg == 0 && live) {
                float4 a = red[0][lane];
#pragma unroll
                for (int r = 1; r < 4; ++r) {
                    const float4 b = red[r][lane];
                    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
                }
                *reinterpret_cast<float4 *>(part + (slab * nk + k) * d + j) = a;
            }
            __syncthreads();
        }
    }
}

// stage 2: out[t] = sum over slabs of part[slab][t].  One workgroup of 16 wavefronts per 64 elements:
// wavefront w adds slabs w, w + 16, ... (coalesced 256-byte reads), the sixteen partial sums are added in
// wavefront order through LDS.
__global__ void __launch_bounds__(1024) attn_slab_sum_kernel(const float *part, int64_t n_slabs, int64_t elems, float *out)
{
    __shared__ float red[16][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 64 + lane;
    float a = 0.f;
    if (t < elems) {
#pragma unroll 4
        for (int64_t s = w; s < n_slabs; s += 16) a += part[s * elems + t];
    }
    red[w][lane] = a;
    __syncthreads();
    if (w == 0 && t < elems) {
        float r = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) r += red[i][lane];
        out[t] = r;
    }
}


// ---- scores of several vector sets in one pass over the table -------------------------------------------
// A node type is the source of some relations and the destination of others, and every one of them takes
// a row score <x_i, vec_k> of the same table with vectors of its own (el with W_r a_r, er with q_r).  One
// pass serves them all: 32 lanes per row (two rows per wavefront), a lane owns four columns and keeps its
// four columns of all (set, head) vectors in registers, so a row costs one 16-byte load per lane, 4 FMAs
// per vector, and one reduce-scatter butterfly after which lane v holds score v.  Tables of at most 128
// columns, at most 32 vectors.  The backward runs the same way: dx[i, :] = sum_v dscore_v[i] vec_v (the
// 32 scalars of a row are broadcast by lane shuffles), dvec_v = sum_i dscore_v[i] x[i, :] through
// per-slab partial sums added in slab order.
constexpr int kMultiSets = 8, kMultiVecs = 32, kMultiCols = 128;
struct ScoreMulti {
    const float *vec[kMultiSets]; // [K][d] each
    float *score[kMultiSets];     // [n][K] each: written by the forward, read (dscore) by the backward
    float *dvec[kMultiSets];      // [K][d] each, or null
    int n_sets, K, NV;            // NV = n_sets * K
};

// pointer j of a table of kMultiSets pointers for a lane-dependent j (a select chain: indexing the kernel
// arguments by a vector register would move them to scratch memory)
__device__ __forceinline__ float *pick(float *const (&tab)[kMultiSets], int j)
{
    float *p = tab[0];
#pragma unroll
    for (int q = 1; q < kMultiSets; ++q) p = j == q ? tab[q] : p;
    return p;
}

template <typename T> __device__ __forceinline__ void load4(const T *p, float f[4]);
template <> __device__ __forceinline__ void load4<float>(const float *p, float f[4])
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t *p, float f[4])
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}

// this lane's four columns (4 l .. 4 l + 3) of the first NVC vectors; zero beyond d or beyond the NV vectors given
template <int NVC> __device__ __forceinline__ void load_vectors(const ScoreMulti &m, int d, int l, float v[NVC][4])
{
#pragma unroll
    for (int vi = 0; vi < NVC; ++vi) {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[vi][c] = 0.f;
        if (vi < m.NV && 4 * l < d) {
            const float4 q = *reinterpret_cast<const float4 *>(m.vec[vi / m.K] + static_cast<int64_t>(vi % m.K) * d + 4 * l);
            v[vi][0] = q.x; v[vi][1] = q.y; v[vi][2] = q.z; v[vi][3] = q.w;
        }
    }
}

// one step of the reduce-scatter over a row's 32 lanes: of its 2 CNT values a lane keeps the half its lane bit
// CNT selects and adds the partner lane's copy of that half (register indices are compile-time constants)
template <int CNT> __device__ __forceinline__ void reduce_scatter_step(float (&acc)[kMultiVecs], int l)
{
    const bool up = (l & CNT) != 0;
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
        const float send = up ? acc[i] : acc[i + CNT];
        const float keep = up ? acc[i + CNT] : acc[i];
        acc[i] = keep + __shfl_xor(send, CNT, 64);
    }
}

template <typename T, int NVC>
__global__ void __launch_bounds__(256) attn_score_multi_kernel(const T *x, int64_t ld_x, int64_t n, int d, ScoreMulti m)
{
    const int lane = threadIdx.x & 63, l = lane & 31, half = lane >> 5;
    float v[NVC][4];
    load_vectors<NVC>(m, d, l, v);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6), n_waves = static_cast<int64_t>(gridDim.x) * 4;
    for (int64_t r0 = wave * 2; r0 < n; r0 += n_waves * 2) { // uniform per wavefront
        const int64_t r = r0 + half;
        float xv[4] = {0.f, 0.f, 0.f, 0.f};
        if (r < n && 4 * l < d) load4<T>(x + r * ld_x + 4 * l, xv);
        float acc[kMultiVecs];
#pragma unroll
        for (int vi = 0; vi < kMultiVecs; ++vi)
            acc[vi] = vi < NVC ? (xv[0] * v[vi < NVC ? vi : 0][0] + xv[1] * v[vi < NVC ? vi : 0][1]) +
                                     (xv[2] * v[vi < NVC ? vi : 0][2] + xv[3] * v[vi < NVC ? vi : 0][3])
                               : 0.f;
        // reduce-scatter over the 32 lanes of the row: each step halves the values a lane keeps (the half its
        // lane bit selects) and adds the partner's; after five steps lane v holds the whole sum of value v
        reduce_scatter_step<16>(acc, l);
        reduce_scatter_step<8>(acc, l);
        reduce_scatter_step<4>(acc, l);
        reduce_scatter_step<2>(acc, l);
        reduce_scatter_step<1>(acc, l);
        if (r < n && l < m.NV) pick(m.score, l / m.K)[r * m.K + l % m.K] = acc[0];
    }
}

template <int NVC>
__global__ void __launch_bounds__(256) attn_score_bwd_multi_input_kernel(int64_t n, int d, ScoreMulti m, float *dx, int64_t ld_dx, float beta)
{
    const int lane = threadIdx.x & 63, l = lane & 31, half = lane >> 5;
    float v[NVC][4];
    load_vectors<NVC>(m, d, l, v);
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6), n_waves = static_cast<int64_t>(gridDim.x) * 4;
    for (int64_t r0 = wave * 2; r0 < n; r0 += n_waves * 2) {
        const int64_t r = r0 + half;
        float ds = 0.f;
        if (r < n && l < m.NV) ds = pick(m.score, l / m.K)[r * m.K + l % m.K];
        float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int vi = 0; vi < NVC; ++vi) {
            const float sv = __shfl(ds, (lane & 32) | vi, 64);
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = fmaf(sv, v[vi][c], o[c]);
        }
        if (r < n && 4 * l < d) {
            float4 *dst = reinterpret_cast<float4 *>(dx + r * ld_dx + 4 * l);
            float4 w4 = make_float4(o[0], o[1], o[2], o[3]);
            if (beta != 0.f) {
                const float4 old = *dst;
                w4.x += old.x; w4.y += old.y; w4.z += old.z; w4.w += old.w;
            }
            *dst = w4;
        }
    }
}

// part[slab][v][128]: the slab's sum over its rows of dscore_v[i] x[i, :]; the two rows a wavefront has in
// flight are added first (lane shuffle), then the four wavefronts in wavefront order through LDS
template <typename T, int NVC>
__global__ void __launch_bounds__(256) attn_score_bwd_multi_param_kernel(const T *x, int64_t ld_x, int64_t n, int d, ScoreMulti m, float *part)
{
    __shared__ float buf[NVC][kMultiCols];
    const int lane = threadIdx.x & 63, l = lane & 31, half = lane >> 5, w = threadIdx.x >> 6;
    const int64_t slab = blockIdx.x;
    const int64_t i0 = slab * kSlabRows, i1 = min(n, i0 + kSlabRows);
    float acc[NVC][4];
#pragma unroll
    for (int vi = 0; vi < NVC; ++vi)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[vi][c] = 0.f;
    for (int64_t r0 = i0 + 2 * w; r0 < i1; r0 += 8) {
        const int64_t r = r0 + half;
        float xv[4] = {0.f, 0.f, 0.f, 0.f}, ds = 0.f;
        if (r < i1 && 4 * l < d) load4<T>(x + r * ld_x + 4 * l, xv);
        if (r < i1 && l < m.NV) ds = pick(m.score, l / m.K)[r * m.K + l % m.K];
#pragma unroll
        for (int vi = 0; vi < NVC; ++vi) {
            const float sv = __shfl(ds, (lane & 32) | vi, 64);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[vi][c] = fmaf(sv, xv[c], acc[vi][c]);
        }
    }
#pragma unroll
    for (int vi = 0; vi < NVC; ++vi)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[vi][c] += __shfl_xor(acc[vi][c], 32, 64);
    for (int q = 0; q < 4; ++q) { // wavefront q adds its sums to the buffer, in order
        if (w == q && half == 0) {
#pragma unroll
            for (int vi = 0; vi < NVC; ++vi)
#pragma unroll
                for (int c = 0; c < 4; ++c) buf[vi][4 * l + c] = (q == 0 ? 0.f : buf[vi][4 * l + c]) + acc[vi][c];
        }
        __syncthreads();
    }
    float *o = part + slab * (NVC * kMultiCols);
    for (int t = threadIdx.x; t < NVC * kMultiCols; t += 256) o[t] = (&buf[0][0])[t];
}

// dvec_v[c] = sum over the slabs, in slab order per wavefront and wavefront order through LDS (as attn_slab_sum_kernel)
__global__ void __launch_bounds__(1024) attn_multi_slab_sum_kernel(const float *part, int64_t n_slabs, int nvc, int d, ScoreMulti m)
{
    __shared__ float red[16][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t elems = static_cast<int64_t>(nvc) * kMultiCols;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 64 + lane;
    float a = 0.f;
    if (t < elems) {
#pragma unroll 4
        for (int64_t s = w; s < n_slabs; s += 16) a += part[s * elems + t];
    }
    red[w][lane] = a;
    __syncthreads();
    const int vi = static_cast<int>(t / kMultiCols), c = static_cast<int>(t % kMultiCols);
    float *out = (t < elems && vi < m.NV) ? pick(m.dvec, vi / m.K) : nullptr;
    if (w == 0 && out && c < d) {
        float r = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) r += red[i][lane];
        out[static_cast<int64_t>(vi % m.K) * d + c] = r;
    }
}

// ---- the source score taken off the input table ------------------------------------------------------
// el[u, k] = <z_u[k, :], a[k, :]> with z_u = W^T h_u equals <h_u, wa[k, :]> with wa[k, j] = sum_f W[j, kF + f] a[k, f]:
// the scores then come from the (narrower, never rounded) input table instead of the stored projection.
// One thread per (k, j); the sum over f runs in order.
template <typename T>
__global__ void __launch_bounds__(256) attn_fold_kernel(const T *W, int64_t ld_w, int d_in, int K, int F, const float *a, float *wa)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= K * d_in) return;
    const int k = t / d_in, j = t - k * d_in;
    const T *w = W + static_cast<int64_t>(j) * ld_w + k * F;
    float acc = 0.f;
    for (int f = 0; f < F; ++f) acc = fmaf(ld1(w + f), a[k * F + f], acc);
    wa[t] = acc;
}

// Its backward: dW[j, kF + f] = beta dW[j, kF + f] + dwa[k, j] a[k, f]   (one thread per element of dW)
__global__ void __launch_bounds__(256) attn_fold_bwd_w_kernel(const float *dwa, const float *a, int d_in, int K, int F, float *dW,
                                                              int64_t ld_dw, float beta)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int d_out = K * F;
    if (t >= d_in * d_out) return;
    const int j = t / d_out, c = t - j * d_out;
    const float v = dwa[(c / F) * d_in + j] * a[c];
    float *o = dW + static_cast<int64_t>(j) * ld_dw + c;
    *o = beta != 0.f ? *o + v : v;
}

// da[k, f] = sum_j dwa[k, j] W[j, kF + f]: one wavefront per (k, f), lanes take j round-robin and are
// combined by a fixed butterfly, so the order of the sum is fixed.
template <typename T>
__global__ void __launch_bounds__(256) attn_fold_bwd_a_kernel(const float *dwa, const T *W, int64_t ld_w, int d_in, int K, int F, float *da)
{
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= K * F) return; // uniform per wavefront
    const int k = c / F;
    float acc = 0.f;
    for (int j = lane; j < d_in; j += 64) acc = fmaf(dwa[k * d_in + j], ld1(W + static_cast<int64_t>(j) * ld_w + c), acc);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) da[c] = acc;
}

heta_status ensure_attn(heta_graph *g, size_t bytes)
{
    bytes = std::max<size_t>(bytes, 256); // never hand out a null workspace (relations without edges)
    if (bytes <= g->attn_bytes) return HETA_OK;
    if (g->d_attn) HETA_HIP(hipFree(g->d_attn)); // waits for earlier users
    g->d_attn = nullptr;
    g->attn_bytes = 0;
    HETA_HIP(hipMalloc(&g->d_attn, bytes));
    g->attn_bytes = bytes;
    return HETA_OK;
}

inline size_t round256(size_t b) { return (b + 255) / 256 * 256; }

heta_status check_attn_args(const char *fn, heta_graph *g, int32_t rel, int32_t d, int32_t heads)
{
    if (!g) return fail(HETA_ERR_INVALID_ARG, "%s: null graph", fn);
    if (rel < 0 || rel >= (int32_t)g->rels.size()) return fail(HETA_ERR_INVALID_ARG, "%s: relation %d out of range", fn, rel);
    if (heads <= 0 || heads > kMaxHeads || d <= 0 || d % heads != 0)
        return fail(HETA_ERR_SHAPE, "%s: need 1 <= heads <= %d dividing d (d=%d heads=%d)", fn, kMaxHeads, d, heads);
    return HETA_OK;
}

} // namespace

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_attn_score(const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d, const float *vec,
                            int32_t heads, int32_t per_head, float *score, void *hip_stream)
{
    if (!vec || (n > 0 && (!x || !score))) return fail(HETA_ERR_INVALID_ARG, "heta_attn_score: null argument");
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "heta_attn_score: bad dtype");
    if (n < 0 || d <= 0 || ld_x < d || heads <= 0 || heads > kMaxHeads || (per_head && d % heads != 0))
        return fail(HETA_ERR_SHAPE, "heta_attn_score: bad shape (n=%lld d=%d ld=%lld heads=%d)", (long long)n, d,
                    (long long)ld_x, heads);
    if (reinterpret_cast<uintptr_t>(x) % dtype_size(dt) || reinterpret_cast<uintptr_t>(vec) % 4 || reinterpret_cast<uintptr_t>(score) % 4)
        return fail(HETA_ERR_INVALID_ARG, "heta_attn_score: pointer not aligned to its element size");
    DotParams p{};
    p.x = x;
    p.ld_x = ld_x;
    p.y = vec;
    p.ld_y = 0;
    p.n = n;
    p.d = d;
    p.K = heads;
    p.F = per_head ? d / heads : d;
    p.per_head = per_head ? 1 : 0;
    p.scale = 1.f;
    p.corr = nullptr;
    p.out = score;
    return launch_rowdot(p, dt, HETA_F32, as_stream(hip_stream));
}

heta_status heta_attn_score_bwd(heta_graph *g, const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d,
                                const float *vec, int32_t heads, int32_t per_head, const float *dscore, float *dx,
                                int64_t ld_dx, float beta, float *dvec, void *hip_stream)
{
    if (!g || !vec || (n > 0 && (!x || !dscore))) return fail(HETA_ERR_INVALID_ARG, "heta_attn_score_bwd: null argument");
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "heta_attn_score_bwd: bad dtype");
    if (n < 0 || d <= 0 || ld_x < d || heads <= 0 || heads > kMaxHeads || (per_head && d % heads != 0) || (dx && ld_dx < d))
        return fail(HETA_ERR_SHAPE, "heta_attn_score_bwd: bad shape (n=%lld d=%d heads=%d)", (long long)n, d, heads);
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "heta_attn_score_bwd: beta must be 0 or 1");
    hipStream_t st = as_stream(hip_stream);
    const int F = per_head ? d / heads : d;
    if (dx && n > 0) {
        const int64_t threads = n * d;
        const int64_t blocks = (threads + 255) / 256;
        if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "heta_attn_score_bwd: too many elements");
        ProfScope prof("attn_score_bwd_input_kernel", st, static_cast<double>(n) * (d * (beta != 0.f ? 8.0 : 4.0) + 4.0 * heads), 0);
        const bool vec4 = d % 4 == 0 && F % 4 == 0 && ld_dx % 4 == 0 && aligned16(dx) && aligned16(vec);
        if (vec4)
            hipLaunchKernelGGL(attn_score_bwd_input_vec_kernel, dim3((unsigned)((threads / 4 + 255) / 256)), dim3(256), 0, st,
                               dscore, vec, n, (int)d, (int)heads, F, per_head ? 1 : 0, dx, ld_dx, beta);
        else
            hipLaunchKernelGGL(attn_score_bwd_input_kernel, dim3((unsigned)blocks), dim3(256), 0, st, dscore, vec, n, (int)d,
                               (int)heads, F, per_head ? 1 : 0, dx, ld_dx, beta);
        HETA_LAUNCH_CHECK("attn_score_bwd_input_kernel");
    }
    if (dvec) {
        const int nk = per_head ? 1 : heads;
        const int64_t elems = static_cast<int64_t>(nk) * d;
        const int64_t n_slabs = (n + kSlabRows - 1) / kSlabRows;
        if (n_slabs == 0) {
            HETA_HIP(hipMemsetAsync(dvec, 0, elems * sizeof(float), st));
            return HETA_OK;
        }
        heta_status e = ensure_attn(g, static_cast<size_t>(n_slabs) * elems * sizeof(float));
        if (e != HETA_OK) return e;
        float *part = static_cast<float *>(g->d_attn);
        {
            ProfScope prof("attn_score_bwd_param_kernel", st, static_cast<double>(n) * (d * dtype_size(dt) + 4.0 * heads), 0);
            const dim3 grid((unsigned)n_slabs, (d + 255) / 256);
            const bool vec4 = d % 4 == 0 && F % 4 == 0 && ld_x % 4 == 0 && reinterpret_cast<uintptr_t>(x) % (4 * dtype_size(dt)) == 0;
            if (vec4) {
#define HETA_PARAM_VEC(TT, KH)                                                                                          \
    hipLaunchKernelGGL((attn_score_bwd_param_vec_kernel<TT, KH>), grid, dim3(256), 0, st, static_cast<const TT *>(x), ld_x, \
                       dscore, n, (int)d, (int)heads, F, part)
                if (dt == HETA_F32) {
                    if (per_head) HETA_PARAM_VEC(float, 0);
                    else if (heads <= 4) HETA_PARAM_VEC(float, 4);
                    else HETA_PARAM_VEC(float, 16);
                } else {
                    if (per_head) HETA_PARAM_VEC(bf16_t, 0);
                    else if (heads <= 4) HETA_PARAM_VEC(bf16_t, 4);
                    else HETA_PARAM_VEC(bf16_t, 16);
                }
#undef HETA_PARAM_VEC
            } else if (dt == HETA_F32) {
                hipLaunchKernelGGL((attn_score_bwd_param_kernel<float>), grid, dim3(256), 0, st, static_cast<const float *>(x), ld_x,
                                   dscore, n, (int)d, (int)heads, F, per_head ? 1 : 0, part);
            } else {
                hipLaunchKernelGGL((attn_score_bwd_param_kernel<bf16_t>), grid, dim3(256), 0, st, static_cast<const bf16_t *>(x), ld_x,
                                   dscore, n, (int)d, (int)heads, F, per_head ? 1 : 0, part);
            }
            HETA_LAUNCH_CHECK("attn_score_bwd_param_kernel");
            hipLaunchKernelGGL(attn_slab_sum_kernel, dim3((unsigned)((elems + 63) / 64)), dim3(1024), 0, st, part, n_slabs, elems, dvec);
            HETA_LAUNCH_CHECK("attn_slab_sum_kernel");
        }
    }
    return HETA_OK;
}

// whether the one-pass kernels take this table and these vector sets
static bool multi_ok(const void *x, heta_dtype dt, int64_t ld_x, int32_t d, int32_t n_sets, int32_t heads, const float *const *vecs)
{
    if (d > kMultiCols || d % 4 || n_sets > kMultiSets || n_sets * heads > kMultiVecs) return false;
    if (reinterpret_cast<uintptr_t>(x) % (4 * dtype_size(dt)) || ld_x % 4) return false;
    for (int j = 0; j < n_sets; ++j)
        if (!aligned16(vecs[j])) return false;
    return true;
}

heta_status heta_attn_score_multi(const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d, int32_t n_sets,
                                  const float *const *vecs, int32_t heads, float *const *scores, void *hip_stream)
{
    const char *who = "heta_attn_score_multi";
    if (n_sets < 0 || (n_sets > 0 && (!vecs || !scores))) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n_sets == 0) return HETA_OK;
    for (int j = 0; j < n_sets; ++j)
        if (!vecs[j] || (n > 0 && !scores[j])) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n > 0 && !x) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (n < 0 || d <= 0 || ld_x < d || heads <= 0 || heads > kMaxHeads)
        return fail(HETA_ERR_SHAPE, "%s: bad shape (n=%lld d=%d ld=%lld heads=%d)", who, (long long)n, d, (long long)ld_x, heads);
    hipStream_t st = as_stream(hip_stream);
    if (!multi_ok(x, dt, ld_x, d, n_sets, heads, vecs)) { // shapes the one-pass kernel does not take: set by set
        for (int j = 0; j < n_sets; ++j) {
            heta_status e = heta_attn_score(x, dt, ld_x, n, d, vecs[j], heads, 0, scores[j], hip_stream);
            if (e != HETA_OK) return e;
        }
        return HETA_OK;
    }
    if (n == 0) return HETA_OK;
    ScoreMulti m{};
    m.n_sets = n_sets;
    m.K = heads;
    m.NV = n_sets * heads;
    for (int j = 0; j < n_sets; ++j) {
        m.vec[j] = vecs[j];
        m.score[j] = scores[j];
    }
    const int64_t blocks = std::min<int64_t>((n + 7) / 8, 256 * 8);
    ProfScope prof("attn_score_multi_kernel", st, static_cast<double>(n) * (d * dtype_size(dt) + 4.0 * m.NV), 0);
#define HETA_SM(TT, NVC) hipLaunchKernelGGL((attn_score_multi_kernel<TT, NVC>), dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const TT *>(x), ld_x, n, (int)d, m)
#define HETA_SM_T(TT) do { if (m.NV <= 8) HETA_SM(TT, 8); else if (m.NV <= 16) HETA_SM(TT, 16); else if (m.NV <= 24) HETA_SM(TT, 24); else HETA_SM(TT, 32); } while (0)
    if (dt == HETA_F32) HETA_SM_T(float);
    else HETA_SM_T(bf16_t);
#undef HETA_SM_T
#undef HETA_SM
    HETA_LAUNCH_CHECK("attn_score_multi_kernel");
    return HETA_OK;
}

heta_status heta_attn_score_bwd_multi(heta_graph *g, const void *x, heta_dtype dt, int64_t ld_x, int64_t n, int32_t d,
                                      int32_t n_sets, const float *const *vecs, int32_t heads, const float *const *dscores,
                                      float *dx, int64_t ld_dx, float beta, float *const *dvecs, void *hip_stream)
{
    const char *who = "heta_attn_score_bwd_multi";
    if (!g || n_sets < 0 || (n_sets > 0 && (!vecs || !dscores))) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n_sets == 0) return HETA_OK;
    for (int j = 0; j < n_sets; ++j)
        if (!vecs[j] || (n > 0 && !dscores[j])) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n > 0 && !x) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (n < 0 || d <= 0 || ld_x < d || heads <= 0 || heads > kMaxHeads || (dx && ld_dx < d))
        return fail(HETA_ERR_SHAPE, "%s: bad shape (n=%lld d=%d heads=%d)", who, (long long)n, d, heads);
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "%s: beta must be 0 or 1", who);
    hipStream_t st = as_stream(hip_stream);
    const bool dx_ok = !dx || (aligned16(dx) && ld_dx % 4 == 0);
    if (!multi_ok(x, dt, ld_x, d, n_sets, heads, vecs) || !dx_ok) { // set by set, accumulating into dx
        for (int j = 0; j < n_sets; ++j) {
            heta_status e = heta_attn_score_bwd(g, x, dt, ld_x, n, d, vecs[j], heads, 0, dscores[j], dx, ld_dx,
                                                j == 0 ? beta : 1.f, dvecs ? dvecs[j] : nullptr, hip_stream);
            if (e != HETA_OK) return e;
        }
        return HETA_OK;
    }
    ScoreMulti m{};
    m.n_sets = n_sets;
    m.K = heads;
    m.NV = n_sets * heads;
    bool any_dvec = false;
    for (int j = 0; j < n_sets; ++j) {
        m.vec[j] = vecs[j];
        m.score[j] = const_cast<float *>(dscores[j]);
        m.dvec[j] = dvecs ? dvecs[j] : nullptr;
        any_dvec = any_dvec || m.dvec[j];
    }
    const int nvc = m.NV <= 8 ? 8 : m.NV <= 16 ? 16 : m.NV <= 24 ? 24 : 32;
    if (dx && n > 0) {
        const int64_t blocks = std::min<int64_t>((n + 7) / 8, 256 * 8);
        ProfScope prof("attn_score_bwd_input_kernel", st, static_cast<double>(n) * (d * (beta != 0.f ? 8.0 : 4.0) + 4.0 * m.NV), 0);
#define HETA_SI(NVC) hipLaunchKernelGGL((attn_score_bwd_multi_input_kernel<NVC>), dim3((unsigned)blocks), dim3(256), 0, st, n, (int)d, m, dx, ld_dx, beta)
        if (nvc == 8) HETA_SI(8); else if (nvc == 16) HETA_SI(16); else if (nvc == 24) HETA_SI(24); else HETA_SI(32);
#undef HETA_SI
        HETA_LAUNCH_CHECK("attn_score_bwd_multi_input_kernel");
    }
    if (any_dvec) {
        const int64_t n_slabs = (n + kSlabRows - 1) / kSlabRows;
        if (n_slabs == 0) {
            for (int j = 0; j < n_sets; ++j)
                if (m.dvec[j]) HETA_HIP(hipMemsetAsync(m.dvec[j], 0, static_cast<size_t>(heads) * d * sizeof(float), st));
            return HETA_OK;
        }
        if (n_slabs > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "%s: too many rows", who);
        heta_status e = ensure_attn(g, static_cast<size_t>(n_slabs) * nvc * kMultiCols * sizeof(float));
        if (e != HETA_OK) return e;
        float *part = static_cast<float *>(g->d_attn);
        ProfScope prof("attn_score_bwd_param_kernel", st, static_cast<double>(n) * (d * dtype_size(dt) + 4.0 * m.NV), 0);
#define HETA_SP(TT, NVC) hipLaunchKernelGGL((attn_score_bwd_multi_param_kernel<TT, NVC>), dim3((unsigned)n_slabs), dim3(256), 0, st, static_cast<const TT *>(x), ld_x, n, (int)d, m, part)
#define HETA_SP_T(TT) do { if (nvc == 8) HETA_SP(TT, 8); else if (nvc == 16) HETA_SP(TT, 16); else if (nvc == 24) HETA_SP(TT, 24); else HETA_SP(TT, 32); } while (0)
        if (dt == HETA_F32) HETA_SP_T(float);
        else HETA_SP_T(bf16_t);
#undef HETA_SP_T
#undef HETA_SP
        HETA_LAUNCH_CHECK("attn_score_bwd_multi_param_kernel");
        const int64_t elems = static_cast<int64_t>(nvc) * kMultiCols;
        hipLaunchKernelGGL(attn_multi_slab_sum_kernel, dim3((unsigned)((elems + 63) / 64)), dim3(1024), 0, st, part, n_slabs, nvc, (int)d, m);
        HETA_LAUNCH_CHECK("attn_multi_slab_sum_kernel");
    }
    return HETA_OK;
}

heta_status heta_attn_fold(const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_in, int32_t d_out, const float *a,
                           int32_t heads, float *wa, void *hip_stream)
{
    if (!W || !a || !wa) return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold: null argument");
    if (!valid_dtype(w_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold: bad dtype");
    if (d_in <= 0 || d_out <= 0 || ld_w < d_out || heads <= 0 || heads > kMaxHeads || d_out % heads != 0 ||
        static_cast<int64_t>(d_in) * d_out > (int64_t(1) << 30))
        return fail(HETA_ERR_SHAPE, "heta_attn_fold: bad shape (d_in=%d d_out=%d ld_w=%lld heads=%d)", d_in, d_out,
                    (long long)ld_w, heads);
    if (reinterpret_cast<uintptr_t>(W) % dtype_size(w_dt) || reinterpret_cast<uintptr_t>(a) % 4 || reinterpret_cast<uintptr_t>(wa) % 4)
        return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold: pointer not aligned to its element size");
    hipStream_t st = as_stream(hip_stream);
    const int F = d_out / heads;
    const unsigned blocks = static_cast<unsigned>((heads * d_in + 255) / 256);
    if (w_dt == HETA_F32)
        hipLaunchKernelGGL(attn_fold_kernel<float>, dim3(blocks), dim3(256), 0, st, static_cast<const float *>(W), ld_w, (int)d_in,
                           (int)heads, F, a, wa);
    else
        hipLaunchKernelGGL(attn_fold_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, static_cast<const bf16_t *>(W), ld_w, (int)d_in,
                           (int)heads, F, a, wa);
    HETA_LAUNCH_CHECK("attn_fold_kernel");
    return HETA_OK;
}

heta_status heta_attn_fold_bwd(const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_in, int32_t d_out, const float *a,
                               int32_t heads, const float *dwa, float *dW, int64_t ld_dw, float beta, float *da,
                               void *hip_stream)
{
    if (!W || !a || !dwa) return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold_bwd: null argument");
    if (!valid_dtype(w_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold_bwd: bad dtype");
    if (d_in <= 0 || d_out <= 0 || ld_w < d_out || heads <= 0 || heads > kMaxHeads || d_out % heads != 0 || (dW && ld_dw < d_out) ||
        static_cast<int64_t>(d_in) * d_out > (int64_t(1) << 30))
        return fail(HETA_ERR_SHAPE, "heta_attn_fold_bwd: bad shape (d_in=%d d_out=%d heads=%d)", d_in, d_out, heads);
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "heta_attn_fold_bwd: beta must be 0 or 1");
    if (reinterpret_cast<uintptr_t>(W) % dtype_size(w_dt) || reinterpret_cast<uintptr_t>(a) % 4 ||
        reinterpret_cast<uintptr_t>(dwa) % 4 || reinterpret_cast<uintptr_t>(dW) % 4 || reinterpret_cast<uintptr_t>(da) % 4)
        return fail(HETA_ERR_INVALID_ARG, "heta_attn_fold_bwd: pointer not aligned to its element size");
    hipStream_t st = as_stream(hip_stream);
    const int F = d_out / heads;
    if (dW) {
        const unsigned blocks = static_cast<unsigned>((static_cast<int64_t>(d_in) * d_out + 255) / 256);
        hipLaunchKernelGGL(attn_fold_bwd_w_kernel, dim3(blocks), dim3(256), 0, st, dwa, a, (int)d_in, (int)heads, F, dW, ld_dw, beta);
        HETA_LAUNCH_CHECK("attn_fold_bwd_w_kernel");
    }
    if (da) {
        const unsigned blocks = static_cast<unsigned>((d_out + 3) / 4);
        if (w_dt == HETA_F32)
            hipLaunchKernelGGL(attn_fold_bwd_a_kernel<float>, dim3(blocks), dim3(256), 0, st, dwa, static_cast<const float *>(W), ld_w,
                               (int)d_in, (int)heads, F, da);
        else
            hipLaunchKernelGGL(attn_fold_bwd_a_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, dwa, static_cast<const bf16_t *>(W), ld_w,
                               (int)d_in, (int)heads, F, da);
        HETA_LAUNCH_CHECK("attn_fold_bwd_a_kernel");
    }
    return HETA_OK;
}

heta_status heta_rel_attn_fwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, void *out,
                              heta_dtype out_dt, int64_t ld_out, float beta, float *smax, float *sinv, void *out_pos,
                              int64_t ld_pos, void *hip_stream)
{
    heta_status e = check_attn_args("heta_rel_attn_fwd", g, rel, d, heads);
    if (e != HETA_OK) return e;
    if (!z || !el || !er || !out || ((smax == nullptr) != (sinv == nullptr)))
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: null argument (smax and sinv go together)");
    if (!valid_dtype(z_dt) || !valid_dtype(out_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: bad dtype");
    if (ld_z < d || ld_out < d || (out_pos && ld_pos < d)) return fail(HETA_ERR_SHAPE, "heta_rel_attn_fwd: need d <= ld");
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "heta_rel_attn_fwd: beta must be 0 or 1");
    if (out_pos && beta != 0.f) return fail(HETA_ERR_SHAPE, "heta_rel_attn_fwd: out_pos needs beta = 0");
    if (reinterpret_cast<uintptr_t>(z) % dtype_size(z_dt) || reinterpret_cast<uintptr_t>(out) % dtype_size(out_dt) ||
        reinterpret_cast<uintptr_t>(out_pos) % dtype_size(out_dt))
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: pointer not aligned to its element size");
    const Relation &r = g->rels[rel];
    hipStream_t st = as_stream(hip_stream);
    const size_t a_bytes = std::max<size_t>(256, round256(static_cast<size_t>(r.n_edges) * heads * sizeof(float)));
    e = ensure_attn(g, (out_pos ? 2 : 1) * a_bytes + hub_scratch_bytes(r.csr, heads));
    if (e != HETA_OK) return e;
    char *base = static_cast<char *>(g->d_attn);
    float *alpha = reinterpret_cast<float *>(base);
    float *alpha_pos = out_pos ? reinterpret_cast<float *>(base + a_bytes) : nullptr;
    float *hub_scratch = reinterpret_cast<float *>(base + (out_pos ? 2 : 1) * a_bytes);
    SweepParams sp{};
    sp.K = heads;
    sp.slope = slope;
    sp.row_a = er;
    sp.nbr_a = el;
    sp.smax = smax;
    sp.sinv = sinv;
    sp.alpha = alpha;
    sp.gate = alpha_pos;
    e = launch_sweeps<SWEEP_FWD>(r.csr, sp, hub_scratch, st, "attn_sweep_fwd");
    if (e != HETA_OK) return e;
    return aggregate_slot_weighted(g, r.csr, z, z_dt, ld_z, d, alpha, heads, out, out_dt, ld_out, beta, st, alpha_pos, out_pos,
                                   ld_pos);
}

heta_status heta_rel_attn_bwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, const float *smax,
                              const float *sinv, const void *o, const void *o_pos, heta_dtype o_dt, int64_t ld_o,
                              const float *grad_out, int64_t ld_go, float *dz, int64_t ld_dz, float *del, float *der,
                              void *hip_stream)
{
    heta_status e = check_attn_args("heta_rel_attn_bwd", g, rel, d, heads);
    if (e != HETA_OK) return e;
    if (!z || !el || !er || !smax || !sinv || !o || !grad_out || !dz || !del || !der)
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: null argument");
    if (!valid_dtype(z_dt) || !valid_dtype(o_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: bad dtype");
    if (ld_z < d || ld_o < d || ld_go < d || ld_dz < d) return fail(HETA_ERR_SHAPE, "heta_rel_attn_bwd: need d <= ld");
    if (reinterpret_cast<uintptr_t>(z) % dtype_size(z_dt) || reinterpret_cast<uintptr_t>(o) % dtype_size(o_dt) ||
        reinterpret_cast<uintptr_t>(o_pos) % dtype_size(o_dt) || reinterpret_cast<uintptr_t>(grad_out) % 4 ||
        reinterpret_cast<uintptr_t>(dz) % 4)
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: pointer not aligned to its element size");
    const Relation &r = g->rels[rel];
    hipStream_t st = as_stream(hip_stream);
    const int K = heads;
    // workspace: two per-slot weight arrays, per-row terms, and one [max rows x d] fp32 intermediate
    const size_t w_bytes = std::max<size_t>(256, round256(static_cast<size_t>(r.n_edges) * K * sizeof(float)));
    const size_t dst_bytes = round256(static_cast<size_t>(r.n_dst) * K * sizeof(float));
    const size_t src_bytes = round256(static_cast<size_t>(r.n_src) * K * sizeof(float));
    const int64_t ld_r = (static_cast<int64_t>(d) + 3) / 4 * 4;
    const size_t r_bytes = round256(static_cast<size_t>(o_pos ? r.n_src : std::max(r.n_dst, r.n_src)) * ld_r * sizeof(float));
    const size_t hub_bytes = round256(std::max(hub_scratch_bytes(r.csr, K), hub_scratch_bytes(r.csc, K)));
    const size_t pack_bytes = 4 * dst_bytes;
    e = ensure_attn(g, 2 * w_bytes + 2 * dst_bytes + src_bytes + r_bytes + hub_bytes + pack_bytes);
    if (e != HETA_OK) return e;
    char *base = static_cast<char *>(g->d_attn);
    float *w_alpha = reinterpret_cast<float *>(base);
    float *w_gate = reinterpret_cast<float *>(base + w_bytes);
    float *dot = reinterpret_cast<float *>(base + 2 * w_bytes);
    float *corr_d = reinterpret_cast<float *>(base + 2 * w_bytes + dst_bytes);
    float *corr_s = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes);
    float *R = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes + src_bytes);
    float *hub_scratch = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes + src_bytes + r_bytes);
    float *nbr_pack = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes + src_bytes + r_bytes + hub_bytes);

    // dot[v, k] = <g[v, k, :], o[v, k, :]>
    DotParams dp{};
    dp.x = grad_out;
    dp.ld_x = ld_go;
    dp.y = o;
    dp.ld_y = ld_o;
    dp.n = r.n_dst;
    dp.d = d;
    dp.K = K;
    dp.F = d / K;
    dp.per_head = 1;
    dp.scale = 1.f;
    dp.corr = nullptr;
    dp.out = dot;
    if (o_pos) { // <g, o_pos> in the same pass over g; der = (1 - slope) <g, o_pos> - corr_d is finished after the sweep
        dp.y2 = o_pos;
        dp.scale2 = 1.f - slope;
        dp.out2 = der;
    }
    e = launch_rowdot(dp, HETA_F32, o_dt, st);
    if (e != HETA_OK) return e;
    dp.y2 = nullptr;

    // Destination side: der = sum_e gate_e <g, z[u_e]> - dot * sum_e gate_e, gate_e = alpha_e * LeakyReLU'.
    SweepParams sp{};
    sp.K = K;
    sp.slope = slope;
    sp.row_a = er;
    sp.nbr_a = el;
    sp.smax = const_cast<float *>(smax);
    sp.sinv = const_cast<float *>(sinv);
    sp.dot = dot;
    sp.corr = corr_d;
    if (o_pos) {
        // gate_e = alpha_e (slope + (1 - slope) [logit_e > 0]), so with o_pos = sum over positive-logit edges of
        // alpha_e z[u_e] (saved by the forward): sum_e gate_e <g, z[u_e]> = slope * dot + (1 - slope) <g, o_pos>,
        // and no feature row is gathered on this side.
        sp.gate = nullptr;
        sp.dot_shift = slope;
        e = launch_sweeps<SWEEP_BWD_CSR>(r.csr, sp, hub_scratch, st, "attn_sweep_bwd_dst");
        if (e != HETA_OK) return e;
        const int64_t total = r.n_dst * K;
        if (total > 0) {
            hipLaunchKernelGGL(attn_sub_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, der, corr_d, total);
            HETA_LAUNCH_CHECK("attn_sub_kernel");
        }
    } else {
        // without it: R[v] = sum_e gate_e z[u_e] by one more weighted aggregation over the CSR
        sp.gate = w_gate;
        sp.dot_shift = 0.f;
        e = launch_sweeps<SWEEP_BWD_CSR>(r.csr, sp, hub_scratch, st, "attn_sweep_bwd_dst");
        if (e != HETA_OK) return e;
        e = aggregate_slot_weighted(g, r.csr, z, z_dt, ld_z, d, w_gate, K, R, HETA_F32, ld_r, 0.f, st);
        if (e != HETA_OK) return e;
        dp.y = R;
        dp.ld_y = ld_r;
        dp.corr = corr_d;
        dp.out = der;
        e = launch_rowdot(dp, HETA_F32, HETA_F32, st);
        if (e != HETA_OK) return e;
    }

    // Source side: alpha and gate per CSC slot; one pass over the gathered gradient rows gives both
    // dz[u] = sum_e alpha_e g[v_e] and R[u] = sum_e gate_e g[v_e]; del = <z, R> - sum_e gate_e dot[v_e].
    if (r.n_dst > 0) {
        const int64_t total = r.n_dst * K;
        hipLaunchKernelGGL(attn_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, er, smax, sinv, dot, r.n_dst, K,
                           nbr_pack);
        HETA_LAUNCH_CHECK("attn_pack_kernel");
    }
    sp.row_a = el;
    sp.nbr_a = er;
    sp.nbr_pack = nbr_pack;
    sp.alpha = w_alpha;
    sp.gate = w_gate;
    sp.corr = corr_s;
    e = launch_sweeps<SWEEP_BWD_CSC>(r.csc, sp, hub_scratch, st, "attn_sweep_bwd_src");
    if (e != HETA_OK) return e;
    // del = <z, R> - corr_s is taken inside the aggregation when the shapes allow it (R is then never written)
    const SecondSumDot zr{z, z_dt, ld_z, corr_s, del};
    bool dot_done = false;
    e = aggregate_slot_weighted(g, r.csc, grad_out, HETA_F32, ld_go, d, w_alpha, K, dz, HETA_F32, ld_dz, 0.f, st, w_gate, R, ld_r,
                                &zr, &dot_done);
    if (e != HETA_OK) return e;
    if (dot_done) return HETA_OK;
    dp.x = z;
    dp.ld_x = ld_z;
    dp.y = R;
    dp.ld_y = ld_r;
    dp.n = r.n_src;
    dp.scale = 1.f;
    dp.corr = corr_s;
    dp.out = del;
    return launch_rowdot(dp, z_dt, HETA_F32, st);
}

} // extern "C"
