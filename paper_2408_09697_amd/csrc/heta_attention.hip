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

// ---- reductions over the W lanes that share one (row, head) -------------------------------------------
template <int W> struct Group;
template <> struct Group<1> {
    static __device__ __forceinline__ float sum(float v, float *) { return v; }
    static __device__ __forceinline__ float max(float v, float *) { return v; }
};
template <> struct Group<64> {
    static __device__ __forceinline__ float sum(float v, float *)
    {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        return v;
    }
    static __device__ __forceinline__ float max(float v, float *)
    {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
        return v;
    }
};
template <> struct Group<1024> { // one workgroup of 16 wavefronts; lds holds 16 floats
    static __device__ __forceinline__ float sum(float v, float *lds)
    {
        v = Group<64>::sum(v, nullptr);
        __syncthreads(); // previous use of lds is over
        if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
        __syncthreads();
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) t += lds[i];
        return t;
    }
    static __device__ __forceinline__ float max(float v, float *lds)
    {
        v = Group<64>::max(v, nullptr);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
        __syncthreads();
        float t = lds[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) t = fmaxf(t, lds[i]);
        return t;
    }
};

// ---- row sweeps ------------------------------------------------------------------------------------------
enum SweepOp { SWEEP_FWD = 0, SWEEP_BWD_CSR = 1, SWEEP_BWD_CSC = 2 };

struct SweepParams {
    const int64_t *sptr;
    const int32_t *sidx;
    const int32_t *perm;
    int64_t q0, q1;       // schedule positions of this launch
    int K;
    float slope;
    const float *row_a;   // [rows][K]  score half of the row side (er for the CSR, el for the CSC)
    const float *nbr_a;   // [nbrs][K]  score half of the neighbour side
    float *smax, *sinv;   // [dst][K]   softmax shift and 1/denominator: written by FWD, read by the others
    const float *dot;     // [dst][K]   <g, o> per head (backward)
    float *alpha;         // [E][K] by edge slot (FWD, BWD_CSC)
    float *gate;          // [E][K] by edge slot (BWD_*)
    float *corr;          // [rows][K]  the scalar term subtracted from the row's score gradient (BWD_*)
};

template <int W, int OP>
__global__ void __launch_bounds__(W == 1 ? 256 : (W == 64 ? 256 : 1024)) attn_sweep_kernel(SweepParams p)
{
    __shared__ float lds[16];
    int64_t q;
    int lane;
    if (W == 1) {
        q = p.q0 + static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
        lane = 0;
    } else if (W == 64) {
        q = p.q0 + static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
        lane = threadIdx.x & 63;
    } else {
        q = p.q0 + blockIdx.x;
        lane = threadIdx.x;
    }
    if (q >= p.q1) return; // uniform over the W lanes of a group (and over the workgroup when W = 1024)
    const int k = blockIdx.y;
    const int K = p.K;
    const int64_t row = p.perm[q];
    const int64_t e0 = p.sptr[q], e1 = p.sptr[q + 1];
    const float ar = p.row_a[row * K + k];
    if (OP == SWEEP_FWD) {
        float m = -INFINITY;
        for (int64_t e = e0 + lane; e < e1; e += W)
            m = fmaxf(m, lrelu(p.nbr_a[static_cast<int64_t>(p.sidx[e]) * K + k] + ar, p.slope));
        m = Group<W>::max(m, lds);
        float den = 0.f;
        for (int64_t e = e0 + lane; e < e1; e += W)
            den += expf(lrelu(p.nbr_a[static_cast<int64_t>(p.sidx[e]) * K + k] + ar, p.slope) - m);
        den = Group<W>::sum(den, lds);
        const bool empty = e1 == e0;
        const float inv = empty ? 0.f : 1.f / den;
        if (empty) m = 0.f;
        for (int64_t e = e0 + lane; e < e1; e += W)
            p.alpha[e * K + k] = expf(lrelu(p.nbr_a[static_cast<int64_t>(p.sidx[e]) * K + k] + ar, p.slope) - m) * inv;
        if (lane == 0 && p.smax) {
            p.smax[row * K + k] = m;
            p.sinv[row * K + k] = inv;
        }
    } else if (OP == SWEEP_BWD_CSR) {
        const float m = p.smax[row * K + k], inv = p.sinv[row * K + k];
        float gs = 0.f;
        for (int64_t e = e0 + lane; e < e1; e += W) {
            const float x = p.nbr_a[static_cast<int64_t>(p.sidx[e]) * K + k] + ar;
            const float gt = expf(lrelu(x, p.slope) - m) * inv * (x > 0.f ? 1.f : p.slope);
            p.gate[e * K + k] = gt;
            gs += gt;
        }
        gs = Group<W>::sum(gs, lds);
        if (lane == 0) p.corr[row * K + k] = p.dot[row * K + k] * gs;
    } else {
        float c = 0.f;
        for (int64_t e = e0 + lane; e < e1; e += W) {
            const int64_t v = p.sidx[e];
            const float x = p.nbr_a[v * K + k] + ar;
            const float a = expf(lrelu(x, p.slope) - p.smax[v * K + k]) * p.sinv[v * K + k];
            const float gt = a * (x > 0.f ? 1.f : p.slope);
            p.alpha[e * K + k] = a;
            p.gate[e * K + k] = gt;
            c += gt * p.dot[v * K + k];
        }
        c = Group<W>::sum(c, lds);
        if (lane == 0) p.corr[row * K + k] = c;
    }
}

template <int OP>
heta_status launch_sweeps(const Schedule &s, SweepParams p, hipStream_t st, const char *name)
{
    if (s.n_rows == 0) return HETA_OK;
    p.sptr = s.d_sptr;
    p.sidx = s.d_sidx;
    p.perm = s.d_perm;
    const int64_t n_long_or_hub = s.rows_with_deg_ge[kShortDegAttn];
    // Algorithmic bytes: per edge and head one 4-byte score of the neighbour and the weights written;
    // per edge one 4-byte id; per row its offsets and per-head terms.
    const double per_edge = 4.0 + p.K * (OP == SWEEP_FWD ? 8.0 : (OP == SWEEP_BWD_CSR ? 8.0 : 24.0));
    ProfScope prof(name, st, per_edge * static_cast<double>(s.n_edges) + static_cast<double>(s.n_rows) * (12.0 + 12.0 * p.K), 0);
    if (s.n_hub_rows > 0) {
        p.q0 = 0;
        p.q1 = s.n_hub_rows;
        hipLaunchKernelGGL((attn_sweep_kernel<1024, OP>), dim3((unsigned)s.n_hub_rows, p.K), dim3(1024), 0, st, p);
        HETA_LAUNCH_CHECK("attn_sweep_kernel");
    }
    if (n_long_or_hub > s.n_hub_rows) {
        p.q0 = s.n_hub_rows;
        p.q1 = n_long_or_hub;
        const int64_t blocks = (p.q1 - p.q0 + 3) / 4;
        hipLaunchKernelGGL((attn_sweep_kernel<64, OP>), dim3((unsigned)blocks, p.K), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_sweep_kernel");
    }
    if (s.n_rows > n_long_or_hub) {
        p.q0 = n_long_or_hub;
        p.q1 = s.n_rows;
        const int64_t blocks = (p.q1 - p.q0 + 255) / 256;
        hipLaunchKernelGGL((attn_sweep_kernel<1, OP>), dim3((unsigned)blocks, p.K), dim3(256), 0, st, p);
        HETA_LAUNCH_CHECK("attn_sweep_kernel");
    }
    return HETA_OK;
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
    const float *corr;
    float *out;
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
    if (lane < p.K) p.out[i * p.K + lane] = res - (p.corr ? p.corr[i * p.K + lane] : 0.f);
}

template <typename TX, typename TY>
heta_status launch_rowdot_t(const DotParams &p, hipStream_t st)
{
    if (p.n == 0) return HETA_OK;
    const size_t sx = sizeof(TX), sy = sizeof(TY);
    const bool vec = (reinterpret_cast<uintptr_t>(p.x) % (4 * sx) == 0) && (p.ld_x % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(p.y) % (4 * sy) == 0) && (p.ld_y % 4 == 0) && (p.d % 4 == 0) &&
                     (p.F % 4 == 0);
    const int64_t blocks = (p.n + 3) / 4;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "attention: too many rows");
    const double bytes = static_cast<double>(p.n) * (p.d * (sx + (p.ld_y ? sy : 0)) + 4.0 * p.K * (p.corr ? 2 : 1));
    ProfScope prof("attn_rowdot_kernel", st, bytes, 0);
    if (vec) hipLaunchKernelGGL((attn_rowdot_kernel<TX, TY, 4>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((attn_rowdot_kernel<TX, TY, 1>), dim3((unsigned)blocks), dim3(256), 0, st, p);
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

// dvec_k[j] = sum_i ds[i, k] x[i, j]: stage 1, one workgroup per (slab of rows, 256 columns), partial sums
// to part[slab][k][j] (per_head: part[slab][j], only k = j / F); stage 2 adds the slabs in order.
constexpr int kSlabRows = 1024;
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

__global__ void __launch_bounds__(256) attn_slab_sum_kernel(const float *part, int64_t n_slabs, int64_t elems, float *out)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= elems) return;
    float a = 0.f;
    for (int64_t s = 0; s < n_slabs; ++s) a += part[s * elems + t];
    out[t] = a;
}

heta_status ensure_attn(heta_graph *g, size_t bytes)
{
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
            if (dt == HETA_F32)
                hipLaunchKernelGGL((attn_score_bwd_param_kernel<float>), grid, dim3(256), 0, st, static_cast<const float *>(x),
                                   ld_x, dscore, n, (int)d, (int)heads, F, per_head ? 1 : 0, part);
            else
                hipLaunchKernelGGL((attn_score_bwd_param_kernel<bf16_t>), grid, dim3(256), 0, st, static_cast<const bf16_t *>(x),
                                   ld_x, dscore, n, (int)d, (int)heads, F, per_head ? 1 : 0, part);
            HETA_LAUNCH_CHECK("attn_score_bwd_param_kernel");
        }
        hipLaunchKernelGGL(attn_slab_sum_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, part, n_slabs, elems, dvec);
        HETA_LAUNCH_CHECK("attn_slab_sum_kernel");
    }
    return HETA_OK;
}

heta_status heta_rel_attn_fwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, void *out,
                              heta_dtype out_dt, int64_t ld_out, float beta, float *smax, float *sinv, void *hip_stream)
{
    heta_status e = check_attn_args("heta_rel_attn_fwd", g, rel, d, heads);
    if (e != HETA_OK) return e;
    if (!z || !el || !er || !out || ((smax == nullptr) != (sinv == nullptr)))
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: null argument (smax and sinv go together)");
    if (!valid_dtype(z_dt) || !valid_dtype(out_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: bad dtype");
    if (ld_z < d || ld_out < d) return fail(HETA_ERR_SHAPE, "heta_rel_attn_fwd: need d <= ld");
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "heta_rel_attn_fwd: beta must be 0 or 1");
    if (reinterpret_cast<uintptr_t>(z) % dtype_size(z_dt) || reinterpret_cast<uintptr_t>(out) % dtype_size(out_dt))
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_fwd: pointer not aligned to its element size");
    const Relation &r = g->rels[rel];
    hipStream_t st = as_stream(hip_stream);
    e = ensure_attn(g, round256(static_cast<size_t>(r.n_edges) * heads * sizeof(float)));
    if (e != HETA_OK) return e;
    float *alpha = static_cast<float *>(g->d_attn);
    SweepParams sp{};
    sp.K = heads;
    sp.slope = slope;
    sp.row_a = er;
    sp.nbr_a = el;
    sp.smax = smax;
    sp.sinv = sinv;
    sp.alpha = alpha;
    e = launch_sweeps<SWEEP_FWD>(r.csr, sp, st, "attn_sweep_fwd");
    if (e != HETA_OK) return e;
    return aggregate_slot_weighted(g, r.csr, z, z_dt, ld_z, d, alpha, heads, out, out_dt, ld_out, beta, st);
}

heta_status heta_rel_attn_bwd(heta_graph *g, int32_t rel, const void *z, heta_dtype z_dt, int64_t ld_z, int32_t d,
                              int32_t heads, const float *el, const float *er, float slope, const float *smax,
                              const float *sinv, const void *o, heta_dtype o_dt, int64_t ld_o, const float *grad_out,
                              int64_t ld_go, float *dz, int64_t ld_dz, float *del, float *der, void *hip_stream)
{
    heta_status e = check_attn_args("heta_rel_attn_bwd", g, rel, d, heads);
    if (e != HETA_OK) return e;
    if (!z || !el || !er || !smax || !sinv || !o || !grad_out || !dz || !del || !der)
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: null argument");
    if (!valid_dtype(z_dt) || !valid_dtype(o_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: bad dtype");
    if (ld_z < d || ld_o < d || ld_go < d || ld_dz < d) return fail(HETA_ERR_SHAPE, "heta_rel_attn_bwd: need d <= ld");
    if (reinterpret_cast<uintptr_t>(z) % dtype_size(z_dt) || reinterpret_cast<uintptr_t>(o) % dtype_size(o_dt) ||
        reinterpret_cast<uintptr_t>(grad_out) % 4 || reinterpret_cast<uintptr_t>(dz) % 4)
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_attn_bwd: pointer not aligned to its element size");
    const Relation &r = g->rels[rel];
    hipStream_t st = as_stream(hip_stream);
    const int K = heads;
    // workspace: two per-slot weight arrays, per-row terms, and one [max rows x d] fp32 intermediate
    const size_t w_bytes = round256(static_cast<size_t>(r.n_edges) * K * sizeof(float));
    const size_t dst_bytes = round256(static_cast<size_t>(r.n_dst) * K * sizeof(float));
    const size_t src_bytes = round256(static_cast<size_t>(r.n_src) * K * sizeof(float));
    const int64_t ld_r = (static_cast<int64_t>(d) + 3) / 4 * 4;
    const size_t r_bytes = round256(static_cast<size_t>(std::max(r.n_dst, r.n_src)) * ld_r * sizeof(float));
    e = ensure_attn(g, 2 * w_bytes + 2 * dst_bytes + src_bytes + r_bytes);
    if (e != HETA_OK) return e;
    char *base = static_cast<char *>(g->d_attn);
    float *w_alpha = reinterpret_cast<float *>(base);
    float *w_gate = reinterpret_cast<float *>(base + w_bytes);
    float *dot = reinterpret_cast<float *>(base + 2 * w_bytes);
    float *corr_d = reinterpret_cast<float *>(base + 2 * w_bytes + dst_bytes);
    float *corr_s = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes);
    float *R = reinterpret_cast<float *>(base + 2 * w_bytes + 2 * dst_bytes + src_bytes);

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
    dp.corr = nullptr;
    dp.out = dot;
    e = launch_rowdot(dp, HETA_F32, o_dt, st);
    if (e != HETA_OK) return e;

    // destination side: gate per CSR slot, R[v] = sum_e gate_e z[u_e], der = <g, R> - dot * sum_e gate_e
    SweepParams sp{};
    sp.K = K;
    sp.slope = slope;
    sp.row_a = er;
    sp.nbr_a = el;
    sp.smax = const_cast<float *>(smax);
    sp.sinv = const_cast<float *>(sinv);
    sp.dot = dot;
    sp.gate = w_gate;
    sp.corr = corr_d;
    e = launch_sweeps<SWEEP_BWD_CSR>(r.csr, sp, st, "attn_sweep_bwd_dst");
    if (e != HETA_OK) return e;
    e = aggregate_slot_weighted(g, r.csr, z, z_dt, ld_z, d, w_gate, K, R, HETA_F32, ld_r, 0.f, st);
    if (e != HETA_OK) return e;
    dp.x = grad_out;
    dp.ld_x = ld_go;
    dp.y = R;
    dp.ld_y = ld_r;
    dp.n = r.n_dst;
    dp.corr = corr_d;
    dp.out = der;
    e = launch_rowdot(dp, HETA_F32, HETA_F32, st);
    if (e != HETA_OK) return e;

    // source side: alpha and gate per CSC slot; dz[u] = sum_e alpha_e g[v_e]; R[u] = sum_e gate_e g[v_e];
    // del = <z, R> - sum_e gate_e dot[v_e]
    sp.row_a = el;
    sp.nbr_a = er;
    sp.alpha = w_alpha;
    sp.gate = w_gate;
    sp.corr = corr_s;
    e = launch_sweeps<SWEEP_BWD_CSC>(r.csc, sp, st, "attn_sweep_bwd_src");
    if (e != HETA_OK) return e;
    e = aggregate_slot_weighted(g, r.csc, grad_out, HETA_F32, ld_go, d, w_alpha, K, dz, HETA_F32, ld_dz, 0.f, st);
    if (e != HETA_OK) return e;
    e = aggregate_slot_weighted(g, r.csc, grad_out, HETA_F32, ld_go, d, w_gate, K, R, HETA_F32, ld_r, 0.f, st);
    if (e != HETA_OK) return e;
    dp.x = z;
    dp.ld_x = ld_z;
    dp.y = R;
    dp.ld_y = ld_r;
    dp.n = r.n_src;
    dp.corr = corr_s;
    dp.out = del;
    return launch_rowdot(dp, z_dt, HETA_F32, st);
}

} // extern "C"
