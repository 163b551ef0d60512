// Sparse optimizer step of a learnable feature table.
//
// Featureless node types carry learnable vectors that are updated after backpropagation
// together with their optimizer states, Adam's moment and variance (Sections 2.2 and 6 of the
// paper; there the update is the DRAM-bound stage that takes a quarter to a third of an epoch).
// Here table and states stay resident in HBM and a mini-batch's rows are updated in one
// streaming pass: Algorithm 1 of the Adam paper on the rows listed in `ids`, with one global
// step counter; rows not listed keep parameters and states bit for bit.
//
// HBM-bound: per element one gradient, moment, variance and parameter read and one moment,
// variance and parameter write (28 bytes with an fp32 table, 24 with a bf16 table), 128-bit
// accesses, one thread per 4 consecutive elements of a row.
#include <cmath>

#include "heta_internal.h"

namespace heta {

using bf16_t = uint16_t;

struct AdamParams {
    void *table;
    int table_bf16;
    int64_t ld_table;
    float *m, *v;
    int64_t ld_state;
    const int64_t *ids; // nullable: identity
    int64_t n, n_table_rows;
    const float *grad;
    int64_t ld_grad;
    int d;
    float lr, beta1, beta2, eps;
    float c1, c2;       // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
};

__device__ __forceinline__ float adam_element(const AdamParams &p, float g, float &m, float &v, float theta)
{
    // every product and sum rounded on its own: which pairs the compiler fuses into an FMA differs from one kernel
    // this function is inlined into to the next, and the single and the multi-table kernel must agree bit for bit
#pragma clang fp contract(off)
    m = p.beta1 * m + (1.f - p.beta1) * g;
    v = p.beta2 * v + (1.f - p.beta2) * g * g;
    return theta - p.lr * (m * p.c1) / (sqrtf(v * p.c2) + p.eps);
}

__device__ __forceinline__ bf16_t adam_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
    return static_cast<bf16_t>((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <int V> // V = 4: 128-bit accesses on whole, aligned chunks; V = 1: element-wise
__device__ __forceinline__ void sparse_adam_body(const AdamParams &p)
{
    const int per_row = (p.d + V - 1) / V;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / per_row;
    if (i >= p.n) return;
    const int c = static_cast<int>(t % per_row) * V;
    const int64_t r = p.ids ? p.ids[i] : i;
    if (r < 0 || r >= p.n_table_rows) return; // a row id outside the table: nothing is read or written for it
    const float *gp = p.grad + i * p.ld_grad + c;
    float *mp = p.m + r * p.ld_state + c, *vp = p.v + r * p.ld_state + c;
    if (V == 4) {
        const float4 g = *reinterpret_cast<const float4 *>(gp);
        float4 m = *reinterpret_cast<const float4 *>(mp), v = *reinterpret_cast<const float4 *>(vp);
        if (p.table_bf16) {
            bf16_t *tp = static_cast<bf16_t *>(p.table) + r * p.ld_table + c;
            const uint2 raw = *reinterpret_cast<const uint2 *>(tp);
            const float x0 = adam_element(p, g.x, m.x, v.x, __uint_as_float(raw.x << 16));
            const float x1 = adam_element(p, g.y, m.y, v.y, __uint_as_float(raw.x & 0xffff0000u));
            const float x2 = adam_element(p, g.z, m.z, v.z, __uint_as_float(raw.y << 16));
            const float x3 = adam_element(p, g.w, m.w, v.w, __uint_as_float(raw.y & 0xffff0000u));
            *reinterpret_cast<uint2 *>(tp) = make_uint2(adam_to_bf16(x0) | (static_cast<uint32_t>(adam_to_bf16(x1)) << 16),
                                                        adam_to_bf16(x2) | (static_cast<uint32_t>(adam_to_bf16(x3)) << 16));
        } else {
            float *tp = static_cast<float *>(p.table) + r * p.ld_table + c;
            float4 x = *reinterpret_cast<const float4 *>(tp);
            x.x = adam_element(p, g.x, m.x, v.x, x.x);
            x.y = adam_element(p, g.y, m.y, v.y, x.y);
            x.z = adam_element(p, g.z, m.z, v.z, x.z);
            x.w = adam_element(p, g.w, m.w, v.w, x.w);
            *reinterpret_cast<float4 *>(tp) = x;
        }
        *reinterpret_cast<float4 *>(mp) = m;
        *reinterpret_cast<float4 *>(vp) = v;
    } else {
        float m = *mp, v = *vp;
        if (p.table_bf16) {
            bf16_t *tp = static_cast<bf16_t *>(p.table) + r * p.ld_table + c;
            *tp = adam_to_bf16(adam_element(p, *gp, m, v, __uint_as_float(static_cast<uint32_t>(*tp) << 16)));
        } else {
            float *tp = static_cast<float *>(p.table) + r * p.ld_table + c;
            *tp = adam_element(p, *gp, m, v, *tp);
        }
        *mp = m;
        *vp = v;
    }
}

template <int V> __global__ void __launch_bounds__(256) sparse_adam_kernel(AdamParams p) { sparse_adam_body<V>(p); }

// several tables in one launch (the weight matrices of a model and its learnable tables after one backward pass):
// blockIdx.y picks the table
constexpr int kAdamMulti = 16;
struct AdamMulti {
    AdamParams p[kAdamMulti];
};
static_assert(sizeof(AdamMulti) <= 3584, "kernel arguments are limited to 4 KB");
template <int V> __global__ void __launch_bounds__(256) sparse_adam_multi_kernel(AdamMulti m) { sparse_adam_body<V>(m.p[blockIdx.y]); }

// checks one update's arguments and fills its parameter block; *vec: 128-bit accesses are possible
static heta_status adam_params(const char *who, void *table, heta_dtype dt, int64_t ld_table, int32_t d, int64_t n_table_rows, float *m,
                               float *v, int64_t ld_state, const int64_t *ids, int64_t n, const float *grad, int64_t ld_grad, float lr,
                               float beta1, float beta2, float eps, int64_t step, AdamParams *out, bool *vec, double *bytes)
{
    if (!table || !m || !v || (n > 0 && !grad)) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (d <= 0 || ld_table < d || ld_state < d || ld_grad < d || n < 0 || n_table_rows < 0)
        return fail(HETA_ERR_SHAPE, "%s: need 0 < d <= every leading dimension and non-negative counts", who);
    if (!ids && n > n_table_rows) return fail(HETA_ERR_SHAPE, "%s: %lld gradient rows for a table of %lld rows", who, (long long)n, (long long)n_table_rows);
    if (step < 1) return fail(HETA_ERR_INVALID_ARG, "%s: the step counter starts at 1", who);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
        return fail(HETA_ERR_INVALID_ARG, "%s: need 0 <= beta1, beta2 < 1 and eps >= 0", who);
    const size_t esz = dtype_size(dt);
    if ((reinterpret_cast<uintptr_t>(table) % esz) || (reinterpret_cast<uintptr_t>(m) & 3u) || (reinterpret_cast<uintptr_t>(v) & 3u) ||
        (reinterpret_cast<uintptr_t>(grad) & 3u))
        return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", who);
    AdamParams p{};
    p.table = table;
    p.table_bf16 = dt == HETA_BF16;
    p.ld_table = ld_table;
    p.m = m;
    p.v = v;
    p.ld_state = ld_state;
    p.ids = ids;
    p.n = n;
    p.n_table_rows = n_table_rows;
    p.grad = grad;
    p.ld_grad = ld_grad;
    p.d = d;
    p.lr = lr;
    p.beta1 = beta1;
    p.beta2 = beta2;
    p.eps = eps;
    p.c1 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(step))));
    p.c2 = static_cast<float>(1.0 / (1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(step))));
    *out = p;
    *vec = d % 4 == 0 && ld_state % 4 == 0 && ld_grad % 4 == 0 && aligned16(m) && aligned16(v) && (n == 0 || aligned16(grad)) &&
           (ld_table * esz) % (4 * esz) == 0 && (reinterpret_cast<uintptr_t>(table) % (4 * esz)) == 0;
    // algorithmic traffic: gradient, both states twice, the parameter twice, one id per row
    *bytes = static_cast<double>(n) * (d * (4.0 + 16.0 + 2.0 * esz) + (ids ? 8.0 : 0.0));
    return HETA_OK;
}

} // namespace heta

using namespace heta;

extern "C" heta_status heta_sparse_adam_multi(int32_t n_items, const heta_adam_item *items, float lr, float beta1, float beta2, float eps,
                                              int64_t step, void *hip_stream)
{
    const char *who = "heta_sparse_adam_multi";
    if (n_items < 0 || (n_items > 0 && !items)) return fail(HETA_ERR_INVALID_ARG, "%s: bad item list", who);
    hipStream_t st = as_stream(hip_stream);
    for (int32_t i0 = 0; i0 < n_items; i0 += kAdamMulti) {
        // every item is checked before anything is launched for this group of up to kAdamMulti
        AdamMulti m{};
        bool vec[kAdamMulti];
        int n_live = 0;
        double bytes = 0;
        for (int32_t i = i0; i < n_items && i < i0 + kAdamMulti; ++i) {
            const heta_adam_item &it = items[i];
            AdamParams p{};
            bool vq = false;
            double b = 0;
            heta_status e = adam_params(who, it.table, it.dt, it.ld_table, it.d, it.n_table_rows, it.m, it.v, it.ld_state, it.ids, it.n,
                                        it.grad, it.ld_grad, lr, beta1, beta2, eps, step, &p, &vq, &b);
            if (e != HETA_OK) return e;
            if (it.n == 0) continue;
            m.p[n_live] = p;
            vec[n_live++] = vq;
            bytes += b;
        }
        if (n_live == 0) continue;
        // one launch for the items that take 128-bit accesses, one for the rest (blockIdx.y = position in the launch)
        for (int pass = 0; pass < 2; ++pass) {
            AdamMulti q{};
            int k = 0;
            int64_t threads_max = 0;
            for (int i = 0; i < n_live; ++i)
                if (vec[i] == (pass == 0)) {
                    q.p[k++] = m.p[i];
                    threads_max = std::max<int64_t>(threads_max, m.p[i].n * (pass == 0 ? m.p[i].d / 4 : m.p[i].d));
                }
            if (k == 0) continue;
            if ((threads_max + 255) / 256 > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "%s: too many elements for one launch", who);
            ProfScope prof("sparse_adam_kernel", st, bytes, 0);
            bytes = 0; // counted once
            const dim3 grid((unsigned)((threads_max + 255) / 256), (unsigned)k);
            if (pass == 0) hipLaunchKernelGGL(sparse_adam_multi_kernel<4>, grid, dim3(256), 0, st, q);
            else hipLaunchKernelGGL(sparse_adam_multi_kernel<1>, grid, dim3(256), 0, st, q);
            HETA_LAUNCH_CHECK("sparse_adam_multi_kernel");
        }
    }
    return HETA_OK;
}

extern "C" heta_status heta_sparse_adam(void *table, heta_dtype dt, int64_t ld_table, int32_t d, int64_t n_table_rows,
                                        float *m, float *v, int64_t ld_state, const int64_t *ids, int64_t n,
                                        const float *grad, int64_t ld_grad, float lr, float beta1, float beta2, float eps,
                                        int64_t step, void *hip_stream)
{
    const char *who = "heta_sparse_adam";
    AdamParams p{};
    bool vec = false;
    double bytes = 0;
    heta_status e = adam_params(who, table, dt, ld_table, d, n_table_rows, m, v, ld_state, ids, n, grad, ld_grad, lr, beta1, beta2, eps, step,
                                &p, &vec, &bytes);
    if (e != HETA_OK) return e;
    if (n == 0) return HETA_OK;
    hipStream_t st = as_stream(hip_stream);
    ProfScope prof("sparse_adam_kernel", st, bytes, 0);
    if (vec) {
        const int64_t threads = n * (d / 4);
        if ((threads + 255) / 256 > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "%s: too many elements for one launch", who);
        hipLaunchKernelGGL(sparse_adam_kernel<4>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, p);
    } else {
        const int64_t threads = n * d;
        if ((threads + 255) / 256 > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "%s: too many elements for one launch", who);
        hipLaunchKernelGGL(sparse_adam_kernel<1>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, p);
    }
    HETA_LAUNCH_CHECK("sparse_adam_kernel");
    return HETA_OK;
}
