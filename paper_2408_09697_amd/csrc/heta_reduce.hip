// Cross-relation aggregation AGG_all = sum (Eq. 1 of the paper, second line; Algorithm 1,
// the designated worker's step) and the backward of its optional activation.  Pure streaming:
// every element is read once per partial and written once, 128 bits per lane where the
// layout allows.
#include "heta_internal.h"

namespace heta {

constexpr int kMaxPartials = 16;

struct ReduceParams {
    const float *part[kMaxPartials];
    int n_partials;
    int64_t ld, ld_out;
    int64_t n_rows;
    int d;
    int relu;
    float *out;
};

template <int V> // V floats per thread (4: vector path, 1: scalar path)
__global__ void __launch_bounds__(256) cross_rel_reduce_kernel(ReduceParams p)
{
    const int per_row = (p.d + V - 1) / V;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / per_row;
    const int c = static_cast<int>(t % per_row) * V;
    if (i >= p.n_rows) return;
    if (V == 4) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < p.n_partials; ++k) {
            const float4 v = *reinterpret_cast<const float4 *>(p.part[k] + i * p.ld + c);
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        if (p.relu) { a.x = fmaxf(a.x, 0.f); a.y = fmaxf(a.y, 0.f); a.z = fmaxf(a.z, 0.f); a.w = fmaxf(a.w, 0.f); }
        *reinterpret_cast<float4 *>(p.out + i * p.ld_out + c) = a;
    } else {
        float a = 0.f;
        for (int k = 0; k < p.n_partials; ++k) a += p.part[k][i * p.ld + c];
        if (p.relu) a = fmaxf(a, 0.f);
        p.out[i * p.ld_out + c] = a;
    }
}

template <int V>
__global__ void __launch_bounds__(256) act_bwd_kernel(int64_t n_rows, int d, int relu, const float *h, int64_t ld_h,
                                                      const float *go, int64_t ld_go, float *gi, int64_t ld_gi)
{
    const int per_row = (d + V - 1) / V;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / per_row;
    const int c = static_cast<int>(t % per_row) * V;
    if (i >= n_rows) return;
    if (V == 4) {
        float4 g = *reinterpret_cast<const float4 *>(go + i * ld_go + c);
        if (relu) {
            const float4 x = *reinterpret_cast<const float4 *>(h + i * ld_h + c);
            g.x = x.x > 0.f ? g.x : 0.f; g.y = x.y > 0.f ? g.y : 0.f;
            g.z = x.z > 0.f ? g.z : 0.f; g.w = x.w > 0.f ? g.w : 0.f;
        }
        *reinterpret_cast<float4 *>(gi + i * ld_gi + c) = g;
    } else {
        float g = go[i * ld_go + c];
        if (relu && !(h[i * ld_h + c] > 0.f)) g = 0.f;
        gi[i * ld_gi + c] = g;
    }
}

// A plain streaming copy of known size: the reference point against which hardware byte
// counters are scaled when the library's kernels are profiled.
__global__ void __launch_bounds__(256) calibration_copy_kernel(const uint4 *src, uint4 *dst, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

// Matrix instructions on registers only, no memory traffic: what the matrix pipes sustain at the clock the
// chip holds under that load.  Each wavefront keeps four independent 32 x 32 accumulators busy (16 MFMAs
// per loop trip, none waiting on another); the operands are zero on one side, so the sums stay zero.
typedef float calib_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 calib_bf16x8 __attribute__((ext_vector_type(8)));
template <bool BF16, bool VARYING>
__global__ void __launch_bounds__(256) calibration_mfma_kernel(int64_t iters, float *sink)
{
    calib_f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    // VARYING: four operand pairs of mixed signs and significands, taken in turn, so that the multipliers and
    // the accumulators see new bits with every instruction (what a kernel on real data makes them do); else one
    // pair with zeros on one side (the sums stay zero)
    float a[4], b[4];
    calib_bf16x8 av[4], bv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t h = (threadIdx.x * 2654435761u + q * 40503u) ^ (threadIdx.x >> 3);
        a[q] = VARYING ? (static_cast<float>(h & 0xffffu) - 32768.f) * (1.f / 32768.f) : static_cast<float>(threadIdx.x & 63) * 0.015625f;
        b[q] = VARYING ? (static_cast<float>((h >> 16) & 0xffffu) - 32768.f) * (1.f / 32768.f) : 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            av[q][v] = static_cast<__bf16>(VARYING ? a[q] * (0.25f + 0.09375f * v) : a[q]);
            bv[q][v] = static_cast<__bf16>(VARYING ? b[q] * (1.f - 0.109375f * v) : 0.f);
        }
    }
    for (int64_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (BF16) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[VARYING ? u : 0], bv[VARYING ? u : 0], acc[j], 0, 0, 0);
                else acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[VARYING ? u : 0], b[VARYING ? u : 0], acc[j], 0, 0, 0);
            }
    }
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += acc[j][v];
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = t;
}

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_cross_rel_reduce(const heta_graph *g, int32_t dst_type, const float *const *partials,
                                  int32_t n_partials, int64_t ld, int32_t d_out, heta_act act,
                                  float *out, int64_t ld_out, void *hip_stream)
{
    if (!g || !partials || !out) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: null argument");
    if (dst_type < 0 || dst_type >= (int32_t)g->ntypes.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: node type %d out of range", dst_type);
    if (n_partials < 1 || n_partials > kMaxPartials)
        return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: n_partials must be in [1, %d]", kMaxPartials);
    if (act != HETA_ACT_NONE && act != HETA_ACT_RELU) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: bad act");
    if (d_out <= 0 || ld < d_out || ld_out < d_out) return fail(HETA_ERR_SHAPE, "heta_cross_rel_reduce: bad shape");
    ReduceParams p{};
    bool vec = (d_out % 4 == 0) && (ld % 4 == 0) && (ld_out % 4 == 0) && aligned16(out);
    for (int k = 0; k < n_partials; ++k) {
        if (!partials[k]) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: partial %d is NULL", k);
        if (reinterpret_cast<uintptr_t>(partials[k]) & 3u)
            return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: partial %d not 4-byte aligned", k);
        vec = vec && aligned16(partials[k]);
        p.part[k] = partials[k];
    }
    if (reinterpret_cast<uintptr_t>(out) & 3u) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_reduce: out not aligned");
    p.n_partials = n_partials;
    p.ld = ld;
    p.ld_out = ld_out;
    p.n_rows = g->ntypes[dst_type].num_nodes;
    p.d = d_out;
    p.relu = (act == HETA_ACT_RELU);
    p.out = out;
    if (p.n_rows == 0) return HETA_OK;
    const int64_t threads = p.n_rows * (vec ? d_out / 4 : d_out);
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "heta_cross_rel_reduce: too large");
    ProfScope prof("cross_rel_reduce_kernel", as_stream(hip_stream),
                   (n_partials + 1.0) * static_cast<double>(p.n_rows) * d_out * 4.0, 0);
    if (vec)
        hipLaunchKernelGGL(cross_rel_reduce_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream), p);
    else
        hipLaunchKernelGGL(cross_rel_reduce_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream), p);
    HETA_LAUNCH_CHECK("cross_rel_reduce_kernel");
    return HETA_OK;
}

heta_status heta_act_bwd(int64_t n_rows, int32_t d, heta_act act, const float *h, int64_t ld_h,
                         const float *grad_out, int64_t ld_go, float *grad_in, int64_t ld_gi, void *hip_stream)
{
    if (!grad_out || !grad_in || (act == HETA_ACT_RELU && !h))
        return fail(HETA_ERR_INVALID_ARG, "heta_act_bwd: null argument");
    if (act != HETA_ACT_NONE && act != HETA_ACT_RELU) return fail(HETA_ERR_INVALID_ARG, "heta_act_bwd: bad act");
    if (n_rows < 0 || d <= 0 || ld_go < d || ld_gi < d || (act == HETA_ACT_RELU && ld_h < d))
        return fail(HETA_ERR_SHAPE, "heta_act_bwd: bad shape");
    if ((reinterpret_cast<uintptr_t>(grad_out) & 3u) || (reinterpret_cast<uintptr_t>(grad_in) & 3u) ||
        (h && (reinterpret_cast<uintptr_t>(h) & 3u)))
        return fail(HETA_ERR_INVALID_ARG, "heta_act_bwd: pointer not 4-byte aligned");
    if (n_rows == 0) return HETA_OK;
    const int relu = (act == HETA_ACT_RELU);
    const bool vec = (d % 4 == 0) && (ld_go % 4 == 0) && (ld_gi % 4 == 0) && aligned16(grad_out) && aligned16(grad_in) &&
                     (!relu || ((ld_h % 4 == 0) && aligned16(h)));
    const int64_t threads = n_rows * (vec ? d / 4 : d);
    const int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "heta_act_bwd: too large");
    ProfScope prof("act_bwd_kernel", as_stream(hip_stream), (relu ? 3.0 : 2.0) * static_cast<double>(n_rows) * d * 4.0, 0);
    if (vec)
        hipLaunchKernelGGL(act_bwd_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream), n_rows, (int)d,
                           relu, h, ld_h, grad_out, ld_go, grad_in, ld_gi);
    else
        hipLaunchKernelGGL(act_bwd_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream), n_rows, (int)d,
                           relu, h, ld_h, grad_out, ld_go, grad_in, ld_gi);
    HETA_LAUNCH_CHECK("act_bwd_kernel");
    return HETA_OK;
}

heta_status heta_calibration_copy(void *dst, const void *src, int64_t n_bytes, void *hip_stream)
{
    if (!dst || !src || n_bytes < 0 || (n_bytes % 16) || !aligned16(dst) || !aligned16(src))
        return fail(HETA_ERR_INVALID_ARG, "heta_calibration_copy: need 16-byte aligned buffers and a size that is a multiple of 16");
    if (n_bytes == 0) return HETA_OK;
    const int64_t n = n_bytes / 16;
    const int64_t blocks = (n + 255) / 256;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "heta_calibration_copy: too large");
    ProfScope prof("calibration_copy_kernel", as_stream(hip_stream), 2.0 * static_cast<double>(n_bytes), 0);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n);
    HETA_LAUNCH_CHECK("calibration_copy_kernel");
    return HETA_OK;
}

heta_status heta_calibration_mfma(heta_dtype dt, int32_t varying, int64_t iters, float *sink, int64_t sink_elems, double *flops_out,
                                  void *hip_stream)
{
    constexpr int kBlocks = 512; // two workgroups of four wavefronts per CU: two wavefronts per SIMD
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "heta_calibration_mfma: bad dtype");
    if (!sink || sink_elems < kBlocks * 4 || iters < 1 || iters > (int64_t(1) << 24))
        return fail(HETA_ERR_INVALID_ARG, "heta_calibration_mfma: need 1 <= iters <= 2^24 and a sink of %d floats", kBlocks * 4);
    const double per_mfma = dt == HETA_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    const double flops = per_mfma * 16.0 * static_cast<double>(iters) * 4.0 * kBlocks;
    if (flops_out) *flops_out = flops;
    ProfScope prof("calibration_mfma_kernel", as_stream(hip_stream), 0, flops);
    const dim3 grid(kBlocks), block(256);
    if (dt == HETA_BF16 && varying) hipLaunchKernelGGL((calibration_mfma_kernel<true, true>), grid, block, 0, as_stream(hip_stream), iters, sink);
    else if (dt == HETA_BF16) hipLaunchKernelGGL((calibration_mfma_kernel<true, false>), grid, block, 0, as_stream(hip_stream), iters, sink);
    else if (varying) hipLaunchKernelGGL((calibration_mfma_kernel<false, true>), grid, block, 0, as_stream(hip_stream), iters, sink);
    else hipLaunchKernelGGL((calibration_mfma_kernel<false, false>), grid, block, 0, as_stream(hip_stream), iters, sink);
    HETA_LAUNCH_CHECK("calibration_mfma_kernel");
    return HETA_OK;
}

} // extern "C"
