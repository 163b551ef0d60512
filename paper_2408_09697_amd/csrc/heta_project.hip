// Per-relation projection on the matrix cores: Z_r = M_r W_r (forward), dM_r = dZ_r W_r^T and
// dW_r = M_r^T dZ_r (backward) - the per-relation weight matrices of an R-GCN-style AGG_r
// (Section 2.1 of the paper).  This is the only dense contraction on the path and the only
// place MFMA is used.
//
// One kernel template computes C[M,N] (+)= A[M,K] . B[K,N] with fp32 accumulation:
//   - a 256-thread workgroup owns a 128 x 128 tile of C, each of its four wavefronts a 64 x 64
//     quarter held as 2 x 2 MFMA 32x32 accumulators (64 VGPRs per lane);
//   - A and B tiles of 32 k-values are staged through LDS in a k-contiguous layout, rows padded
//     by 16 bytes so that the 128-bit fragment reads of 8 consecutive lanes fall on distinct banks;
//   - an operand is described by how it lies in memory: "k-contiguous" (element (r,k) at
//     base[r*ld + k], copied with 128-bit loads/stores) or "r-contiguous" (element (r,k) at
//     base[k*ld + r], transposed on the way into LDS);
//   - fp32 operands use v_mfma_f32_32x32x2_f32; as soon as one operand is bf16 both are fed as
//     bf16 to v_mfma_f32_32x32x16_bf16.  The k index a lane supplies only has to agree between
//     the A and B fragments, so each lane reads 16 contiguous bytes and spreads them over
//     consecutive MFMAs;
//   - the weight gradient contracts over graph rows: the row range is split over grid.z,
//     partial products go to the workspace and are added in split order (no atomics).
#include <algorithm>

#include "heta_internal.h"

namespace heta {

using bf16_t = uint16_t;
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128, BN = 128, BK = 32;

struct GemmParams {
    const void *A;
    int64_t lda;
    int a_vec;          // 128-bit loads allowed for A
    const void *B;
    int64_t ldb;
    int b_vec;
    int64_t M, N, K;
    float *C;           // output, or partial buffer [split][M][ldc] when `partial`
    int64_t ldc;
    const float *row_scale;
    float beta;
    int64_t k_per_split; // multiple of BK; grid.z = n_split ranges of this many k-values
    int n_split;
    int partial;         // write raw partial products per split instead of the finished output
};

__device__ __forceinline__ bf16_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return static_cast<bf16_t>((u >> 16) | 0x40u);
    return static_cast<bf16_t>((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <typename S, typename CT> __device__ __forceinline__ CT convert(S v);
template <> __device__ __forceinline__ float convert<float, float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t convert<float, bf16_t>(float v) { return to_bf16(v); }
template <> __device__ __forceinline__ bf16_t convert<bf16_t, bf16_t>(bf16_t v) { return v; }

// LDS row stride in elements of CT: 32 k-values + 16 bytes of padding
template <typename CT> struct LdsStride { static constexpr int value = BK + 16 / (int)sizeof(CT); };

// Moves a [ROWS x BK] operand tile global -> registers -> LDS.
//   RC == false: element (r,k) at base[r*ld + k]   (k-contiguous)
//   RC == true : element (r,k) at base[k*ld + r]   (r-contiguous, transposed into LDS)
template <typename S, typename CT, bool RC, int ROWS>
struct TileLoader {
    static constexpr int E = 16 / (int)sizeof(S);
    static constexpr int NCH = ROWS * BK / E / 256;
    static constexpr int SA = LdsStride<CT>::value;
    S regs[NCH][E];

    __device__ __forceinline__ void load(const S *base, int64_t ld, int64_t r0, int64_t R, int64_t k0, int64_t K,
                                         bool vec, int tid)
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int q = tid + 256 * i;
            int r, k;
            if (RC) { k = q % BK; r = (q / BK) * E; }
            else { r = q / (BK / E); k = (q % (BK / E)) * E; }
            const int64_t gr = r0 + r, gk = k0 + k;
#pragma unroll
            for (int j = 0; j < E; ++j) regs[i][j] = S(0);
            if (gr >= R || gk >= K) continue;
            const S *src = RC ? base + gk * ld + gr : base + gr * ld + gk;
            const int64_t left = RC ? R - gr : K - gk; // valid elements along the contiguous direction
            if (vec) {
                union { uint4 u; S s[E]; } t;
                t.u = *reinterpret_cast<const uint4 *>(src);
#pragma unroll
                for (int j = 0; j < E; ++j) if (j < left) regs[i][j] = t.s[j];
            } else {
#pragma unroll
                for (int j = 0; j < E; ++j) if (j < left) regs[i][j] = src[j];
            }
        }
    }

    __device__ __forceinline__ void store(CT *lds, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int q = tid + 256 * i;
            if (RC) {
                const int k = q % BK, r = (q / BK) * E;
#pragma unroll
                for (int j = 0; j < E; ++j) lds[(r + j) * SA + k] = convert<S, CT>(regs[i][j]);
            } else {
                const int r = q / (BK / E), k = (q % (BK / E)) * E;
                CT tmp[E];
#pragma unroll
                for (int j = 0; j < E; ++j) tmp[j] = convert<S, CT>(regs[i][j]);
                CT *dst = lds + r * SA + k;
                if (sizeof(CT) * E == 16) *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(tmp);
                else *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(tmp);
            }
        }
    }
};

template <typename CT, typename SA_T, bool A_RC, typename SB_T, bool B_RC>
__global__ void __launch_bounds__(256) gemm_kernel(GemmParams p)
{
    constexpr int S = LdsStride<CT>::value;
    __shared__ __attribute__((aligned(16))) CT As[BM * S];
    __shared__ __attribute__((aligned(16))) CT Bs[BN * S];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x) * BM, n0 = static_cast<int64_t>(blockIdx.y) * BN;
    const int64_t kbeg = static_cast<int64_t>(blockIdx.z) * p.k_per_split;
    const int64_t kend = min(p.K, kbeg + p.k_per_split);

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    TileLoader<SA_T, CT, A_RC, BM> la;
    TileLoader<SB_T, CT, B_RC, BN> lb;
    const SA_T *A = static_cast<const SA_T *>(p.A);
    const SB_T *B = static_cast<const SB_T *>(p.B);

    if (kbeg < kend) {
        la.load(A, p.lda, m0, p.M, kbeg, kend, p.a_vec, tid);
        lb.load(B, p.ldb, n0, p.N, kbeg, kend, p.b_vec, tid);
    }
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads(); // previous tile fully consumed
        la.store(As, tid);
        lb.store(Bs, tid);
        __syncthreads();
        if (k0 + BK < kend) { // next tile's global loads fly during the MFMAs
            la.load(A, p.lda, m0, p.M, k0 + BK, kend, p.a_vec, tid);
            lb.load(B, p.ldb, n0, p.N, k0 + BK, kend, p.b_vec, tid);
        }
        if constexpr (sizeof(CT) == 4) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 8) {
                float4 a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    a[i] = *reinterpret_cast<const float4 *>(&As[(wm + i * 32 + l32) * S + kk + 4 * half]);
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    b[j] = *reinterpret_cast<const float4 *>(&Bs[(wn + j * 32 + l32) * S + kk + 4 * half]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].x, b[j].x, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].y, b[j].y, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].z, b[j].z, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].w, b[j].w, acc[i][j], 0, 0, 0);
                    }
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                union Frag { uint4 u; bf16x8 v; } a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    a[i].u = *reinterpret_cast<const uint4 *>(&As[(wm + i * 32 + l32) * S + kk + 8 * half]);
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    b[j].u = *reinterpret_cast<const uint4 *>(&Bs[(wn + j * 32 + l32) * S + kk + 8 * half]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
            }
        }
    }

    // epilogue: accumulator register v of lane (half, l32) is C[8*(v/4) + 4*half + v%4][l32] of its 32x32 tile
    float *C = p.C + (p.partial ? static_cast<int64_t>(blockIdx.z) * p.M * p.ldc : 0);
    const bool direct = !p.partial;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn + j * 32 + l32;
            if (n >= p.N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm + i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (m >= p.M) continue;
                float val = acc[i][j][v];
                float *o = C + m * p.ldc + n;
                if (direct) {
                    if (p.row_scale) val *= p.row_scale[m];
                    if (p.beta != 0.f) val += p.beta * *o;
                }
                *o = val;
            }
        }
}

// dW[m, n] = beta * dW[m, n] + sum over splits (in split order) of part[s][m][n]
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float *part, int n_split, int64_t M, int64_t N,
                                                            float *out, int64_t ldo, float beta)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= M * N) return;
    const int64_t m = t / N, n = t % N;
    float a = 0.f;
    for (int s = 0; s < n_split; ++s) a += part[(static_cast<int64_t>(s) * M + m) * N + n];
    float *o = out + m * ldo + n;
    *o = (beta != 0.f) ? beta * *o + a : a;
}

template <typename CT, typename SA_T, bool A_RC, typename SB_T, bool B_RC>
static heta_status launch_gemm(const GemmParams &p, hipStream_t st)
{
    const int64_t mt = (p.M + BM - 1) / BM, nt = (p.N + BN - 1) / BN;
    if (mt > 0x7fffffff || nt > 65535) return fail(HETA_ERR_UNSUPPORTED, "projection: matrix too large for one launch");
    // algorithmic traffic: both operands once, the output once (twice when accumulating)
    const double bytes = static_cast<double>(p.M) * p.K * sizeof(SA_T) + static_cast<double>(p.K) * p.N * sizeof(SB_T) +
                         static_cast<double>(p.M) * p.N * 4.0 * (p.beta != 0.f ? 2.0 : 1.0);
    ProfScope prof(sizeof(CT) == 4 ? (p.partial ? "gemm_wgrad_f32" : "gemm_f32") : (p.partial ? "gemm_wgrad_bf16" : "gemm_bf16"),
                   st, bytes, 2.0 * p.M * p.N * p.K);
    hipLaunchKernelGGL((gemm_kernel<CT, SA_T, A_RC, SB_T, B_RC>), dim3((unsigned)mt, (unsigned)nt, (unsigned)std::max(1, p.n_split)),
                       dim3(256), 0, st, p);
    HETA_LAUNCH_CHECK("gemm_kernel");
    return HETA_OK;
}

static bool vec_ok(const void *ptr, int64_t ld, heta_dtype dt)
{
    return aligned16(ptr) && (ld * (int64_t)dtype_size(dt)) % 16 == 0;
}

template <bool A_RC, bool B_RC>
static heta_status dispatch_gemm(GemmParams p, heta_dtype a_dt, heta_dtype b_dt, hipStream_t st)
{
    p.a_vec = vec_ok(p.A, p.lda, a_dt);
    p.b_vec = vec_ok(p.B, p.ldb, b_dt);
    if (a_dt == HETA_F32 && b_dt == HETA_F32) return launch_gemm<float, float, A_RC, float, B_RC>(p, st);
    if (a_dt == HETA_F32 && b_dt == HETA_BF16) return launch_gemm<bf16_t, float, A_RC, bf16_t, B_RC>(p, st);
    if (a_dt == HETA_BF16 && b_dt == HETA_F32) return launch_gemm<bf16_t, bf16_t, A_RC, float, B_RC>(p, st);
    return launch_gemm<bf16_t, bf16_t, A_RC, bf16_t, B_RC>(p, st);
}

static heta_status project_impl(int64_t n_rows, const void *in, heta_dtype in_dt, int64_t ld_in, int32_t d_in,
                                const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_out, int32_t transW,
                                const float *row_scale, float *out, int64_t ld_out, float beta, hipStream_t st,
                                const char *who)
{
    if (!in || !W || !out) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (!valid_dtype(in_dt) || !valid_dtype(w_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (n_rows < 0 || d_in <= 0 || d_out <= 0) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
    if (ld_in < d_in || ld_out < d_out || ld_w < (transW ? d_in : d_out))
        return fail(HETA_ERR_SHAPE, "%s: leading dimension smaller than the row width", who);
    if ((reinterpret_cast<uintptr_t>(in) % dtype_size(in_dt)) || (reinterpret_cast<uintptr_t>(W) % dtype_size(w_dt)) ||
        (reinterpret_cast<uintptr_t>(out) & 3u))
        return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", who);
    if (n_rows == 0) return HETA_OK;
    GemmParams p{};
    p.A = in;
    p.lda = ld_in;
    p.B = W;
    p.ldb = ld_w;
    p.M = n_rows;
    p.N = d_out;
    p.K = d_in;
    p.C = out;
    p.ldc = ld_out;
    p.row_scale = row_scale;
    p.beta = beta;
    p.k_per_split = (static_cast<int64_t>(d_in) + BK - 1) / BK * BK;
    p.n_split = 1;
    p.partial = 0;
    // B[k][n] = W[k][n] is n-contiguous (r-contiguous in the loader's terms); W^T is k-contiguous
    return transW ? dispatch_gemm<false, false>(p, in_dt, w_dt, st) : dispatch_gemm<false, true>(p, in_dt, w_dt, st);
}

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_project(int64_t n_rows, const void *in, heta_dtype in_dt, int64_t ld_in, int32_t d_in,
                         const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_out, int32_t transW,
                         const float *row_scale, float *out, int64_t ld_out, float beta, void *hip_stream)
{
    return project_impl(n_rows, in, in_dt, ld_in, d_in, W, w_dt, ld_w, d_out, transW, row_scale, out, ld_out, beta,
                        as_stream(hip_stream), "heta_project");
}

heta_status heta_rel_project(const heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                             int64_t ld_in, int32_t d_in, const void *W, heta_dtype w_dt, int64_t ld_w,
                             int32_t d_out, int32_t transW, const float *row_scale, float *out,
                             int64_t ld_out, float beta, void *hip_stream)
{
    if (!g) return fail(HETA_ERR_INVALID_ARG, "heta_rel_project: graph is NULL");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_project: relation %d out of range", rel);
    return project_impl(g->rels[rel].n_dst, in, in_dt, ld_in, d_in, W, w_dt, ld_w, d_out, transW, row_scale, out,
                        ld_out, beta, as_stream(hip_stream), "heta_rel_project");
}

heta_status heta_rel_project_wgrad(heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                                   int64_t ld_in, int32_t d_in, const float *gout, int64_t ld_go,
                                   int32_t d_out, float *dW, int64_t ld_dw, float beta, void *hip_stream)
{
    if (!g || !in || !gout || !dW) return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: null argument");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: relation %d out of range", rel);
    if (!valid_dtype(in_dt)) return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: bad dtype");
    if (d_in <= 0 || d_out <= 0 || ld_in < d_in || ld_go < d_out || ld_dw < d_out)
        return fail(HETA_ERR_SHAPE, "heta_rel_project_wgrad: bad sizes");
    if ((reinterpret_cast<uintptr_t>(in) % dtype_size(in_dt)) || (reinterpret_cast<uintptr_t>(gout) & 3u) ||
        (reinterpret_cast<uintptr_t>(dW) & 3u))
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: pointer not aligned to its element size");
    hipStream_t st = as_stream(hip_stream);
    const int64_t n_rows = g->rels[rel].n_dst;
    const int64_t mt = (d_in + BM - 1) / BM, nt = (d_out + BN - 1) / BN;
    const int64_t k_tiles = (n_rows + BK - 1) / BK;
    int64_t n_split = std::max<int64_t>(1, std::min<int64_t>(k_tiles, (1024 + mt * nt - 1) / (mt * nt)));
    const int64_t tiles_per_split = std::max<int64_t>(1, (k_tiles + n_split - 1) / n_split);
    n_split = std::max<int64_t>(1, (k_tiles + tiles_per_split - 1) / tiles_per_split);
    const size_t part_bytes = static_cast<size_t>(n_split) * d_in * d_out * sizeof(float);
    heta_status e = ensure_workspace(g, part_bytes);
    if (e != HETA_OK) return e;
    GemmParams p{};
    p.A = in;          // A[m = column of `in`][k = graph row] : r-contiguous
    p.lda = ld_in;
    p.B = gout;        // B[k = graph row][n] : r-contiguous
    p.ldb = ld_go;
    p.M = d_in;
    p.N = d_out;
    p.K = n_rows;
    p.C = static_cast<float *>(g->d_ws);
    p.ldc = d_out;
    p.row_scale = nullptr;
    p.beta = 0.f;
    p.k_per_split = tiles_per_split * BK;
    p.n_split = static_cast<int>(n_split);
    p.partial = 1;
    e = dispatch_gemm<true, true>(p, in_dt, HETA_F32, st);
    if (e != HETA_OK) return e;
    const int64_t total = static_cast<int64_t>(d_in) * d_out;
    ProfScope prof("splitk_reduce_kernel", st, (p.n_split + 1.0) * total * 4.0, 0);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float *>(g->d_ws), p.n_split, (int64_t)d_in, (int64_t)d_out, dW, ld_dw, beta);
    HETA_LAUNCH_CHECK("splitk_reduce_kernel");
    return HETA_OK;
}

} // extern "C"
