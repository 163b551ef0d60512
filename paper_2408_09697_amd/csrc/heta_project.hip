// Per-relation projection on the matrix cores: Z_r = M_r W_r (forward), dM_r = dZ_r W_r^T and
// dW_r = M_r^T dZ_r (backward) - the per-relation weight matrices of an R-GCN-style AGG_r
// (Section 2.1 of the paper) - and the same three products for all relations into one
// destination type at once, where the forward then is Eq. 1 in one pass:
// H_t = sum_r M_r W_r, a single contraction over the concatenated k ranges of the relations.
// This is the only dense contraction on the path and the only place MFMA is used.
//
// One kernel template computes C[M,N] (+)= A[M,K] . B[K,N] with fp32 accumulation:
//   - a workgroup of 2 x WN wavefronts owns a 128 x (64*WN) tile of C, each wavefront a 64 x 64
//     block held as 2 x 2 MFMA 32x32 accumulators (64 VGPRs per lane); WN = 4 (512 threads,
//     256 output columns) lets a 256-wide projection read its input rows from HBM exactly once;
//   - A and B tiles of 32 k-values are staged through LDS in a k-contiguous layout, rows padded
//     by 16 bytes so that the 128-bit fragment reads of 8 consecutive lanes fall on distinct
//     banks; the global loads of tile i+1 are issued before the MFMAs of tile i and only
//     touched (masked, converted, stored to LDS) after them;
//   - an operand is described by how it lies in memory: "k-contiguous" (element (r,k) at
//     base[r*ld + k], copied with 128-bit loads/stores) or "r-contiguous" (element (r,k) at
//     base[k*ld + r], transposed on the way into LDS);
//   - fp32 operands use v_mfma_f32_32x32x2_f32; as soon as one operand is bf16 both are fed as
//     bf16 to v_mfma_f32_32x32x16_bf16.  The k index a lane supplies only has to agree between
//     the A and B fragments, so each lane reads 16 contiguous bytes and spreads them over
//     consecutive MFMAs;
//   - a launch carries up to 8 "segments": either summed into one output (k-concatenation, the
//     fused forward) or independent products that share an operand (all dM_r or all dW_r of a
//     destination type), scheduled next to each other so the shared operand is fetched from
//     HBM once and served from cache to the others;
//   - the weight gradient contracts over graph rows: the row range is split over workgroups,
//     partial products go to the workspace and are added in split order (no atomics).
#include <algorithm>

#include "heta_gemm.h"
#include "heta_test_hooks.h"

namespace heta {

template <typename CT, typename SA_T, bool A_RC, typename SB_T, bool B_RC, int WN, bool VEC, int BK, bool B_SPLIT = false>
__global__ void __launch_bounds__(128 * WN) gemm_kernel(GemmParams p)
{
    constexpr int NT = 128 * WN, BN = 64 * WN;
    __shared__ __attribute__((aligned(16))) CT As[LdsTile<CT, A_RC, BM, BK>::elems];
    __shared__ __attribute__((aligned(16))) CT Bs[LdsTile<CT, B_RC, BN, BK>::elems];
    // B_SPLIT: an fp32 B is fed to the bf16 MFMAs as two terms (rounded value + what the rounding left)
    __shared__ __attribute__((aligned(16))) CT Bs_lo[B_SPLIT ? LdsTile<CT, B_RC, BN, BK>::elems : 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave / WN) * 64, wn = (wave % WN) * 64;
    const int half = lane >> 5, l32 = lane & 31;

    // workgroup id -> (XCD, position in that XCD's queue) -> (outer, inner).  Workgroups are dealt
    // round-robin to the 8 XCDs; the tiles that share an operand get consecutive positions of ONE
    // XCD's queue and meet in its L2: for a row-parallel product the column tiles and batch
    // segments of a row block (inner), one row block per outer step; for a split contraction
    // (weight gradient) every tile and segment of one split (they share that split's rows of both
    // operands), one split per outer step.
    const int n_batch = p.batch ? p.n_seg : 1;
    const int64_t inner = p.nt * n_batch * (p.partial ? p.mt : 1);
    const int64_t n_outer = p.partial ? p.n_split : p.mt;
    const int64_t xcd = blockIdx.x % 8, jq = blockIdx.x / 8;
    const int64_t in_idx = jq % inner, outer = (jq / inner) * 8 + xcd;
    if (outer >= n_outer) return;
    const int s0 = p.batch ? static_cast<int>(in_idx % n_batch) : 0;
    const int64_t rest = in_idx / n_batch;
    const int64_t n0 = (rest % p.nt) * BN;
    const int64_t m0 = (p.partial ? rest / p.nt : outer) * BM;
    const int64_t split = p.partial ? outer : 0;
    const GemmSeg &out_seg = p.seg[s0];
    if (m0 >= out_seg.M || n0 >= out_seg.N) return; // uniform per workgroup (smaller segment of a batch)
    const int s_end = p.batch ? s0 + 1 : p.n_seg;
    const int rows_a = static_cast<int>(min(out_seg.M - m0, static_cast<int64_t>(BM)));
    const int rows_b = static_cast<int>(min(out_seg.N - n0, static_cast<int64_t>(BN)));

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    TileLoader<SA_T, CT, A_RC, BM, NT, VEC, BK> la;
    TileLoader<SB_T, CT, B_RC, BN, NT, VEC, BK> lb;

    // The tile sequence runs over the k range of this split in every segment of the block.
    // (ls, lk, lend) describe the tile whose loads are issued next.
    const int64_t kb = split * p.k_per_split;
    int ls = s0 - 1;
    int64_t lk = 0, lend = 0;
    auto next_segment = [&]() -> bool {
        for (++ls; ls < s_end; ++ls) {
            const GemmSeg &g = p.seg[ls];
            lend = min(g.K, kb + p.k_per_split);
            if (kb < lend) {
                lk = kb;
                la.init(static_cast<const SA_T *>(g.A), g.lda, m0, kb, tid);
                lb.init(static_cast<const SB_T *>(g.B), g.ldb, n0, kb, tid);
                return true;
            }
        }
        return false;
    };
    auto issue = [&]() {
        const int k_left = static_cast<int>(min(lend - lk, static_cast<int64_t>(BK)));
        la.load(rows_a, k_left, tid);
        lb.load(rows_b, k_left, tid);
        lk += BK;
    };
    bool have = next_segment();
    if (have) issue();
    while (have) {
        __syncthreads(); // previous tile fully consumed
        la.store(As, tid);
        lb.store(Bs, tid);
        if constexpr (B_SPLIT) lb.store_residual(Bs_lo, tid);
        __syncthreads();
        // start the next tile's loads; they complete behind the MFMAs below
        have = lk < lend || next_segment();
        if (have) issue();
        if constexpr (sizeof(CT) == 4) {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 8) {
                float a[2][4], b[2][4];
#pragma unroll
                for (int i = 0; i < 2; ++i) frag_f32<A_RC, BM, BK>(As, wm + i * 32 + l32, kk, half, a[i]);
#pragma unroll
                for (int j = 0; j < 2; ++j) frag_f32<B_RC, BN, BK>(Bs, wn + j * 32 + l32, kk, half, b[j]);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[j][t], acc[i][j], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK; kk += 16) {
                union Frag { uint4 u; bf16x8 v; } a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i].u = frag_bf16<A_RC, BM, BK>(As, wm + i * 32 + l32, kk, half);
#pragma unroll
                for (int j = 0; j < 2; ++j) b[j].u = frag_bf16<B_RC, BN, BK>(Bs, wn + j * 32 + l32, kk, half);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
                if constexpr (B_SPLIT) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) b[j].u = frag_bf16<B_RC, BN, BK>(Bs_lo, wn + j * 32 + l32, kk, half);
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[j].v, acc[i][j], 0, 0, 0);
                }
            }
        }
    }

    // epilogue: accumulator register v of lane (half, l32) is C[8*(v/4) + 4*half + v%4][l32] of its 32x32 tile
    float *C = out_seg.C + (p.partial ? split * out_seg.M * out_seg.ldc : 0);
    const bool direct = !p.partial;
    const bool plain = !direct || (!p.row_scale && p.beta == 0.f && !p.relu);
    const bool interior = rows_a == BM && rows_b == BN;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int nl = wn + j * 32 + l32;
            float *col = C + (m0 + wm + i * 32 + 4 * half) * out_seg.ldc + n0 + nl;
            if (p.out_bf16) { // bf16 output: same element mapping, 16-bit stores
                if (nl >= rows_b) continue;
                bf16_t *hcol = reinterpret_cast<bf16_t *>(out_seg.C) + (m0 + wm + i * 32 + 4 * half) * out_seg.ldc + n0 + nl;
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (wm + i * 32 + 8 * (v / 4) + 4 * half + (v % 4) < rows_a)
                        hcol[(8 * (v / 4) + (v % 4)) * out_seg.ldc] = to_bf16(acc[i][j][v]);
                continue;
            }
            if (interior && plain) {
#pragma unroll
                for (int v = 0; v < 16; ++v) col[(8 * (v / 4) + (v % 4)) * out_seg.ldc] = acc[i][j][v];
                continue;
            }
            if (nl >= rows_b) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ml = wm + i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (ml >= rows_a) continue;
                float val = acc[i][j][v];
                float *o = col + (8 * (v / 4) + (v % 4)) * out_seg.ldc;
                if (direct) {
                    if (p.row_scale) val *= p.row_scale[m0 + ml];
                    if (p.beta != 0.f) val += p.beta * *o;
                    if (p.relu) val = fmaxf(val, 0.f);
                }
                *o = val;
            }
        }
}

// out[m, n] = beta * out[m, n] + sum over splits (in split order) of part[s][m][n], for every segment of
// a batched weight gradient in one launch (blockIdx.y = segment)
struct SplitSegs { // passed by value
    const float *part[kMaxSeg];
    float *out[kMaxSeg];
    int64_t M[kMaxSeg], ldo[kMaxSeg];
};
__global__ void __launch_bounds__(256) splitk_reduce_kernel(SplitSegs g, int n_split, int64_t N, float beta)
{
    const int seg = blockIdx.y;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t total = g.M[seg] * N;
    if (t >= total) return;
    const float *part = g.part[seg];
    const int64_t m = t / N, n = t % N;
    float a = 0.f;
    int s = 0;
    for (; s + 8 <= n_split; s += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = part[static_cast<int64_t>(s + u) * total + t];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += v[u];
    }
    for (; s < n_split; ++s) a += part[static_cast<int64_t>(s) * total + t];
    float *o = g.out[seg] + m * g.ldo[seg] + n;
    *o = (beta != 0.f) ? beta * *o + a : a;
}

// out[n][k] = W[k][n]: bf16 weight matrices laid out k-contiguous, the form the direct-to-LDS
// pipeline can copy into LDS as is (an n-contiguous bf16 operand would need pair interleaving).
// blockIdx.z picks the matrix: the weights of every segment of a product in one launch.
struct PackSegs {
    const bf16_t *W[kMaxSeg];
    bf16_t *out[kMaxSeg];
    int64_t ldw[kMaxSeg];
    int K[kMaxSeg], ld_out[kMaxSeg];
};
__global__ void __launch_bounds__(256) pack_weight_kernel(PackSegs q, int N)
{
    __shared__ bf16_t tile[32][33];
    const int s = blockIdx.z;
    const bf16_t *W = q.W[s];
    bf16_t *out = q.out[s];
    const int64_t ldw = q.ldw[s];
    const int K = q.K[s], ld_out = q.ld_out[s];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5; // 32 x 8
    const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    if (k0 >= ld_out) return; // uniform per workgroup: a narrower matrix of the launch
    for (int r = ty; r < 32; r += 8)
        tile[r][tx] = (k0 + r < K && n0 + tx < N) ? W[static_cast<int64_t>(k0 + r) * ldw + n0 + tx] : bf16_t(0);
    __syncthreads();
    for (int r = ty; r < 32; r += 8)
        if (n0 + r < N && k0 + tx < ld_out) out[static_cast<int64_t>(n0 + r) * ld_out + k0 + tx] = (k0 + tx < K) ? tile[tx][r] : bf16_t(0);
}

// ---- host side -------------------------------------------------------------------------------------

static void gemm_cost(const GemmParams &p, heta_dtype a_dt, heta_dtype b_dt, double *bytes, double *flops);
// test hook: route every projection through the register-staged kernel
static bool g_force_staged = false;

static bool vec_ok(const void *ptr, int64_t ld, heta_dtype dt)
{
    return aligned16(ptr) && (ld * (int64_t)dtype_size(dt)) % 16 == 0;
}

template <typename CT, typename SA_T, bool A_RC, typename SB_T, bool B_RC, int WN, bool VEC>
static heta_status launch_gemm(GemmParams &p, hipStream_t st, int bk)
{
    constexpr int BN = 64 * WN;
    int64_t mt = 0, nt = 0;
    double bytes = 0, flops = 0;
    gemm_cost(p, sizeof(SA_T) == 4 ? HETA_F32 : HETA_BF16, sizeof(SB_T) == 4 ? HETA_F32 : HETA_BF16, &bytes, &flops);
    for (int s = 0; s < p.n_seg; ++s) {
        mt = std::max(mt, (p.seg[s].M + BM - 1) / BM);
        nt = std::max(nt, (p.seg[s].N + BN - 1) / BN);
    }
    p.mt = mt;
    p.nt = nt;
    const int64_t inner = nt * (p.batch ? p.n_seg : 1) * (p.partial ? mt : 1);
    const int64_t n_outer = p.partial ? std::max(1, p.n_split) : mt;
    const int64_t blocks = (n_outer + 7) / 8 * 8 * inner;
    if (blocks <= 0) return HETA_OK;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "projection: matrix too large for one launch");
    ProfScope prof(sizeof(CT) == 4 ? (p.partial ? "gemm_wgrad_f32" : "gemm_f32") : (p.partial ? "gemm_wgrad_bf16" : "gemm_bf16"),
                   st, bytes, flops);
    if constexpr (sizeof(CT) == 2 && A_RC && B_RC && sizeof(SB_T) == 4) {
        if (p.split_b) {
            hipLaunchKernelGGL((gemm_kernel<CT, SA_T, A_RC, SB_T, B_RC, WN, VEC, 64, true>), dim3((unsigned)blocks), dim3(128 * WN), 0, st, p);
            HETA_LAUNCH_CHECK("gemm_kernel");
            return HETA_OK;
        }
    }
    if (sizeof(CT) == 2 && A_RC && B_RC && bk == 64)
        hipLaunchKernelGGL((gemm_kernel<CT, SA_T, A_RC, SB_T, B_RC, WN, VEC, (sizeof(CT) == 2 && A_RC && B_RC) ? 64 : 32>),
                           dim3((unsigned)blocks), dim3(128 * WN), 0, st, p);
    else
        hipLaunchKernelGGL((gemm_kernel<CT, SA_T, A_RC, SB_T, B_RC, WN, VEC, 32>), dim3((unsigned)blocks), dim3(128 * WN), 0, st, p);
    HETA_LAUNCH_CHECK("gemm_kernel");
    return HETA_OK;
}

// work and algorithmic traffic of a launch: every distinct operand once, every output once
// (twice when accumulating)
static void gemm_cost(const GemmParams &p, heta_dtype a_dt, heta_dtype b_dt, double *bytes, double *flops)
{
    *bytes = 0;
    *flops = 0;
    const int n_out = p.batch ? p.n_seg : 1;
    for (int s = 0; s < p.n_seg; ++s) {
        const GemmSeg &g = p.seg[s];
        *flops += 2.0 * g.M * g.N * g.K;
        bool a_seen = false, b_seen = false;
        for (int q = 0; q < s; ++q) {
            a_seen = a_seen || p.seg[q].A == g.A;
            b_seen = b_seen || p.seg[q].B == g.B;
        }
        if (!a_seen) *bytes += static_cast<double>(g.M) * g.K * dtype_size(a_dt);
        if (!b_seen) *bytes += static_cast<double>(g.K) * g.N * dtype_size(b_dt);
        if (s < n_out) *bytes += static_cast<double>(g.M) * g.N * (p.out_bf16 ? 2.0 : 4.0) * ((p.beta != 0.f && !p.partial) ? 2.0 : 1.0);
    }
}

template <bool A_RC, bool B_RC>
static heta_status dispatch_gemm(GemmParams &p, heta_dtype a_dt, heta_dtype b_dt, hipStream_t st, int bk = 32)
{
    if (!g_force_staged) {
        // the direct-to-LDS pipeline takes every launch whose operands have 16-byte rows
        double bytes, flops;
        gemm_cost(p, a_dt, b_dt, &bytes, &flops);
        const bool f32 = a_dt == HETA_F32 && b_dt == HETA_F32;
        const char *name = f32 ? (p.partial ? "gemm_wgrad_f32" : "gemm_f32") : (p.partial ? "gemm_wgrad_bf16" : "gemm_bf16");
        bool handled = false;
        heta_status e = launch_gemm_direct(p, a_dt, b_dt, A_RC, B_RC, st, name, bytes, flops, &handled);
        if (e != HETA_OK || handled) return e;
    }
    int64_t n_max = 0;
    bool vec = true; // 128-bit loads need every operand of the launch to qualify
    for (int s = 0; s < p.n_seg; ++s) {
        vec = vec && vec_ok(p.seg[s].A, p.seg[s].lda, a_dt) && vec_ok(p.seg[s].B, p.seg[s].ldb, b_dt);
        n_max = std::max(n_max, p.seg[s].N);
    }
    const bool wide = n_max > 128;
#define HETA_GEMM(CT, SA, SB)                                                                                   \
    return wide ? (vec ? launch_gemm<CT, SA, A_RC, SB, B_RC, 4, true>(p, st, bk)                                    \
                       : launch_gemm<CT, SA, A_RC, SB, B_RC, 4, false>(p, st, bk))                                  \
                : (vec ? launch_gemm<CT, SA, A_RC, SB, B_RC, 2, true>(p, st, bk)                                    \
                       : launch_gemm<CT, SA, A_RC, SB, B_RC, 2, false>(p, st, bk))
    if (a_dt == HETA_F32 && b_dt == HETA_F32) { HETA_GEMM(float, float, float); }
    if (a_dt == HETA_F32 && b_dt == HETA_BF16) { HETA_GEMM(bf16_t, float, bf16_t); }
    if (a_dt == HETA_BF16 && b_dt == HETA_F32) { HETA_GEMM(bf16_t, bf16_t, float); }
    HETA_GEMM(bf16_t, bf16_t, bf16_t);
#undef HETA_GEMM
}

static bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

// the handle's buffer for rewritten weight matrices holds at least `bytes`
static heta_status ensure_pack(heta_graph *owner, size_t bytes)
{
    if (bytes <= owner->pack_bytes) return HETA_OK;
    if (owner->d_pack) {
        HETA_HIP(hipDeviceSynchronize()); // earlier readers
        scratch_free(owner->d_pack);
    }
    owner->d_pack = nullptr;
    owner->pack_bytes = 0;
    HETA_HIP(scratch_alloc(&owner->d_pack, bytes * 2));
    owner->pack_bytes = bytes * 2;
    return HETA_OK;
}

// fp32 x fp32 products through a graph handle whose B operands are weight matrices (forward, input gradient):
// the weights are rewritten once per launch as the three bf16 terms the product is fed with, into the handle's
// packing buffer, and the k loop splits only A.  Launches the direct pipeline would not take, or would give its
// small tiles, are left as they are.  trans: B(k, n) = W[n*ldb + k].
static heta_status pack_f32_weights(heta_graph *owner, GemmParams &p, int trans, hipStream_t st)
{
    if (!owner || g_force_staged || g_f32_native || p.partial || gemm_direct_small(p)) return HETA_OK;
    size_t bytes = 0;
    for (int s = 0; s < p.n_seg; ++s) {
        const GemmSeg &g = p.seg[s];
        if (!aligned16(g.A) || (g.lda * 4) % 16 || !aligned16(g.B) || (g.ldb * 4) % 16) return HETA_OK;
        bytes += (split3_weight_bytes(g.K, g.N) + 255) / 256 * 256;
    }
    heta_status e = ensure_pack(owner, bytes);
    if (e != HETA_OK) return e;
    char *dst = static_cast<char *>(owner->d_pack);
    for (int s = 0; s < p.n_seg; ++s) {
        GemmSeg &g = p.seg[s];
        e = pack_split3_weights(static_cast<const float *>(g.B), g.ldb, g.K, g.N, trans, dst, &g, st);
        if (e != HETA_OK) return e;
        dst += (split3_weight_bytes(g.K, g.N) + 255) / 256 * 256;
    }
    return HETA_OK;
}

// out = beta*out + row_scale * sum_s in_s . (W_s or W_s^T)
static heta_status project_impl(int64_t n_rows, int n_seg, const void *const *ins, heta_dtype in_dt, const int64_t *ld_in,
                                const int32_t *d_in, const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w,
                                int32_t d_out, int32_t transW, const float *row_scale, int relu, void *out,
                                int64_t ld_out, float beta, hipStream_t st, const char *who, heta_graph *pack_owner = nullptr,
                                heta_dtype out_dt = HETA_F32, void *const *outs = nullptr, const int64_t *ld_outs = nullptr)
{
    // outs != nullptr: n_seg independent products, one output each (out / ld_out unused); else one summed output
    if (outs && n_seg >= 1) {
        if (!ld_outs) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
        for (int s = 0; s < n_seg && s < kMaxSeg; ++s) {
            if (!outs[s]) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
            if (ld_outs[s] < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
            if (misaligned(outs[s], dtype_size(valid_dtype(out_dt) ? out_dt : HETA_F32)))
                return fail(HETA_ERR_INVALID_ARG, "%s: out not aligned to its element size", who);
        }
        out = outs[0];
        ld_out = ld_outs[0];
    }
    if (!ins || !Ws || !out || !ld_in || !d_in || !ld_w) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n_seg < 1 || n_seg > kMaxSeg) return fail(HETA_ERR_INVALID_ARG, "%s: between 1 and %d inputs", who, kMaxSeg);
    if (!valid_dtype(in_dt) || !valid_dtype(w_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    for (int s = 0; s < n_seg; ++s)
        if (!ins[s] || !Ws[s]) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n_rows < 0 || d_out <= 0 || ld_out < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
    if (!valid_dtype(out_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (misaligned(out, dtype_size(out_dt))) return fail(HETA_ERR_INVALID_ARG, "%s: out not aligned to its element size", who);
    if (out_dt == HETA_BF16 && (beta != 0.f || row_scale || relu))
        return fail(HETA_ERR_UNSUPPORTED, "%s: a bf16 output takes no beta, row_scale or activation", who);
    GemmParams p{};
    p.out_bf16 = out_dt == HETA_BF16;
    for (int s = 0; s < n_seg; ++s) {
        if (d_in[s] <= 0 || ld_in[s] < d_in[s] || ld_w[s] < (transW ? d_in[s] : d_out))
            return fail(HETA_ERR_SHAPE, "%s: leading dimension smaller than the row width", who);
        if (misaligned(ins[s], dtype_size(in_dt)) || misaligned(Ws[s], dtype_size(w_dt)))
            return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", who);
        GemmSeg &g = p.seg[s];
        g.A = ins[s];
        g.lda = ld_in[s];
        g.B = Ws[s];
        g.ldb = ld_w[s];
        g.C = static_cast<float *>(outs ? outs[s] : out); // typed by p.out_bf16 in the kernels' epilogue
        g.ldc = outs ? ld_outs[s] : ld_out;
        g.M = n_rows;
        g.N = d_out;
        g.K = d_in[s];
    }
    if (n_rows == 0) return HETA_OK;
    p.n_seg = n_seg;
    p.batch = outs ? 1 : 0;
    p.row_scale = row_scale;
    p.beta = beta;
    p.relu = relu;
    p.k_per_split = int64_t(1) << 40;
    p.n_split = 1;
    p.partial = 0;
    if (in_dt == HETA_F32 && w_dt == HETA_F32) {
        heta_status pe = pack_f32_weights(pack_owner, p, transW, st);
        if (pe != HETA_OK) return pe;
    }
    // B[k][n] = W[k][n] is n-contiguous (r-contiguous in the loader's terms); W^T is k-contiguous
    if (transW) return dispatch_gemm<false, false>(p, in_dt, w_dt, st);
    if (pack_owner && !g_force_staged && w_dt == HETA_BF16) {
        // forward with bf16 weights and a graph handle: the small W_r are first rewritten k-contiguous into the
        // handle's packing buffer, so that both operands can stream into LDS without a register stage (fp32
        // inputs, an inner layer's embeddings, are rounded to bf16 when their fragments are read, as the
        // register-staged kernel rounds them when it stages them)
        bool ok = true;
        size_t bytes = 0;
        for (int s = 0; s < n_seg; ++s) {
            ok = ok && aligned16(ins[s]) && (ld_in[s] * static_cast<int64_t>(dtype_size(in_dt))) % 16 == 0;
            bytes += static_cast<size_t>(d_out) * ((d_in[s] + 7) / 8 * 8) * 2 + 256;
        }
        if (ok) {
            heta_status pe = ensure_pack(pack_owner, bytes);
            if (pe != HETA_OK) return pe;
            char *dst = static_cast<char *>(pack_owner->d_pack);
            PackSegs q{};
            int ldp_max = 0;
            for (int s = 0; s < n_seg; ++s) {
                const int ldp = (d_in[s] + 7) / 8 * 8;
                q.W[s] = static_cast<const bf16_t *>(Ws[s]);
                q.out[s] = reinterpret_cast<bf16_t *>(dst);
                q.ldw[s] = ld_w[s];
                q.K[s] = d_in[s];
                q.ld_out[s] = ldp;
                ldp_max = std::max(ldp_max, ldp);
                p.seg[s].B = dst;
                p.seg[s].ldb = ldp;
                dst += (static_cast<size_t>(d_out) * ldp * 2 + 255) / 256 * 256;
            }
            hipLaunchKernelGGL(pack_weight_kernel, dim3((d_out + 31) / 32, (ldp_max + 31) / 32, n_seg), dim3(256), 0, st, q, d_out);
            HETA_LAUNCH_CHECK("pack_weight_kernel");
            return dispatch_gemm<false, false>(p, in_dt, w_dt, st);
        }
    }
    return dispatch_gemm<false, true>(p, in_dt, w_dt, st);
}

// dW_s = beta*dW_s + in_s^T . gout over n_rows graph rows, all s in one launch
static heta_status wgrad_impl(heta_graph *g, int64_t n_rows, int n_seg, const void *const *ins, heta_dtype in_dt,
                              const int64_t *ld_in, const int32_t *d_in, const float *gout, int64_t ld_go, int32_t d_out,
                              float *const *dW, const int64_t *ld_dw, float beta, hipStream_t st, const char *who,
                              int gout_two_terms = 0, const float *const *gouts = nullptr, const int64_t *ld_gos = nullptr)
{
    // gouts != nullptr: every segment has its own gradient operand (gout / ld_go unused)
    if (gouts && n_seg >= 1) {
        if (!ld_gos) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
        for (int s = 0; s < n_seg && s < kMaxSeg; ++s) {
            if (!gouts[s]) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
            if (ld_gos[s] < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
            if (misaligned(gouts[s], 4)) return fail(HETA_ERR_INVALID_ARG, "%s: gout not 4-byte aligned", who);
        }
        gout = gouts[0];
        ld_go = ld_gos[0];
    }
    if (!g || !ins || !gout || !dW || !ld_in || !d_in || !ld_dw) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n_seg < 1 || n_seg > kMaxSeg) return fail(HETA_ERR_INVALID_ARG, "%s: between 1 and %d inputs", who, kMaxSeg);
    if (!valid_dtype(in_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (d_out <= 0 || ld_go < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
    if (misaligned(gout, 4)) return fail(HETA_ERR_INVALID_ARG, "%s: gout not 4-byte aligned", who);
    GemmParams p{};
    int64_t out_elems = 0, tiles = 0;
    // bf16 inputs with 16-byte rows take the all-direct kernel: 128 x 128 tiles, three workgroups per CU (wider and
    // taller tiles below)
    bool bf16_direct = in_dt == HETA_BF16 && !g_force_staged;
    for (int s = 0; s < n_seg && bf16_direct; ++s)
        bf16_direct = ins[s] && vec_ok(ins[s], ld_in[s], in_dt) && vec_ok(gouts ? gouts[s] : gout, gouts ? ld_gos[s] : ld_go, HETA_F32);
    // fp32 inputs on the direct pipeline (six bf16 terms per product): 128 x 128 tiles, three workgroups per CU
    bool f32_terms = in_dt == HETA_F32 && !g_force_staged && !g_f32_native;
    for (int s = 0; s < n_seg && f32_terms; ++s)
        f32_terms = ins[s] && vec_ok(ins[s], ld_in[s], in_dt) && vec_ok(gouts ? gouts[s] : gout, gouts ? ld_gos[s] : ld_go, HETA_F32);
    int d_in_max = 0;
    for (int s = 0; s < n_seg; ++s) d_in_max = std::max(d_in_max, d_in[s]);
    const bool tall = bf16_direct && d_in_max > 128; // 320 x 128 tiles, one 512-thread workgroup per CU
    const bool wide_direct = bf16_direct && !tall && d_out > 128; // 128 x 256 tiles, two 512-thread workgroups per CU
    const bool tall_wide = tall && d_out > 128;                   // 320 x 256 or 256 x 256 tiles, one workgroup per CU
    const int BN = (d_out > 128 && (!bf16_direct || wide_direct || tall_wide) && !f32_terms) ? 256 : 128;
    int BMt = tall ? 320 : BM;
    if (tall_wide) { // the tile height the launch will choose (wgrad_tile_rows): the one that pads the input columns less
        int64_t pad320 = 0, pad256 = 0;
        for (int s = 0; s < n_seg; ++s) {
            pad320 += (static_cast<int64_t>(d_in[s]) + 319) / 320 * 320;
            pad256 += (static_cast<int64_t>(d_in[s]) + 255) / 256 * 256;
        }
        if (pad256 < pad320) BMt = 256;
    }
    for (int s = 0; s < n_seg; ++s) {
        if (!ins[s] || !dW[s]) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
        if (d_in[s] <= 0 || ld_in[s] < d_in[s] || ld_dw[s] < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
        if (misaligned(ins[s], dtype_size(in_dt)) || misaligned(dW[s], 4))
            return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", who);
        GemmSeg &q = p.seg[s];
        q.A = ins[s];      // A[m = column of `in`][k = graph row] : r-contiguous
        q.lda = ld_in[s];
        q.B = gouts ? gouts[s] : gout; // B[k = graph row][n] : r-contiguous
        q.ldb = gouts ? ld_gos[s] : ld_go;
        q.M = d_in[s];
        q.N = d_out;
        q.K = n_rows;
        q.ldc = d_out;
        out_elems += static_cast<int64_t>(d_in[s]) * d_out;
        tiles += ((d_in[s] + BMt - 1) / BMt) * ((d_out + BN - 1) / BN);
    }
    // Split the graph rows so that the workgroups fill the chip exactly once and never spill into a
    // second, nearly empty round.  Workgroups are dealt round-robin to the 8 XCDs (32 CUs each) and
    // the kernel keeps the `tiles` output tiles of one split on one XCD, so a split costs `tiles`
    // workgroup slots of its XCD: 2 resident 512-thread workgroups per CU (3 or 4 of 256 threads).
    // Each split keeps at least 4 k-tiles (a few thousand graph rows still spread over the chip: a
    // workgroup's k-tiles are latency-bound when few workgroups run).
    const int64_t BK = in_dt == HETA_F32 ? 32 : 64;
    const int64_t k_tiles = (n_rows + BK - 1) / BK;
    const int64_t slots_per_xcd = 32 * (tall ? 1 : wide_direct ? 2 : (bf16_direct || f32_terms) ? 3 : (d_out > 128 ? 2 : (in_dt == HETA_F32 ? 3 : 4)));
    // a split's workgroups are (largest segment's row tiles) x (column tiles) x (segments), all on one XCD
    int64_t mt_max = 1;
    for (int s = 0; s < n_seg; ++s) mt_max = std::max<int64_t>(mt_max, (d_in[s] + BMt - 1) / BMt);
    const int64_t slots_per_split = std::max<int64_t>(tiles, mt_max * ((d_out + BN - 1) / BN) * n_seg);
    const int64_t splits_per_xcd = std::max<int64_t>(1, slots_per_xcd / std::max<int64_t>(1, slots_per_split));
    int64_t n_split = std::max<int64_t>(1, std::min<int64_t>((k_tiles + 3) / 4, 8 * splits_per_xcd));
    const int64_t tiles_per_split = std::max<int64_t>(1, (k_tiles + n_split - 1) / n_split);
    n_split = std::max<int64_t>(1, (k_tiles + tiles_per_split - 1) / tiles_per_split);
    heta_status e = ensure_workspace(g, static_cast<size_t>(n_split) * out_elems * sizeof(float));
    if (e != HETA_OK) return e;
    float *ws = static_cast<float *>(g->d_ws);
    int64_t off = 0;
    for (int s = 0; s < n_seg; ++s) {
        p.seg[s].C = ws + off;
        off += n_split * static_cast<int64_t>(d_in[s]) * d_out;
    }
    p.n_seg = n_seg;
    p.batch = 1;
    p.row_scale = nullptr;
    p.beta = 0.f;
    p.relu = 0;
    p.k_per_split = tiles_per_split * BK;
    p.n_split = static_cast<int>(n_split);
    p.partial = 1;
    p.split_b = (gout_two_terms && in_dt == HETA_BF16) ? 1 : 0;
    e = dispatch_gemm<true, true>(p, in_dt, HETA_F32, st, static_cast<int>(BK));
    if (e != HETA_OK) return e;
    {
        SplitSegs segs{};
        int64_t total_max = 0;
        double bytes = 0;
        for (int s = 0; s < n_seg; ++s) {
            const int64_t total = static_cast<int64_t>(d_in[s]) * d_out;
            segs.part[s] = static_cast<const float *>(p.seg[s].C);
            segs.out[s] = dW[s];
            segs.M[s] = d_in[s];
            segs.ldo[s] = ld_dw[s];
            total_max = std::max(total_max, total);
            bytes += (n_split + 1.0) * total * 4.0;
        }
        ProfScope prof("splitk_reduce_kernel", st, bytes, 0);
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((total_max + 255) / 256), (unsigned)n_seg), dim3(256), 0, st, segs,
                           static_cast<int>(n_split), (int64_t)d_out, beta);
        HETA_LAUNCH_CHECK("splitk_reduce_kernel");
    }
    return HETA_OK;
}

static heta_status check_type(const heta_graph *g, int32_t t, const char *who)
{
    if (!g) return fail(HETA_ERR_INVALID_ARG, "%s: graph is NULL", who);
    if (t < 0 || t >= (int32_t)g->ntypes.size()) return fail(HETA_ERR_INVALID_ARG, "%s: node type %d out of range", who, t);
    return HETA_OK;
}

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_projection_f32_native(int32_t on)
{
    g_f32_native = on != 0;
    return HETA_OK;
}

heta_status heta_projection_force_staged(int32_t on)
{
    g_force_staged = on != 0;
    return HETA_OK;
}

heta_status heta_project(int64_t n_rows, const void *in, heta_dtype in_dt, int64_t ld_in, int32_t d_in,
                         const void *W, heta_dtype w_dt, int64_t ld_w, int32_t d_out, int32_t transW,
                         const float *row_scale, void *out, heta_dtype out_dt, int64_t ld_out, float beta,
                         void *hip_stream)
{
    return project_impl(n_rows, 1, &in, in_dt, &ld_in, &d_in, &W, w_dt, &ld_w, d_out, transW, row_scale, 0, out, ld_out,
                        beta, as_stream(hip_stream), "heta_project", nullptr, out_dt);
}

heta_status heta_rel_project(heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                             int64_t ld_in, int32_t d_in, const void *W, heta_dtype w_dt, int64_t ld_w,
                             int32_t d_out, int32_t transW, const float *row_scale, void *out,
                             heta_dtype out_dt, int64_t ld_out, float beta, void *hip_stream)
{
    if (!g) return fail(HETA_ERR_INVALID_ARG, "heta_rel_project: graph is NULL");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_project: relation %d out of range", rel);
    return project_impl(g->rels[rel].n_dst, 1, &in, in_dt, &ld_in, &d_in, &W, w_dt, &ld_w, d_out, transW, row_scale, 0,
                        out, ld_out, beta, as_stream(hip_stream), "heta_rel_project", g, out_dt);
}

heta_status heta_rel_project_wgrad(heta_graph *g, int32_t rel, const void *in, heta_dtype in_dt,
                                   int64_t ld_in, int32_t d_in, const float *gout, int64_t ld_go,
                                   int32_t d_out, float *dW, int64_t ld_dw, float beta, void *hip_stream)
{
    if (!g) return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: null argument");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_rel_project_wgrad: relation %d out of range", rel);
    return wgrad_impl(g, g->rels[rel].n_dst, 1, &in, in_dt, &ld_in, &d_in, gout, ld_go, d_out, &dW, &ld_dw, beta,
                      as_stream(hip_stream), "heta_rel_project_wgrad");
}

heta_status heta_project_batch(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt, const int64_t *ld_in,
                               const int32_t *d_in, const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w, int32_t d_out,
                               int32_t transW, void *const *outs, heta_dtype out_dt, const int64_t *ld_out, void *hip_stream)
{
    if (!outs || !ld_out) return fail(HETA_ERR_INVALID_ARG, "heta_project_batch: null argument");
    return project_impl(n_rows, n, ins, in_dt, ld_in, d_in, Ws, w_dt, ld_w, d_out, transW, nullptr, 0, nullptr, 0, 0.f,
                        as_stream(hip_stream), "heta_project_batch", g, out_dt, outs, ld_out);
}

heta_status heta_project_sum(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt, const int64_t *ld_in,
                             const int32_t *d_in, const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w, int32_t d_out,
                             int32_t transW, float *out, int64_t ld_out, float beta, void *hip_stream)
{
    return project_impl(n_rows, n, ins, in_dt, ld_in, d_in, Ws, w_dt, ld_w, d_out, transW, nullptr, 0, out, ld_out, beta,
                        as_stream(hip_stream), "heta_project_sum", g);
}

heta_status heta_project_wgrad_batch(heta_graph *g, int64_t n_rows, int32_t n, const void *const *ins, heta_dtype in_dt,
                                     const int64_t *ld_in, const int32_t *d_in, const float *const *gouts,
                                     const int64_t *ld_go, int32_t d_out, float *const *dW, const int64_t *ld_dw, float beta,
                                     int32_t gout_two_terms, void *hip_stream)
{
    if (!g || !gouts || !ld_go) return fail(HETA_ERR_INVALID_ARG, "heta_project_wgrad_batch: null argument");
    if (n_rows < 0) return fail(HETA_ERR_SHAPE, "heta_project_wgrad_batch: negative row count");
    return wgrad_impl(g, n_rows, n, ins, in_dt, ld_in, d_in, nullptr, 0, d_out, dW, ld_dw, beta, as_stream(hip_stream),
                      "heta_project_wgrad_batch", gout_two_terms, gouts, ld_go);
}

heta_status heta_cross_rel_project(heta_graph *g, int32_t dst_type, int32_t n, const void *const *ins,
                                   heta_dtype in_dt, const int64_t *ld_in, const int32_t *d_in,
                                   const void *const *Ws, heta_dtype w_dt, const int64_t *ld_w, int32_t d_out,
                                   heta_act act, float *out, int64_t ld_out, float beta, void *hip_stream)
{
    heta_status e = check_type(g, dst_type, "heta_cross_rel_project");
    if (e != HETA_OK) return e;
    if (act != HETA_ACT_NONE && act != HETA_ACT_RELU) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_project: bad act");
    return project_impl(g->ntypes[dst_type].num_nodes, n, ins, in_dt, ld_in, d_in, Ws, w_dt, ld_w, d_out, 0, nullptr,
                        act == HETA_ACT_RELU, out, ld_out, beta, as_stream(hip_stream), "heta_cross_rel_project", g);
}

heta_status heta_cross_rel_project_bwd(const heta_graph *g, int32_t dst_type, int32_t n, const float *gout,
                                       int64_t ld_go, int32_t d_out, const void *const *Ws, heta_dtype w_dt,
                                       const int64_t *ld_w, const int32_t *d_in, void *const *dM,
                                       heta_dtype dm_dt, const int64_t *ld_dm, void *hip_stream)
{
    const char *who = "heta_cross_rel_project_bwd";
    heta_status e = check_type(g, dst_type, who);
    if (e != HETA_OK) return e;
    if (!gout || !Ws || !ld_w || !d_in || !dM || !ld_dm) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
    if (n < 1 || n > kMaxSeg) return fail(HETA_ERR_INVALID_ARG, "%s: between 1 and %d relations", who, kMaxSeg);
    if (!valid_dtype(w_dt) || !valid_dtype(dm_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", who);
    if (d_out <= 0 || ld_go < d_out) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
    if (misaligned(gout, 4)) return fail(HETA_ERR_INVALID_ARG, "%s: gout not 4-byte aligned", who);
    const int64_t n_rows = g->ntypes[dst_type].num_nodes;
    GemmParams p{};
    for (int s = 0; s < n; ++s) {
        if (!Ws[s] || !dM[s]) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", who);
        if (d_in[s] <= 0 || ld_w[s] < d_out || ld_dm[s] < d_in[s]) return fail(HETA_ERR_SHAPE, "%s: bad sizes", who);
        if (misaligned(Ws[s], dtype_size(w_dt)) || misaligned(dM[s], dtype_size(dm_dt)))
            return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", who);
        GemmSeg &q = p.seg[s];
        q.A = gout;
        q.lda = ld_go;
        q.B = Ws[s];   // B[k][n] = W[n][k]: W is [d_in, d_out] row-major, k-contiguous
        q.ldb = ld_w[s];
        q.C = static_cast<float *>(dM[s]); // typed by p.out_bf16 in the kernels' epilogue
        q.ldc = ld_dm[s];
        q.M = n_rows;
        q.N = d_in[s];
        q.K = d_out;
    }
    if (n_rows == 0) return HETA_OK;
    p.n_seg = n;
    p.batch = 1;
    p.row_scale = nullptr;
    p.beta = 0.f;
    p.relu = 0;
    p.k_per_split = int64_t(1) << 40;
    p.n_split = 1;
    p.partial = 0;
    p.out_bf16 = dm_dt == HETA_BF16;
    if (w_dt == HETA_F32) { // the handle's packing buffer is scratch memory, not part of the graph it describes
        e = pack_f32_weights(const_cast<heta_graph *>(g), p, 1, as_stream(hip_stream));
        if (e != HETA_OK) return e;
    }
    return dispatch_gemm<false, false>(p, HETA_F32, w_dt, as_stream(hip_stream));
}

heta_status heta_cross_rel_project_wgrad(heta_graph *g, int32_t dst_type, int32_t n, const void *const *ins,
                                         heta_dtype in_dt, const int64_t *ld_in, const int32_t *d_in,
                                         const float *gout, int64_t ld_go, int32_t d_out, float *const *dW,
                                         const int64_t *ld_dw, float beta, int32_t gout_two_terms, void *hip_stream)
{
    heta_status e = check_type(g, dst_type, "heta_cross_rel_project_wgrad");
    if (e != HETA_OK) return e;
    return wgrad_impl(g, g->ntypes[dst_type].num_nodes, n, ins, in_dt, ld_in, d_in, gout, ld_go, d_out, dW, ld_dw, beta,
                      as_stream(hip_stream), "heta_cross_rel_project_wgrad", gout_two_terms);
}

} // extern "C"
