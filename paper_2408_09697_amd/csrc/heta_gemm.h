// GEMM building blocks shared by the translation units that hold the projection kernels
// (not part of the ABI): problem description, LDS tile layouts, the register-staged tile
// loader and the MFMA fragment readers.
#pragma once

#include "heta_internal.h"

namespace heta {

using bf16_t = uint16_t;
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128;
// BK, the k-values per tile, is a template parameter: 32, or 64 for the bf16 weight gradient,
// whose long k loop is bound by per-tile overhead rather than by MFMA work.
constexpr int kMaxSeg = 8;

struct GemmSeg {
    const void *A;
    int64_t lda;
    const void *B;
    int64_t ldb;
    float *C;           // output of this segment (batch mode) - segment 0's is used in sum mode
    int64_t ldc;
    int64_t M, N, K;
    // optional: B rewritten as three bf16 terms (pack_split3_weights), [term][k / 8][n_pad][8 k-values]
    const void *B3;
    int32_t ko, n_pad;  // k-octets (K rounded up to 16, over 8) and columns (N rounded up to 128) of B3
};

struct GemmParams {
    GemmSeg seg[kMaxSeg];
    int n_seg;
    int batch;           // 0: C_0 (+)= sum_s A_s B_s ; 1: C_s (+)= A_s B_s for every s
    const float *row_scale;
    float beta;
    int relu;
    int split_b;         // bf16 product with an fp32 B: feed B as two bf16 terms (value = hi + lo, 16 significant bits)
    int out_bf16;        // outputs are bf16 [M][ldc] (plain stores only: no beta, scale, activation, split)
    int64_t k_per_split; // multiple of BK
    int n_split;
    int partial;         // write raw partial products [split][M][ldc] (ldc = N) instead of the output
    int64_t mt, nt;      // tile counts (maximum over the segments in batch mode)
};

__device__ __forceinline__ bf16_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return static_cast<bf16_t>((u >> 16) | 0x40u);
    return static_cast<bf16_t>((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// two fp32 values -> two bf16 in one 32-bit word (lo in the low half), round to nearest even, with the
// packed hardware convert (v_cvt_pk_bf16_f32)
typedef float floatx2_pk __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_pk __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi)
{
    const floatx2_pk f = {lo, hi};
    const bf16x2_pk h = __builtin_convertvector(f, bf16x2_pk);
    return *reinterpret_cast<const uint32_t *>(&h);
}
__device__ __forceinline__ uint32_t pack2_bf16(bf16_t lo, bf16_t hi) { return static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16); }

template <typename S, typename CT> __device__ __forceinline__ CT convert(S v);
template <> __device__ __forceinline__ float convert<float, float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t convert<float, bf16_t>(float v) { return to_bf16(v); }
template <> __device__ __forceinline__ bf16_t convert<bf16_t, bf16_t>(bf16_t v) { return v; }

// ---- LDS tile layouts ------------------------------------------------------------------------------
// A k-contiguous operand (element (r,k) at base[r*ld + k]) is kept r-major in LDS, rows of one
// tile's k-values (128 bytes) padded by 16 bytes: copied with 128-bit stores, fragments read with one 128-bit load
// (8 consecutive lanes fall on distinct banks).
// An r-contiguous operand (element (r,k) at base[k*ld + r]) is kept k-major, exactly as it lies
// in memory, so that global loads stay coalesced along r and LDS stores stay 128-bit:
//   fp32 compute: Ls[k][r]; a fragment is four 32-bit reads (lanes along r: conflict-free);
//   bf16 compute: Ls[k/2][r] of 32-bit words holding the pair (k, k+1); a fragment is four
//   32-bit reads that deliver eight consecutive k-values.
// The k index a lane supplies to an MFMA only has to agree between the A and B fragments; all
// three layouts hand lane (half, l32) the k-values kk + (4|8)*half + 0..(3|7) in order.
template <typename CT, int BK> struct LdsStride { static constexpr int value = BK + 16 / (int)sizeof(CT); };
template <typename CT, bool RC, int ROWS, int BK> struct LdsTile {
    static constexpr int elems = RC ? BK * ROWS : ROWS * LdsStride<CT, BK>::value;
};

template <bool RC, int ROWS, int BK>
__device__ __forceinline__ void frag_f32(const float *tile, int r, int kk, int half, float f[4])
{
    if (RC) {
#pragma unroll
        for (int t = 0; t < 4; ++t) f[t] = tile[(kk + 4 * half + t) * ROWS + r];
    } else {
        const float4 v = *reinterpret_cast<const float4 *>(&tile[r * LdsStride<float, BK>::value + kk + 4 * half]);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
}

template <bool RC, int ROWS, int BK>
__device__ __forceinline__ uint4 frag_bf16(const bf16_t *tile, int r, int kk, int half)
{
    if (RC) {
        const uint32_t *w = reinterpret_cast<const uint32_t *>(tile);
        const int kp = kk / 2 + 4 * half;
        return make_uint4(w[(kp + 0) * ROWS + r], w[(kp + 1) * ROWS + r], w[(kp + 2) * ROWS + r], w[(kp + 3) * ROWS + r]);
    }
    return *reinterpret_cast<const uint4 *>(&tile[r * LdsStride<bf16_t, BK>::value + kk + 8 * half]);
}

// Moves a [ROWS x BK] operand tile global -> registers -> LDS with NT threads (layouts above).
// Every thread owns a fixed set of 16-byte chunks of the tile; its global addresses are set up
// once per segment and advanced by one tile per load().  load() only issues the global loads;
// masking of ragged edges, conversion and (for bf16 pairs) interleaving happen in store().
// VEC selects 128-bit loads (rows 16-byte aligned) against element-wise loads.
template <typename S, typename CT, bool RC, int ROWS, int NT, bool VEC, int BK>
struct TileLoader {
    static constexpr bool PAIR = RC && sizeof(CT) == 2;
    static constexpr int E = 16 / (int)sizeof(S);
    static constexpr int CPR = ROWS / E;                                 // chunks along r (r-contiguous operands)
    static constexpr int ITEMS = PAIR ? (BK / 2) * CPR : ROWS * BK / E;  // work items per tile
    static constexpr int NI = (ITEMS + NT - 1) / NT;                     // items per thread
    static constexpr int LPI = PAIR ? 2 : 1;                             // global chunks per item
    static constexpr int SA = LdsStride<CT, BK>::value;
    const S *ptr[NI];
    int64_t step, ld_;
    uint4 raw[NI][LPI];
    int left[NI][LPI]; // valid elements of the chunk (0 = nothing loaded)

    __device__ __forceinline__ static int row_of(int q) { return RC ? (q % CPR) * E : q / (BK / E); }
    __device__ __forceinline__ static int k_of(int q) { return RC ? (q / CPR) * LPI : (q % (BK / E)) * E; }

    __device__ __forceinline__ void init(const S *base, int64_t ld, int64_t r0, int64_t k0, int tid)
    {
        step = RC ? BK * ld : BK;
        ld_ = ld;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = tid + NT * i;
            const int64_t gr = r0 + row_of(q), gk = k0 + k_of(q);
            ptr[i] = RC ? base + gk * ld + gr : base + gr * ld + gk;
        }
    }

    // rows_left / k_left: valid rows and k-values of this tile (may exceed the tile size)
    __device__ __forceinline__ void load(int rows_left, int k_left, int tid)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = tid + NT * i;
#pragma unroll
            for (int l = 0; l < LPI; ++l) {
                const int lr = rows_left - row_of(q), lk = k_left - (k_of(q) + l);
                const bool in = (ITEMS % NT == 0 || q < ITEMS) && lr > 0 && lk > 0;
                left[i][l] = in ? min(E, RC ? lr : lk) : 0;
                raw[i][l] = make_uint4(0u, 0u, 0u, 0u);
                if (in) {
                    const S *src = ptr[i] + (l ? ld_ : 0);
                    if (VEC) {
                        raw[i][l] = *reinterpret_cast<const uint4 *>(src);
                    } else {
                        union { uint4 u; S s[E]; } t;
                        t.u = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                        for (int j = 0; j < E; ++j) if (j < left[i][l]) t.s[j] = src[j];
                        raw[i][l] = t.u;
                    }
                }
            }
            ptr[i] += step;
        }
    }

    // second term of an fp32 operand fed as two bf16 terms: what rounding to bf16 left over, in the
    // same LDS layout as store() (pair-interleaved r-contiguous operands only)
    __device__ __forceinline__ void store_residual(CT *lds, int tid) const
    {
        static_assert(sizeof(S) == 4, "only an fp32 operand has a residual");
        if constexpr (PAIR && sizeof(S) == 4) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int q = tid + NT * i;
                if (ITEMS % NT != 0 && q >= ITEMS) continue;
                union Chunk { uint4 u; float s[E]; } t[LPI];
#pragma unroll
                for (int l = 0; l < LPI; ++l) {
                    t[l].u = raw[i][l];
                    if (VEC && left[i][l] < E) {
#pragma unroll
                        for (int j = 0; j < E; ++j) if (j >= left[i][l]) t[l].s[j] = 0.f;
                    }
                }
                const int r = row_of(q), k = k_of(q);
                uint32_t w[E];
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const float a = t[0].s[j], b = t[LPI - 1].s[j];
                    const uint32_t hi = pack2_bf16(a, b); // the pair as store() writes it
                    const float ra = a - __uint_as_float(hi << 16);
                    const float rb = b - __uint_as_float(hi & 0xffff0000u);
                    w[j] = pack2_bf16(ra, rb);
                }
                uint32_t *dst = reinterpret_cast<uint32_t *>(lds) + (k / 2) * ROWS + r;
#pragma unroll
                for (int j = 0; j < E; j += 4) *reinterpret_cast<uint4 *>(dst + j) = make_uint4(w[j], w[j + 1], w[j + 2], w[j + 3]);
            }
        }
    }

    __device__ __forceinline__ void store(CT *lds, int tid) const
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int q = tid + NT * i;
            if (ITEMS % NT != 0 && q >= ITEMS) continue;
            union Chunk { uint4 u; S s[E]; } t[LPI];
#pragma unroll
            for (int l = 0; l < LPI; ++l) {
                t[l].u = raw[i][l];
                if (VEC && left[i][l] < E) { // a chunk that straddles the edge: the load brought in padding
#pragma unroll
                    for (int j = 0; j < E; ++j) if (j >= left[i][l]) t[l].s[j] = S(0);
                }
            }
            const int r = row_of(q), k = k_of(q);
            if (PAIR) {
                uint32_t w[E];
#pragma unroll
                for (int j = 0; j < E; ++j) w[j] = pack2_bf16(t[0].s[j], t[LPI - 1].s[j]);
                uint32_t *dst = reinterpret_cast<uint32_t *>(lds) + (k / 2) * ROWS + r;
#pragma unroll
                for (int j = 0; j < E; j += 4) *reinterpret_cast<uint4 *>(dst + j) = make_uint4(w[j], w[j + 1], w[j + 2], w[j + 3]);
            } else if (RC) {
                *reinterpret_cast<uint4 *>(lds + k * ROWS + r) = t[0].u; // fp32 compute: S == CT == float
            } else if constexpr (sizeof(S) == 4 && sizeof(CT) == 2) { // fp32 -> bf16, k-contiguous: packed converts
                uint32_t w[E / 2];
#pragma unroll
                for (int j = 0; j < E / 2; ++j) w[j] = pack2_bf16(t[0].s[2 * j], t[0].s[2 * j + 1]);
                *reinterpret_cast<uint2 *>(lds + r * SA + k) = make_uint2(w[0], w[1]);
            } else {
                CT tmp[E];
#pragma unroll
                for (int j = 0; j < E; ++j) tmp[j] = convert<S, CT>(t[0].s[j]);
                CT *dst = lds + r * SA + k;
                if (sizeof(CT) * E == 16) *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(tmp);
                else *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(tmp);
            }
        }
    }
};

// The direct-to-LDS pipeline (heta_gemm_direct.hip).  Sets *handled when it launched the product;
// otherwise the caller falls back to the register-staged kernel.
extern bool g_f32_native; // test switch, see heta_test_hooks.h
// Bytes of the three-term form of a K x N fp32 operand, and the kernel that writes it: B(k, n) = W[k*ldw + n]
// (trans = 0) or W[n*ldw + k] (trans = 1); x = h + m + l in bf16, zero beyond K and N.  out must be 16-byte aligned.
size_t split3_weight_bytes(int64_t K, int64_t N);
heta_status pack_split3_weights(const float *W, int64_t ldw, int64_t K, int64_t N, int trans, void *out, GemmSeg *seg,
                                hipStream_t st);
// whether the direct pipeline would give this launch its 64 x 64 tiles (too few 128 x 128 tiles to fill the chip)
bool gemm_direct_small(const GemmParams &p);
int wgrad_tile_rows(const GemmParams &p);
heta_status launch_gemm_direct(GemmParams &p, heta_dtype a_dt, heta_dtype b_dt, bool a_rc, bool b_rc, hipStream_t st,
                               const char *name, double bytes, double flops, bool *handled);

} // namespace heta
