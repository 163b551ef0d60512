// Fused forward of one destination type for inference: relation-specific aggregation, projection
// and cross-relation sum in one kernel (Eq. 1 of the paper, both lines; Algorithm 1, the aggregation
// and AGG_all steps), without the aggregated features M_r ever reaching HBM:
//
//     H_t[v, :] = act( sum_r ( (sum | mean)_{e in r, v_e = v} H0_s[u_e] ) W_r )
//
// One workgroup of four wavefronts owns 64 consecutive destination rows and all d_out <= 256 output
// columns (each wavefront 64 columns: 2 x 2 MFMA tiles of 32 x 32 in registers).  For every relation
// into the type and every chunk of up to 128 input columns it
//   A. aggregates the chunk of its 64 rows into LDS: a lane group per row (one 16-byte piece of the
//      chunk per lane) walks the row's in-edges by row id with four neighbour rows in flight; rows of at
//      least 512 edges are not walked here - the ordinary hub-chunk kernels have reduced them into a
//      compact array beforehand and the lane group copies the finished row;
//   B. multiplies the LDS tile by the chunk's rows of W_r with MFMAs (v_mfma_f32_32x32x2_f32, or
//      v_mfma_f32_32x32x16_bf16 when tables and weights are bf16: the tile is then stored as bf16,
//      the same rounding the unfused path applies when it stores M_r), W_r fragments read straight
//      from a k-contiguous copy in global memory, one k-step ahead (W_r is small and stays in L2; no
//      other wavefront of the workgroup needs a wavefront's columns, so LDS would not save anything).
// Training keeps the unfused path: M_r is an operand of dW_r and has to exist in HBM there.
#include <algorithm>
#include <vector>

#include "heta_gemm.h"

namespace heta {

namespace {

constexpr int kFusedRows = 64;   // destination rows per workgroup
constexpr int kFusedKC = 128;    // input columns per chunk
constexpr int kFusedMaxSeg = 16;

struct FusedSeg {
    const int64_t *ptr;      // CSR by row id
    const int32_t *idx;
    const void *table;
    int64_t ld;              // elements
    const int64_t *gid;      // nullable
    const void *W;           // packed [d_out][ldw]: k-contiguous, zero padded to whole k-steps
    int64_t ldw;
    int d_in;
    const int32_t *hub_slot; // [n_rows] index among the hub rows, for rows of >= kHubMinDeg edges
    const float *hub_rows;   // [n_hub][ld_hub] aggregated (and scaled) hub rows
    int64_t ld_hub;
};

struct FusedParams {
    FusedSeg seg[kFusedMaxSeg];
    int n_seg;
    int64_t n_rows;
    int d_out;
    int mean, relu;
    float *out;
    int64_t ld_out;
};

template <typename T> struct FusedTraits;
template <> struct FusedTraits<float> {
    static constexpr int EPC = 4;                   // elements per 16-byte piece
    static constexpr int SA = kFusedKC + 4;         // LDS row stride (elements)
};
template <> struct FusedTraits<bf16_t> {
    static constexpr int EPC = 8;
    static constexpr int SA = kFusedKC + 8;
};

// one 16-byte piece of a source row, widened to fp32 when added
template <typename T> struct Chunk16;
template <> struct Chunk16<float> {
    float4 v;
    __device__ __forceinline__ void load(const float *p) { v = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void zero() { v = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void add_to(float *a) const { a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w; }
};
template <> struct Chunk16<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void zero() { v = make_uint4(0u, 0u, 0u, 0u); }
    __device__ __forceinline__ void add_to(float *a) const
    {
        a[0] += __uint_as_float(v.x << 16); a[1] += __uint_as_float(v.x & 0xffff0000u);
        a[2] += __uint_as_float(v.y << 16); a[3] += __uint_as_float(v.y & 0xffff0000u);
        a[4] += __uint_as_float(v.z << 16); a[5] += __uint_as_float(v.z & 0xffff0000u);
        a[6] += __uint_as_float(v.w << 16); a[7] += __uint_as_float(v.w & 0xffff0000u);
    }
};

template <typename T> __device__ __forceinline__ void store_lds(T *dst, const float *a);
template <> __device__ __forceinline__ void store_lds<float>(float *dst, const float *a)
{
    *reinterpret_cast<float4 *>(dst) = make_float4(a[0], a[1], a[2], a[3]);
}
template <> __device__ __forceinline__ void store_lds<bf16_t>(bf16_t *dst, const float *a)
{
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w[i] = static_cast<uint32_t>(to_bf16(a[2 * i])) | (static_cast<uint32_t>(to_bf16(a[2 * i + 1])) << 16);
    *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
}

template <typename T>
__global__ void __launch_bounds__(256) fused_fwd_kernel(FusedParams p)
{
    constexpr int EPC = FusedTraits<T>::EPC, SA = FusedTraits<T>::SA;
    constexpr int L = kFusedKC / EPC;   // lanes per row chunk: 32 (fp32) or 16 (bf16)
    constexpr int NG = 256 / L;         // lane groups per workgroup: 8 or 16
    constexpr int U = 8;                // neighbour rows in flight per lane group
    __shared__ __attribute__((aligned(16))) T As[kFusedRows * SA];
    __shared__ __attribute__((aligned(16))) float part_s[NG][2][kFusedKC]; // a lane group's partial sums of the rows it shares
    __shared__ int64_t ptr_s[kFusedRows + 1];
    __shared__ int eff_s[kFusedRows + 1];  // prefix of the edges walked here (rows below the hub threshold)
    __shared__ int head_row[NG], tail_row[NG];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int wn = wave * 64;
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * kFusedRows;
    const int rows = static_cast<int>(min(static_cast<int64_t>(kFusedRows), p.n_rows - v0));
    const int grp = tid / L, l = tid % L;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    for (int s = 0; s < p.n_seg; ++s) {
        const FusedSeg &g = p.seg[s];
        __syncthreads(); // the previous relation's last chunk has been consumed
        if (tid <= rows) ptr_s[tid] = g.ptr[v0 + tid];
        __syncthreads();
        if (wave == 0) { // eff_s: inclusive scan over the 64 rows of (degree, or 0 for hub and absent rows)
            int dg = 0;
            if (lane < rows) {
                const int64_t d64 = ptr_s[lane + 1] - ptr_s[lane];
                dg = d64 < kHubMinDeg ? static_cast<int>(d64) : 0;
            }
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_up(dg, off, 64);
                if (lane >= off) dg += t;
            }
            eff_s[lane + 1] = dg;
            if (lane == 0) eff_s[0] = 0;
        }
        __syncthreads();
        // The tile's edges (hub rows excluded) are cut into NG equal slices, one per lane group, so the
        // groups finish together whatever the degrees are; a row cut by a slice boundary is summed from
        // the groups' partial sums in group order.
        const int e_eff = eff_s[kFusedRows];
        const int per = (e_eff + NG - 1) / NG;
        const int sl_a = min(grp * per, e_eff), sl_b = min(sl_a + per, e_eff);
        const T *table = static_cast<const T *>(g.table);
        for (int kc = 0; kc < g.d_in; kc += kFusedKC) {
            // ---- A: aggregate columns [kc, kc + 128) of the tile's rows into LDS ------------------
            const int col = kc + l * EPC;
            const bool col_ok = col < g.d_in; // d_in is a multiple of EPC
            if (l == 0) {
                head_row[grp] = -1;
                tail_row[grp] = -1;
            }
            // rows without walked edges: zero, or the finished hub row
            for (int r = grp; r < kFusedRows; r += NG) {
                if (r < rows && eff_s[r + 1] > eff_s[r]) continue;
                float a[EPC];
#pragma unroll
                for (int i = 0; i < EPC; ++i) a[i] = 0.f;
                if (r < rows && col_ok && ptr_s[r + 1] - ptr_s[r] >= kHubMinDeg) {
                    const float *h = g.hub_rows + static_cast<int64_t>(g.hub_slot[v0 + r]) * g.ld_hub + col;
#pragma unroll
                    for (int i = 0; i < EPC; ++i) a[i] = h[i];
                }
                store_lds<T>(&As[r * SA + l * EPC], a);
            }
            // This group's slice.  Loads are issued U edges at a time regardless of row boundaries, and the
            // neighbour ids of the next batch are fetched before the current batch's rows are consumed, so a
            // batch costs one memory round trip; the accumulate side tracks the row boundaries.
            if (sl_a < sl_b) {
                const int64_t p0 = ptr_s[0];
                const bool no_hubs = ptr_s[rows] - p0 == e_eff; // then the tile's edges are consecutive in the CSR
                int r = 0;
                while (eff_s[r + 1] <= sl_a) ++r; // first row with an edge in the slice
                int r_beg = eff_s[r], r_end = eff_s[r + 1];
                int rl = r, rl_end = r_end;       // load-side cursor (only needed around hub rows)
                auto edge_pos = [&](int x) -> int64_t {
                    if (no_hubs) return p0 + x;
                    while (x >= rl_end) {
                        ++rl;
                        rl_end = eff_s[rl + 1];
                    }
                    return ptr_s[rl] - eff_s[rl] + x;
                };
                int seg_a = sl_a;
                float a[EPC];
#pragma unroll
                for (int t = 0; t < EPC; ++t) a[t] = 0.f;
                int32_t ids[U];
#pragma unroll
                for (int u = 0; u < U; ++u) ids[u] = sl_a + u < sl_b ? g.idx[edge_pos(sl_a + u)] : 0;
                for (int i = sl_a; i < sl_b; i += U) {
                    Chunk16<T> v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (i + u < sl_b && col_ok) {
                            const int64_t row = g.gid ? g.gid[ids[u]] : static_cast<int64_t>(ids[u]);
                            v[u].load(table + row * g.ld + col);
                        } else {
                            v[u].zero();
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) ids[u] = i + U + u < sl_b ? g.idx[edge_pos(i + U + u)] : 0;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int x = i + u;
                        if (x >= sl_b) break;
                        v[u].add_to(a);
                        const int seg_b = min(r_end, sl_b);
                        if (x + 1 != seg_b) continue;
                        // the segment [seg_a, seg_b) of row r is complete
                        if (seg_a == r_beg && seg_b == r_end) { // the whole row
                            if (p.mean) {
                                const float sc = 1.f / static_cast<float>(r_end - r_beg);
#pragma unroll
                                for (int t = 0; t < EPC; ++t) a[t] *= sc;
                            }
                            store_lds<T>(&As[r * SA + l * EPC], a);
                        } else { // a piece of a row shared with other groups
                            const int which = seg_a > r_beg ? 0 : 1; // 0: the row began in an earlier slice; 1: it begins here
#pragma unroll
                            for (int t = 0; t < EPC; ++t) part_s[grp][which][l * EPC + t] = a[t];
                            if (l == 0) (which ? tail_row : head_row)[grp] = r;
                        }
#pragma unroll
                        for (int t = 0; t < EPC; ++t) a[t] = 0.f;
                        seg_a = seg_b;
                        if (seg_b < sl_b) {
                            do { ++r; } while (eff_s[r + 1] == eff_s[r]); // next row with walked edges
                            r_beg = eff_s[r];
                            r_end = eff_s[r + 1];
                        }
                    }
                }
            }
            __syncthreads();
            // shared rows: the group where the row begins adds the pieces in group order
            if (tail_row[grp] >= 0) {
                const int r = tail_row[grp];
                float a[EPC];
#pragma unroll
                for (int t = 0; t < EPC; ++t) a[t] = part_s[grp][1][l * EPC + t];
                for (int g2 = grp + 1; g2 < NG && head_row[g2] == r; ++g2)
#pragma unroll
                    for (int t = 0; t < EPC; ++t) a[t] += part_s[g2][0][l * EPC + t];
                if (p.mean) {
                    const float sc = 1.f / static_cast<float>(eff_s[r + 1] - eff_s[r]);
#pragma unroll
                    for (int t = 0; t < EPC; ++t) a[t] *= sc;
                }
                store_lds<T>(&As[r * SA + l * EPC], a);
            }
            __syncthreads();
            // ---- B: acc += As[64 x kw] * W[kc .. kc + kw, :] ---------------------------------------
            const int kw = min(kFusedKC, g.d_in - kc);
            if (wn < p.d_out) { // uniform per wavefront
                // W is packed k-contiguous ([n][ldw], zero padded): a fragment is one 16-byte load, issued one
                // k-step ahead of the MFMAs that use it
                const T *Wp = static_cast<const T *>(g.W);
                const int n0 = wn + l32, n1 = wn + 32 + l32;
                const T *w0 = Wp + static_cast<int64_t>(min(n0, p.d_out - 1)) * g.ldw + kc + EPC * half;
                const T *w1 = Wp + static_cast<int64_t>(min(n1, p.d_out - 1)) * g.ldw + kc + EPC * half;
                constexpr int KS = sizeof(T) == 4 ? 8 : 16; // k-values per step
                uint4 nb0 = *reinterpret_cast<const uint4 *>(w0), nb1 = *reinterpret_cast<const uint4 *>(w1);
                for (int kk = 0; kk < kw; kk += KS) {
                    const uint4 cb0 = nb0, cb1 = nb1;
                    if (kk + KS < kw) {
                        nb0 = *reinterpret_cast<const uint4 *>(w0 + kk + KS);
                        nb1 = *reinterpret_cast<const uint4 *>(w1 + kk + KS);
                    }
                    if constexpr (sizeof(T) == 4) {
                        float fa[2][4];
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            const float4 t = *reinterpret_cast<const float4 *>(&As[(i * 32 + l32) * SA + kk + 4 * half]);
                            fa[i][0] = t.x; fa[i][1] = t.y; fa[i][2] = t.z; fa[i][3] = t.w;
                        }
                        const float fb[2][4] = {{__uint_as_float(cb0.x), __uint_as_float(cb0.y), __uint_as_float(cb0.z), __uint_as_float(cb0.w)},
                                                {__uint_as_float(cb1.x), __uint_as_float(cb1.y), __uint_as_float(cb1.z), __uint_as_float(cb1.w)}};
#pragma unroll
                        for (int t = 0; t < 4; ++t)
#pragma unroll
                            for (int i = 0; i < 2; ++i)
#pragma unroll
                                for (int j = 0; j < 2; ++j)
                                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t], fb[j][t], acc[i][j], 0, 0, 0);
                    } else {
                        union Frag { uint4 u; bf16x8 v; } fa[2], fb[2];
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            fa[i].u = *reinterpret_cast<const uint4 *>(&As[(i * 32 + l32) * SA + kk + 8 * half]);
                        fb[0].u = cb0;
                        fb[1].u = cb1;
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int j = 0; j < 2; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
                    }
                }
            }
            __syncthreads(); // before the next chunk overwrites the tile
        }
    }
    // epilogue: accumulator register v of lane (half, l32) is C[8*(v/4) + 4*half + v%4][l32] of its 32x32 tile
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = wn + j * 32 + l32;
            if (n >= p.d_out) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (r >= rows) continue;
                float val = acc[i][j][v];
                if (p.relu) val = fmaxf(val, 0.f);
                p.out[(v0 + r) * p.ld_out + n] = val;
            }
        }
}

// hub_slot[perm[h]] = h for the hub rows of a schedule
__global__ void __launch_bounds__(256) hub_slot_kernel(const int32_t *perm, int64_t n_hub, int32_t *slot)
{
    const int64_t h = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (h < n_hub) slot[perm[h]] = static_cast<int32_t>(h);
}

// out[n][k] = W[k][n] for k < K, 0 for K <= k < ld_out: the weight matrix k-contiguous
template <typename T>
__global__ void __launch_bounds__(256) fused_pack_kernel(const T *W, int64_t ldw, int K, int N, T *out, int ld_out)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= static_cast<int64_t>(N) * ld_out) return;
    const int n = static_cast<int>(t / ld_out), k = static_cast<int>(t % ld_out);
    out[t] = k < K ? W[static_cast<int64_t>(k) * ldw + n] : T(0);
}

} // namespace

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_cross_rel_aggregate_project(heta_graph *g, int32_t dst_type, int32_t n, const int32_t *rels,
                                             heta_reduce op, const void *const *tables, heta_dtype dt,
                                             const int64_t *ld_table, const int32_t *d_table, const int64_t *n_table_rows,
                                             const int64_t *const *src_gid, const void *const *W, const int64_t *ld_w,
                                             int32_t d_out, heta_act act, float *out, int64_t ld_out, void *hip_stream)
{
    if (!g || !rels || !tables || !ld_table || !d_table || !n_table_rows || !W || !ld_w || !out)
        return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: null argument");
    if (dst_type < 0 || dst_type >= (int32_t)g->ntypes.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: node type %d out of range", dst_type);
    if (n < 1 || n > kFusedMaxSeg)
        return fail(HETA_ERR_SHAPE, "heta_cross_rel_aggregate_project: 1..%d relations per call (got %d)", kFusedMaxSeg, n);
    if (op != HETA_SUM && op != HETA_MEAN) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: bad reduce op");
    if (act != HETA_ACT_NONE && act != HETA_ACT_RELU) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: bad activation");
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: bad dtype");
    if (d_out < 1 || d_out > 256 || ld_out < d_out)
        return fail(HETA_ERR_UNSUPPORTED, "heta_cross_rel_aggregate_project: needs 1 <= d_out <= 256 and ld_out >= d_out (d_out=%d)", d_out);
    const int64_t n_rows = g->ntypes[dst_type].num_nodes;
    if (n_rows == 0) return HETA_OK;
    hipStream_t st = as_stream(hip_stream);
    const size_t esz = dtype_size(dt);
    const int epc = static_cast<int>(16 / esz);
    FusedParams p{};
    p.n_seg = n;
    p.n_rows = n_rows;
    p.d_out = d_out;
    p.mean = (op == HETA_MEAN);
    p.relu = (act == HETA_ACT_RELU);
    p.out = out;
    p.ld_out = ld_out;
    // packed bf16 weights of this call: one region of the handle's packing buffer
    size_t pack_elems = 0;
    std::vector<int> d_in(n);
    for (int s = 0; s < n; ++s) {
        const int32_t ri = rels[s];
        if (ri < 0 || ri >= (int32_t)g->rels.size() || g->rels[ri].dst_type != dst_type)
            return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: relation %d does not end in node type %d", ri, dst_type);
        const Relation &r = g->rels[ri];
        d_in[s] = d_table[s];
        if ((!tables[s] && r.n_edges > 0) || !W[s]) // a relation without edges never reads its table
            return fail(HETA_ERR_INVALID_ARG, "heta_cross_rel_aggregate_project: null table or W (relation %d)", ri);
        if (d_in[s] < 1 || d_in[s] % epc != 0 || ld_table[s] < d_in[s] || (ld_table[s] * (int64_t)esz) % 16 != 0 || !aligned16(tables[s]))
            return fail(HETA_ERR_UNSUPPORTED,
                        "heta_cross_rel_aggregate_project: source rows must be 16-byte aligned multiples of 16 bytes (relation %d, d=%d)", ri,
                        d_in[s]);
        if (ld_w[s] < d_out) return fail(HETA_ERR_SHAPE, "heta_cross_rel_aggregate_project: ld_w < d_out (relation %d)", ri);
        const int64_t *gid = src_gid ? src_gid[s] : nullptr;
        if (n_table_rows[s] < 0 || (!gid && n_table_rows[s] < r.n_src))
            return fail(HETA_ERR_SHAPE, "heta_cross_rel_aggregate_project: table of relation %d has too few rows", ri);
        pack_elems += static_cast<size_t>(d_out) * ((d_in[s] + 15) / 16 * 16);
    }
    if (pack_elems * esz > g->pack_bytes) {
        if (g->d_pack) {
            HETA_HIP(hipDeviceSynchronize()); // earlier readers
            scratch_free(g->d_pack);
        }
        g->d_pack = nullptr;
        g->pack_bytes = 0;
        HETA_HIP(scratch_alloc(&g->d_pack, pack_elems * esz));
        g->pack_bytes = pack_elems * esz;
    }
    size_t pack_off = 0;
    for (int s = 0; s < n; ++s) {
        Relation &r = g->rels[rels[s]];
        FusedSeg &f = p.seg[s];
        f.ptr = r.csr.d_ptr;
        f.idx = r.csr.d_idx;
        f.table = tables[s];
        f.ld = ld_table[s];
        f.gid = src_gid ? src_gid[s] : nullptr;
        f.d_in = d_in[s];
        {
            const int ldp = (d_in[s] + 15) / 16 * 16;
            const int64_t total = static_cast<int64_t>(d_out) * ldp;
            const unsigned pb = (unsigned)((total + 255) / 256);
            char *dst = static_cast<char *>(g->d_pack) + pack_off * esz;
            if (dt == HETA_BF16)
                hipLaunchKernelGGL((fused_pack_kernel<bf16_t>), dim3(pb), dim3(256), 0, st, static_cast<const bf16_t *>(W[s]), ld_w[s],
                                   d_in[s], (int)d_out, reinterpret_cast<bf16_t *>(dst), ldp);
            else
                hipLaunchKernelGGL((fused_pack_kernel<float>), dim3(pb), dim3(256), 0, st, static_cast<const float *>(W[s]), ld_w[s],
                                   d_in[s], (int)d_out, reinterpret_cast<float *>(dst), ldp);
            HETA_LAUNCH_CHECK("fused_pack_kernel");
            f.W = dst;
            f.ldw = ldp;
            pack_off += static_cast<size_t>(total);
        }
        // hub rows: slot map (once per relation) and their aggregated rows (every call)
        f.hub_slot = nullptr;
        f.hub_rows = nullptr;
        f.ld_hub = (static_cast<int64_t>(d_in[s]) + 3) / 4 * 4;
        if (r.csr.n_hub_rows > 0) {
            if (!r.d_hub_slot) {
                HETA_HIP(hipMalloc(reinterpret_cast<void **>(&r.d_hub_slot), static_cast<size_t>(r.n_dst) * sizeof(int32_t)));
                hipLaunchKernelGGL(hub_slot_kernel, dim3((unsigned)((r.csr.n_hub_rows + 255) / 256)), dim3(256), 0, st, r.csr.d_perm,
                                   r.csr.n_hub_rows, r.d_hub_slot);
                HETA_LAUNCH_CHECK("hub_slot_kernel");
            }
            const size_t need = static_cast<size_t>(r.csr.n_hub_rows) * f.ld_hub * sizeof(float);
            if (need > r.hub_rows_bytes) {
                if (r.d_hub_rows) HETA_HIP(hipFree(r.d_hub_rows));
                r.d_hub_rows = nullptr;
                r.hub_rows_bytes = 0;
                HETA_HIP(hipMalloc(reinterpret_cast<void **>(&r.d_hub_rows), need));
                r.hub_rows_bytes = need;
            }
            heta_status e = aggregate_hub_rows(g, r.csr, tables[s], dt, ld_table[s], d_in[s], f.gid, p.mean, r.d_hub_rows, f.ld_hub, st);
            if (e != HETA_OK) return e;
            f.hub_slot = r.d_hub_slot;
            f.hub_rows = r.d_hub_rows;
        }
    }
    const int64_t blocks = (n_rows + kFusedRows - 1) / kFusedRows;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "heta_cross_rel_aggregate_project: too many rows");
    double bytes = static_cast<double>(n_rows) * d_out * 4.0, flops = 0;
    for (int s = 0; s < n; ++s) {
        const Relation &r = g->rels[rels[s]];
        bytes += static_cast<double>(r.n_edges) * (d_in[s] * esz + 4.0) + static_cast<double>(r.n_dst) * 8.0 +
                 static_cast<double>(d_in[s]) * d_out * esz;
        flops += 2.0 * static_cast<double>(r.n_dst) * d_in[s] * d_out;
    }
    ProfScope prof("fused_fwd_kernel", st, bytes, flops);
    if (dt == HETA_F32) hipLaunchKernelGGL((fused_fwd_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((fused_fwd_kernel<bf16_t>), dim3((unsigned)blocks), dim3(256), 0, st, p);
    HETA_LAUNCH_CHECK("fused_fwd_kernel");
    return HETA_OK;
}

} // extern "C"
