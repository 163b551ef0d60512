// Relation-specific aggregation, forward and backward, as one segmented gather-reduce.
//
// Forward (Eq. 1 of the paper, first line, with a GCN-style sum/mean as AGG_r) walks a
// relation's CSR: output row v adds the source rows of v's in-edges.  Backward (Algorithm 1,
// local backpropagation) walks the CSC: output row u adds the gradient rows of the
// destinations of u's out-edges, weighted by 1/deg for the mean.  Both are
//
//     out[r] = beta * out[r] + scale(r) * sum_{e in [ptr[r], ptr[r+1])} w[idx[e]] * table[row(idx[e])]
//
// so one family of kernels serves both, and nothing is scattered: every output row is
// written by exactly one lane group, which makes the result independent of scheduling.
//
// Mapping to the machine (wave64, HBM-bound):
//   - A row of d elements is cut into 16-byte chunks; a "lane group" of L lanes (L = the
//     power of two covering the chunks, at most 64, each lane holding one or two chunks)
//     reads a whole neighbour row with one 128-bit load per lane, fully coalesced.
//   - Rows are scheduled by degree (perm = rows by descending degree) and the kernels walk the
//     schedule-ordered copy of the adjacency (sptr / sidx), so what a wavefront needs before
//     its first feature load is consecutive in memory:
//       hub rows   (>= 512 edges): cut into 256-edge chunks, one wavefront per chunk, partial
//                  sums to a workspace, a second kernel adds the partials in chunk order;
//       long rows  (32 .. 511 edges): one wavefront per row; its 64/L lane groups take the
//                  row's edges round-robin, several loads in flight each, and are combined at
//                  the end with cross-lane shuffles;
//       short rows (< 32 edges: the bulk of a power-law graph, incl. empty rows): one wavefront
//                  per batch of up to 64 rows of EQUAL degree k.  Where the batch starts, in
//                  rows and in edges, follows from the degree histogram alone, so the wavefront
//                  fetches its up to 256 neighbour ids and its row ids with coalesced loads whose
//                  addresses depend on nothing, parks them in LDS, and then streams feature
//                  rows: lane group g owns rows g, g + 64/L, ... and keeps 8 row loads in
//                  flight across row boundaries - two dependent memory round trips per
//                  wavefront instead of four, and 8 KB in flight per wavefront.
//   - Neighbour ids of a long row are fetched 64 at a time with one coalesced load and
//     broadcast with lane shuffles.
#include <algorithm>
#include <mutex>
#include <utility>
#include <vector>

#include "heta_internal.h"

namespace heta {

constexpr int kShortDeg = 32;      // rows of fewer edges are batched by degree
constexpr int kBatchIds = 256;     // neighbour ids a batch wavefront parks in LDS
constexpr int kWaveSplitMaxItems = 2048; // long rows + hub chunks up to which a relation's items get a workgroup each

struct AggParams {
    const int64_t *sptr;   // schedule-ordered row offsets
    const int32_t *sidx;   // schedule-ordered neighbour ids
    const int32_t *perm;
    const HubChunk *hub_chunks;
    const int64_t *hub_chunk_ptr;
    const void *table;
    int64_t ld;            // elements
    const int64_t *gid;    // nullable: neighbour id -> table row
    const float *edge_w;   // nullable: weight per neighbour id
    const float *slot_w;   // nullable: weight per (edge position in sidx, head): [n_edges][heads]
    int heads;             // with slot_w: number of heads, columns [h*head_dim, (h+1)*head_dim) use weight h
    int head_dim;
    const float *slot_w2;  // nullable (with slot_w only): a second weight array; the same gathered rows are
    void *out2;            // reduced a second time with it into out2 (same type and leading dimension rules as out)
    int64_t ld_out2;
    int mean;              // divide the row sum by the row's degree
    int hub_only;          // reduce the hub rows only, into out[h] for the h-th hub row of the schedule
    int wave_split;        // few long rows / hub chunks: four wavefronts per item (agg_wave_split_kernel)
    // With slot_w2, instead of storing the second sum: dot_out[row, k] = <second sum of head k, dot_z[row, head k]> -
    // dot_corr[row, k] (the attention backward needs only this dot of the gate-weighted sum, not the sum itself).
    const void *dot_z;     // nullable; rows indexed like out, ld_z elements apart, fp32 or bf16 (dot_z_bf16)
    int64_t ld_z;
    int dot_z_bf16;
    const float *dot_corr; // nullable
    float *dot_out;        // [n_rows][heads]
    int combine_dot;       // set on the hub combine launch that finishes dot_out
    void *out;
    int64_t ld_out;
    int out_bf16;
    float beta;            // 0 or 1
    float *ws;             // hub partials [slot][ws_stride]; with slot_w2 the second sum follows at +ws_ld
    int64_t ws_ld;
    int64_t ws_stride;
    int d;
    int64_t n_hub_chunks, n_hub_rows;
    int64_t n_wave_items;  // hub chunks + long rows
    int64_t n_rows;
    // short rows, bucket b holds the rows of degree k = kShortDeg - 1 - b:
    int32_t batch0[kShortDeg + 1]; // first batch (wavefront) of bucket b; batch0[kShortDeg] = number of batches
    int32_t row0[kShortDeg + 1];   // schedule position of the bucket's first row; row0[kShortDeg] = n_rows
    int64_t edge0[kShortDeg];      // position of its first neighbour id in sidx
};

using bf16_t = uint16_t;

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return static_cast<bf16_t>((u >> 16) | 0x40u);
    return static_cast<bf16_t>((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// One chunk of a row: EPC elements of T, read as one load.
template <typename T, int EPC> struct Chunk;
template <> struct Chunk<float, 4> {
    float4 v;
    __device__ __forceinline__ void load(const float *p) { v = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ void zero() { v = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void add_to(float *a, float w) const
    {
        a[0] = fmaf(w, v.x, a[0]); a[1] = fmaf(w, v.y, a[1]); a[2] = fmaf(w, v.z, a[2]); a[3] = fmaf(w, v.w, a[3]);
    }
    __device__ __forceinline__ void add_to(float *a) const { a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w; }
};
template <> struct Chunk<float, 1> {
    float v;
    __device__ __forceinline__ void load(const float *p) { v = *p; }
    __device__ __forceinline__ void zero() { v = 0.f; }
    __device__ __forceinline__ void add_to(float *a, float w) const { a[0] = fmaf(w, v, a[0]); }
    __device__ __forceinline__ void add_to(float *a) const { a[0] += v; }
};
template <> struct Chunk<bf16_t, 8> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void zero() { v = make_uint4(0u, 0u, 0u, 0u); }
    __device__ __forceinline__ void widen(float *f) const
    {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    __device__ __forceinline__ void add_to(float *a, float w) const
    {
        float f[8];
        widen(f);
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = fmaf(w, f[i], a[i]);
    }
    __device__ __forceinline__ void add_to(float *a) const
    {
        float f[8];
        widen(f);
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] += f[i];
    }
};
template <> struct Chunk<bf16_t, 1> {
    bf16_t v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *p; }
    __device__ __forceinline__ void zero() { v = 0; }
    __device__ __forceinline__ void add_to(float *a, float w) const { a[0] = fmaf(w, bf16_to_f32(v), a[0]); }
    __device__ __forceinline__ void add_to(float *a) const { a[0] += bf16_to_f32(v); }
};

// Final store of one lane's chunk of an output row: scale, optional accumulate, element guard.
// Whole chunks on 16-byte aligned rows go out as 128-bit stores (fp32: one per 4 elements; bf16:
// one per 8 elements, or a 64-bit store for a 4-element chunk).
template <int EPC>
__device__ __forceinline__ void store_out(const AggParams &p, void *out, int64_t ld_out, int64_t row, int col0,
                                          const float *acc, float scale)
{
    const bool whole = col0 + EPC <= p.d;
    if (p.out_bf16) {
        bf16_t *o = static_cast<bf16_t *>(out) + row * ld_out + col0;
        if constexpr (EPC % 4 == 0) {
            if (whole && ((ld_out & 7) == 0) && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
                float v[EPC];
#pragma unroll
                for (int i = 0; i < EPC; ++i) v[i] = acc[i] * scale;
                if (p.beta != 0.f) {
#pragma unroll
                    for (int i = 0; i < EPC; ++i) v[i] += bf16_to_f32(o[i]);
                }
                uint32_t w[EPC / 2];
#pragma unroll
                for (int i = 0; i < EPC / 2; ++i)
                    w[i] = static_cast<uint32_t>(f32_to_bf16(v[2 * i])) | (static_cast<uint32_t>(f32_to_bf16(v[2 * i + 1])) << 16);
                if constexpr (EPC == 8) *reinterpret_cast<uint4 *>(o) = make_uint4(w[0], w[1], w[2], w[3]);
                else *reinterpret_cast<uint2 *>(o) = make_uint2(w[0], w[1]);
                return;
            }
        }
#pragma unroll
        for (int i = 0; i < EPC; ++i)
            if (col0 + i < p.d) {
                float v = acc[i] * scale;
                if (p.beta != 0.f) v += bf16_to_f32(o[i]);
                o[i] = f32_to_bf16(v);
            }
    } else {
        float *o = static_cast<float *>(out) + row * ld_out + col0;
        if constexpr (EPC % 4 == 0) {
            if (whole && ((ld_out & 3) == 0) && ((reinterpret_cast<uintptr_t>(out) & 15u) == 0)) {
#pragma unroll
                for (int q = 0; q < EPC / 4; ++q) {
                    float4 v = make_float4(acc[4 * q] * scale, acc[4 * q + 1] * scale, acc[4 * q + 2] * scale, acc[4 * q + 3] * scale);
                    if (p.beta != 0.f) {
                        const float4 old = *reinterpret_cast<const float4 *>(o + 4 * q);
                        v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
                    }
                    *reinterpret_cast<float4 *>(o + 4 * q) = v;
                }
                return;
            }
        }
#pragma unroll
        for (int i = 0; i < EPC; ++i)
            if (col0 + i < p.d) {
                float v = acc[i] * scale;
                if (p.beta != 0.f) v += o[i];
                o[i] = v;
            }
    }
}

template <int EPC>
__device__ __forceinline__ void store_out(const AggParams &p, int64_t row, int col0, const float *acc, float scale)
{
    store_out<EPC>(p, p.out, p.ld_out, row, col0, acc, scale);
}

__device__ __forceinline__ float row_scale(const AggParams &p, int64_t deg)
{
    if (!p.mean) return 1.f;
    return deg > 0 ? 1.f / static_cast<float>(deg) : 0.f;
}

// The dot form of the second sum's store: acc2 holds EPC consecutive columns (from col0) of the row's second
// sum; the lanes of a head (head_dim / EPC of them, a power of two, consecutive) add their partial dots.  Every
// lane of the row's lane group calls it (lanes beyond the row's width contribute 0).
template <int EPC>
__device__ __forceinline__ void dot_store(const AggParams &p, int64_t row, int col0, const float *acc2, float scale, int l)
{
    float part = 0.f;
    const bool live = col0 < p.d;
    if (live) { // the host has checked that z's chunks of EPC elements are aligned as vectors
        if (p.dot_z_bf16) {
            const uint16_t *z = static_cast<const uint16_t *>(p.dot_z) + row * p.ld_z + col0;
#pragma unroll
            for (int q = 0; q < EPC / 4; ++q) {
                const uint2 raw = *reinterpret_cast<const uint2 *>(z + 4 * q);
                part = fmaf(acc2[4 * q + 0], __uint_as_float(raw.x << 16), part);
                part = fmaf(acc2[4 * q + 1], __uint_as_float(raw.x & 0xffff0000u), part);
                part = fmaf(acc2[4 * q + 2], __uint_as_float(raw.y << 16), part);
                part = fmaf(acc2[4 * q + 3], __uint_as_float(raw.y & 0xffff0000u), part);
            }
        } else {
            const float *z = static_cast<const float *>(p.dot_z) + row * p.ld_z + col0;
#pragma unroll
            for (int q = 0; q < EPC / 4; ++q) {
                const float4 v = *reinterpret_cast<const float4 *>(z + 4 * q);
                part = fmaf(acc2[4 * q + 0], v.x, part);
                part = fmaf(acc2[4 * q + 1], v.y, part);
                part = fmaf(acc2[4 * q + 2], v.z, part);
                part = fmaf(acc2[4 * q + 3], v.w, part);
            }
        }
    }
    part *= scale;
    const int lph = p.head_dim / EPC;
    for (int off = lph >> 1; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if (live && (l & (lph - 1)) == 0) {
        const int64_t at = row * p.heads + col0 / p.head_dim;
        p.dot_out[at] = part - (p.dot_corr ? p.dot_corr[at] : 0.f);
    }
}

// ---- short rows: one wavefront per batch of equal-degree rows ---------------------------------------
// Rows per batch for degree k and G lane groups: about 16 row loads per lane group (two fills of its
// load pipeline), at most 64 rows and kBatchIds neighbour ids - small enough that a block of a sampled
// mini-batch with wide rows (G = 1) still spreads over the whole chip.
__host__ __device__ inline int batch_rows(int k, int G)
{
    if (k == 0) return 64;
    int r = G * (16 / k > 1 ? 16 / k : 1);
    r = r < kBatchIds / k ? r : kBatchIds / k;
    return r < 64 ? r : 64;
}

template <typename T, int EPC, int L, int CPL, bool DUAL>
__device__ __forceinline__ void agg_batch_body(const AggParams &p, const unsigned bx = blockIdx.x)
{
    constexpr int G = 64 / L;          // lane groups = rows in progress per wavefront
    constexpr int U = CPL == 1 ? 8 : 4; // row loads in flight per lane group
    __shared__ int32_t ids_s[4][kBatchIds];
    __shared__ float w_s[4][kBatchIds];
    __shared__ int32_t row_s[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w = bx * 4 + wave;
    const bool active = w < p.batch0[kShortDeg]; // uniform per wavefront; idle wavefronts still reach the barrier
    int k = 0, nrows = 0;
    int64_t e0 = 0;
    if (active) {
        int b = 0;
        while (w >= p.batch0[b + 1]) ++b; // at most kShortDeg scalar steps
        k = kShortDeg - 1 - b;
        const int R = batch_rows(k, G);
        const int first = (w - p.batch0[b]) * R;
        const int q0 = p.row0[b] + first;
        nrows = min(R, p.row0[b + 1] - q0);
        e0 = p.edge0[b] + static_cast<int64_t>(first) * k;
        const int n_ids = nrows * k;
        // level 1: everything below has an address that depends on no load
        if (lane < nrows) row_s[wave][lane] = p.perm[q0 + lane];
#pragma unroll
        for (int c = 0; c < kBatchIds / 64; ++c) {
            const int i = c * 64 + lane;
            if (i < n_ids) {
                const int id = p.sidx[e0 + i];
                ids_s[wave][i] = p.gid ? static_cast<int32_t>(p.gid[id]) : id;
                if (p.edge_w) w_s[wave][i] = p.edge_w[id];
            }
        }
    }
    __syncthreads();
    if (!active) return;
    const int g = lane / L, l = lane % L;
    const int n_chunks = (p.d + EPC - 1) / EPC;
    const int ch0 = blockIdx.y * (L * CPL) + l;
    const T *table = static_cast<const T *>(p.table);
    if (k == 0) { // empty rows: exactly 0 (or untouched when accumulating)
        if (p.beta == 0.f) {
            float zero[EPC];
#pragma unroll
            for (int i = 0; i < EPC; ++i) zero[i] = 0.f;
            for (int r = g; r < nrows; r += G)
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int ch = ch0 + c * L;
                    if (ch < n_chunks) {
                        store_out<EPC>(p, row_s[wave][r], ch * EPC, zero, 0.f);
                        if (DUAL && !p.dot_out) store_out<EPC>(p, p.out2, p.ld_out2, row_s[wave][r], ch * EPC, zero, 0.f);
                    }
                }
        }
        if constexpr (DUAL && CPL == 1) { // an empty row's second sum is zero: its dot is zero
            if (p.dot_out) {
                float zero[EPC];
#pragma unroll
                for (int i = 0; i < EPC; ++i) zero[i] = 0.f;
                for (int r = g; r < nrows; r += G) dot_store<EPC>(p, row_s[wave][r], ch0 * EPC, zero, 0.f, l);
            }
        }
        return;
    }
    const float scale = p.mean ? 1.f / static_cast<float>(k) : 1.f;
    const bool weighted = p.edge_w || p.slot_w;
    int head[CPL]; // head of each of this lane's chunks (per-head edge weights)
#pragma unroll
    for (int c = 0; c < CPL; ++c) head[c] = p.slot_w ? min((ch0 + c * L) * EPC / p.head_dim, p.heads - 1) : 0;
    float acc[CPL][EPC], acc2[DUAL ? CPL : 1][EPC];
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < EPC; ++i) {
            acc[c][i] = 0.f;
            if (DUAL) acc2[c][i] = 0.f;
        }
    // Lane group g walks the slots (row g + G*rl, edge j) of its rows in order; rl and j are the same
    // for every group, so the slot bookkeeping is scalar.
    const int rounds = (nrows + G - 1) / G;
    int rl = 0, j = 0; // slot at which the next load is issued
    const int total = rounds * k;
    for (int s0 = 0; s0 < total; s0 += U) {
        Chunk<T, EPC> v[U][CPL];
        float ww[U][CPL], ww2[DUAL ? U : 1][CPL];
        int rl_u = rl, j_u = j;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = g + rl_u * G;
            const bool ok = s0 + u < total && r < nrows;
            const int i = ok ? r * k + j_u : 0;
            const int rid = ids_s[wave][i];
            const T *rp = table + static_cast<int64_t>(rid) * p.ld;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                const int ch = ch0 + c * L;
                ww[u][c] = p.edge_w ? w_s[wave][i] : 1.f;
                if (ok && ch < n_chunks) {
                    v[u][c].load(rp + static_cast<int64_t>(ch) * EPC);
                    if (p.slot_w) ww[u][c] = p.slot_w[(e0 + i) * p.heads + head[c]];
                    if (DUAL) ww2[u][c] = p.slot_w2[(e0 + i) * p.heads + head[c]];
                } else {
                    v[u][c].zero();
                    if (DUAL) ww2[u][c] = 0.f;
                }
            }
            if (++j_u == k) {
                j_u = 0;
                ++rl_u;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (s0 + u < total) {
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    if (weighted) v[u][c].add_to(acc[c], ww[u][c]);
                    else v[u][c].add_to(acc[c]);
                    if (DUAL) v[u][c].add_to(acc2[c], ww2[u][c]);
                }
                if (++j == k) { // last edge of the row: store it, start the next
                    const int r = g + rl * G;
                    if (r < nrows) {
                        const int64_t row = row_s[wave][r];
#pragma unroll
                        for (int c = 0; c < CPL; ++c) {
                            const int ch = ch0 + c * L;
                            if (ch < n_chunks) {
                                store_out<EPC>(p, row, ch * EPC, acc[c], scale);
                                if (DUAL && !p.dot_out) store_out<EPC>(p, p.out2, p.ld_out2, row, ch * EPC, acc2[c], scale);
                            }
                        }
                        if constexpr (DUAL && CPL == 1) {
                            if (p.dot_out) dot_store<EPC>(p, row, ch0 * EPC, acc2[0], scale, l);
                        }
                    }
#pragma unroll
                    for (int c = 0; c < CPL; ++c)
#pragma unroll
                        for (int i = 0; i < EPC; ++i) {
                            acc[c][i] = 0.f;
                            if (DUAL) acc2[c][i] = 0.f;
                        }
                    j = 0;
                    ++rl;
                }
            }
        }
    }
}

// ---- long rows and hub chunks: one wavefront per item ----------------------------------------------
// SPLIT: the four wavefronts of a workgroup share one item, wavefront s taking the 64-edge segments s, s + 4,
// ...; their sums are added through LDS in wavefront order.  For launches of few items (the long rows of a
// sampled block), where one wavefront per item leaves most of the chip idle behind a serial walk of up to 511
// edges.
template <typename T, int EPC, int L, int CPL, bool DUAL, bool SPLIT = false>
__device__ __forceinline__ void agg_wave_body(const AggParams &p, const unsigned bx = blockIdx.x)
{
    constexpr int G = 64 / L;            // lane groups per wavefront
    constexpr int U = CPL == 2 ? 4 : ((G >= 16) ? 1 : ((G >= 8) ? 2 : ((G >= 4) ? 4 : 8))); // edges in flight per group and step
    constexpr int NACC = CPL * EPC * (DUAL ? 2 : 1);
    __shared__ float part_s[SPLIT ? 3 : 1][SPLIT ? NACC : 1][SPLIT ? L : 1]; // wavefronts 1..3, one value per (sum element, lane of group 0)
    const int lane = threadIdx.x & 63;
    const int ws = SPLIT ? static_cast<int>(threadIdx.x >> 6) : 0;
    const int64_t w = SPLIT ? static_cast<int64_t>(bx) : static_cast<int64_t>(bx) * 4 + (threadIdx.x >> 6);
    if (w >= p.n_wave_items) return;     // uniform per wavefront (per workgroup with SPLIT)
    int64_t e0, e1, row = -1;
    int slot = -1;
    if (w < p.n_hub_chunks) {
        const HubChunk c = p.hub_chunks[w];
        e0 = c.e0;
        e1 = c.e0 + c.len;
        slot = c.slot;
    } else {
        const int64_t q = p.n_hub_rows + (w - p.n_hub_chunks);
        row = p.perm[q];
        e0 = p.sptr[q];
        e1 = p.sptr[q + 1];
    }
    const int g = lane / L, l = lane % L;
    const int n_chunks = (p.d + EPC - 1) / EPC;
    const int ch0 = blockIdx.y * (L * CPL) + l;
    const T *table = static_cast<const T *>(p.table);
    const bool weighted = p.edge_w || p.slot_w;
    int head[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) head[c] = p.slot_w ? min((ch0 + c * L) * EPC / p.head_dim, p.heads - 1) : 0;
    float acc[CPL][EPC], acc2[DUAL ? CPL : 1][EPC];
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < EPC; ++i) {
            acc[c][i] = 0.f;
            if (DUAL) acc2[c][i] = 0.f;
        }

    for (int64_t base = e0 + 64 * ws; base < e1; base += SPLIT ? 256 : 64) {
        const int cnt = static_cast<int>(min(static_cast<int64_t>(64), e1 - base));
        int rid = 0;
        float wv = 1.f;
        if (lane < cnt) {
            const int c = p.sidx[base + lane];
            rid = p.gid ? static_cast<int>(p.gid[c]) : c;
            if (p.edge_w) wv = p.edge_w[c];
        }
        for (int j = 0; j < cnt; j += G * U) {
            Chunk<T, EPC> v[U][CPL];
            float ww[U][CPL], ww2[DUAL ? U : 1][CPL];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = j + u * G + g;
                const bool ok = k < cnt;
                const int r = __shfl(rid, k & 63, 64);
                const float wn = __shfl(wv, k & 63, 64);
                const T *rp = table + static_cast<int64_t>(r) * p.ld;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int ch = ch0 + c * L;
                    ww[u][c] = wn;
                    if (ok && ch < n_chunks) {
                        v[u][c].load(rp + static_cast<int64_t>(ch) * EPC);
                        if (p.slot_w) ww[u][c] = p.slot_w[(base + k) * p.heads + head[c]];
                        if (DUAL) ww2[u][c] = p.slot_w2[(base + k) * p.heads + head[c]];
                    } else {
                        v[u][c].zero();
                        if (DUAL) ww2[u][c] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    if (weighted) v[u][c].add_to(acc[c], ww[u][c]);
                    else v[u][c].add_to(acc[c]);
                    if (DUAL) v[u][c].add_to(acc2[c], ww2[u][c]);
                }
        }
    }
    // combine the lane groups (fixed butterfly order)
#pragma unroll
    for (int off = L; off < 64; off <<= 1)
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int i = 0; i < EPC; ++i) {
                acc[c][i] += __shfl_xor(acc[c][i], off, 64);
                if (DUAL) acc2[c][i] += __shfl_xor(acc2[c][i], off, 64);
            }
    if constexpr (SPLIT) {
        if (ws > 0 && g == 0) {
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int i = 0; i < EPC; ++i) {
                    part_s[ws - 1][c * EPC + i][l] = acc[c][i];
                    if (DUAL) part_s[ws - 1][CPL * EPC + c * EPC + i][l] = acc2[c][i];
                }
        }
        __syncthreads();
        if (ws > 0) return;
        if (g == 0) {
#pragma unroll
            for (int q = 0; q < 3; ++q)
#pragma unroll
                for (int c = 0; c < CPL; ++c)
#pragma unroll
                    for (int i = 0; i < EPC; ++i) {
                        acc[c][i] += part_s[q][c * EPC + i][l];
                        if (DUAL) acc2[c][i] += part_s[q][CPL * EPC + c * EPC + i][l];
                    }
        }
    }
    if (g != 0) return;
    if (slot >= 0) {
        float *o = p.ws + static_cast<int64_t>(slot) * p.ws_stride;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const int ch = ch0 + c * L;
            if (ch < n_chunks) {
#pragma unroll
                for (int i = 0; i < EPC; ++i) {
                    o[ch * EPC + i] = acc[c][i];
                    if (DUAL) o[p.ws_ld + ch * EPC + i] = acc2[c][i];
                }
            }
        }
    } else {
        const float scale = row_scale(p, e1 - e0);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const int ch = ch0 + c * L;
            if (ch < n_chunks) {
                store_out<EPC>(p, row, ch * EPC, acc[c], scale);
                if (DUAL && !p.dot_out) store_out<EPC>(p, p.out2, p.ld_out2, row, ch * EPC, acc2[c], scale);
            }
        }
        if constexpr (DUAL && CPL == 1) {
            if (p.dot_out) dot_store<EPC>(p, row, ch0 * EPC, acc2[0], scale, l);
        }
    }
}

// ---- hub rows: add the chunk partials in chunk order -------------------------------------------------
// One workgroup of 16 wavefronts per (hub row, tile of 256 columns); wavefront w adds the partials
// w, w+16, w+32, ... (four loads in flight) and the sixteen sums are combined through LDS in
// wavefront order, so the summation order is fixed.
constexpr int kCombineWaves = 16;
__device__ __forceinline__ void agg_hub_combine_body(const AggParams &p)
{
    __shared__ float4 part[kCombineWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t h = blockIdx.x;
    if (h >= p.n_hub_rows) return; // whole workgroup (a launch over several relations is as wide as the widest)
    const int64_t row = p.hub_only ? h : p.perm[h];
    const int64_t s0 = p.hub_chunk_ptr[h], s1 = p.hub_chunk_ptr[h + 1];
    const int col0 = (blockIdx.y * 64 + lane) * 4;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col0 < p.ws_ld) {
        for (int64_t s = s0 + wave; s < s1; s += 4 * kCombineWaves) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t t = s + kCombineWaves * u;
                if (t < s1) v[u] = *reinterpret_cast<const float4 *>(p.ws + t * p.ws_stride + col0);
                else v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) { a.x += v[u].x; a.y += v[u].y; a.z += v[u].z; a.w += v[u].w; }
        }
    }
    part[wave][lane] = a;
    __syncthreads();
    if (wave != 0 || (col0 >= p.d && !p.combine_dot)) return;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < kCombineWaves; ++k) {
        const float4 v = part[k][lane];
        acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    }
    const float scale = row_scale(p, p.sptr[h + 1] - p.sptr[h]);
    if (p.combine_dot) dot_store<4>(p, row, col0, acc, scale, lane); // all 64 lanes of wavefront 0 (one 256-column tile)
    else store_out<4>(p, row, col0, acc, scale);
}

// The kernels proper.  The single-relation forms take the parameters of their relation; the multi forms
// take up to kAggMulti parameter blocks and blockIdx.z picks one, so that the small relations of a
// sampled mini-batch block share one launch (and one launch latency) instead of queueing behind each
// other.  Every body guards its own item count, so a grid as wide as the widest relation is safe.
constexpr int kAggMulti = 4;
struct AggMulti {
    AggParams p[kAggMulti];
};
static_assert(sizeof(AggMulti) <= 3584, "kernel arguments are limited to 4 KB");

template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_batch_kernel(AggParams p) { agg_batch_body<T, EPC, L, CPL, DUAL>(p); }
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_wave_kernel(AggParams p) { agg_wave_body<T, EPC, L, CPL, DUAL>(p); }
__global__ void __launch_bounds__(64 * kCombineWaves) agg_hub_combine_kernel(AggParams p) { agg_hub_combine_body(p); }

template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_batch_multi_kernel(AggMulti m) { agg_batch_body<T, EPC, L, CPL, DUAL>(m.p[blockIdx.z]); }
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_wave_multi_kernel(AggMulti m) { agg_wave_body<T, EPC, L, CPL, DUAL>(m.p[blockIdx.z]); }
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_wave_split_kernel(AggParams p) { agg_wave_body<T, EPC, L, CPL, DUAL, true>(p); }
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_wave_split_multi_kernel(AggMulti m) { agg_wave_body<T, EPC, L, CPL, DUAL, true>(m.p[blockIdx.z]); }
__global__ void __launch_bounds__(64 * kCombineWaves) agg_hub_combine_multi_kernel(AggMulti m) { agg_hub_combine_body(m.p[blockIdx.z]); }
// Both row classes of a small launch in one grid: the first `wave_blocks` workgroups along x walk the split long rows,
// the rest the batches of short rows.  A sampled block has a handful of long rows; as a launch of their own they
// keep a few CUs busy for a serial walk of several hundred edges while the rest of the chip waits for the next kernel.
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_pair_kernel(AggParams p, unsigned wave_blocks)
{
    if (blockIdx.x < wave_blocks) agg_wave_body<T, EPC, L, CPL, DUAL, true>(p, blockIdx.x);
    else agg_batch_body<T, EPC, L, CPL, DUAL>(p, blockIdx.x - wave_blocks);
}
template <typename T, int EPC, int L, int CPL, bool DUAL>
__global__ void __launch_bounds__(256) agg_pair_multi_kernel(AggMulti m, unsigned wave_blocks)
{
    if (blockIdx.x < wave_blocks) agg_wave_body<T, EPC, L, CPL, DUAL, true>(m.p[blockIdx.z], blockIdx.x);
    else agg_batch_body<T, EPC, L, CPL, DUAL>(m.p[blockIdx.z], blockIdx.x - wave_blocks);
}

// ---- launch ---------------------------------------------------------------------------------------
constexpr int64_t kPairWaveBlocks = 256; // split long rows up to which both row classes share a launch
// algorithmic bytes of the two row classes of one call (for the optional profiler)
struct AggCost {
    double wave_bytes = 0, group_bytes = 0;
    bool timed = true; // false: no event brackets (the entry point that must not allocate)
};

template <typename T, int EPC, int L, int CPL, bool DUAL = false>
static heta_status launch_pair(const AggParams *ps, int n, int n_super, hipStream_t st, const AggCost &cost)
{
    if constexpr (!DUAL && EPC > 1) { // the two-weight form exists for the 128-bit paths
        if (ps[0].slot_w2) return launch_pair<T, EPC, L, CPL, true>(ps, n, n_super, st, cost);
    }
    const bool split = ps[0].wave_split != 0; // the same for every item of a launch (part of the plan's key)
    int64_t wave_blocks = 0, batch_blocks = 0;
    for (int i = 0; i < n; ++i) {
        wave_blocks = std::max<int64_t>(wave_blocks, split ? ps[i].n_wave_items : (ps[i].n_wave_items + 3) / 4);
        batch_blocks = std::max<int64_t>(batch_blocks, (ps[i].batch0[kShortDeg] + 3) / 4);
    }
    if (wave_blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "aggregate: too many long rows");
    AggMulti m{};
    if (n > 1)
        for (int i = 0; i < n; ++i) m.p[i] = ps[i];
    if (split && wave_blocks > 0 && wave_blocks <= kPairWaveBlocks && batch_blocks > 0) {
        ProfScope prof(cost.timed ? "agg_batch_kernel" : nullptr, st, cost.wave_bytes + cost.group_bytes, 0);
        const unsigned blocks = static_cast<unsigned>(wave_blocks + batch_blocks);
        if (n == 1)
            hipLaunchKernelGGL((agg_pair_kernel<T, EPC, L, CPL, DUAL>), dim3(blocks, n_super), dim3(256), 0, st, ps[0], (unsigned)wave_blocks);
        else
            hipLaunchKernelGGL((agg_pair_multi_kernel<T, EPC, L, CPL, DUAL>), dim3(blocks, n_super, n), dim3(256), 0, st, m, (unsigned)wave_blocks);
        HETA_LAUNCH_CHECK("agg_pair_kernel");
        return HETA_OK;
    }
    if (wave_blocks > 0) {
        ProfScope prof(cost.timed ? "agg_wave_kernel" : nullptr, st, cost.wave_bytes, 0);
        if (split && n == 1)
            hipLaunchKernelGGL((agg_wave_split_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)wave_blocks, n_super), dim3(256), 0, st, ps[0]);
        else if (split)
            hipLaunchKernelGGL((agg_wave_split_multi_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)wave_blocks, n_super, n), dim3(256), 0, st, m);
        else if (n == 1)
            hipLaunchKernelGGL((agg_wave_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)wave_blocks, n_super), dim3(256), 0, st, ps[0]);
        else
            hipLaunchKernelGGL((agg_wave_multi_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)wave_blocks, n_super, n), dim3(256), 0, st, m);
        HETA_LAUNCH_CHECK("agg_wave_kernel");
    }
    if (batch_blocks > 0) {
        ProfScope prof(cost.timed ? "agg_batch_kernel" : nullptr, st, cost.group_bytes, 0);
        if (n == 1)
            hipLaunchKernelGGL((agg_batch_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)batch_blocks, n_super), dim3(256), 0, st, ps[0]);
        else
            hipLaunchKernelGGL((agg_batch_multi_kernel<T, EPC, L, CPL, DUAL>), dim3((unsigned)batch_blocks, n_super, n), dim3(256), 0, st, m);
        HETA_LAUNCH_CHECK("agg_batch_kernel");
    }
    return HETA_OK;
}

template <typename T, int EPC>
static heta_status launch_vec(const AggParams *ps, int n, int n_chunks, hipStream_t st, const AggCost &c)
{
    if (n_chunks <= 1) return launch_pair<T, EPC, 1, 1>(ps, n, 1, st, c);
    if (n_chunks <= 2) return launch_pair<T, EPC, 2, 1>(ps, n, 1, st, c);
    if (n_chunks <= 4) return launch_pair<T, EPC, 4, 1>(ps, n, 1, st, c);
    if (n_chunks <= 8) return launch_pair<T, EPC, 8, 1>(ps, n, 1, st, c);
    if (n_chunks <= 16) return launch_pair<T, EPC, 16, 1>(ps, n, 1, st, c);
    if (n_chunks <= 32) return launch_pair<T, EPC, 32, 1>(ps, n, 1, st, c);
    if (n_chunks <= 64) return launch_pair<T, EPC, 64, 1>(ps, n, 1, st, c);
    return launch_pair<T, EPC, 64, 2>(ps, n, (n_chunks + 127) / 128, st, c);
}

// Everything about one aggregation that the host decides before a launch: the filled-in kernel
// parameters (all but the address of the hub partials), the kernel family it takes, the bytes of hub
// partials it needs and its algorithmic bytes.
struct AggPlan {
    AggParams p;
    heta_dtype in_dt = HETA_F32;
    bool vec = false, dual = false;
    int n_chunks = 0;
    size_t ws_need = 0;
    AggCost cost;
    double hub_bytes = 0;
    int64_t n_hub_rows = 0;
    // relations with equal keys run the same kernel instantiation with the same grid.y
    int key() const { return (in_dt == HETA_F32 ? 0 : 1) | (vec ? 2 : 0) | (dual ? 4 : 0) | (p.wave_split ? 8 : 0) | (n_chunks << 4); }
};

static bool agg_vectorized(const AggParams &p, heta_dtype in_dt)
{
    const size_t esz = dtype_size(in_dt);
    // with per-head weights a lane's chunk must not straddle two heads
    return aligned16(p.table) && ((p.ld * esz) % 16 == 0) && (!p.slot_w || p.head_dim % static_cast<int>(16 / esz) == 0);
}

static heta_status plan_aggregate(const Schedule &s, AggParams p, heta_dtype in_dt, AggPlan *plan)
{
    const size_t esz = dtype_size(in_dt);
    const bool vec = agg_vectorized(p, in_dt);
    const bool dual = p.slot_w2 != nullptr;
    const int epc = vec ? static_cast<int>(16 / esz) : 1;
    const int n_chunks = (p.d + epc - 1) / epc;
    int L = 64; // lanes per row, as the dispatch picks them
    if (vec) {
        L = 1;
        while (L < n_chunks && L < 64) L <<= 1;
    }
    const int G = 64 / L;
    // rows with at least this many edges get a whole wavefront
    const int wave_min = kShortDeg;
    const int64_t n_long_or_hub = s.rows_with_deg_ge[wave_min];
    p.sptr = s.d_sptr;
    p.sidx = s.d_sidx;
    p.perm = s.d_perm;
    p.hub_chunks = s.d_hub_chunks;
    p.hub_chunk_ptr = s.d_hub_chunk_ptr;
    p.n_hub_chunks = s.n_hub_chunks;
    p.n_hub_rows = s.n_hub_rows;
    p.n_wave_items = s.n_hub_chunks + (p.hub_only ? 0 : n_long_or_hub - s.n_hub_rows);
    // at most two wavefronts per SIMD's worth of items: spread each over a workgroup (decided per relation, so
    // that a relation is summed in the same order whatever shares its launch)
    p.wave_split = p.n_wave_items <= kWaveSplitMaxItems;
    p.n_rows = s.n_rows;
    // short rows: bucket b = degree kShortDeg - 1 - b, in schedule order (descending degree)
    int64_t batches = 0;
    for (int b = 0; b < kShortDeg; ++b) {
        const int k = kShortDeg - 1 - b;
        const int64_t first = s.rows_with_deg_ge[k + 1], count = s.rows_with_deg_ge[k] - first;
        p.batch0[b] = static_cast<int32_t>(batches);
        p.row0[b] = static_cast<int32_t>(first);
        p.edge0[b] = s.edges_with_deg_ge[k + 1];
        if (!p.hub_only) batches += (count + batch_rows(k, G) - 1) / batch_rows(k, G);
        if (batches > 0x7ffffff0) return fail(HETA_ERR_UNSUPPORTED, "aggregate: too many short rows");
    }
    p.batch0[kShortDeg] = static_cast<int32_t>(batches);
    p.row0[kShortDeg] = static_cast<int32_t>(s.n_rows);
    p.ws_ld = (static_cast<int64_t>(p.d) + 7) / 8 * 8;
    p.ws_stride = dual ? 2 * p.ws_ld : p.ws_ld;
    p.ws = nullptr;
    if (s.n_hub_rows > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "aggregate: too many hub rows");
    plan->ws_need = static_cast<size_t>(s.n_hub_chunks) * p.ws_stride * sizeof(float);
    // Algorithmic bytes per row class: one neighbour row and one 4-byte index per edge, one 8-byte
    // row pointer and one output row per row.  Hub rows' outputs are written by the combine kernel.
    const double osz = p.out_bf16 ? 2.0 : 4.0;
    const double per_edge = static_cast<double>(p.d) * esz + 4.0 + (p.slot_w ? 4.0 * p.heads : 0.0) + (dual ? 4.0 * p.heads : 0.0);
    const double per_row = 8.0 + p.d * osz * (dual ? 2.0 : 1.0);
    const double e_wave = static_cast<double>(s.edges_with_deg_ge[wave_min]);
    const double r_long = static_cast<double>(n_long_or_hub - s.n_hub_rows);
    plan->cost.wave_bytes = e_wave * per_edge + r_long * per_row;
    plan->cost.group_bytes = (static_cast<double>(s.n_edges) - e_wave) * per_edge +
                             static_cast<double>(s.n_rows - n_long_or_hub) * per_row;
    plan->hub_bytes = static_cast<double>(s.n_hub_rows) * per_row;
    plan->n_hub_rows = s.n_hub_rows;
    plan->p = p;
    plan->in_dt = in_dt;
    plan->vec = vec;
    plan->dual = dual;
    plan->n_chunks = n_chunks;
    return HETA_OK;
}

// Launches n planned aggregations of one key (n = 1: the single-relation kernels) whose hub partial
// addresses are set.
static heta_status launch_plans(const AggPlan *plans, int n, hipStream_t st, bool timed)
{
    AggParams ps[kAggMulti];
    AggCost cost;
    cost.timed = timed;
    double hub_bytes = 0;
    int64_t hub_rows = 0;
    for (int i = 0; i < n; ++i) {
        ps[i] = plans[i].p;
        cost.wave_bytes += plans[i].cost.wave_bytes;
        cost.group_bytes += plans[i].cost.group_bytes;
        hub_bytes += plans[i].hub_bytes;
        hub_rows = std::max(hub_rows, plans[i].n_hub_rows);
    }
    const AggPlan &f = plans[0];
    heta_status e;
    if (f.in_dt == HETA_F32)
        e = f.vec ? launch_vec<float, 4>(ps, n, f.n_chunks, st, cost) : launch_pair<float, 1, 64, 2>(ps, n, (f.n_chunks + 127) / 128, st, cost);
    else
        e = f.vec ? launch_vec<bf16_t, 8>(ps, n, f.n_chunks, st, cost) : launch_pair<bf16_t, 1, 64, 2>(ps, n, (f.n_chunks + 127) / 128, st, cost);
    if (e != HETA_OK) return e;
    if (hub_rows > 0) {
        const int tiles = static_cast<int>((f.p.ws_ld + 255) / 256);
        ProfScope prof(timed ? "agg_hub_combine_kernel" : nullptr, st, hub_bytes, 0);
        if (n == 1) {
            hipLaunchKernelGGL(agg_hub_combine_kernel, dim3((unsigned)hub_rows, tiles), dim3(64 * kCombineWaves), 0, st, ps[0]);
            HETA_LAUNCH_CHECK("agg_hub_combine_kernel");
            if (f.dual) {
                AggParams p2 = ps[0];
                p2.ws = ps[0].ws + ps[0].ws_ld;
                p2.out = ps[0].out2;
                p2.ld_out = ps[0].ld_out2;
                p2.combine_dot = ps[0].dot_out ? 1 : 0;
                hipLaunchKernelGGL(agg_hub_combine_kernel, dim3((unsigned)hub_rows, tiles), dim3(64 * kCombineWaves), 0, st, p2);
                HETA_LAUNCH_CHECK("agg_hub_combine_kernel");
            }
        } else {
            AggMulti m{};
            for (int i = 0; i < n; ++i) m.p[i] = ps[i];
            hipLaunchKernelGGL(agg_hub_combine_multi_kernel, dim3((unsigned)hub_rows, tiles, n), dim3(64 * kCombineWaves), 0, st, m);
            HETA_LAUNCH_CHECK("agg_hub_combine_kernel");
        }
    }
    return HETA_OK;
}

// The shared entry of forward and backward.  With fixed_ws the hub partials go to that buffer of
// fixed_ws_bytes instead of the handle's grow-on-demand workspace, and nothing is allocated: a shape
// that does not fit is an error, and the launches are not bracketed by profiling events.
static heta_status run_aggregate(heta_graph *g, const Schedule &s, AggParams p, heta_dtype in_dt,
                                 int64_t table_elems_ld, hipStream_t st, float *fixed_ws = nullptr,
                                 size_t fixed_ws_bytes = 0)
{
    (void)table_elems_ld;
    if (s.n_rows == 0) return HETA_OK;
    if (p.slot_w2 && !agg_vectorized(p, in_dt)) { // the two-weight kernels exist for the 128-bit paths only: two passes otherwise
        AggParams a = p, b = p;
        a.slot_w2 = nullptr;
        b.slot_w = p.slot_w2;
        b.slot_w2 = nullptr;
        b.out = p.out2;
        b.ld_out = p.ld_out2;
        heta_status e1 = run_aggregate(g, s, a, in_dt, table_elems_ld, st);
        return e1 != HETA_OK ? e1 : run_aggregate(g, s, b, in_dt, table_elems_ld, st);
    }
    AggPlan plan;
    heta_status e = plan_aggregate(s, p, in_dt, &plan);
    if (e != HETA_OK) return e;
    if (plan.ws_need > 0) {
        if (fixed_ws) {
            if (plan.ws_need > fixed_ws_bytes)
                return fail(HETA_ERR_UNSUPPORTED,
                            "aggregate: %lld hub chunks of %d columns need %zu bytes of partial sums, the fixed scratch "
                            "holds %zu; use the allocating entry point",
                            (long long)s.n_hub_chunks, p.d, plan.ws_need, fixed_ws_bytes);
            plan.p.ws = fixed_ws;
        } else {
            e = ensure_workspace(g, plan.ws_need);
            if (e != HETA_OK) return e;
            plan.p.ws = static_cast<float *>(g->d_ws);
        }
    }
    return launch_plans(&plan, 1, st, fixed_ws == nullptr);
}

// Several independent aggregations (no two write the same output) in as few launches as their kernel
// families allow: plans of one key share launches of up to kAggMulti relations, each with a region of
// its own in the hub-partial workspace.
static heta_status run_aggregate_multi(heta_graph *g, std::vector<AggPlan> &plans, hipStream_t st)
{
    size_t total = 0;
    for (const AggPlan &pl : plans) total += (pl.ws_need + 255) / 256 * 256;
    if (total > 0) {
        heta_status e = ensure_workspace(g, total);
        if (e != HETA_OK) return e;
        size_t off = 0;
        for (AggPlan &pl : plans) {
            if (pl.ws_need > 0) pl.p.ws = reinterpret_cast<float *>(static_cast<char *>(g->d_ws) + off);
            off += (pl.ws_need + 255) / 256 * 256;
        }
    }
    std::vector<char> done(plans.size(), 0);
    for (size_t i = 0; i < plans.size(); ++i) {
        if (done[i]) continue;
        AggPlan group[kAggMulti];
        int n = 0;
        for (size_t j = i; j < plans.size() && n < kAggMulti; ++j)
            if (!done[j] && plans[j].key() == plans[i].key()) {
                group[n++] = plans[j];
                done[j] = 1;
            }
        heta_status e = launch_plans(group, n, st, true);
        if (e != HETA_OK) return e;
    }
    return HETA_OK;
}

// Weighted aggregation with one weight per (edge slot of the schedule, head): the second half of the
// attention aggregation (heta_attention.hip computes the weights).
heta_status aggregate_slot_weighted(heta_graph *g, const Schedule &s, const void *table, heta_dtype dt, int64_t ld,
                                    int d, const float *slot_w, int heads, void *out, heta_dtype out_dt,
                                    int64_t ld_out, float beta, hipStream_t st, const float *slot_w2, void *out2,
                                    int64_t ld_out2, const SecondSumDot *dot, bool *dot_done)
{
    AggParams p{};
    p.table = table;
    p.ld = ld;
    p.slot_w = slot_w;
    p.slot_w2 = slot_w2;
    p.out2 = out2;
    p.ld_out2 = ld_out2;
    p.heads = heads;
    p.head_dim = d / heads;
    p.out = out;
    p.ld_out = ld_out;
    p.out_bf16 = (out_dt == HETA_BF16);
    p.beta = beta;
    p.d = d;
    if (dot_done) *dot_done = false;
    if (dot && slot_w2 && dot->z && dot->out) {
        // the dot form needs: the 128-bit path, one chunk per lane (a row inside one lane group), heads that are a
        // power-of-two number of chunks wide for both the row kernels' chunk (16 bytes of the gathered type) and the
        // hub combine's (4 columns), z rows whose chunks are aligned, a single 256-column tile in the combine
        const int epc = static_cast<int>(16 / dtype_size(dt));
        const int hd = p.head_dim, lph = hd / epc, lph4 = hd / 4;
        const size_t zsz = dtype_size(dot->z_dt);
        const bool ok = agg_vectorized(p, dt) && d % epc == 0 && d / epc <= 64 && d <= 256 && hd % epc == 0 && hd % 4 == 0 &&
                        lph > 0 && (lph & (lph - 1)) == 0 && (lph4 & (lph4 - 1)) == 0 &&
                        reinterpret_cast<uintptr_t>(dot->z) % (epc * zsz) == 0 && dot->ld_z % epc == 0;
        if (ok) {
            p.dot_z = dot->z;
            p.ld_z = dot->ld_z;
            p.dot_z_bf16 = dot->z_dt == HETA_BF16;
            p.dot_corr = dot->corr;
            p.dot_out = dot->out;
            if (dot_done) *dot_done = true;
        }
    }
    return run_aggregate(g, s, p, dt, ld, st);
}

// The hub rows of a schedule only (rows of at least kHubMinDeg edges), reduced into a compact fp32
// array: out[h] is the sum (or mean) of the h-th row of the schedule order.  For callers that handle
// all other rows themselves (the fused aggregate-and-project kernel).
heta_status aggregate_hub_rows(heta_graph *g, const Schedule &s, const void *table, heta_dtype dt, int64_t ld, int d,
                               const int64_t *gid, int mean, float *out, int64_t ld_out, hipStream_t st)
{
    if (s.n_hub_rows == 0) return HETA_OK;
    AggParams p{};
    p.table = table;
    p.ld = ld;
    p.gid = gid;
    p.mean = mean;
    p.hub_only = 1;
    p.out = out;
    p.ld_out = ld_out;
    p.d = d;
    return run_aggregate(g, s, p, dt, ld, st);
}

// ---- plain row gather and id check -------------------------------------------------------------------
template <typename V>
__global__ void __launch_bounds__(256) gather_rows_kernel(const V *table, int64_t ld_v, const int64_t *gid,
                                                          int64_t n, int per_row, V *out, int64_t ld_out_v)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t i = t / per_row;
    const int c = static_cast<int>(t % per_row);
    if (i >= n) return;
    out[i * ld_out_v + c] = table[gid[i] * ld_v + c];
}

__global__ void __launch_bounds__(256) check_ids_kernel(const int64_t *ids, int64_t n, int64_t limit, int *flag)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n && (ids[i] < 0 || ids[i] >= limit)) *flag = 1; // every writer stores the same value
}

// ---- fixed scratch of the entry point that allocates nothing ------------------------------------------
// Hub-row partial sums of heta_rel_aggregate_fwd_noalloc.  The array lives in the code object, so every
// device the library runs on holds a copy of its own until the process ends.  In host code its name is
// only a handle for hipGetSymbolAddress: kernels get the per-device address looked up below.
constexpr size_t kNoallocScratchBytes = static_cast<size_t>(HETA_NOALLOC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

constexpr int kMaxDevices = 64;
static float *g_scratch_ptr[kMaxDevices];          // per device, filled once with that device current
static std::once_flag g_scratch_once[kMaxDevices];

// Address of the current device's copy of `scratch` (looked up on the first call per device).
static heta_status noalloc_scratch(float **out)
{
    int dev = 0;
    HETA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(HETA_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices);
    hipError_t err = hipSuccess;
    std::call_once(g_scratch_once[dev], [&] {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        g_scratch_ptr[dev] = err == hipSuccess ? static_cast<float *>(ptr) : nullptr;
    });
    if (err != hipSuccess || !g_scratch_ptr[dev])
        return fail(HETA_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev,
                    err != hipSuccess ? hipGetErrorString(err) : "no address");
    *out = g_scratch_ptr[dev];
    return HETA_OK;
}

heta_status noalloc_scratch_init()
{
    float *p = nullptr;
    return noalloc_scratch(&p);
}

} // namespace heta

using namespace heta;

// argument checks shared by the two forward entry points
static heta_status check_fwd_args(const char *fn, heta_graph *g, int32_t rel, heta_reduce op, const void *src_table,
                                  heta_dtype in_dt, int64_t ld_src, int32_t d, int64_t n_table_rows,
                                  const int64_t *src_gid, void *out, heta_dtype out_dt, int64_t ld_out, float beta)
{
    if (!g || !src_table || !out) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", fn);
    if (rel < 0 || rel >= (int32_t)g->rels.size()) return fail(HETA_ERR_INVALID_ARG, "%s: relation %d out of range", fn, rel);
    if (op != HETA_SUM && op != HETA_MEAN) return fail(HETA_ERR_INVALID_ARG, "%s: bad reduce op", fn);
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "%s: beta must be 0 or 1", fn);
    if (!valid_dtype(in_dt) || !valid_dtype(out_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", fn);
    if (d <= 0 || ld_src < d || ld_out < d)
        return fail(HETA_ERR_SHAPE, "%s: need 0 < d <= ld (d=%d ld_src=%lld ld_out=%lld)", fn, d, (long long)ld_src,
                    (long long)ld_out);
    const Relation &r = g->rels[rel];
    if (n_table_rows < 0 || n_table_rows >= (int64_t(1) << 31)) return fail(HETA_ERR_SHAPE, "%s: n_table_rows outside [0, 2^31)", fn);
    if (!src_gid && n_table_rows < r.n_src)
        return fail(HETA_ERR_SHAPE, "%s: table has %lld rows, relation needs %lld", fn, (long long)n_table_rows,
                    (long long)r.n_src);
    if ((reinterpret_cast<uintptr_t>(src_table) % dtype_size(in_dt)) || (reinterpret_cast<uintptr_t>(out) % dtype_size(out_dt)))
        return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", fn);
    return HETA_OK;
}

static AggParams fwd_params(heta_reduce op, const void *src_table, int64_t ld_src, int32_t d, const int64_t *src_gid,
                            void *out, heta_dtype out_dt, int64_t ld_out, float beta)
{
    AggParams p{};
    p.table = src_table;
    p.ld = ld_src;
    p.gid = src_gid;
    p.edge_w = nullptr;
    p.mean = (op == HETA_MEAN);
    p.out = out;
    p.ld_out = ld_out;
    p.out_bf16 = (out_dt == HETA_BF16);
    p.beta = beta;
    p.d = d;
    return p;
}

static heta_status check_bwd_args(const char *fn, heta_graph *g, int32_t rel, heta_reduce op, const void *grad_out,
                                  heta_dtype go_dt, int64_t ld_go, int32_t d, float *grad_src, int64_t ld_gs, float beta)
{
    if (!g || !grad_out || !grad_src) return fail(HETA_ERR_INVALID_ARG, "%s: null argument", fn);
    if (rel < 0 || rel >= (int32_t)g->rels.size()) return fail(HETA_ERR_INVALID_ARG, "%s: relation %d out of range", fn, rel);
    if (op != HETA_SUM && op != HETA_MEAN) return fail(HETA_ERR_INVALID_ARG, "%s: bad reduce op", fn);
    if (!valid_dtype(go_dt)) return fail(HETA_ERR_INVALID_ARG, "%s: bad dtype", fn);
    if (d <= 0 || ld_go < d || ld_gs < d)
        return fail(HETA_ERR_SHAPE, "%s: need 0 < d <= ld (d=%d ld_go=%lld ld_gs=%lld)", fn, d, (long long)ld_go,
                    (long long)ld_gs);
    if (beta != 0.f && beta != 1.f) return fail(HETA_ERR_SHAPE, "%s: beta must be 0 or 1", fn);
    if ((reinterpret_cast<uintptr_t>(grad_out) % dtype_size(go_dt)) || (reinterpret_cast<uintptr_t>(grad_src) & 3u))
        return fail(HETA_ERR_INVALID_ARG, "%s: pointer not aligned to its element size", fn);
    return HETA_OK;
}

static AggParams bwd_params(const Relation &r, heta_reduce op, const void *grad_out, int64_t ld_go, int32_t d,
                            float *grad_src, int64_t ld_gs, float beta)
{
    AggParams p{};
    p.table = grad_out;
    p.ld = ld_go;
    p.gid = nullptr;
    p.edge_w = (op == HETA_MEAN) ? r.d_inv_deg : nullptr;
    p.mean = 0;
    p.out = grad_src;
    p.ld_out = ld_gs;
    p.out_bf16 = 0;
    p.beta = beta;
    p.d = d;
    return p;
}

extern "C" {

heta_status heta_rel_aggregate_fwd(heta_graph *g, int32_t rel, heta_reduce op, const void *src_table,
                                   heta_dtype in_dt, int64_t ld_src, int32_t d, int64_t n_table_rows,
                                   const int64_t *src_gid, void *out, heta_dtype out_dt, int64_t ld_out,
                                   float beta, void *hip_stream)
{
    heta_status e = check_fwd_args("heta_rel_aggregate_fwd", g, rel, op, src_table, in_dt, ld_src, d, n_table_rows, src_gid,
                                   out, out_dt, ld_out, beta);
    if (e != HETA_OK) return e;
    const AggParams p = fwd_params(op, src_table, ld_src, d, src_gid, out, out_dt, ld_out, beta);
    return run_aggregate(g, g->rels[rel].csr, p, in_dt, ld_src, as_stream(hip_stream));
}

heta_status heta_rel_aggregate_fwd_noalloc(heta_graph *g, int32_t rel, heta_reduce op, const void *src_table,
                                           heta_dtype in_dt, int64_t ld_src, int32_t d, int64_t n_table_rows,
                                           const int64_t *src_gid, void *out, heta_dtype out_dt, int64_t ld_out,
                                           float beta, void *hip_stream)
{
    heta_status e = check_fwd_args("heta_rel_aggregate_fwd_noalloc", g, rel, op, src_table, in_dt, ld_src, d, n_table_rows,
                                   src_gid, out, out_dt, ld_out, beta);
    if (e != HETA_OK) return e;
    float *ws = nullptr;
    e = noalloc_scratch(&ws);
    if (e != HETA_OK) return e;
    const AggParams p = fwd_params(op, src_table, ld_src, d, src_gid, out, out_dt, ld_out, beta);
    // Every partial row the combine kernel reads is written by this call's own chunk kernel first, so
    // what an earlier call left in the array is never read and nothing needs clearing.
    return run_aggregate(g, g->rels[rel].csr, p, in_dt, ld_src, as_stream(hip_stream), ws, kNoallocScratchBytes);
}

heta_status heta_rel_aggregate_bwd(heta_graph *g, int32_t rel, heta_reduce op, const void *grad_out,
                                   heta_dtype go_dt, int64_t ld_go, int32_t d, float *grad_src, int64_t ld_gs,
                                   float beta, void *hip_stream)
{
    heta_status e = check_bwd_args("heta_rel_aggregate_bwd", g, rel, op, grad_out, go_dt, ld_go, d, grad_src, ld_gs, beta);
    if (e != HETA_OK) return e;
    const Relation &r = g->rels[rel];
    return run_aggregate(g, r.csc, bwd_params(r, op, grad_out, ld_go, d, grad_src, ld_gs, beta), go_dt, ld_go,
                         as_stream(hip_stream));
}

// Byte ranges [lo, hi) of the outputs of the items of one multi call must not overlap.
static heta_status check_disjoint(const char *fn, const std::vector<std::pair<uintptr_t, uintptr_t>> &ranges)
{
    for (size_t i = 0; i < ranges.size(); ++i)
        for (size_t j = i + 1; j < ranges.size(); ++j)
            if (ranges[i].first < ranges[j].second && ranges[j].first < ranges[i].second)
                return fail(HETA_ERR_INVALID_ARG, "%s: the outputs of items %zu and %zu overlap", fn, i, j);
    return HETA_OK;
}

static std::pair<uintptr_t, uintptr_t> out_range(const void *out, int64_t rows, int64_t ld, int32_t d, size_t esz)
{
    const uintptr_t lo = reinterpret_cast<uintptr_t>(out);
    return {lo, rows > 0 ? lo + static_cast<uintptr_t>(((rows - 1) * ld + d) * static_cast<int64_t>(esz)) : lo};
}

heta_status heta_rel_aggregate_fwd_multi(heta_graph *g, int32_t n, const heta_agg_item *items, heta_reduce op,
                                         heta_dtype in_dt, heta_dtype out_dt, void *hip_stream)
{
    const char *fn = "heta_rel_aggregate_fwd_multi";
    if (n < 0 || (n > 0 && !items)) return fail(HETA_ERR_INVALID_ARG, "%s: bad item array", fn);
    if (n == 0) return HETA_OK;
    try {
        std::vector<AggPlan> plans;
        std::vector<std::pair<uintptr_t, uintptr_t>> ranges;
        for (int32_t i = 0; i < n; ++i) {
            const heta_agg_item &it = items[i];
            heta_status e = check_fwd_args(fn, g, it.rel, op, it.in, in_dt, it.ld_in, it.d, it.n_table_rows, it.src_gid,
                                           it.out, out_dt, it.ld_out, it.beta);
            if (e != HETA_OK) return e;
            const Relation &r = g->rels[it.rel];
            ranges.push_back(out_range(it.out, r.n_dst, it.ld_out, it.d, dtype_size(out_dt)));
            if (r.csr.n_rows == 0) continue;
            AggPlan pl;
            e = plan_aggregate(r.csr, fwd_params(op, it.in, it.ld_in, it.d, it.src_gid, it.out, out_dt, it.ld_out, it.beta),
                               in_dt, &pl);
            if (e != HETA_OK) return e;
            plans.push_back(pl);
        }
        heta_status e = check_disjoint(fn, ranges);
        if (e != HETA_OK) return e;
        return run_aggregate_multi(g, plans, as_stream(hip_stream));
    } catch (const std::bad_alloc &) {
        return fail(HETA_ERR_OOM, "%s: host allocation failed", fn);
    } catch (...) {
        return fail(HETA_ERR_DEVICE, "%s: unexpected exception", fn);
    }
}

heta_status heta_rel_aggregate_bwd_multi(heta_graph *g, int32_t n, const heta_agg_item *items, heta_reduce op,
                                         heta_dtype in_dt, void *hip_stream)
{
    const char *fn = "heta_rel_aggregate_bwd_multi";
    if (n < 0 || (n > 0 && !items)) return fail(HETA_ERR_INVALID_ARG, "%s: bad item array", fn);
    if (n == 0) return HETA_OK;
    try {
        std::vector<AggPlan> plans;
        std::vector<std::pair<uintptr_t, uintptr_t>> ranges;
        for (int32_t i = 0; i < n; ++i) {
            const heta_agg_item &it = items[i];
            heta_status e = check_bwd_args(fn, g, it.rel, op, it.in, in_dt, it.ld_in, it.d, static_cast<float *>(it.out),
                                           it.ld_out, it.beta);
            if (e != HETA_OK) return e;
            const Relation &r = g->rels[it.rel];
            ranges.push_back(out_range(it.out, r.n_src, it.ld_out, it.d, sizeof(float)));
            if (r.csc.n_rows == 0) continue;
            AggPlan pl;
            e = plan_aggregate(r.csc, bwd_params(r, op, it.in, it.ld_in, it.d, static_cast<float *>(it.out), it.ld_out, it.beta),
                               in_dt, &pl);
            if (e != HETA_OK) return e;
            plans.push_back(pl);
        }
        heta_status e = check_disjoint(fn, ranges);
        if (e != HETA_OK) return e;
        return run_aggregate_multi(g, plans, as_stream(hip_stream));
    } catch (const std::bad_alloc &) {
        return fail(HETA_ERR_OOM, "%s: host allocation failed", fn);
    } catch (...) {
        return fail(HETA_ERR_DEVICE, "%s: unexpected exception", fn);
    }
}

heta_status heta_feature_gather(const void *table, heta_dtype dt, int64_t ld_table, int32_t d,
                                int64_t n_table_rows, const int64_t *gid, int64_t n, void *out,
                                int64_t ld_out, void *hip_stream)
{
    if (!table || !gid || !out) return fail(HETA_ERR_INVALID_ARG, "heta_feature_gather: null argument");
    if (!valid_dtype(dt)) return fail(HETA_ERR_INVALID_ARG, "heta_feature_gather: bad dtype");
    if (d <= 0 || ld_table < d || ld_out < d || n < 0 || n_table_rows < 0)
        return fail(HETA_ERR_SHAPE, "heta_feature_gather: bad shape");
    if (n == 0) return HETA_OK;
    const size_t esz = dtype_size(dt);
    if ((reinterpret_cast<uintptr_t>(table) % esz) || (reinterpret_cast<uintptr_t>(out) % esz))
        return fail(HETA_ERR_INVALID_ARG, "heta_feature_gather: pointer not aligned to its element size");
    hipStream_t st = as_stream(hip_stream);
    const size_t row_bytes = static_cast<size_t>(d) * esz;
    const bool vec = aligned16(table) && aligned16(out) && (ld_table * esz) % 16 == 0 && (ld_out * esz) % 16 == 0 &&
                     row_bytes % 16 == 0;
    if (vec) {
        const int per_row = static_cast<int>(row_bytes / 16);
        const int64_t threads = n * per_row;
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           static_cast<const uint4 *>(table), (int64_t)(ld_table * esz / 16), gid, n, per_row,
                           static_cast<uint4 *>(out), (int64_t)(ld_out * esz / 16));
    } else if (esz == 4) {
        const int64_t threads = n * d;
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           static_cast<const uint32_t *>(table), ld_table, gid, n, (int)d,
                           static_cast<uint32_t *>(out), ld_out);
    } else {
        const int64_t threads = n * d;
        hipLaunchKernelGGL(gather_rows_kernel<uint16_t>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           static_cast<const uint16_t *>(table), ld_table, gid, n, (int)d,
                           static_cast<uint16_t *>(out), ld_out);
    }
    HETA_LAUNCH_CHECK("gather_rows_kernel");
    return HETA_OK;
}

heta_status heta_check_ids(const int64_t *ids, int64_t n, int64_t limit, void *hip_stream)
{
    if (n < 0 || (n > 0 && !ids)) return fail(HETA_ERR_INVALID_ARG, "heta_check_ids: bad arguments");
    if (n == 0) return HETA_OK;
    hipStream_t st = as_stream(hip_stream);
    int *flag = nullptr;
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(&flag), sizeof(int)));
    int h = 0;
    hipError_t e = hipMemcpyAsync(flag, &h, sizeof(int), hipMemcpyHostToDevice, st);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(check_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ids, n, limit, flag);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(flag);
    if (e != hipSuccess) return fail(HETA_ERR_DEVICE, "heta_check_ids: %s", hipGetErrorString(e));
    if (h) return fail(HETA_ERR_INVALID_ARG, "heta_check_ids: an id lies outside [0, %lld)", (long long)limit);
    return HETA_OK;
}

} // extern "C"
