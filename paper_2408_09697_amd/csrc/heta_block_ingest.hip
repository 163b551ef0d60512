// Ingest of a whole sampled block on the device: the index data of up to 32 small relations at once.
//
// A mini-batch block (Section 2.2 of the paper: the sampled k-hop neighbourhood, one bipartite graph per
// relation and hop) has a handful of relations of 10^3 .. 10^5 edges each.  The per-relation device
// pipeline costs twenty launches per relation, the host path a few hundred microseconds of CPU work and
// an upload (plus a download when the block was sampled on the device).  Here the relations of a block
// are treated as ONE block-diagonal bipartite graph over the concatenated destination rows, source nodes
// and edges, so that every step is one launch (or one sort / one scan) for the whole block:
//
//   rows kernel     degrees, 1/deg, validation, degree histograms, sort keys (relation, 512 - min(deg, 512))
//   edges kernel    validation, the CSR's neighbour ids copied, (global source id, global edge id) pairs
//   sort            stable LSD radix sort of those pairs = the transpose of every relation at once
//   colptr, rows    column offsets by binary search in the sorted keys; the CSC's degrees, keys, histograms
//   sort            one stable sort of all CSR and CSC rows by (schedule, capped degree) = every schedule's
//                   row order (a relation's rows stay contiguous because the schedule id leads the key)
//   scan, fill      schedule-ordered offsets and neighbour ids, hub chunk lists
//
// Values are written relation-local (row ids, neighbour ids, offsets) into per-relation slices of one
// arena, so the aggregation kernels see exactly what the other ingest paths produce; the results are
// bit-identical to theirs.  Everything is deterministic: integer atomics only count, every placement is
// by rank.  Inputs are sanitised as they are read (offsets clamped into [0, E], ids into [0, n_src)), so
// a malformed CSR cannot send any later access out of bounds; it is reported after the one
// synchronisation at the end.
#include <algorithm>
#include <cstring>
#include <vector>

#include "heta_internal.h"

namespace heta {

namespace {

constexpr int kMaxBlockRels = 32;

struct BlockTables { // passed by value
    int n_rel;
    int64_t dst_off[kMaxBlockRels + 1];  // destination rows of relation i are global rows [dst_off[i], dst_off[i+1])
    int64_t src_off[kMaxBlockRels + 1];  // its source nodes
    int64_t edge_off[kMaxBlockRels + 1]; // its edges
    int64_t hub_off[2 * kMaxBlockRels + 1];    // chunk descriptors of schedule s (s < n_rel: CSR of relation s; else CSC of s - n_rel)
    int64_t hubptr_off[2 * kMaxBlockRels + 1]; // its chunk range array
};

struct BlockInputs { // passed by value
    const int64_t *rowptr[kMaxBlockRels];
    const int32_t *col[kMaxBlockRels];
};

// largest i < n with off[i] <= x (off non-decreasing, off[0] <= x): the segment that owns x; among segments
// starting at the same offset the last one, which is the non-empty one
__device__ __forceinline__ int seg_of(const int64_t *off, int n, int64_t x)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid;
        else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ int64_t last_le64(const int64_t *a, int64_t n, int64_t x)
{
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (a[mid] <= x) lo = mid;
        else hi = mid;
    }
    return lo;
}

enum : unsigned long long { kBadPtr0 = 1, kBadDecrease = 2, kBadTotal = 3, kBadCol = 4 };

// The error word holds the complement of the smallest (kind, relation, position) reported, 0 while nothing is:
// it is cleared by the same fill as the counters beside it.
__device__ __forceinline__ void report(unsigned long long *err, unsigned long long kind, int rel, int64_t at)
{
    atomicMax(err, ~((kind << 56) | (static_cast<unsigned long long>(rel) << 48) | static_cast<unsigned long long>(at)));
}

__device__ __forceinline__ int64_t clamp64(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

// One thread per global row of one direction.  CSR (CSC = 0): offsets come from the caller's rowptr, sanitised;
// CSC (CSC = 1): from the global column offsets found in the sorted keys.  Writes the relation-local offsets,
// the global offsets (CSR only; the CSC's are an input), 1/deg (CSR only), the schedule sort pair and the
// degree histograms of the row's schedule.
constexpr int kBlkRowsThreads = 1024; // rows per workgroup of blk_rows_kernel
constexpr int kBlkLocalSched = 4;     // schedules whose histograms a workgroup keeps in LDS
template <int CSC>
__device__ __forceinline__ void blk_rows_body(const unsigned bx, const BlockTables &t, const BlockInputs &in, int64_t n_rows_total,
                                              int64_t sched_pos0, int64_t *ptr_local, int64_t *ptr_global, float *inv_deg, uint32_t *key,
                                              uint32_t *val, unsigned long long *hist, unsigned long long *err)
{
    // degree histograms of the workgroup's rows: the schedule of its first row and the three after it (a workgroup's
    // 1,024 consecutive rows rarely span more) are counted in LDS and reach the global counters once per workgroup and
    // bin; counted per wavefront, the few thousand wavefronts of a block queued up on the counters of degrees 1 and 2
    __shared__ unsigned int rows_s[kBlkLocalSched][kDegHist];
    __shared__ unsigned long long edges_s[kBlkLocalSched][kDegHist];
    __shared__ int sched0_s;
    for (int k = threadIdx.x; k < kBlkLocalSched * kDegHist; k += kBlkRowsThreads) {
        (&rows_s[0][0])[k] = 0;
        (&edges_s[0][0])[k] = 0;
    }
    if (threadIdx.x == 0) {
        const int64_t R0 = static_cast<int64_t>(bx) * kBlkRowsThreads;
        const int rel0 = R0 < n_rows_total ? seg_of(CSC ? t.src_off : t.dst_off, t.n_rel, R0) : 0;
        sched0_s = CSC ? t.n_rel + rel0 : rel0;
    }
    __syncthreads();
    const int sched0 = sched0_s;
    const int64_t R = static_cast<int64_t>(bx) * kBlkRowsThreads + threadIdx.x;
    const bool live = R < n_rows_total;
    uint32_t hkey = 0xffffffffu; // (schedule, capped degree) of this lane's row, for the histogram at the end
    int64_t hdeg = 0;
    if (live) {
    const int64_t *off = CSC ? t.src_off : t.dst_off;
    const int rel = seg_of(off, t.n_rel, R);
    const int64_t v = R - off[rel], n_local = off[rel + 1] - off[rel];
    const int64_t E = t.edge_off[rel + 1] - t.edge_off[rel];
    int64_t p0, p1;
    if (CSC) {
        p0 = ptr_global[R] - t.edge_off[rel];
        p1 = ptr_global[R + 1] - t.edge_off[rel];
    } else {
        const int64_t *rp = in.rowptr[rel];
        const int64_t r0 = rp[v], r1 = rp[v + 1];
        if (v == 0 && r0 != 0) report(err, kBadPtr0, rel, 0);
        if (r1 < r0) report(err, kBadDecrease, rel, v);
        if (v == n_local - 1 && r1 != E) report(err, kBadTotal, rel, 0);
        p0 = v == 0 ? 0 : clamp64(r0, 0, E);
        p1 = v == n_local - 1 ? E : clamp64(r1, p0, E);
        ptr_global[R] = t.edge_off[rel] + p0;
        if (R == n_rows_total - 1) ptr_global[n_rows_total] = t.edge_off[t.n_rel];
        inv_deg[R] = p1 > p0 ? 1.0f / static_cast<float>(p1 - p0) : 0.0f;
    }
    int64_t *pl = ptr_local + off[rel] + rel; // each relation's slice has one more entry than rows
    pl[v] = p0;
    if (v == n_local - 1) pl[n_local] = E;
    const int64_t deg = p1 - p0;
    const int capped = static_cast<int>(min(deg, static_cast<int64_t>(kHubMinDeg)));
    const int sched = CSC ? t.n_rel + rel : rel;
    key[sched_pos0 + R] = (static_cast<uint32_t>(sched) << 10) | static_cast<uint32_t>(kHubMinDeg - capped);
    val[sched_pos0 + R] = static_cast<uint32_t>(sched_pos0 + R);
    hkey = (static_cast<uint32_t>(sched) << 10) | static_cast<uint32_t>(capped);
    hdeg = deg;
    }
    if (live) {
        const int sched = static_cast<int>(hkey >> 10), capped = static_cast<int>(hkey & 1023u);
        const int ls = sched - sched0;
        if (ls >= 0 && ls < kBlkLocalSched) {
            atomicAdd(&rows_s[ls][capped], 1u);
            atomicAdd(&edges_s[ls][capped], static_cast<unsigned long long>(hdeg));
        } else { // a workgroup that spans more than four schedules: straight to the global counters
            unsigned long long *h = hist + static_cast<int64_t>(sched) * 2 * kDegHist;
            atomicAdd(&h[capped], 1ull);
            atomicAdd(&h[kDegHist + capped], static_cast<unsigned long long>(hdeg));
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < kBlkLocalSched * kDegHist; k += kBlkRowsThreads) {
        const unsigned int n = (&rows_s[0][0])[k];
        if (n) {
            unsigned long long *h = hist + static_cast<int64_t>(sched0 + k / kDegHist) * 2 * kDegHist;
            atomicAdd(&h[k % kDegHist], static_cast<unsigned long long>(n));
            atomicAdd(&h[kDegHist + k % kDegHist], (&edges_s[0][0])[k]);
        }
    }
}

// One thread per global edge: the caller's neighbour id, checked and sanitised, goes to the CSR's own copy and,
// as a global source id, into the transpose's sort key; the value is the global edge id.
__device__ __forceinline__ void blk_edges_body(const int64_t e, const BlockTables &t, const BlockInputs &in, int64_t n_edges_total,
                                               int32_t *csr_idx, uint32_t *key, uint32_t *val, unsigned long long *err)
{
    if (e >= n_edges_total) return;
    const int rel = seg_of(t.edge_off, t.n_rel, e);
    const int64_t le = e - t.edge_off[rel], n_src = t.src_off[rel + 1] - t.src_off[rel];
    int64_t c = in.col[rel][le];
    if (c < 0 || c >= n_src) {
        report(err, kBadCol, rel, le);
        c = clamp64(c, 0, max(n_src - 1, static_cast<int64_t>(0)));
    }
    csr_idx[e] = static_cast<int32_t>(c);
    key[e] = static_cast<uint32_t>(t.src_off[rel] + c);
    val[e] = static_cast<uint32_t>(e);
}

template <int CSC>
__global__ void __launch_bounds__(kBlkRowsThreads) blk_rows_kernel(BlockTables t, BlockInputs in, int64_t n_rows_total, int64_t sched_pos0,
                                                                   int64_t *ptr_local, int64_t *ptr_global, float *inv_deg, uint32_t *key,
                                                                   uint32_t *val, unsigned long long *hist, unsigned long long *err)
{
    blk_rows_body<CSC>(blockIdx.x, t, in, n_rows_total, sched_pos0, ptr_local, ptr_global, inv_deg, key, val, hist, err);
}
// The two kernels that read the caller's arrays in one grid (they depend on nothing and on each other not at all):
// the first row_blocks workgroups take the CSR rows, the rest 1,024 edges each.
__global__ void __launch_bounds__(kBlkRowsThreads) blk_rows_edges_kernel(BlockTables t, BlockInputs in, unsigned row_blocks, int64_t n_rows_total,
                                                                         int64_t *ptr_local, int64_t *ptr_global, float *inv_deg, uint32_t *row_key,
                                                                         uint32_t *row_val, unsigned long long *hist, int64_t n_edges_total,
                                                                         int32_t *csr_idx, uint32_t *edge_key, uint32_t *edge_val,
                                                                         unsigned long long *err)
{
    if (blockIdx.x < row_blocks)
        blk_rows_body<0>(blockIdx.x, t, in, n_rows_total, 0, ptr_local, ptr_global, inv_deg, row_key, row_val, hist, err);
    else
        blk_edges_body(static_cast<int64_t>(blockIdx.x - row_blocks) * kBlkRowsThreads + threadIdx.x, t, in, n_edges_total, csr_idx, edge_key,
                       edge_val, err);
}

// global column offsets: colG[U] = number of sorted keys below U, U in [0, n_src_total]
__device__ __forceinline__ void blk_colptr_body(const int64_t U, const uint32_t *sorted_keys, int64_t n_edges, int64_t n_src_total, int64_t *colG)
{
    if (U > n_src_total) return;
    int64_t lo = 0, hi = n_edges;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (sorted_keys[mid] < static_cast<uint32_t>(U)) lo = mid + 1;
        else hi = mid;
    }
    colG[U] = lo;
}

// csc_idx[p] = relation-local destination row of the edge at sorted position p (the block-diagonal structure
// keeps a relation's columns, and so its CSC slots, contiguous: p is already the slot's global position)
__device__ __forceinline__ void blk_csc_idx_body(const int64_t p, const BlockTables &t, const uint32_t *sorted_edge, int64_t n_edges_total,
                                                 const int64_t *ptrG_csr, int64_t n_dst_total, int32_t *csc_idx)
{
    if (p >= n_edges_total) return;
    const int64_t e = sorted_edge[p];
    const int64_t R = last_le64(ptrG_csr, n_dst_total, e); // the last row starting at or before e owns it (empty rows share offsets)
    const int rel = seg_of(t.edge_off, t.n_rel, e);
    csc_idx[p] = static_cast<int32_t>(R - t.dst_off[rel]);
}

// both readers of the transpose sort's result in one grid: the first col_blocks workgroups the column offsets
__global__ void __launch_bounds__(256) blk_colptr_csc_idx_kernel(BlockTables t, unsigned col_blocks, const uint32_t *sorted_keys,
                                                                 const uint32_t *sorted_edge, int64_t n_edges_total, int64_t n_src_total,
                                                                 int64_t *colG, const int64_t *ptrG_csr, int64_t n_dst_total, int32_t *csc_idx)
{
    if (blockIdx.x < col_blocks)
        blk_colptr_body(static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x, sorted_keys, n_edges_total, n_src_total, colG);
    else
        blk_csc_idx_body(static_cast<int64_t>(blockIdx.x - col_blocks) * 256 + threadIdx.x, t, sorted_edge, n_edges_total, ptrG_csr, n_dst_total,
                         csc_idx);
}

// Sorted position Q of the schedule sort -> that row's place in its schedule: the row order (relation-local
// ids), its degree, and the number of 256-edge chunks if it is a hub row.
__global__ void __launch_bounds__(256) blk_perm_kernel(BlockTables t, const uint32_t *sorted_row, int64_t n_dst_total, int64_t n_total,
                                                       const int64_t *ptrG_csr, const int64_t *ptrG_csc, int32_t *csr_perm,
                                                       int32_t *csc_perm, int64_t *sdeg, int64_t *cnt)
{
    const int64_t Q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (Q >= n_total) return;
    const int64_t g = sorted_row[Q]; // global row: CSR rows first, then CSC rows; the sort keeps the two sides apart
    int64_t deg;
    if (Q < n_dst_total) {
        const int rel = seg_of(t.dst_off, t.n_rel, g);
        csr_perm[Q] = static_cast<int32_t>(g - t.dst_off[rel]);
        deg = ptrG_csr[g + 1] - ptrG_csr[g];
    } else {
        const int64_t U = g - n_dst_total;
        const int rel = seg_of(t.src_off, t.n_rel, U);
        csc_perm[Q - n_dst_total] = static_cast<int32_t>(U - t.src_off[rel]);
        deg = ptrG_csc[U + 1] - ptrG_csc[U];
    }
    sdeg[Q] = deg;
    cnt[Q] = deg >= kHubMinDeg ? (deg + kHubChunk - 1) / kHubChunk : 0;
}

// Relation-local schedule offsets, hub chunk ranges and hub chunk descriptors from the two global scans.
// sptrG: exclusive scan of sdeg over all Q (CSR side counts from 0, CSC side continues from the edge total);
// chunkG: exclusive scan of cnt.
__device__ __forceinline__ void blk_sptr_body(const int64_t Q, const BlockTables &t, int64_t n_dst_total, int64_t n_total, const int64_t *sptrG,
                                              const int64_t *chunkG, const int64_t *sdeg, int64_t *csr_sptr, int64_t *csc_sptr,
                                              int64_t *hub_chunk_ptr, HubChunk *hub_chunks, int64_t *n_chunks_out)
{
    if (Q >= n_total) return;
    const bool csc = Q >= n_dst_total;
    const int64_t *off = csc ? t.src_off : t.dst_off;
    const int64_t P = csc ? Q - n_dst_total : Q;       // position within its side
    const int rel = seg_of(off, t.n_rel, P);
    const int sched = csc ? t.n_rel + rel : rel;
    const int64_t q = P - off[rel], n_local = off[rel + 1] - off[rel];
    const int64_t start = (csc ? n_dst_total : 0) + off[rel];              // first Q of this schedule
    const int64_t e_base = sptrG[start], c_base = chunkG[start];
    int64_t *sp = (csc ? csc_sptr : csr_sptr) + off[rel] + rel;
    const int64_t s0 = sptrG[Q] - e_base;
    sp[q] = s0;
    if (q == n_local - 1) sp[n_local] = sptrG[Q + 1] - e_base;
    // chunk ranges: entry h for every hub row h and the one after the last (non-hub rows add no chunks, so the
    // running count simply stays); the slice holds E / 512 + 2 entries, more than hub rows + 1
    const int64_t E = t.edge_off[rel + 1] - t.edge_off[rel];
    const int64_t cap = E / kHubMinDeg + 2;
    int64_t *cp = hub_chunk_ptr + t.hubptr_off[sched];
    if (q < cap) cp[q] = chunkG[Q] - c_base;
    if (q == n_local - 1) {
        if (q + 1 < cap) cp[q + 1] = chunkG[Q + 1] - c_base;
        n_chunks_out[sched] = chunkG[Q + 1] - c_base;
    }
    const int64_t deg = sdeg[Q];
    if (deg >= kHubMinDeg) {
        HubChunk *hc = hub_chunks + t.hub_off[sched];
        const int64_t room = t.hub_off[sched + 1] - t.hub_off[sched]; // never exceeded by a well-formed CSR
        const int64_t c0 = chunkG[Q] - c_base, nc = (deg + kHubChunk - 1) / kHubChunk;
        for (int64_t c = 0; c < nc && c0 + c < room; ++c) { // a hub row's chunks: at most a few thousand, written by its one thread
            HubChunk d;
            d.e0 = s0 + c * kHubChunk;
            d.len = static_cast<int32_t>(min(static_cast<int64_t>(kHubChunk), s0 + deg - d.e0));
            d.slot = static_cast<int32_t>(c0 + c);
            hc[c0 + c] = d;
        }
    }
}

// sidx of both directions: slot e' of the concatenated schedule-ordered adjacency (CSR slots first, then CSC
// slots) takes the neighbour id of its row's (e' - row start)-th edge
__device__ __forceinline__ void blk_sidx_body(const int64_t x, int64_t n_edges_total, int64_t n_dst_total, int64_t n_src_total,
                                              const int64_t *sptrG, const uint32_t *sorted_row, const int64_t *ptrG_csr,
                                              const int64_t *ptrG_csc, const int32_t *csr_idx, const int32_t *csc_idx,
                                              int32_t *csr_sidx, int32_t *csc_sidx)
{
    if (x >= 2 * n_edges_total) return;
    if (x < n_edges_total) {
        const int64_t Q = last_le64(sptrG, n_dst_total, x);
        const int64_t g = sorted_row[Q];
        // (the clamp only matters for a malformed CSR, whose offsets need not add up: it is reported, never followed out of bounds)
        csr_sidx[x] = csr_idx[clamp64(ptrG_csr[g] + (x - sptrG[Q]), 0, n_edges_total - 1)];
    } else {
        const int64_t Q = n_dst_total + last_le64(sptrG + n_dst_total, n_src_total, x);
        const int64_t U = static_cast<int64_t>(sorted_row[Q]) - n_dst_total;
        csc_sidx[x - n_edges_total] = csc_idx[clamp64(ptrG_csc[U] + (x - sptrG[Q]), 0, n_edges_total - 1)];
    }
}

// both consumers of the two row scans in one grid: the first sptr_blocks workgroups the schedule offsets and hub chunks
__global__ void __launch_bounds__(256) blk_sptr_sidx_kernel(BlockTables t, unsigned sptr_blocks, int64_t n_dst_total, int64_t n_src_total,
                                                            int64_t n_total, int64_t n_edges_total, const int64_t *sptrG, const int64_t *chunkG,
                                                            const int64_t *sdeg, int64_t *csr_sptr, int64_t *csc_sptr, int64_t *hub_chunk_ptr,
                                                            HubChunk *hub_chunks, int64_t *n_chunks_out, const uint32_t *sorted_row,
                                                            const int64_t *ptrG_csr, const int64_t *ptrG_csc, const int32_t *csr_idx,
                                                            const int32_t *csc_idx, int32_t *csr_sidx, int32_t *csc_sidx)
{
    if (blockIdx.x < sptr_blocks)
        blk_sptr_body(static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x, t, n_dst_total, n_total, sptrG, chunkG, sdeg, csr_sptr, csc_sptr,
                      hub_chunk_ptr, hub_chunks, n_chunks_out);
    else
        blk_sidx_body(static_cast<int64_t>(blockIdx.x - sptr_blocks) * 256 + threadIdx.x, n_edges_total, n_dst_total, n_src_total, sptrG,
                      sorted_row, ptrG_csr, ptrG_csc, csr_idx, csc_idx, csr_sidx, csc_sidx);
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <typename T> T *carve(char *&cursor, size_t n)
{
    T *p = reinterpret_cast<T *>(cursor);
    cursor += align_up(std::max<size_t>(n, 1) * sizeof(T), 256);
    return p;
}

template <typename T> size_t carve_size(size_t n) { return align_up(std::max<size_t>(n, 1) * sizeof(T), 256); }

} // namespace

int block_ingest_max_relations() { return kMaxBlockRels; }

// Builds the listed relations (registered already in their graphs: types, sizes; no arrays yet) from their CSRs;
// `names` says how an error message calls each.
// rowptr / col: DEVICE arrays per listed relation.  On success the relations' schedules point into *arena_out
// (one pool block, to be released with scratch_free when the graph goes) and carry their host-side histograms.
// Synchronous.
heta_status build_block_on_device(const std::vector<Relation *> &rels, const std::vector<std::string> &names,
                                  const int64_t *const *rowptr, const int32_t *const *col, void **arena_out, hipStream_t st)
{
    *arena_out = nullptr;
    const int n_rel = static_cast<int>(rels.size());
    if (n_rel == 0) return HETA_OK;
    if (n_rel > kMaxBlockRels) return fail(HETA_ERR_UNSUPPORTED, "block ingest takes at most %d relations at once", kMaxBlockRels);
    BlockTables t{};
    BlockInputs in{};
    t.n_rel = n_rel;
    size_t hub_total = 0, hubptr_total = 0;
    for (int i = 0; i < n_rel; ++i) {
        const Relation &r = *rels[i];
        t.dst_off[i + 1] = t.dst_off[i] + r.n_dst;
        t.src_off[i + 1] = t.src_off[i] + r.n_src;
        t.edge_off[i + 1] = t.edge_off[i] + r.n_edges;
        in.rowptr[i] = rowptr[i];
        in.col[i] = col[i];
    }
    for (int s = 0; s < 2 * n_rel; ++s) { // chunk descriptors / chunk ranges per schedule: the same bounds as the host path's
        const int64_t E = rels[s % n_rel]->n_edges;
        t.hub_off[s] = static_cast<int64_t>(hub_total);
        t.hubptr_off[s] = static_cast<int64_t>(hubptr_total);
        hub_total += static_cast<size_t>(E / kHubChunk + E / kHubMinDeg + 1);
        hubptr_total += static_cast<size_t>(E / kHubMinDeg + 2);
    }
    t.hub_off[2 * n_rel] = static_cast<int64_t>(hub_total);
    t.hubptr_off[2 * n_rel] = static_cast<int64_t>(hubptr_total);
    for (int i = 0; i < n_rel; ++i) { // what needs no look at the arrays is rejected before anything is launched
        const Relation &r = *rels[i];
        if (r.n_edges > 0 && r.n_dst == 0)
            return fail(HETA_ERR_BAD_CSR, "%s: rowptr[n_dst] differs from num_edges = %lld", names[i].c_str(), (long long)r.n_edges);
        if (r.n_edges > 0 && r.n_src == 0) return fail(HETA_ERR_BAD_CSR, "%s: col[0] outside [0, 0)", names[i].c_str());
    }
    const int64_t nR = t.dst_off[n_rel], nS = t.src_off[n_rel], nE = t.edge_off[n_rel], nQ = nR + nS;
    if (nQ >= (int64_t(1) << 31) || nE >= (int64_t(1) << 31)) return fail(HETA_ERR_UNSUPPORTED, "block too large for the block ingest");

    // ---- the arena: everything the relations keep ------------------------------------------------------
    const size_t arena_bytes = 2 * carve_size<int64_t>(nR + n_rel) + 2 * carve_size<int64_t>(nS + n_rel) + carve_size<int64_t>(hubptr_total) +
                               carve_size<HubChunk>(hub_total) + 4 * carve_size<int32_t>(nE) + carve_size<int32_t>(nR) +
                               carve_size<int32_t>(nS) + carve_size<float>(nR);
    void *arena = nullptr;
    HETA_HIP(scratch_alloc(&arena, arena_bytes));
    char *cur = static_cast<char *>(arena);
    int64_t *csr_ptr = carve<int64_t>(cur, nR + n_rel), *csr_sptr = carve<int64_t>(cur, nR + n_rel);
    int64_t *csc_ptr = carve<int64_t>(cur, nS + n_rel), *csc_sptr = carve<int64_t>(cur, nS + n_rel);
    int64_t *hub_chunk_ptr = carve<int64_t>(cur, hubptr_total);
    HubChunk *hub_chunks = carve<HubChunk>(cur, hub_total);
    int32_t *csr_idx = carve<int32_t>(cur, nE), *csr_sidx = carve<int32_t>(cur, nE);
    int32_t *csc_idx = carve<int32_t>(cur, nE), *csc_sidx = carve<int32_t>(cur, nE);
    int32_t *csr_perm = carve<int32_t>(cur, nR), *csc_perm = carve<int32_t>(cur, nS);
    float *inv_deg = carve<float>(cur, nR);

    // ---- scratch: one pool block ---------------------------------------------------------------------------
    const int64_t n_sort = std::max(nE, nQ);
    const int64_t hist_elems = sort_hist_elems(std::max<int64_t>(n_sort, 1));
    const size_t n_hist = static_cast<size_t>(2 * n_rel) * 2 * kDegHist;
    const size_t scratch_bytes = carve_size<int64_t>(nR + 1) + carve_size<int64_t>(nS + 1) + 2 * carve_size<int64_t>(nQ) +
                                 2 * carve_size<int64_t>(nQ + 1) + carve_size<int64_t>(2 * scan_scratch_elems(nQ + 1)) +
                                 4 * carve_size<uint32_t>(n_sort) + 2 * carve_size<uint32_t>(hist_elems) +
                                 carve_size<uint32_t>(scan_scratch_elems(hist_elems)) + carve_size<unsigned long long>(n_hist + 1) +
                                 carve_size<int64_t>(2 * n_rel);
    void *scratch = nullptr;
    hipError_t he = scratch_alloc(&scratch, scratch_bytes);
    if (he != hipSuccess) {
        scratch_free(arena);
        return fail(he == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE, "block ingest: %s", hipGetErrorString(he));
    }
    cur = static_cast<char *>(scratch);
    int64_t *ptrG_csr = carve<int64_t>(cur, nR + 1), *ptrG_csc = carve<int64_t>(cur, nS + 1);
    int64_t *sdeg = carve<int64_t>(cur, nQ), *cnt = carve<int64_t>(cur, nQ);
    int64_t *sptrG = carve<int64_t>(cur, nQ + 1), *chunkG = carve<int64_t>(cur, nQ + 1);
    int64_t *tile_sums = carve<int64_t>(cur, 2 * scan_scratch_elems(nQ + 1)); // two scans share a launch set
    uint32_t *keyA = carve<uint32_t>(cur, n_sort), *valA = carve<uint32_t>(cur, n_sort);
    uint32_t *keyB = carve<uint32_t>(cur, n_sort), *valB = carve<uint32_t>(cur, n_sort);
    uint32_t *shist = carve<uint32_t>(cur, hist_elems), *soffs = carve<uint32_t>(cur, hist_elems);
    uint32_t *stile = carve<uint32_t>(cur, scan_scratch_elems(hist_elems));
    unsigned long long *hist = carve<unsigned long long>(cur, n_hist + 1); // the last entry is the error word
    int64_t *n_chunks_dev = carve<int64_t>(cur, 2 * n_rel);
    unsigned long long *err = hist + n_hist;

    heta_status e = HETA_OK;
    auto finish = [&](heta_status s) { // the pool wants idle blocks
        (void)hipStreamSynchronize(st);
        scratch_free(scratch);
        if (s != HETA_OK) scratch_free(arena);
        return s;
    };
#define HETA_BLK(call)                                                                                             \
    do {                                                                                                           \
        hipError_t e_ = (call);                                                                                    \
        if (e_ != hipSuccess) return finish(fail(HETA_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_))); \
    } while (0)
#define HETA_BLK_LAUNCHED(name)                                                                                    \
    do {                                                                                                           \
        hipError_t e_ = hipGetLastError();                                                                         \
        if (e_ != hipSuccess) return finish(fail(HETA_ERR_DEVICE, "launch of %s failed: %s", name, hipGetErrorString(e_))); \
    } while (0)
    auto blocks_for = [](int64_t n) { return dim3(static_cast<unsigned>((std::max<int64_t>(n, 1) + 255) / 256)); };

    // offsets of relations without rows, chunk ranges of schedules without hub rows: zero unless written
    HETA_BLK(hipMemsetAsync(arena, 0, reinterpret_cast<char *>(hub_chunks) - static_cast<char *>(arena), st));
    // one fill for the histograms, the error word and the chunk counts (consecutive pieces)
    HETA_BLK(hipMemsetAsync(hist, 0, reinterpret_cast<char *>(n_chunks_dev + 2 * n_rel) - reinterpret_cast<char *>(hist), st));
    // the schedule sort's pairs: CSR rows at [0, nR), CSC rows at [nR, nQ) of keyB / valB (keyA / valA serve the transpose first)
    auto blocks_of = [](int64_t n, int64_t per) { return static_cast<unsigned>((n + per - 1) / per); };
    if (nR == 0) HETA_BLK(hipMemsetAsync(ptrG_csr, 0, sizeof(int64_t), st));
    uint32_t *ks = keyA, *vs = valA;
    if (nR > 0 || nE > 0) { // CSR rows and edges, both straight from the caller's arrays, in one launch
        const unsigned rb = blocks_of(nR, kBlkRowsThreads), eb = blocks_of(nE, kBlkRowsThreads);
        hipLaunchKernelGGL(blk_rows_edges_kernel, dim3(rb + eb), dim3(kBlkRowsThreads), 0, st, t, in, rb, nR, csr_ptr, ptrG_csr, inv_deg, keyB,
                           valB, hist, nE, csr_idx, keyA, valA, err);
        HETA_BLK_LAUNCHED("blk_rows_edges_kernel");
    }
    // The transpose sort's ping-pong partner: keyB / valB already hold the CSR rows' schedule pairs, so the partner is the
    // arena's two sidx arrays (nE 32-bit words each), which nothing touches before the final fill.
    uint32_t *keyT = reinterpret_cast<uint32_t *>(csr_sidx), *valT = reinterpret_cast<uint32_t *>(csc_sidx);
    if (nE > 0) {
        int bits = 1;
        while ((int64_t(1) << bits) < std::max<int64_t>(nS, 2)) ++bits;
        if ((e = device_sort_pairs_u32_async(keyA, valA, keyT, valT, nE, int64_t(1) << bits, &ks, &vs, shist, soffs, stile, st)) != HETA_OK)
            return finish(e);
    }
    {
        const unsigned cb = blocks_of(nS + 1, 256), ib = blocks_of(nE, 256);
        hipLaunchKernelGGL(blk_colptr_csc_idx_kernel, dim3(cb + ib), dim3(256), 0, st, t, cb, ks, vs, nE, nS, ptrG_csc, ptrG_csr, nR, csc_idx);
        HETA_BLK_LAUNCHED("blk_colptr_csc_idx_kernel");
    }
    if (nS > 0) {
        hipLaunchKernelGGL(blk_rows_kernel<1>, dim3(static_cast<unsigned>((nS + kBlkRowsThreads - 1) / kBlkRowsThreads)), dim3(kBlkRowsThreads), 0, st, t, in, nS, nR, csc_ptr, ptrG_csc, (float *)nullptr, keyB,
                           valB, hist, err);
        HETA_BLK_LAUNCHED("blk_rows_kernel");
    }
    // every schedule's row order: one stable sort by (schedule, 512 - capped degree); 2 n_rel <= 64 schedules: 16 bits
    uint32_t *ks2 = keyB, *vs2 = valB;
    if (nQ > 0) {
        // the transpose's results (ks / vs) are consumed; (keyA, valA) is free as the partner unless the sort ended there
        uint32_t *pk = keyA, *pv = valA;
        if ((e = device_sort_pairs_u32_async(keyB, valB, pk, pv, nQ, int64_t(1) << 16, &ks2, &vs2, shist, soffs, stile, st)) != HETA_OK)
            return finish(e);
        hipLaunchKernelGGL(blk_perm_kernel, blocks_for(nQ), dim3(256), 0, st, t, vs2, nR, nQ, ptrG_csr, ptrG_csc, csr_perm, csc_perm, sdeg, cnt);
        HETA_BLK_LAUNCHED("blk_perm_kernel");
    }
    if ((e = device_exclusive_scan2_i64_async(sdeg, cnt, nQ, sptrG, chunkG, nQ + 1, tile_sums, st)) != HETA_OK) return finish(e);
    if (nQ > 0 || nE > 0) {
        const unsigned sb = blocks_of(nQ, 256), xb = blocks_of(2 * nE, 256);
        hipLaunchKernelGGL(blk_sptr_sidx_kernel, dim3(sb + xb), dim3(256), 0, st, t, sb, nR, nS, nQ, nE, sptrG, chunkG, sdeg, csr_sptr, csc_sptr,
                           hub_chunk_ptr, hub_chunks, n_chunks_dev, vs2, ptrG_csr, ptrG_csc, csr_idx, csc_idx, csr_sidx, csc_sidx);
        HETA_BLK_LAUNCHED("blk_sptr_sidx_kernel");
    }
    // histograms, the error word and the chunk counts come back through a page-locked buffer of the thread's own
    // (hist, err and n_chunks_dev are consecutive in the scratch block: 256-byte aligned pieces)
    static thread_local void *t_back = nullptr;
    static thread_local size_t t_back_cap = 0;
    // one copy: the host buffer mirrors the device layout from hist to the end of the chunk counts
    const size_t back_hist = reinterpret_cast<char *>(n_chunks_dev) - reinterpret_cast<char *>(hist);
    const size_t back_total = back_hist + 2 * n_rel * sizeof(int64_t);
    if (back_total > t_back_cap) {
        if (t_back) (void)hipHostFree(t_back);
        t_back = nullptr;
        t_back_cap = 0;
        const size_t cap = std::max<size_t>(back_total, (size_t(2) * kMaxBlockRels * 2 * kDegHist + 1) * 8 + 2 * kMaxBlockRels * 8 + 512);
        HETA_BLK(hipHostMalloc(&t_back, cap, hipHostMallocDefault));
        t_back_cap = cap;
    }
    unsigned long long *h = static_cast<unsigned long long *>(t_back);
    int64_t *n_chunks = reinterpret_cast<int64_t *>(static_cast<char *>(t_back) + back_hist);
    HETA_BLK(hipMemcpyAsync(h, hist, back_total, hipMemcpyDeviceToHost, st));
    HETA_BLK(hipStreamSynchronize(st));
#undef HETA_BLK
#undef HETA_BLK_LAUNCHED
    if (h[n_hist] != 0) {
        const unsigned long long bad = ~h[n_hist];
        const unsigned long long kind = bad >> 56, at = bad & ((1ull << 48) - 1);
        const int which = static_cast<int>((bad >> 48) & 0xff);
        const Relation &r = *rels[which];
        const char *name = names[which].c_str();
        if (kind == kBadPtr0) e = fail(HETA_ERR_BAD_CSR, "%s: rowptr[0] is not 0", name);
        else if (kind == kBadDecrease) e = fail(HETA_ERR_BAD_CSR, "%s: rowptr decreases at row %llu", name, at);
        else if (kind == kBadTotal) e = fail(HETA_ERR_BAD_CSR, "%s: rowptr[n_dst] differs from num_edges = %lld", name, (long long)r.n_edges);
        else e = fail(HETA_ERR_BAD_CSR, "%s: col[%llu] outside [0, %lld)", name, at, (long long)r.n_src);
        return finish(e);
    }
    for (int i = 0; i < n_rel; ++i) {
        Relation &r = *rels[i];
        for (int side = 0; side < 2; ++side) {
            Schedule &s = side ? r.csc : r.csr;
            const int sched = side ? n_rel + i : i;
            const int64_t row0 = side ? t.src_off[i] : t.dst_off[i];
            s.d_ptr = (side ? csc_ptr : csr_ptr) + row0 + i;
            s.d_sptr = (side ? csc_sptr : csr_sptr) + row0 + i;
            s.d_idx = (side ? csc_idx : csr_idx) + t.edge_off[i];
            s.d_sidx = (side ? csc_sidx : csr_sidx) + t.edge_off[i];
            s.d_perm = (side ? csc_perm : csr_perm) + row0;
            s.d_hub_chunks = hub_chunks + t.hub_off[sched];
            s.d_hub_chunk_ptr = hub_chunk_ptr + t.hubptr_off[sched];
            const unsigned long long *hh = h + static_cast<size_t>(sched) * 2 * kDegHist;
            int64_t rows = 0, edges = 0;
            for (int k = kHubMinDeg; k >= 0; --k) {
                rows += static_cast<int64_t>(hh[k]);
                edges += static_cast<int64_t>(hh[kDegHist + k]);
                s.rows_with_deg_ge[k] = rows;
                s.edges_with_deg_ge[k] = edges;
            }
            s.n_hub_rows = s.rows_with_deg_ge[kHubMinDeg];
            s.n_hub_chunks = n_chunks[sched];
        }
        r.d_inv_deg = inv_deg + t.dst_off[i];
        r.host_built = true; // its arrays are slices of an arena of the graph, not allocations of its own
    }
    *arena_out = arena;
    return finish(HETA_OK);
}

} // namespace heta
