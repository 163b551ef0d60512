// Internal declarations shared by the translation units of libheta (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <memory>
#include <string>
#include <vector>

#include "heta.h"

namespace heta {

// ---- error reporting ---------------------------------------------------------------------------
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
heta_status fail(heta_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

#define HETA_HIP(call)                                                                               \
    do {                                                                                             \
        hipError_t e_ = (call);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return ::heta::fail(e_ == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE,         \
                                "%s failed: %s", #call, hipGetErrorString(e_));                      \
    } while (0)

#define HETA_LAUNCH_CHECK(name)                                                                      \
    do {                                                                                             \
        hipError_t e_ = hipGetLastError();                                                           \
        if (e_ != hipSuccess)                                                                        \
            return ::heta::fail(HETA_ERR_DEVICE, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- row schedule of one direction of one relation ----------------------------------------------
// Rows are the reduction's output rows: destinations for the CSR (forward), sources for the CSC
// (backward).  `perm` lists the rows by descending degree (stable, so ascending row id within a
// degree).  Rows of at least kHubMinDeg edges ("hub rows", the head of a power-law degree
// distribution) come first in `perm`; each is cut into chunks of kHubChunk edges that separate
// wavefronts reduce into partial rows of the workspace, and a second kernel adds a hub row's
// partials in chunk order.
constexpr int kHubMinDeg = 512;
constexpr int kHubChunk = 256;
constexpr int kDegHist = 513; // rows_with_deg_ge[k] for k in [0, 512]

struct HubChunk {       // one wavefront's share of a hub row
    int64_t e0;         // first edge (position in the schedule-ordered neighbour array)
    int32_t len;        // number of edges (<= kHubChunk)
    int32_t slot;       // partial row in the workspace
};

struct Schedule {
    int64_t n_rows = 0, n_edges = 0;
    int64_t *d_ptr = nullptr;     // [n_rows + 1] offsets by row id (the CSR / CSC itself)
    int32_t *d_idx = nullptr;     // [n_edges] neighbour ids in that order
    int32_t *d_perm = nullptr;    // [n_rows] rows by descending degree
    // The same adjacency laid out in schedule order: position q holds row perm[q], its neighbours
    // are sidx[sptr[q] .. sptr[q+1]).  The kernels walk only this copy, so a wavefront's row
    // offsets and neighbour ids are consecutive in memory and, for rows of fewer than kHubMinDeg
    // edges, computable from the degree histogram without a load.
    int64_t *d_sptr = nullptr;    // [n_rows + 1]
    int32_t *d_sidx = nullptr;    // [n_edges]
    int64_t n_hub_rows = 0;       // perm[0 .. n_hub_rows) are hub rows
    int64_t n_hub_chunks = 0;
    HubChunk *d_hub_chunks = nullptr;    // [n_hub_chunks], grouped by hub row in perm order
    int64_t *d_hub_chunk_ptr = nullptr;  // [n_hub_rows + 1] chunk range of each hub row
    int64_t rows_with_deg_ge[kDegHist];  // host: number of rows whose degree is >= k
    int64_t edges_with_deg_ge[kDegHist]; // host: number of edges in those rows
};

struct Relation {
    int32_t src_type = 0, dst_type = 0;
    int64_t n_src = 0, n_dst = 0, n_edges = 0;
    Schedule csr;                 // rows = destinations, idx = sources
    Schedule csc;                 // rows = sources, idx = destinations
    float *d_inv_deg = nullptr;   // [n_dst] 1/deg_r(v), 0 for zero-degree rows
    int32_t *d_hub_slot = nullptr; // [n_dst] position of a destination among the CSR schedule's hub rows, built on first use
    float *d_hub_rows = nullptr;   // aggregated hub rows of the fused forward, grown on demand
    size_t hub_rows_bytes = 0;
    bool host_built = false;      // its device arrays are slices of the graph's arena, not allocations of their own
    int32_t shares = -1;          // >= 0: csr / csc are relation `shares`' csc / csr (a declared reverse); only d_inv_deg is its own
};

} // namespace heta

struct heta_graph {
    int device = 0;
    std::vector<heta_ntype> ntypes;
    std::vector<heta::Relation> rels;
    void *d_arena = nullptr;      // every host-built relation's arrays: one allocation, one copy
    // the arrays of the relations built by the whole-block device ingest; the blocks of one heta_graph_create_batch
    // call share one allocation, released with the last of them
    std::shared_ptr<void> block_arena;
    // workspace for hub-row partials and split weight-gradient partials; grown on demand
    void *d_ws = nullptr;
    size_t ws_bytes = 0;
    // k-contiguous copies of the bf16 weight matrices of the projection in flight; grown on demand
    void *d_pack = nullptr;
    size_t pack_bytes = 0;
    // per-edge attention weights, per-row score terms and one [rows x d] intermediate of the
    // attention aggregation; grown on demand
    void *d_attn = nullptr;
    size_t attn_bytes = 0;
};

namespace heta {
// Brackets one kernel launch with HIP events when profiling is on (see heta_profile_enable);
// `bytes` and `flops` are the algorithmic traffic and work of that launch.
bool profiling_on();
class ProfScope {
public:
    ProfScope(const char *name, hipStream_t st, double bytes, double flops);
    ~ProfScope();
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;

private:
    bool active_;
    hipStream_t stream_;
    size_t index_ = 0;
};

// Device-side ingest (heta_ingest.hip).  All three are synchronous on `st` when they return.
heta_status validate_csr_on_device(int32_t index, const int64_t *d_ptr, const int32_t *d_col, int64_t n_dst, int64_t n_src,
                                   int64_t n_edges, hipStream_t st);
// csc.d_ptr / csc.d_idx (allocated here) = stable transpose of csr.d_ptr / csr.d_idx
heta_status transpose_on_device(const Schedule &csr, int64_t n_src, Schedule &csc, hipStream_t st);
// everything of s beyond d_ptr / d_idx (allocated here); inv_deg (optional, [n_rows]) = 1/degree
heta_status build_schedule_on_device(Schedule &s, float *inv_deg, hipStream_t st);

// Whole-block ingest (heta_block_ingest.hip): the index data of up to block_ingest_max_relations() relations of g
// (listed in `which`, registered already) from their DEVICE CSR arrays, in one pass; *arena_out owns their arrays.
int block_ingest_max_relations();
heta_status build_block_on_device(const std::vector<Relation *> &rels, const std::vector<std::string> &names,
                                  const int64_t *const *rowptr, const int32_t *const *col, void **arena_out, hipStream_t st);

// out[i] = in[0] + ... + in[i-1] for i < n_out (in[j] = 0 for j >= n_in); synchronous on st.
heta_status device_exclusive_scan_i64(const int64_t *in, int64_t n_in, int64_t *out, int64_t n_out, hipStream_t st);
// Stable sort of n (key, value) pairs by keys in [0, key_limit); (keys, vals) and (keys_tmp, vals_tmp) are
// ping-pong buffers, *keys_res / *vals_res point at whichever holds the result; synchronous on st.
heta_status device_sort_pairs_u32(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n,
                                  int64_t key_limit, uint32_t **keys_res, uint32_t **vals_res, hipStream_t st);

// Asynchronous forms with caller-provided scratch: tile_sums of scan_scratch_elems(n_out) elements; hist and offs of
// sort_hist_elems(n) elements each and tile_sums of scan_scratch_elems(sort_hist_elems(n)) elements.
int64_t scan_scratch_elems(int64_t n_out);
int64_t sort_hist_elems(int64_t n);
heta_status device_exclusive_scan2_i64_async(const int64_t *inA, const int64_t *inB, int64_t n_in, int64_t *outA, int64_t *outB,
                                             int64_t n_out, int64_t *tile_sums, hipStream_t st);
heta_status device_exclusive_scan_i64_async(const int64_t *in, int64_t n_in, int64_t *out, int64_t n_out, int64_t *tile_sums,
                                            hipStream_t st);
heta_status device_sort_pairs_u32_async(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n,
                                        int64_t key_limit, uint32_t **keys_res, uint32_t **vals_res, uint32_t *hist, uint32_t *offs,
                                        uint32_t *tile_sums, hipStream_t st);

// Short-lived device scratch from a recycling pool (blocks up to 16 MiB; larger ones are plain hipMalloc).
// scratch_free requires the block to be idle: synchronise first.
hipError_t scratch_alloc(void **out, size_t bytes);
void scratch_free(void *p);

// Makes sure g's workspace holds `bytes`; growing frees and reallocates (device synchronising).
heta_status ensure_workspace(heta_graph *g, size_t bytes);
// out[r] = beta out[r] + sum_e slot_w[e][head of the column] table[idx[e]] over the rows of s; slot_w is
// indexed by the edge's position in s.d_sidx.  With slot_w2 the same gathered rows are reduced a second
// time, with those weights, into out2 (same element type as out).  Uses g's workspace for hub rows.
// dot: instead of storing the second sum, dot->out[row, k] = <second sum of head k, dot->z[row, head k]> - dot->corr[row, k];
// *dot_done tells whether the shapes allowed it (else out2 was written as usual and the caller takes the dot itself).
struct SecondSumDot {
    const void *z;
    heta_dtype z_dt;
    int64_t ld_z;
    const float *corr; // nullable
    float *out;
};
heta_status aggregate_slot_weighted(heta_graph *g, const Schedule &s, const void *table, heta_dtype dt, int64_t ld,
                                    int d, const float *slot_w, int heads, void *out, heta_dtype out_dt,
                                    int64_t ld_out, float beta, hipStream_t st, const float *slot_w2 = nullptr,
                                    void *out2 = nullptr, int64_t ld_out2 = 0, const SecondSumDot *dot = nullptr,
                                    bool *dot_done = nullptr);
// out[h] (fp32, compact) = sum or mean of the h-th hub row of s (rows of >= kHubMinDeg edges lead the schedule)
heta_status aggregate_hub_rows(heta_graph *g, const Schedule &s, const void *table, heta_dtype dt, int64_t ld, int d,
                               const int64_t *gid, int mean, float *out, int64_t ld_out, hipStream_t st);
// Looks up the current device's address of the fixed scratch array of heta_rel_aggregate_fwd_noalloc
// (heta_aggregate.hip); heta_graph_create calls it so that the look-up happens at set-up time.
heta_status noalloc_scratch_init();
inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t dtype_size(heta_dtype dt) { return dt == HETA_F32 ? 4 : 2; }
inline bool valid_dtype(int dt) { return dt == HETA_F32 || dt == HETA_BF16; }
} // namespace heta
