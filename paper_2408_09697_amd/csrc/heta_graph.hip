// Graph ingest: validation, degrees, stable CSR -> CSC transpose, degree-sorted row schedules.
//
// A heterogeneous graph is handed over as its mono-relation subgraphs (Section 2.1 of the
// paper), one CSR over destination rows per relation.  Everything index-shaped that the
// aggregation kernels need later is derived here once and kept on the device: by the kernels of
// heta_ingest.hip for relations of real size, by the host code below for the small blocks of a
// sampled mini-batch, where launch latency would dominate.  Both produce the same arrays.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <system_error>
#include <thread>
#include <unordered_map>
#include <utility>

#include "heta_internal.h"
#include "heta_test_hooks.h"

namespace heta {

static thread_local std::string g_last_error;

void set_error(const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
}

heta_status fail(heta_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return st;
}

// ---- recycled device blocks for short-lived scratch ---------------------------------------------------
// Sampling a mini-batch and ingesting its blocks makes dozens of small allocations per iteration; each
// hipMalloc / hipFree pair costs tens of microseconds and hipFree waits for the device.  Blocks of up to
// 16 MiB are rounded to a power of two and kept on a free list per (device, size) when released, up to
// 256 MiB in total; larger ones go straight to hipMalloc / hipFree.  A block must be idle when it is
// released (the callers synchronise first).
namespace {
constexpr size_t kPoolMaxBlock = size_t(16) << 20, kPoolMaxCached = size_t(256) << 20;
std::mutex g_pool_mu;
std::unordered_map<void *, std::pair<int, size_t>> g_pool_blocks;     // live pooled block -> (device, size class)
std::map<std::pair<int, size_t>, std::vector<void *>> g_pool_free;
size_t g_pool_cached = 0;
} // namespace

hipError_t scratch_alloc(void **out, size_t bytes)
{
    *out = nullptr;
    size_t cls = 256;
    while (cls < bytes) cls <<= 1;
    if (cls > kPoolMaxBlock) return hipMalloc(out, bytes);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        auto it = g_pool_free.find({dev, cls});
        if (it != g_pool_free.end() && !it->second.empty()) {
            *out = it->second.back();
            it->second.pop_back();
            g_pool_cached -= cls;
            return hipSuccess;
        }
    }
    e = hipMalloc(out, cls);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(g_pool_mu);
    g_pool_blocks[*out] = {dev, cls};
    return hipSuccess;
}

void scratch_free(void *p)
{
    if (!p) return;
    {
        std::lock_guard<std::mutex> lk(g_pool_mu);
        auto it = g_pool_blocks.find(p);
        if (it != g_pool_blocks.end()) {
            const size_t cls = it->second.second;
            if (g_pool_cached + cls <= kPoolMaxCached) {
                g_pool_free[it->second].push_back(p);
                g_pool_cached += cls;
                return;
            }
            g_pool_blocks.erase(it);
        }
    }
    (void)hipFree(p);
}

heta_status ensure_workspace(heta_graph *g, size_t bytes)
{
    if (bytes <= g->ws_bytes)
        return HETA_OK;
    // From the recycling pool: a sampled block's graph lives for one iteration, and a fresh hipMalloc for
    // its workspace cost more than the block's whole weight gradient.
    if (g->d_ws) {
        HETA_HIP(hipDeviceSynchronize()); // everything that may still read the old buffer
        scratch_free(g->d_ws);
        g->d_ws = nullptr;
        g->ws_bytes = 0;
    }
    size_t want = bytes + bytes / 4;
    HETA_HIP(scratch_alloc(&g->d_ws, want));
    g->ws_bytes = want;
    return HETA_OK;
}

template <typename T>
[[maybe_unused]] static heta_status upload(T **dst, const T *src, size_t n)
{
    *dst = nullptr;
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(dst), std::max<size_t>(n, 1) * sizeof(T)));
    if (n)
        HETA_HIP(hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice));
    return HETA_OK;
}

// Host-built relations are assembled in one host buffer and reach the device with one
// allocation and one copy: byte offsets here, pointers once the device address is known.
// The buffer is page-locked (a pageable source would be staged by the runtime at a fraction of the
// link's rate, which was most of a mini-batch block's ingest time) and kept per thread for the next graph.
struct PinnedRegion {
    char *p = nullptr;
    size_t cap = 0;
};
static thread_local PinnedRegion t_pinned; // never freed: it lives as long as the thread builds graphs
// Small relations handed over as DEVICE arrays are built on the host: their arrays come back through
// this second page-locked buffer, all copies of a graph queued at once and awaited together.
static thread_local PinnedRegion t_download;

struct StagedCsr {
    const int64_t *ptr = nullptr;
    const int32_t *col = nullptr;
};

static bool takes_device_path(int64_t E, int64_t n_dst, int64_t n_src);

static heta_status download_small_relations(const std::vector<heta_ntype> &nts, const heta_relation *rels, int32_t n_rels,
                                            std::vector<StagedCsr> &staged)
{
    staged.assign(n_rels, StagedCsr());
    std::vector<size_t> off_ptr(n_rels, 0), off_col(n_rels, 0);
    size_t total = 0;
    for (int32_t i = 0; i < n_rels; ++i) {
        const int64_t n_dst = nts[rels[i].dst_type].num_nodes, n_src = nts[rels[i].src_type].num_nodes, E = rels[i].num_edges;
        if (takes_device_path(E, n_dst, n_src)) continue;
        off_ptr[i] = total;
        total += (static_cast<size_t>(n_dst) + 1) * sizeof(int64_t);
        off_col[i] = total;
        total += (static_cast<size_t>(std::max<int64_t>(E, 1)) * sizeof(int32_t) + 7) / 8 * 8;
    }
    if (total == 0) return HETA_OK;
    if (total > t_download.cap) {
        const size_t cap = std::max<size_t>(std::max<size_t>(t_download.cap * 2, total), size_t(1) << 20);
        void *q = nullptr;
        if (hipHostMalloc(&q, cap, hipHostMallocDefault) != hipSuccess)
            return fail(HETA_ERR_OOM, "heta_graph_create: page-locked host allocation of %zu bytes failed", cap);
        if (t_download.p) (void)hipHostFree(t_download.p);
        t_download.p = static_cast<char *>(q);
        t_download.cap = cap;
    }
    for (int32_t i = 0; i < n_rels; ++i) {
        const int64_t n_dst = nts[rels[i].dst_type].num_nodes, n_src = nts[rels[i].src_type].num_nodes, E = rels[i].num_edges;
        if (takes_device_path(E, n_dst, n_src)) continue;
        int64_t *hp = reinterpret_cast<int64_t *>(t_download.p + off_ptr[i]);
        int32_t *hc = reinterpret_cast<int32_t *>(t_download.p + off_col[i]);
        HETA_HIP(hipMemcpyAsync(hp, rels[i].csr_rowptr, (n_dst + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, nullptr));
        if (E) HETA_HIP(hipMemcpyAsync(hc, rels[i].csr_col, E * sizeof(int32_t), hipMemcpyDeviceToHost, nullptr));
        staged[i].ptr = hp;
        staged[i].col = hc;
    }
    HETA_HIP(hipStreamSynchronize(nullptr));
    return HETA_OK;
}

struct HostPack {
    size_t size = 0;
    bool failed = false;
    const char *data() const { return t_pinned.p; }
    // makes room for `need` bytes, keeping the first `size`
    bool reserve(size_t need)
    {
        if (need <= t_pinned.cap) return true;
        size_t cap = std::max<size_t>(std::max<size_t>(t_pinned.cap * 2, need), size_t(1) << 20);
        void *q = nullptr;
        if (hipHostMalloc(&q, cap, hipHostMallocDefault) != hipSuccess) {
            failed = true;
            return false;
        }
        if (size) std::memcpy(q, t_pinned.p, size);
        if (t_pinned.p) (void)hipHostFree(t_pinned.p);
        t_pinned.p = static_cast<char *>(q);
        t_pinned.cap = cap;
        return true;
    }
    template <typename T> size_t add(const T *data_in, size_t n)
    {
        const size_t off = (size + 255) / 256 * 256;
        const size_t end = off + std::max<size_t>(n, 1) * sizeof(T);
        if (!reserve(end)) return 0;
        if (n) std::memcpy(t_pinned.p + off, data_in, n * sizeof(T));
        size = end;
        return off;
    }
};

struct ScheduleOffsets {
    size_t ptr, idx, perm, sptr, sidx, hub_chunks, hub_chunk_ptr;
};

// Every array of a host-built relation has a size known from (rows, edges) alone, hub chunks up to a
// bound, so the whole graph is laid out in the page-locked buffer first and the builders write their
// results in place: no allocation and no copy per relation (fresh std::vectors of this size are
// mapped and page-faulted anew on every call, which was most of a block's ingest time).
static size_t take(size_t &cursor, size_t bytes)
{
    const size_t off = (cursor + 255) / 256 * 256;
    cursor = off + std::max<size_t>(bytes, 1);
    return off;
}

static size_t hub_chunk_bound(int64_t n_edges) // sum over hub rows of ceil(deg / chunk) <= E / chunk + E / min hub degree
{
    return static_cast<size_t>(n_edges / kHubChunk + n_edges / kHubMinDeg + 1);
}

static void lay_out(const Schedule &s, size_t &cursor, ScheduleOffsets &off)
{
    const size_t rows = static_cast<size_t>(s.n_rows), edges = static_cast<size_t>(s.n_edges);
    off.ptr = take(cursor, (rows + 1) * sizeof(int64_t));
    off.idx = take(cursor, edges * sizeof(int32_t));
    off.perm = take(cursor, rows * sizeof(int32_t));
    off.sptr = take(cursor, (rows + 1) * sizeof(int64_t));
    off.sidx = take(cursor, edges * sizeof(int32_t));
    off.hub_chunks = take(cursor, hub_chunk_bound(s.n_edges) * sizeof(HubChunk));
    off.hub_chunk_ptr = take(cursor, (static_cast<size_t>(s.n_edges / kHubMinDeg) + 2) * sizeof(int64_t));
}

// Host build of one direction's schedule (small relations): the same arrays the device path produces.
// `base + off.ptr` and `base + off.idx` already hold the adjacency by row id.
static heta_status build_schedule_on_host(Schedule &s, char *base, const ScheduleOffsets &off)
{
    const int64_t n_rows = s.n_rows;
    const int64_t *ptr = reinterpret_cast<const int64_t *>(base + off.ptr);
    const int32_t *idx = reinterpret_cast<const int32_t *>(base + off.idx);
    int32_t *perm = reinterpret_cast<int32_t *>(base + off.perm);
    int64_t *sptr = reinterpret_cast<int64_t *>(base + off.sptr);
    int32_t *sidx = reinterpret_cast<int32_t *>(base + off.sidx);
    HubChunk *chunks = reinterpret_cast<HubChunk *>(base + off.hub_chunks);
    int64_t *chunk_ptr = reinterpret_cast<int64_t *>(base + off.hub_chunk_ptr);
    // counting sort of the rows by min(degree, kHubMinDeg), descending, stable
    int64_t bucket[kHubMinDeg + 2] = {0}, bucket_edges[kHubMinDeg + 2] = {0};
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t deg = ptr[r + 1] - ptr[r], d = std::min<int64_t>(deg, kHubMinDeg);
        bucket[d] += 1;
        bucket_edges[d] += deg;
    }
    int64_t run = 0, run_edges = 0;
    for (int k = kHubMinDeg; k >= 0; --k) {
        run += bucket[k];
        run_edges += bucket_edges[k];
        s.rows_with_deg_ge[k] = run;
        s.edges_with_deg_ge[k] = run_edges;
    }
    int64_t start[kHubMinDeg + 1];
    for (int k = 0; k <= kHubMinDeg; ++k)
        start[k] = (k == kHubMinDeg) ? 0 : s.rows_with_deg_ge[k + 1];
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t d = std::min<int64_t>(ptr[r + 1] - ptr[r], kHubMinDeg);
        perm[start[d]++] = static_cast<int32_t>(r);
    }
    // the adjacency in schedule order
    sptr[0] = 0;
    for (int64_t q = 0; q < n_rows; ++q) {
        const int64_t r = perm[q], deg = ptr[r + 1] - ptr[r];
        std::copy(idx + ptr[r], idx + ptr[r] + deg, sidx + sptr[q]);
        sptr[q + 1] = sptr[q] + deg;
    }
    s.n_hub_rows = s.rows_with_deg_ge[kHubMinDeg];
    const size_t bound = hub_chunk_bound(s.n_edges);
    size_t n_chunks = 0;
    chunk_ptr[0] = 0;
    for (int64_t h = 0; h < s.n_hub_rows; ++h) {
        for (int64_t e = sptr[h]; e < sptr[h + 1]; e += kHubChunk) {
            if (n_chunks >= bound) return fail(HETA_ERR_UNSUPPORTED, "hub chunk bound %zu exceeded", bound);
            HubChunk c;
            c.e0 = e;
            c.len = static_cast<int32_t>(std::min<int64_t>(kHubChunk, sptr[h + 1] - e));
            c.slot = static_cast<int32_t>(n_chunks);
            chunks[n_chunks++] = c;
        }
        chunk_ptr[h + 1] = static_cast<int64_t>(n_chunks);
    }
    if (n_chunks >= (size_t(1) << 31))
        return fail(HETA_ERR_UNSUPPORTED, "too many hub chunks (%zu)", n_chunks);
    s.n_hub_chunks = static_cast<int64_t>(n_chunks);
    return HETA_OK;
}

static void resolve(Schedule &s, const ScheduleOffsets &off, char *base)
{
    s.d_ptr = reinterpret_cast<int64_t *>(base + off.ptr);
    s.d_idx = reinterpret_cast<int32_t *>(base + off.idx);
    s.d_perm = reinterpret_cast<int32_t *>(base + off.perm);
    s.d_sptr = reinterpret_cast<int64_t *>(base + off.sptr);
    s.d_sidx = reinterpret_cast<int32_t *>(base + off.sidx);
    s.d_hub_chunks = reinterpret_cast<HubChunk *>(base + off.hub_chunks);
    s.d_hub_chunk_ptr = reinterpret_cast<int64_t *>(base + off.hub_chunk_ptr);
}

static void free_schedule(Schedule &s)
{
    (void)hipFree(s.d_ptr);
    (void)hipFree(s.d_idx);
    (void)hipFree(s.d_perm);
    (void)hipFree(s.d_sptr);
    (void)hipFree(s.d_sidx);
    (void)hipFree(s.d_hub_chunks);
    (void)hipFree(s.d_hub_chunk_ptr);
    s = Schedule();
}

static void destroy(heta_graph *g)
{
    if (!g)
        return;
    (void)hipDeviceSynchronize();
    for (auto &r : g->rels) {
        (void)hipFree(r.d_hub_slot);
        (void)hipFree(r.d_hub_rows);
        if (r.host_built) continue; // its arrays live in the graph's arena
        if (r.shares >= 0) {        // a declared reverse: the schedules belong to the relation it names
            (void)hipFree(r.d_inv_deg);
            continue;
        }
        free_schedule(r.csr);
        free_schedule(r.csc);
        (void)hipFree(r.d_inv_deg);
    }
    scratch_free(g->d_arena); // the device is idle here
    g->block_arena.reset(); // released with the last graph that shares it
    scratch_free(g->d_ws);
    scratch_free(g->d_pack);
    (void)hipFree(g->d_attn);
    delete g;
}

// Host-only checks of one relation's arguments and CSR; touches no device.
static heta_status validate_relation(const std::vector<heta_ntype> &ntypes, const heta_relation &in,
                                     int32_t index, const int64_t *ptr, const int32_t *col)
{
    const int64_t n_dst = ntypes[in.dst_type].num_nodes, n_src = ntypes[in.src_type].num_nodes;
    const int64_t E = in.num_edges;
    if (ptr[0] != 0)
        return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr[0] = %lld, expected 0", index, (long long)ptr[0]);
    for (int64_t v = 0; v < n_dst; ++v)
        if (ptr[v + 1] < ptr[v])
            return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr decreases at row %lld", index, (long long)v);
    if (ptr[n_dst] != E)
        return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr[n_dst] = %lld but num_edges = %lld", index,
                    (long long)ptr[n_dst], (long long)E);
    for (int64_t e = 0; e < E; ++e)
        if (col[e] < 0 || col[e] >= n_src)
            return fail(HETA_ERR_BAD_CSR, "relation %d: col[%lld] = %d outside [0, %lld)", index,
                        (long long)e, col[e], (long long)n_src);
    return HETA_OK;
}

static heta_status check_relation_args(const std::vector<heta_ntype> &ntypes, const heta_relation &in,
                                       int32_t index)
{
    const int32_t n_nt = static_cast<int32_t>(ntypes.size());
    if (in.src_type < 0 || in.src_type >= n_nt || in.dst_type < 0 || in.dst_type >= n_nt)
        return fail(HETA_ERR_INVALID_ARG, "relation %d: node type out of range", index);
    if (in.num_edges < 0)
        return fail(HETA_ERR_INVALID_ARG, "relation %d: negative num_edges", index);
    if (!in.csr_rowptr || (in.num_edges > 0 && !in.csr_col))
        return fail(HETA_ERR_INVALID_ARG, "relation %d: null CSR pointer", index);
    if ((in.csc_colptr != nullptr) != (in.csc_row != nullptr) && in.num_edges > 0)
        return fail(HETA_ERR_INVALID_ARG, "relation %d: csc_colptr and csc_row come together or not at all", index);
    if (in.reverse_of < -1 || in.reverse_of >= index)
        return fail(HETA_ERR_INVALID_ARG, "relation %d: reverse_of = %d must be -1 or the index of an earlier relation", index,
                    in.reverse_of);
    return HETA_OK;
}

// reverse_of against the relation it names (both argument structs are already checked on their own)
static heta_status check_reverse_args(const heta_relation *rels, int32_t index)
{
    const heta_relation &in = rels[index];
    if (in.reverse_of < 0) return HETA_OK;
    const heta_relation &base = rels[in.reverse_of];
    if (base.reverse_of >= 0)
        return fail(HETA_ERR_INVALID_ARG, "relation %d: reverse_of names relation %d, which is itself declared a reverse", index,
                    in.reverse_of);
    if (base.src_type != in.dst_type || base.dst_type != in.src_type || base.num_edges != in.num_edges)
        return fail(HETA_ERR_BAD_CSR, "relation %d is not the transpose of relation %d: node types or edge counts differ", index,
                    in.reverse_of);
    return HETA_OK;
}

// ---- element-wise comparison of index arrays on the device -------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) arrays_differ_kernel(const T *a, const T *b, int64_t n, int *flag)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n && a[i] != b[i]) *flag = 1; // every writer stores the same value
}

__global__ void __launch_bounds__(256) inv_degree_kernel(const int64_t *ptr, int64_t n, float *inv)
{
    const int64_t v = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (v >= n) return;
    const int64_t d = ptr[v + 1] - ptr[v];
    inv[v] = d > 0 ? 1.0f / static_cast<float>(d) : 0.0f;
}

// *differ = whether caller[0..n) (host array, or device array with on_device) differs from dev[0..n).  Synchronous.
template <typename T>
static heta_status differs_from_device(const T *caller, bool on_device, const T *dev, int64_t n, bool *differ)
{
    *differ = false;
    if (n <= 0) return HETA_OK;
    T *tmp = nullptr;
    int *flag = nullptr;
    heta_status st = HETA_OK;
    auto done = [&](heta_status s) {
        (void)hipFree(tmp);
        (void)hipFree(flag);
        return s;
    };
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&flag), sizeof(int));
    if (e == hipSuccess) e = hipMemset(flag, 0, sizeof(int));
    const T *a = caller;
    if (e == hipSuccess && !on_device) {
        e = hipMalloc(reinterpret_cast<void **>(&tmp), n * sizeof(T));
        if (e == hipSuccess) e = hipMemcpy(tmp, caller, n * sizeof(T), hipMemcpyHostToDevice);
        a = tmp;
    }
    if (e != hipSuccess) return done(fail(e == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE, "heta_graph_create: %s", hipGetErrorString(e)));
    const int64_t blocks = (n + 255) / 256;
    if (blocks > 0x7fffffff) return done(fail(HETA_ERR_UNSUPPORTED, "heta_graph_create: index array too long to compare"));
    hipLaunchKernelGGL(arrays_differ_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, nullptr, a, dev, n, flag);
    int h = 0;
    e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpy(&h, flag, sizeof(int), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return done(fail(HETA_ERR_DEVICE, "heta_graph_create: %s", hipGetErrorString(e)));
    *differ = h != 0;
    return done(st);
}

// Relations below this many edges + rows are ingested on the host: a few microseconds of CPU work
// beat the launch latencies of the device pipeline (sampled mini-batch blocks); everything larger
// is built by the kernels of heta_ingest.hip.  heta_ingest_force() overrides the choice.
constexpr int64_t kDeviceIngestMin = 1 << 18;
// The small relations of one graph together (a sampled block) go through the whole-block device ingest when they
// add up to this many edges + rows (and are at most 32); below it the host builds them faster than ~40 launches run.
constexpr int64_t kBlockIngestMin = 1 << 16;
static int g_ingest_mode = 0; // 0 = by size, 1 = host, 2 = per-relation device kernels, 3 = small relations by the whole-block device ingest

// A host-built relation waits in the graph's host buffer until every relation is built; then one
// allocation and one copy bring all of them to the device and the offsets become pointers.
struct PendingRelation {
    size_t rel;
    ScheduleOffsets csr, csc;
    size_t inv;
};

static bool takes_device_path(int64_t E, int64_t n_dst, int64_t n_src)
{
    return g_ingest_mode == 2 || ((g_ingest_mode == 0 || g_ingest_mode == 3) && E + n_dst + n_src >= kDeviceIngestMin);
}

// whether the small relations of a graph (those that do not take the per-relation device path) are built together on the device
static bool takes_block_path(const std::vector<heta_ntype> &nts, const heta_relation *rels, int32_t n_rels)
{
    if (g_ingest_mode == 1 || g_ingest_mode == 2) return false;
    int64_t work = 0;
    int32_t n_small = 0;
    for (int32_t i = 0; i < n_rels; ++i) {
        const int64_t n_dst = nts[rels[i].dst_type].num_nodes, n_src = nts[rels[i].src_type].num_nodes, E = rels[i].num_edges;
        if (takes_device_path(E, n_dst, n_src)) continue;
        work += E + n_dst + n_src;
        ++n_small;
    }
    if (n_small == 0 || n_small > block_ingest_max_relations()) return false;
    return g_ingest_mode == 3 || work >= kBlockIngestMin;
}

// One small relation of a graph about to be built: relation `index` of `rels`, registered in g; graph_no is the
// graph's position in a batch (-1: a single heta_graph_create), used in error messages only.
struct SmallRef {
    heta_graph *g;
    const heta_relation *rels;
    int32_t index;
    int graph_no;
};

// The listed small relations (of one graph, or of all graphs of a batch) through the whole-block device ingest.
// Host arrays are staged through the page-locked buffer and one device block first; supplied CSCs and declared
// reverses are then checked against what was built.  The graphs share the one arena that holds the arrays.
static heta_status build_small_relations_on_device(const std::vector<SmallRef> &refs, bool on_device)
{
    const size_t n = refs.size();
    if (n == 0) return HETA_OK;
    std::vector<const int64_t *> ptrs(n);
    std::vector<const int32_t *> cols(n);
    std::vector<Relation *> built(n);
    std::vector<std::string> names(n);
    for (size_t k = 0; k < n; ++k) {
        built[k] = &refs[k].g->rels[refs[k].index];
        names[k] = refs[k].graph_no < 0 ? "relation " + std::to_string(refs[k].index)
                                        : "graph " + std::to_string(refs[k].graph_no) + " relation " + std::to_string(refs[k].index);
    }
    void *staging = nullptr;
    if (on_device) {
        for (size_t k = 0; k < n; ++k) {
            ptrs[k] = refs[k].rels[refs[k].index].csr_rowptr;
            cols[k] = refs[k].rels[refs[k].index].csr_col;
        }
    } else {
        HostPack pack;
        std::vector<size_t> off_ptr(n), off_col(n);
        size_t total = 0;
        for (size_t k = 0; k < n; ++k) {
            const Relation &r = *built[k];
            off_ptr[k] = take(total, (static_cast<size_t>(r.n_dst) + 1) * sizeof(int64_t));
            off_col[k] = take(total, static_cast<size_t>(r.n_edges) * sizeof(int32_t));
        }
        if (!pack.reserve(total)) return fail(HETA_ERR_OOM, "heta_graph_create: page-locked host allocation of %zu bytes failed", total);
        for (size_t k = 0; k < n; ++k) {
            const Relation &r = *built[k];
            const heta_relation &in = refs[k].rels[refs[k].index];
            std::memcpy(t_pinned.p + off_ptr[k], in.csr_rowptr, (r.n_dst + 1) * sizeof(int64_t));
            if (r.n_edges) std::memcpy(t_pinned.p + off_col[k], in.csr_col, r.n_edges * sizeof(int32_t));
        }
        HETA_HIP(scratch_alloc(&staging, total));
        hipError_t e = hipMemcpyAsync(staging, t_pinned.p, total, hipMemcpyHostToDevice, nullptr);
        if (e != hipSuccess) {
            (void)hipStreamSynchronize(nullptr);
            scratch_free(staging);
            return fail(HETA_ERR_DEVICE, "heta_graph_create: %s", hipGetErrorString(e));
        }
        for (size_t k = 0; k < n; ++k) {
            ptrs[k] = reinterpret_cast<const int64_t *>(static_cast<char *>(staging) + off_ptr[k]);
            cols[k] = reinterpret_cast<const int32_t *>(static_cast<char *>(staging) + off_col[k]);
        }
    }
    // The build runs on a stream of the library's own (per thread and device, default priority, non-blocking): its inputs
    // are complete (host arrays; device arrays the caller has finished, as for every synchronous call) and it is complete
    // when the call returns.  On the legacy default stream every one of its ~45 launches would first be ordered against
    // all other streams of the process, which costs more than the kernels run.
    static thread_local hipStream_t t_stream[64] = {};
    int dev = 0;
    HETA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(HETA_ERR_UNSUPPORTED, "device index %d beyond 64", dev);
    if (!t_stream[dev]) HETA_HIP(hipStreamCreateWithFlags(&t_stream[dev], hipStreamNonBlocking));
    if (staging) HETA_HIP(hipStreamSynchronize(nullptr)); // the staged arrays have arrived
    void *arena = nullptr;
    heta_status st = build_block_on_device(built, names, ptrs.data(), cols.data(), &arena, t_stream[dev]); // synchronous
    scratch_free(staging);
    if (st != HETA_OK) return st;
    {
        std::shared_ptr<void> shared(arena, [](void *p) { scratch_free(p); });
        for (const SmallRef &ref : refs) ref.g->block_arena = shared;
    }
    for (size_t k = 0; k < n; ++k) {
        const heta_relation &in = refs[k].rels[refs[k].index];
        const Relation &rel = *built[k];
        const char *name = names[k].c_str();
        bool d1 = false, d2 = false;
        if (in.csc_colptr) {
            if ((st = differs_from_device(in.csc_colptr, on_device, rel.csc.d_ptr, rel.n_src + 1, &d1)) != HETA_OK) return st;
            if ((st = differs_from_device(in.csc_row, on_device, rel.csc.d_idx, rel.n_edges, &d2)) != HETA_OK) return st;
            if (d1 || d2)
                return fail(HETA_ERR_BAD_CSR, "%s: the supplied CSC is not the transposed adjacency of its CSR (columns in "
                                              "ascending edge order)", name);
        }
        if (in.reverse_of >= 0) {
            const Relation &base = refs[k].g->rels[in.reverse_of];
            if ((st = differs_from_device(in.csr_rowptr, on_device, base.csc.d_ptr, rel.n_dst + 1, &d1)) != HETA_OK) return st;
            if ((st = differs_from_device(in.csr_col, on_device, base.csc.d_idx, rel.n_edges, &d2)) != HETA_OK) return st;
            if (d1 || d2) return fail(HETA_ERR_BAD_CSR, "%s: its CSR is not the transposed adjacency of relation %d", name, in.reverse_of);
        }
    }
    return HETA_OK;
}

// Registers relation `index` in g; a large relation is built on the device right away, a small one
// is left for build_on_host (device_path tells which).
static heta_status ingest_relation(heta_graph *g, const heta_relation &in, int32_t index, bool on_device, bool &device_path)
{
    g->rels.emplace_back();
    Relation &rel = g->rels.back(); // owned by g from here on: destroy(g) releases whatever was allocated
    rel.src_type = in.src_type;
    rel.dst_type = in.dst_type;
    rel.n_src = g->ntypes[in.src_type].num_nodes;
    rel.n_dst = g->ntypes[in.dst_type].num_nodes;
    rel.n_edges = in.num_edges;
    const int64_t E = in.num_edges, n_dst = rel.n_dst, n_src = rel.n_src;
    hipStream_t st = nullptr;
    rel.csr.n_rows = n_dst;
    rel.csr.n_edges = E;
    rel.csc.n_rows = n_src;
    rel.csc.n_edges = E;

    device_path = takes_device_path(E, n_dst, n_src);
    if (!device_path) return HETA_OK;
    if (in.reverse_of >= 0) {
        // A declared reverse: its CSR must be the named relation's CSC; then it keeps no arrays of its own
        // but 1/deg.  (The named relation has the same size, so it took the device path as well.)
        const Relation &base = g->rels[in.reverse_of];
        bool d1 = false, d2 = false;
        heta_status vst = differs_from_device(in.csr_rowptr, on_device, base.csc.d_ptr, n_dst + 1, &d1);
        if (vst == HETA_OK) vst = differs_from_device(in.csr_col, on_device, base.csc.d_idx, E, &d2);
        if (vst != HETA_OK) return vst;
        if (d1 || d2)
            return fail(HETA_ERR_BAD_CSR, "relation %d: its CSR is not the transposed adjacency of relation %d", index, in.reverse_of);
        if (in.csc_colptr) {
            vst = differs_from_device(in.csc_colptr, on_device, base.csr.d_ptr, n_src + 1, &d1);
            if (vst != HETA_OK) return vst;
            if (d1) return fail(HETA_ERR_BAD_CSR, "relation %d: the supplied CSC does not match the CSR of relation %d", index, in.reverse_of);
        }
        rel.csr = base.csc;
        rel.csc = base.csr;
        rel.shares = in.reverse_of;
        HETA_HIP(hipMalloc(reinterpret_cast<void **>(&rel.d_inv_deg), std::max<int64_t>(n_dst, 1) * sizeof(float)));
        if (n_dst > 0) {
            hipLaunchKernelGGL(inv_degree_kernel, dim3((unsigned)((n_dst + 255) / 256)), dim3(256), 0, st, rel.csr.d_ptr, n_dst, rel.d_inv_deg);
            HETA_LAUNCH_CHECK("inv_degree_kernel");
            HETA_HIP(hipStreamSynchronize(st));
        }
        return HETA_OK;
    }
    // the CSR itself: a device copy of the caller's arrays
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(&rel.csr.d_ptr), (n_dst + 1) * sizeof(int64_t)));
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(&rel.csr.d_idx), std::max<int64_t>(E, 1) * sizeof(int32_t)));
    const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    HETA_HIP(hipMemcpy(rel.csr.d_ptr, in.csr_rowptr, (n_dst + 1) * sizeof(int64_t), kind));
    if (E) HETA_HIP(hipMemcpy(rel.csr.d_idx, in.csr_col, E * sizeof(int32_t), kind));
    if (on_device) { // host arrays were validated before the device was touched
        heta_status vst = validate_csr_on_device(index, rel.csr.d_ptr, rel.csr.d_idx, n_dst, n_src, E, st);
        if (vst != HETA_OK) return vst;
    }
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(&rel.d_inv_deg), std::max<int64_t>(n_dst, 1) * sizeof(float)));
    heta_status e;
    if ((e = transpose_on_device(rel.csr, n_src, rel.csc, st)) != HETA_OK) return e;
    if (in.csc_colptr) { // a supplied CSC must be the one just derived
        bool d1 = false, d2 = false;
        if ((e = differs_from_device(in.csc_colptr, on_device, rel.csc.d_ptr, n_src + 1, &d1)) != HETA_OK) return e;
        if ((e = differs_from_device(in.csc_row, on_device, rel.csc.d_idx, E, &d2)) != HETA_OK) return e;
        if (d1 || d2)
            return fail(HETA_ERR_BAD_CSR, "relation %d: the supplied CSC is not the transposed adjacency of its CSR (columns in "
                                          "ascending edge order)", index);
    }
    if ((e = build_schedule_on_device(rel.csr, rel.d_inv_deg, st)) != HETA_OK) return e;
    return build_schedule_on_device(rel.csc, nullptr, st);
}

// Host build of one small relation: 1/deg, the stable transpose, both schedules, written in place into
// the relation's slices of the page-locked buffer.  Touches no device and no state shared with other
// relations, so the relations of a graph are built by several threads; a failure is returned with its
// message (the thread-local error slot belongs to the worker).
struct SmallLayout {
    ScheduleOffsets csr, csc; // in the page-locked buffer
    size_t inv;               // 1/deg, in the page-locked buffer
    size_t cursor;            // fill positions of the transpose, in the scratch arena
};

struct HostBuilt {
    heta_status status = HETA_OK;
    std::string message;
};

static void build_on_host(const std::vector<heta_ntype> &ntypes, const heta_relation &in, int32_t index, Relation &rel,
                          const int64_t *ptr, const int32_t *col, bool validate, char *base, const SmallLayout &lay,
                          char *scratch, HostBuilt &out)
{
    const int64_t E = rel.n_edges, n_dst = rel.n_dst, n_src = rel.n_src;
    if (validate) { // arrays that came from the device: checked now that they are on the host
        out.status = validate_relation(ntypes, in, index, ptr, col);
        if (out.status != HETA_OK) {
            out.message = g_last_error;
            return;
        }
    }
    std::memcpy(base + lay.csr.ptr, ptr, (n_dst + 1) * sizeof(int64_t));
    if (E) std::memcpy(base + lay.csr.idx, col, E * sizeof(int32_t));
    float *inv_deg = reinterpret_cast<float *>(base + lay.inv);
    for (int64_t v = 0; v < n_dst; ++v) {
        const int64_t d = ptr[v + 1] - ptr[v];
        inv_deg[v] = d > 0 ? 1.0f / static_cast<float>(d) : 0.0f;
    }
    // stable transpose: column u keeps its edges in ascending original edge position
    int64_t *colptr = reinterpret_cast<int64_t *>(base + lay.csc.ptr);
    int32_t *row = reinterpret_cast<int32_t *>(base + lay.csc.idx);
    int64_t *cursor = reinterpret_cast<int64_t *>(scratch + lay.cursor);
    std::fill(colptr, colptr + n_src + 1, int64_t(0));
    for (int64_t e = 0; e < E; ++e)
        colptr[col[e] + 1] += 1;
    for (int64_t u = 0; u < n_src; ++u)
        colptr[u + 1] += colptr[u];
    std::copy(colptr, colptr + n_src, cursor);
    for (int64_t v = 0; v < n_dst; ++v)
        for (int64_t e = ptr[v]; e < ptr[v + 1]; ++e)
            row[cursor[col[e]]++] = static_cast<int32_t>(v);
    if ((out.status = build_schedule_on_host(rel.csr, base, lay.csr)) == HETA_OK)
        out.status = build_schedule_on_host(rel.csc, base, lay.csc);
    if (out.status != HETA_OK) out.message = g_last_error;
}

static thread_local std::vector<char> t_scratch; // the transposes' fill positions; grows, never shrinks

// Builds every small relation of the graph on the host, several at a time: at most 8 workers, which
// covers the relation counts of the paper's graphs (5 to 14 per block) and leaves cores to the caller's
// other threads.  Largest relations first, dealt by an atomic counter.
static heta_status build_small_relations(heta_graph *g, const heta_relation *rels, const std::vector<int32_t> &small,
                                         bool on_device, const std::vector<StagedCsr> &staged, HostPack &pack,
                                         std::vector<PendingRelation> &pending)
{
    if (small.empty()) return HETA_OK;
    // the layout of the whole graph, in relation order
    std::vector<SmallLayout> lay(small.size());
    size_t total = pack.size, scratch_total = 0;
    for (size_t k = 0; k < small.size(); ++k) {
        const Relation &rel = g->rels[small[k]];
        lay_out(rel.csr, total, lay[k].csr);
        lay_out(rel.csc, total, lay[k].csc);
        lay[k].inv = take(total, static_cast<size_t>(rel.n_dst) * sizeof(float));
        lay[k].cursor = take(scratch_total, static_cast<size_t>(rel.n_src) * sizeof(int64_t));
    }
    if (!pack.reserve(total)) return fail(HETA_ERR_OOM, "heta_graph_create: page-locked host allocation of %zu bytes failed", total);
    pack.size = total;
    if (t_scratch.size() < scratch_total) t_scratch.resize(scratch_total);
    char *base = t_pinned.p, *scratch = t_scratch.data();

    std::vector<size_t> order(small.size());
    for (size_t k = 0; k < order.size(); ++k) order[k] = k;
    auto work = [&](size_t k) { const Relation &r = g->rels[small[k]]; return r.n_edges + r.n_dst + r.n_src; };
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return work(a) > work(b); });
    std::vector<HostBuilt> built(small.size());
    std::atomic<size_t> next{0};
    auto run = [&]() {
        for (size_t j = next.fetch_add(1); j < order.size(); j = next.fetch_add(1)) {
            const size_t k = order[j];
            const int32_t i = small[k];
            const int64_t *ptr = on_device ? staged[i].ptr : rels[i].csr_rowptr;
            const int32_t *col = on_device ? staged[i].col : rels[i].csr_col;
            build_on_host(g->ntypes, rels[i], i, g->rels[i], ptr, col, on_device, base, lay[k], scratch, built[k]);
        }
    };
    int64_t total_work = 0;
    for (size_t k = 0; k < small.size(); ++k) total_work += work(k);
    // below ~64 k elements of work a thread's start costs more than it saves
    const size_t n_threads = total_work < (int64_t(1) << 16) ? 1 : std::min<size_t>(order.size(), 8);
    std::vector<std::thread> workers;
    try {
        for (size_t t = 1; t < n_threads; ++t) workers.emplace_back(run);
    } catch (const std::system_error &) { // no more threads to be had: the caller's thread does what is left
    }
    run();
    for (std::thread &w : workers) w.join();
    for (size_t k = 0; k < small.size(); ++k)
        if (built[k].status != HETA_OK) return fail(built[k].status, "%s", built[k].message.c_str());
    // Supplied CSCs and declared reverses of host-built relations are checked against what was just built
    // (small relations keep arrays of their own either way: sharing pays for the large, device-built ones).
    std::vector<char> fetched;
    auto on_host = [&](const void *p, size_t bytes, const void **out) -> heta_status { // caller's array as host memory
        *out = p;
        if (!on_device || bytes == 0) return HETA_OK;
        fetched.resize(bytes);
        HETA_HIP(hipMemcpy(fetched.data(), p, bytes, hipMemcpyDeviceToHost));
        *out = fetched.data();
        return HETA_OK;
    };
    for (size_t k = 0; k < small.size(); ++k) {
        const int32_t i = small[k];
        const heta_relation &in = rels[i];
        const Relation &rel = g->rels[i];
        const void *q = nullptr;
        if (in.csc_colptr) {
            heta_status st = on_host(in.csc_colptr, (rel.n_src + 1) * sizeof(int64_t), &q);
            if (st != HETA_OK) return st;
            bool bad = std::memcmp(q, base + lay[k].csc.ptr, (rel.n_src + 1) * sizeof(int64_t)) != 0;
            if (!bad && rel.n_edges) {
                if ((st = on_host(in.csc_row, rel.n_edges * sizeof(int32_t), &q)) != HETA_OK) return st;
                bad = std::memcmp(q, base + lay[k].csc.idx, rel.n_edges * sizeof(int32_t)) != 0;
            }
            if (bad)
                return fail(HETA_ERR_BAD_CSR, "relation %d: the supplied CSC is not the transposed adjacency of its CSR (columns in "
                                              "ascending edge order)", i);
        }
        if (in.reverse_of >= 0) {
            size_t kj = small.size();
            for (size_t t = 0; t < small.size(); ++t)
                if (small[t] == in.reverse_of) kj = t;
            if (kj == small.size()) return fail(HETA_ERR_BAD_CSR, "relation %d is not the transpose of relation %d", i, in.reverse_of);
            const int64_t *ptr = on_device ? staged[i].ptr : in.csr_rowptr;
            const int32_t *col = on_device ? staged[i].col : in.csr_col;
            if (std::memcmp(ptr, base + lay[kj].csc.ptr, (rel.n_dst + 1) * sizeof(int64_t)) != 0 ||
                (rel.n_edges && std::memcmp(col, base + lay[kj].csc.idx, rel.n_edges * sizeof(int32_t)) != 0))
                return fail(HETA_ERR_BAD_CSR, "relation %d: its CSR is not the transposed adjacency of relation %d", i, in.reverse_of);
        }
    }
    for (size_t k = 0; k < small.size(); ++k) {
        PendingRelation pr;
        pr.rel = static_cast<size_t>(small[k]);
        pr.csr = lay[k].csr;
        pr.csc = lay[k].csc;
        pr.inv = lay[k].inv;
        g->rels[small[k]].host_built = true;
        pending.push_back(pr);
    }
    return HETA_OK;
}

// one allocation and one copy for every host-built relation of the graph
static heta_status upload_host_built(heta_graph *g, const HostPack &pack, const std::vector<PendingRelation> &pending)
{
    if (pending.empty()) return HETA_OK;
    if (pack.failed) return fail(HETA_ERR_OOM, "heta_graph_create: page-locked host allocation failed");
    HETA_HIP(scratch_alloc(&g->d_arena, pack.size));
    HETA_HIP(hipMemcpy(g->d_arena, pack.data(), pack.size, hipMemcpyHostToDevice));
    char *base = static_cast<char *>(g->d_arena);
    for (const PendingRelation &pr : pending) {
        Relation &rel = g->rels[pr.rel];
        resolve(rel.csr, pr.csr, base);
        resolve(rel.csc, pr.csc, base);
        rel.d_inv_deg = reinterpret_cast<float *>(base + pr.inv);
    }
    return HETA_OK;
}

} // namespace heta

using namespace heta;

extern "C" {

const char *heta_last_error(void) { return g_last_error.c_str(); }
const char *heta_version(void) { return "0.1"; }

// everything of a heta_graph_create call that can be rejected on the host, before the device is touched
// everything of a heta_graph_create call that can be rejected without walking the relations' arrays
static heta_status check_create_args(const heta_ntype *ntypes, int32_t n_ntypes, const heta_relation *rels, int32_t n_rels,
                                     uint32_t flags)
{
    if (!ntypes || n_ntypes <= 0)
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_create: need at least one node type");
    if (n_rels < 0 || (n_rels > 0 && !rels))
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_create: bad relation array");
    if (flags & ~HETA_PTRS_ON_DEVICE)
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_create: unknown flag bits 0x%x", flags);
    for (int32_t t = 0; t < n_ntypes; ++t) {
        if (ntypes[t].num_nodes < 0 || ntypes[t].num_nodes >= (int64_t(1) << 31))
            return fail(HETA_ERR_INVALID_ARG, "node type %d: num_nodes %lld outside [0, 2^31)", t,
                        (long long)ntypes[t].num_nodes);
        if (ntypes[t].feat_dim < 0)
            return fail(HETA_ERR_INVALID_ARG, "node type %d: negative feat_dim", t);
    }
    std::vector<heta_ntype> nts(ntypes, ntypes + n_ntypes);
    for (int32_t i = 0; i < n_rels; ++i) {
        heta_status st = check_relation_args(nts, rels[i], i);
        if (st == HETA_OK) st = check_reverse_args(rels, i);
        if (st != HETA_OK)
            return st;
    }
    return HETA_OK;
}

// The CSRs of host arrays, walked on the host before the device is touched.  small_on_device: the small relations go
// through the whole-block device build, whose kernels check the same properties and fail the call the same way; only
// the large relations (uploaded and built one by one) are walked here then.
static heta_status validate_host_arrays(const heta_ntype *ntypes, int32_t n_ntypes, const heta_relation *rels, int32_t n_rels,
                                        bool small_on_device)
{
    std::vector<heta_ntype> nts(ntypes, ntypes + n_ntypes);
    for (int32_t i = 0; i < n_rels; ++i) {
        const bool large = takes_device_path(rels[i].num_edges, nts[rels[i].dst_type].num_nodes, nts[rels[i].src_type].num_nodes);
        if (!large && small_on_device) continue;
        heta_status st = validate_relation(nts, rels[i], i, rels[i].csr_rowptr, rels[i].csr_col);
        if (st != HETA_OK) return st;
    }
    return HETA_OK;
}

// a new handle with its node types, on the current device
static heta_status new_graph(const heta_ntype *ntypes, int32_t n_ntypes, heta_graph **out)
{
    heta_graph *g = new (std::nothrow) heta_graph();
    if (!g)
        return fail(HETA_ERR_OOM, "heta_graph_create: host allocation failed");
    g->ntypes.assign(ntypes, ntypes + n_ntypes);
    hipError_t e = hipGetDevice(&g->device);
    if (e != hipSuccess) {
        delete g;
        return fail(HETA_ERR_DEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
    }
    // set-up time: this device's address of the fixed scratch of heta_rel_aggregate_fwd_noalloc
    heta_status st = noalloc_scratch_init();
    if (st != HETA_OK) {
        delete g;
        return st;
    }
    *out = g;
    return HETA_OK;
}

heta_status heta_graph_create(const heta_ntype *ntypes, int32_t n_ntypes, const heta_relation *rels,
                              int32_t n_rels, uint32_t flags, heta_graph **out)
{
    if (!out)
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_create: out is NULL");
    heta_status st0 = check_create_args(ntypes, n_ntypes, rels, n_rels, flags);
    if (st0 != HETA_OK) return st0;
    if (!(flags & HETA_PTRS_ON_DEVICE)) {
        const std::vector<heta_ntype> nts(ntypes, ntypes + n_ntypes);
        st0 = validate_host_arrays(ntypes, n_ntypes, rels, n_rels, takes_block_path(nts, rels, n_rels));
        if (st0 != HETA_OK) return st0;
    }
    const bool on_device = (flags & HETA_PTRS_ON_DEVICE) != 0;
    heta_graph *g = nullptr;
    st0 = new_graph(ntypes, n_ntypes, &g);
    if (st0 != HETA_OK) return st0;
    try {
        g->rels.reserve(n_rels);
        HostPack pack;
        std::vector<PendingRelation> pending;
        std::vector<StagedCsr> staged(n_rels);
        const bool block_path = takes_block_path(g->ntypes, rels, n_rels);
        if (on_device && !block_path) {
            heta_status st = download_small_relations(g->ntypes, rels, n_rels, staged);
            if (st != HETA_OK) {
                destroy(g);
                return st;
            }
        }
        std::vector<int32_t> small;
        for (int32_t i = 0; i < n_rels; ++i) {
            bool device_path = false;
            heta_status st = ingest_relation(g, rels[i], i, on_device, device_path);
            if (st != HETA_OK) {
                destroy(g);
                return st;
            }
            if (!device_path) small.push_back(i);
        }
        heta_status st;
        if (block_path) {
            std::vector<SmallRef> refs;
            for (int32_t i : small) refs.push_back(SmallRef{g, rels, i, -1});
            st = build_small_relations_on_device(refs, on_device);
        } else {
            st = build_small_relations(g, rels, small, on_device, staged, pack, pending);
            if (st == HETA_OK) st = upload_host_built(g, pack, pending);
        }
        if (st != HETA_OK) {
            destroy(g);
            return st;
        }
    } catch (const std::bad_alloc &) {
        destroy(g);
        return fail(HETA_ERR_OOM, "heta_graph_create: host allocation failed");
    }
    *out = g;
    return HETA_OK;
}

heta_status heta_graph_create_batch(int32_t n_graphs, const heta_ntype *const *ntypes, const int32_t *n_ntypes,
                                    const heta_relation *const *rels, const int32_t *n_rels, uint32_t flags, heta_graph **out)
{
    if (n_graphs < 0 || (n_graphs > 0 && (!ntypes || !n_ntypes || !rels || !n_rels || !out)))
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_create_batch: null argument");
    for (int32_t q = 0; q < n_graphs; ++q) out[q] = nullptr;
    for (int32_t q = 0; q < n_graphs; ++q) {
        heta_status st = check_create_args(ntypes[q], n_ntypes[q], rels[q], n_rels[q], flags);
        if (st != HETA_OK) return st;
    }
    const bool on_device = (flags & HETA_PTRS_ON_DEVICE) != 0;
    // The small relations of all graphs go through one whole-block build when together they qualify for it; otherwise
    // (too few edges for the device to pay, too many relations for one build, or a forced path) graph by graph.
    bool together = g_ingest_mode == 0 || g_ingest_mode == 3;
    if (together) {
        int64_t work = 0, n_small = 0;
        for (int32_t q = 0; q < n_graphs; ++q)
            for (int32_t i = 0; i < n_rels[q]; ++i) {
                const heta_relation &r = rels[q][i];
                const int64_t n_dst = ntypes[q][r.dst_type].num_nodes, n_src = ntypes[q][r.src_type].num_nodes;
                if (takes_device_path(r.num_edges, n_dst, n_src)) continue;
                work += r.num_edges + n_dst + n_src;
                ++n_small;
            }
        together = n_small > 0 && n_small <= block_ingest_max_relations() && (g_ingest_mode == 3 || work >= kBlockIngestMin);
    }
    if (together && !on_device)
        for (int32_t q = 0; q < n_graphs; ++q) {
            heta_status st = validate_host_arrays(ntypes[q], n_ntypes[q], rels[q], n_rels[q], true);
            if (st != HETA_OK) return st;
        }
    if (!together) {
        for (int32_t q = 0; q < n_graphs; ++q) {
            heta_status st = heta_graph_create(ntypes[q], n_ntypes[q], rels[q], n_rels[q], flags, &out[q]);
            if (st != HETA_OK) {
                for (int32_t p = 0; p < q; ++p) {
                    destroy(out[p]);
                    out[p] = nullptr;
                }
                return st;
            }
        }
        return HETA_OK;
    }
    std::vector<heta_graph *> made;
    auto undo = [&](heta_status st) {
        for (heta_graph *g : made) destroy(g);
        for (int32_t q = 0; q < n_graphs; ++q) out[q] = nullptr;
        return st;
    };
    try {
        std::vector<SmallRef> refs;
        for (int32_t q = 0; q < n_graphs; ++q) {
            heta_graph *g = nullptr;
            heta_status st = new_graph(ntypes[q], n_ntypes[q], &g);
            if (st != HETA_OK) return undo(st);
            made.push_back(g);
            g->rels.reserve(n_rels[q]);
            for (int32_t i = 0; i < n_rels[q]; ++i) {
                bool device_path = false;
                st = ingest_relation(g, rels[q][i], i, on_device, device_path);
                if (st != HETA_OK) return undo(st);
                if (!device_path) refs.push_back(SmallRef{g, rels[q], i, q});
            }
        }
        heta_status st = build_small_relations_on_device(refs, on_device);
        if (st != HETA_OK) return undo(st);
    } catch (const std::bad_alloc &) {
        return undo(fail(HETA_ERR_OOM, "heta_graph_create_batch: host allocation failed"));
    }
    for (int32_t q = 0; q < n_graphs; ++q) out[q] = made[q];
    return HETA_OK;
}

heta_status heta_ingest_force(int32_t mode)
{
    if (mode < 0 || mode > 3) return fail(HETA_ERR_INVALID_ARG, "heta_ingest_force: mode must be 0, 1, 2 or 3");
    g_ingest_mode = mode;
    return HETA_OK;
}

heta_status heta_graph_destroy(heta_graph *g)
{
    destroy(g);
    return HETA_OK;
}

heta_status heta_graph_get_csc(const heta_graph *g, int32_t rel, int64_t *colptr, int32_t *row)
{
    if (!g || !colptr || !row)
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_get_csc: null argument");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_get_csc: relation %d out of range", rel);
    const Relation &r = g->rels[rel];
    HETA_HIP(hipMemcpy(colptr, r.csc.d_ptr, (r.n_src + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (r.n_edges)
        HETA_HIP(hipMemcpy(row, r.csc.d_idx, r.n_edges * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (r.shares >= 0) {
        // The shared array is the named relation's CSR, whose rows hold their neighbours in the caller's order;
        // the transposed adjacency in ascending edge order lists each column's rows in non-decreasing order.
        for (int64_t u = 0; u < r.n_src; ++u) std::sort(row + colptr[u], row + colptr[u + 1]);
    }
    return HETA_OK;
}

heta_status heta_graph_index_bytes(const heta_graph *g, int64_t *bytes)
{
    if (!g || !bytes) return fail(HETA_ERR_INVALID_ARG, "heta_graph_index_bytes: null argument");
    auto schedule_bytes = [](const Schedule &s) {
        return (s.n_rows + 1) * 8 * 2 + s.n_edges * 4 * 2 + s.n_rows * 4 + s.n_hub_chunks * static_cast<int64_t>(sizeof(HubChunk)) +
               (s.n_hub_rows + 1) * 8;
    };
    int64_t total = 0;
    for (const Relation &r : g->rels) {
        total += r.n_dst * 4; // 1/deg
        if (r.shares < 0) total += schedule_bytes(r.csr) + schedule_bytes(r.csc);
    }
    *bytes = total;
    return HETA_OK;
}

static heta_status heta_graph_get_degrees_impl(const heta_graph *g, int32_t rel, int64_t *in_deg)
{
    if (!g || !in_deg)
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_get_degrees: null argument");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_graph_get_degrees: relation %d out of range", rel);
    const Relation &r = g->rels[rel];
    // taken from the schedule (row ids by descending degree + schedule-ordered offsets), so that
    // the read-back covers what the aggregation kernels actually walk
    std::vector<int64_t> sptr(r.n_dst + 1);
    std::vector<int32_t> perm(std::max<int64_t>(r.n_dst, 1));
    HETA_HIP(hipMemcpy(sptr.data(), r.csr.d_sptr, (r.n_dst + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (r.n_dst)
        HETA_HIP(hipMemcpy(perm.data(), r.csr.d_perm, r.n_dst * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int64_t v = 0; v < r.n_dst; ++v)
        in_deg[v] = -1;
    for (int64_t q = 0; q < r.n_dst; ++q)
        if (perm[q] >= 0 && perm[q] < r.n_dst)
            in_deg[perm[q]] = sptr[q + 1] - sptr[q];
    return HETA_OK;
}

// No exception crosses the boundary: host containers may throw std::bad_alloc.
heta_status heta_graph_get_degrees(const heta_graph *g, int32_t rel, int64_t *in_deg)
{
    try {
        return heta_graph_get_degrees_impl(g, rel, in_deg);
    } catch (const std::bad_alloc &) {
        return fail(HETA_ERR_OOM, "heta_graph_get_degrees: host allocation failed");
    } catch (...) {
        return fail(HETA_ERR_DEVICE, "heta_graph_get_degrees: unexpected exception");
    }
}

} // extern "C"
