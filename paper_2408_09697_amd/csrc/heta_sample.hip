// k-hop neighbour sampling on the device (Section 2.2 of the paper and the sampling step of
// Algorithm 1: every iteration samples a fixed number of neighbours per relation for the nodes of the
// mini-batch, hop by hop; fan-outs such as {25, 20}, Section 8.1).
//
// Rule per (destination, relation): all in-edges if the in-degree is at most the fan-out, otherwise
// `fanout` distinct edge slots uniformly without replacement, by Floyd's subset algorithm (Bentley &
// Floyd, CACM 1987) driven by a counter-based generator, SplitMix64 (Steele, Lea, Flood, OOPSLA 2014):
// destination v draws from the stream keyed mix(seed ^ mix(v)), its j-th number is mix(key + j), and a
// number is mapped below n by the high half of (its high 32 bits) * n.  The result therefore depends
// on (seed, v) only - not on the launch shape or on which other destinations are sampled.
//
// One wavefront per destination: lane i holds the i-th chosen slot, membership is one ballot, and the
// ascending order of the output is each lane's rank among the chosen slots.  The unique source ids of a
// node type and the local ids of the sampled edges come from one radix sort of all sampled ids.
#include <algorithm>
#include <vector>

#include <new>

#include "heta_internal.h"

namespace heta {

namespace {

constexpr int kMaxFanout = 64;
constexpr unsigned long long kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ inline unsigned long long mix(unsigned long long x)
{
    unsigned long long z = x + kGamma;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ bool id_ok(int64_t v, int64_t n_rows) { return v >= 0 && v < n_rows; }

__device__ __forceinline__ void count_one(const int64_t *ptr, int64_t n_rows, const int64_t *dst_ids, int64_t i, int fanout,
                                          int64_t *cnt, int *bad)
{
    const int64_t v = dst_ids[i];
    if (!id_ok(v, n_rows)) {
        *bad = 1; // every writer stores the same value
        cnt[i] = 0;
        return;
    }
    const int64_t deg = ptr[v + 1] - ptr[v];
    cnt[i] = deg < fanout ? deg : fanout;
}

// one wavefront: the sampled in-edges of destination i, ascending edge slot, at out[rowptr[i] ...]
__device__ __forceinline__ void fill_one(const int64_t *ptr, const int32_t *idx, int64_t n_rows, const int64_t *dst_ids, int64_t i,
                                         int fanout, unsigned long long seed, const int64_t *rowptr, int64_t *out, int lane)
{
    const int64_t v = dst_ids[i];
    if (!id_ok(v, n_rows)) return;
    const int64_t start = ptr[v], deg = ptr[v + 1] - start;
    const int64_t base = rowptr[i];
    if (deg <= fanout) {
        if (lane < deg) out[base + lane] = idx[start + lane];
        return;
    }
    const unsigned long long key = mix(seed ^ mix(static_cast<unsigned long long>(v)));
    int64_t mine = -1; // lane c holds the c-th chosen slot
    for (int step = 0; step < fanout; ++step) {
        const int64_t j = deg - fanout + step;
        const unsigned long long r = mix(key + static_cast<unsigned long long>(step));
        const int64_t t = static_cast<int64_t>(((r >> 32) * static_cast<unsigned long long>(j + 1)) >> 32);
        const bool present = __ballot(mine == t) != 0ull;
        if (lane == step) mine = present ? j : t;
    }
    int rank = 0;
    for (int c = 0; c < fanout; ++c) {
        const int64_t other = __shfl(mine, c, 64);
        rank += other < mine ? 1 : 0;
    }
    if (lane < fanout) out[base + rank] = idx[start + mine];
}

__global__ void __launch_bounds__(256) sample_count_kernel(const int64_t *ptr, int64_t n_rows, const int64_t *dst_ids,
                                                           int64_t n, int fanout, int64_t *cnt, int *bad)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    count_one(ptr, n_rows, dst_ids, i, fanout, cnt, bad);
}

__global__ void __launch_bounds__(256) sample_fill_kernel(const int64_t *ptr, const int32_t *idx, int64_t n_rows,
                                                          const int64_t *dst_ids, int64_t n, int fanout,
                                                          unsigned long long seed, const int64_t *rowptr, int64_t *out)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (i >= n) return; // uniform per wavefront
    fill_one(ptr, idx, n_rows, dst_ids, i, fanout, seed, rowptr, out, lane);
}

// ---- several relations per launch (a hop of a mini-batch): blockIdx.y = item ------------------------------------
constexpr int kFusedItems = 32;
struct FusedSample { // passed by value
    int n, fanout;
    const int64_t *ptr[kFusedItems];
    const int32_t *idx[kFusedItems];
    int64_t n_rows[kFusedItems];
    const int64_t *dst[kFusedItems];
    int64_t n_dst[kFusedItems];
    int64_t off[kFusedItems + 1]; // item r's counts sit at cnt_all[off[r] ...]; off[n] = total
    unsigned long long seed[kFusedItems];
    int64_t *rowptr[kFusedItems];
    int64_t *out[kFusedItems];
};

__global__ void __launch_bounds__(256) sample_count_multi_kernel(FusedSample f, int64_t *cnt_all, int *bad)
{
    const int r = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= f.n_dst[r]) return;
    count_one(f.ptr[r], f.n_rows[r], f.dst[r], i, f.fanout, cnt_all + f.off[r], bad + r);
}

// scan_all = exclusive scan of all items' counts laid end to end; an item's row offsets restart at 0
__global__ void __launch_bounds__(256) sample_rowptr_multi_kernel(FusedSample f, const int64_t *scan_all, int64_t *counts)
{
    const int r = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i > f.n_dst[r]) return;
    const int64_t first = scan_all[f.off[r]];
    f.rowptr[r][i] = scan_all[f.off[r] + i] - first;
    if (i == f.n_dst[r]) counts[r] = scan_all[f.off[r] + i] - first;
}

__global__ void __launch_bounds__(256) sample_fill_multi_kernel(FusedSample f)
{
    const int r = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (i >= f.n_dst[r]) return; // uniform per wavefront
    fill_one(f.ptr[r], f.idx[r], f.n_rows[r], f.dst[r], i, f.fanout, f.seed[r], f.rowptr[r], f.out[r], lane);
}

// ---- unique + relabel ----------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) gather_keys_kernel(const int64_t *ids, int64_t n, int64_t offset, int64_t limit,
                                                          uint32_t *keys, uint32_t *vals, int *bad)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t v = ids[i];
    if (v < 0 || v >= limit) *bad = 1;
    keys[offset + i] = static_cast<uint32_t>(v);
    vals[offset + i] = static_cast<uint32_t>(offset + i);
}

__global__ void __launch_bounds__(256) head_flag_kernel(const uint32_t *keys, int64_t n, int64_t *head)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    head[i] = (i == 0 || keys[i] != keys[i - 1]) ? 1 : 0;
}

// before[i] = number of heads before i; the element's unique index is before[i] + head[i] - 1
__global__ void __launch_bounds__(256) unique_scatter_kernel(const uint32_t *keys, const uint32_t *vals, const int64_t *head,
                                                             const int64_t *before, int64_t n, int64_t *unique_ids,
                                                             int32_t *local_all)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t u = before[i] + head[i] - 1;
    if (head[i]) unique_ids[u] = keys[i];
    local_all[vals[i]] = static_cast<int32_t>(u);
}

// ---- several id sets per launch: the set's index rides in the key's high bits ---------------------------------
constexpr int kFusedLists = 64;
struct FusedLists { // passed by value
    int n_lists, shift; // shift: bits of the id part of a key
    const int64_t *ids[kFusedLists];
    int64_t len[kFusedLists];
    int64_t off[kFusedLists]; // position of the list's first id in the concatenation of all sets
    int64_t limit[kFusedLists];
    uint32_t group[kFusedLists];
};
struct FusedGroups { // passed by value
    int n, shift;
    int64_t base[kFusedItems + 1]; // set g occupies [base[g], base[g+1]) of the sorted array
    int64_t *uniq[kFusedItems];
};

__global__ void __launch_bounds__(256) gather_keys_multi_kernel(FusedLists f, uint32_t *keys, uint32_t *vals, int *bad)
{
    const int l = blockIdx.y;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= f.len[l]) return;
    const int64_t v = f.ids[l][i];
    const bool ok = v >= 0 && v < f.limit[l];
    if (!ok) bad[f.group[l]] = 1;
    // an id out of range must not reach another set's key range (the sets' sizes in the sorted array are relied on)
    keys[f.off[l] + i] = (f.group[l] << f.shift) | (ok ? static_cast<uint32_t>(v) : 0u);
    vals[f.off[l] + i] = static_cast<uint32_t>(f.off[l] + i);
}

__global__ void __launch_bounds__(256) unique_scatter_multi_kernel(FusedGroups f, const uint32_t *keys, const uint32_t *vals,
                                                                   const int64_t *head, const int64_t *before, int64_t n,
                                                                   int32_t *local_all)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t key = keys[i];
    const int g = static_cast<int>(key >> f.shift);
    const int64_t u = before[i] + head[i] - 1 - before[f.base[g]];
    if (head[i]) f.uniq[g][u] = static_cast<int64_t>(key & ((1u << f.shift) - 1u));
    local_all[vals[i]] = static_cast<int32_t>(u);
}

__global__ void __launch_bounds__(64) group_counts_kernel(FusedGroups f, const int64_t *before, int64_t *counts)
{
    const int g = threadIdx.x;
    if (g < f.n) counts[g] = before[f.base[g + 1]] - before[f.base[g]];
}

// scratch of one call, from the recycling pool (released idle: every entry point below synchronises its
// stream before it returns, and the destructor waits for the device in case an error path did not)
struct Scratch {
    char *p = nullptr;
    size_t cursor = 0;
    ~Scratch()
    {
        if (!p) return;
        (void)hipDeviceSynchronize(); // a no-op wait after the entry point's own synchronisation; covers error paths
        scratch_free(p);
    }
    static size_t padded(size_t bytes) { return (std::max<size_t>(bytes, 1) + 255) / 256 * 256; }
    heta_status alloc(size_t bytes)
    {
        hipError_t e = scratch_alloc(reinterpret_cast<void **>(&p), std::max<size_t>(bytes, 256));
        if (e != hipSuccess)
            return fail(e == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE, "allocation of sampler scratch failed: %s",
                        hipGetErrorString(e));
        return HETA_OK;
    }
    template <typename T> T *take(size_t n) // slices were sized with padded() before alloc()
    {
        T *q = reinterpret_cast<T *>(p + cursor);
        cursor += padded(n * sizeof(T));
        return q;
    }
};

// Counts and error flags come back through page-locked slots, so that the copies are asynchronous and a
// whole batch is awaited once (a copy into pageable memory blocks the host until it has landed).
struct Slot {
    int64_t count;
    int32_t bad;
    int32_t pad;
};
struct PinnedSlots {
    Slot *p = nullptr;
    size_t cap = 0;
};
static thread_local PinnedSlots t_slots; // never freed: it lives as long as the thread samples

static heta_status slots_reserve(size_t n)
{
    if (n <= t_slots.cap) return HETA_OK;
    const size_t cap = std::max<size_t>(n, 64);
    void *q = nullptr;
    if (hipHostMalloc(&q, cap * sizeof(Slot), hipHostMallocDefault) != hipSuccess)
        return fail(HETA_ERR_OOM, "page-locked host allocation of %zu result slots failed", cap);
    if (t_slots.p) (void)hipHostFree(t_slots.p);
    t_slots.p = static_cast<Slot *>(q);
    t_slots.cap = cap;
    return HETA_OK;
}

} // namespace

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_sample_neighbors_batch(const heta_graph *g, int32_t n, const int32_t *rels, const int64_t *const *dst_ids,
                                        const int64_t *n_dst, int32_t fanout, const uint64_t *seeds, int64_t *const *rowptr,
                                        int64_t *const *src_ids, int64_t *n_sampled, void *hip_stream)
{
    if (!g || n < 0 || (n > 0 && (!rels || !dst_ids || !n_dst || !seeds || !rowptr || !src_ids || !n_sampled)))
        return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: null argument");
    if (fanout < 1 || fanout > kMaxFanout)
        return fail(HETA_ERR_SHAPE, "heta_sample_neighbors: need 1 <= fanout <= %d", kMaxFanout);
    size_t bytes = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (rels[i] < 0 || rels[i] >= (int32_t)g->rels.size())
            return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: relation %d out of range", rels[i]);
        if (n_dst[i] < 0) return fail(HETA_ERR_SHAPE, "heta_sample_neighbors: need n_dst >= 0");
        if (!rowptr[i] || (n_dst[i] > 0 && (!dst_ids[i] || !src_ids[i])))
            return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: null argument");
        n_sampled[i] = 0;
        if (n_dst[i] == 0) continue;
        bytes += Scratch::padded(static_cast<size_t>(n_dst[i]) * sizeof(int64_t)) +
                 Scratch::padded(static_cast<size_t>(scan_scratch_elems(n_dst[i] + 1)) * sizeof(int64_t));
    }
    if (n == 0) return HETA_OK;
    hipStream_t st = as_stream(hip_stream);
    Scratch scratch;
    heta_status e;
    int64_t all_dst = 0;
    for (int32_t i = 0; i < n; ++i) all_dst += n_dst[i];
    if (n <= kFusedItems && all_dst > 0) {
        // every item in the same launches: counts of all items end to end, one scan, row offsets per item
        FusedSample f{};
        f.n = n;
        f.fanout = fanout;
        int64_t total = 0, n_max = 0;
        for (int32_t i = 0; i < n; ++i) {
            const Relation &r = g->rels[rels[i]];
            f.ptr[i] = r.csr.d_ptr;
            f.idx[i] = r.csr.d_idx;
            f.n_rows[i] = r.n_dst;
            f.dst[i] = dst_ids[i];
            f.n_dst[i] = n_dst[i];
            f.off[i] = total;
            f.seed[i] = seeds[i];
            f.rowptr[i] = rowptr[i];
            f.out[i] = src_ids[i];
            total += n_dst[i];
            n_max = std::max(n_max, n_dst[i]);
        }
        f.off[n] = total;
        if (total >= (int64_t(1) << 31)) return fail(HETA_ERR_UNSUPPORTED, "heta_sample_neighbors: more than 2^31 destinations");
        const size_t T = static_cast<size_t>(total);
        const size_t fused_bytes = Scratch::padded(static_cast<size_t>(n) * sizeof(int)) + Scratch::padded(T * sizeof(int64_t)) +
                                   Scratch::padded((T + 1) * sizeof(int64_t)) +
                                   Scratch::padded(static_cast<size_t>(scan_scratch_elems(total + 1)) * sizeof(int64_t)) +
                                   Scratch::padded(static_cast<size_t>(n) * sizeof(int64_t));
        if ((e = scratch.alloc(fused_bytes)) != HETA_OK || (e = slots_reserve(2 * static_cast<size_t>(n))) != HETA_OK) return e;
        int *bad = scratch.take<int>(static_cast<size_t>(n));
        int64_t *cnt_all = scratch.take<int64_t>(T), *scan_all = scratch.take<int64_t>(T + 1);
        int64_t *tsum = scratch.take<int64_t>(static_cast<size_t>(scan_scratch_elems(total + 1)));
        int64_t *counts = scratch.take<int64_t>(static_cast<size_t>(n));
        HETA_HIP(hipMemsetAsync(bad, 0, static_cast<size_t>(n) * sizeof(int), st));
        hipLaunchKernelGGL(sample_count_multi_kernel, dim3((unsigned)((n_max + 255) / 256), (unsigned)n), dim3(256), 0, st, f,
                           cnt_all, bad);
        HETA_LAUNCH_CHECK("sample_count_multi_kernel");
        if ((e = device_exclusive_scan_i64_async(cnt_all, total, scan_all, total + 1, tsum, st)) != HETA_OK) return e;
        hipLaunchKernelGGL(sample_rowptr_multi_kernel, dim3((unsigned)((n_max + 1 + 255) / 256), (unsigned)n), dim3(256), 0, st, f,
                           scan_all, counts);
        HETA_LAUNCH_CHECK("sample_rowptr_multi_kernel");
        hipLaunchKernelGGL(sample_fill_multi_kernel, dim3((unsigned)((n_max + 3) / 4), (unsigned)n), dim3(256), 0, st, f);
        HETA_LAUNCH_CHECK("sample_fill_multi_kernel");
        // counts in slots [0, n), flags in slots [n, 2n) (their .bad fields), one copy each
        int64_t *h_counts = reinterpret_cast<int64_t *>(t_slots.p);
        int *h_bad = reinterpret_cast<int *>(t_slots.p + n);
        HETA_HIP(hipMemcpyAsync(h_counts, counts, static_cast<size_t>(n) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        HETA_HIP(hipMemcpyAsync(h_bad, bad, static_cast<size_t>(n) * sizeof(int), hipMemcpyDeviceToHost, st));
        HETA_HIP(hipStreamSynchronize(st));
        for (int32_t i = 0; i < n; ++i)
            if (h_bad[i])
                return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: a destination id of relation %d lies outside [0, %lld)",
                            rels[i], (long long)g->rels[rels[i]].n_dst);
        for (int32_t i = 0; i < n; ++i) n_sampled[i] = h_counts[i];
        return HETA_OK;
    }
    bytes += Scratch::padded(static_cast<size_t>(n) * sizeof(int));
    if ((e = scratch.alloc(bytes)) != HETA_OK || (e = slots_reserve(static_cast<size_t>(n))) != HETA_OK) return e;
    int *bad = scratch.take<int>(static_cast<size_t>(n));
    HETA_HIP(hipMemsetAsync(bad, 0, static_cast<size_t>(n) * sizeof(int), st));
    // per relation count -> scan -> fill -> count and flag to the host, all asynchronous; one synchronisation for the batch
    for (int32_t i = 0; i < n; ++i) {
        const Relation &r = g->rels[rels[i]];
        t_slots.p[i].count = 0;
        t_slots.p[i].bad = 0;
        if (n_dst[i] == 0) {
            HETA_HIP(hipMemsetAsync(rowptr[i], 0, sizeof(int64_t), st));
            continue;
        }
        int64_t *cnt = scratch.take<int64_t>(static_cast<size_t>(n_dst[i]));
        int64_t *tsum = scratch.take<int64_t>(static_cast<size_t>(scan_scratch_elems(n_dst[i] + 1)));
        hipLaunchKernelGGL(sample_count_kernel, dim3((unsigned)((n_dst[i] + 255) / 256)), dim3(256), 0, st, r.csr.d_ptr, r.n_dst,
                           dst_ids[i], n_dst[i], (int)fanout, cnt, bad + i);
        HETA_LAUNCH_CHECK("sample_count_kernel");
        if ((e = device_exclusive_scan_i64_async(cnt, n_dst[i], rowptr[i], n_dst[i] + 1, tsum, st)) != HETA_OK) return e;
        hipLaunchKernelGGL(sample_fill_kernel, dim3((unsigned)((n_dst[i] + 3) / 4)), dim3(256), 0, st, r.csr.d_ptr, r.csr.d_idx,
                           r.n_dst, dst_ids[i], n_dst[i], (int)fanout, (unsigned long long)seeds[i], rowptr[i], src_ids[i]);
        HETA_LAUNCH_CHECK("sample_fill_kernel");
        HETA_HIP(hipMemcpyAsync(&t_slots.p[i].bad, bad + i, sizeof(int), hipMemcpyDeviceToHost, st));
        HETA_HIP(hipMemcpyAsync(&t_slots.p[i].count, rowptr[i] + n_dst[i], sizeof(int64_t), hipMemcpyDeviceToHost, st));
    }
    HETA_HIP(hipStreamSynchronize(st));
    for (int32_t i = 0; i < n; ++i)
        if (t_slots.p[i].bad)
            return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: a destination id of relation %d lies outside [0, %lld)",
                        rels[i], (long long)g->rels[rels[i]].n_dst);
    for (int32_t i = 0; i < n; ++i) n_sampled[i] = t_slots.p[i].count;
    return HETA_OK;
}

heta_status heta_sample_neighbors(const heta_graph *g, int32_t rel, const int64_t *dst_ids, int64_t n_dst, int32_t fanout,
                                  uint64_t seed, int64_t *rowptr, int64_t *src_ids, int64_t *n_sampled, void *hip_stream)
{
    if (!n_sampled) return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: null argument");
    return heta_sample_neighbors_batch(g, 1, &rel, &dst_ids, &n_dst, fanout, &seed, &rowptr, &src_ids, n_sampled, hip_stream);
}

static heta_status heta_unique_relabel_batch_impl(int32_t n_groups, const int32_t *group_ptr, const int64_t *const *lists,
                                      const int64_t *lens, const int64_t *id_limit, int64_t *const *unique_ids,
                                      int64_t *n_unique, int32_t *const *local, void *hip_stream)
{
    if (n_groups < 0 || (n_groups > 0 && (!group_ptr || !id_limit || !unique_ids || !n_unique)))
        return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null argument");
    if (n_groups == 0) return HETA_OK;
    if (group_ptr[0] != 0) return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: group_ptr[0] must be 0");
    std::vector<int64_t> totals(n_groups, 0);
    size_t bytes = Scratch::padded(static_cast<size_t>(n_groups) * sizeof(int));
    for (int32_t gidx = 0; gidx < n_groups; ++gidx) {
        if (group_ptr[gidx + 1] < group_ptr[gidx]) return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: group_ptr decreases");
        if (group_ptr[gidx + 1] > group_ptr[gidx] && (!lists || !lens || !local))
            return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null argument");
        if (id_limit[gidx] < 0 || id_limit[gidx] > (int64_t(1) << 31))
            return fail(HETA_ERR_SHAPE, "heta_unique_relabel: id_limit outside [0, 2^31]");
        for (int32_t l = group_ptr[gidx]; l < group_ptr[gidx + 1]; ++l) {
            if (lens[l] < 0 || (lens[l] > 0 && (!lists[l] || !local[l])))
                return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: list %d is null or has a negative length", l);
            totals[gidx] += lens[l];
        }
        n_unique[gidx] = 0;
        const int64_t total = totals[gidx];
        if (total == 0) continue;
        if (total >= (int64_t(1) << 31)) return fail(HETA_ERR_UNSUPPORTED, "heta_unique_relabel: more than 2^31 ids");
        if (!unique_ids[gidx]) return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null unique_ids");
        const size_t N = static_cast<size_t>(total), n_hist = static_cast<size_t>(sort_hist_elems(total));
        bytes += 4 * Scratch::padded(N * sizeof(uint32_t)) + 2 * Scratch::padded(n_hist * sizeof(uint32_t)) +
                 Scratch::padded(static_cast<size_t>(scan_scratch_elems(static_cast<int64_t>(n_hist))) * sizeof(uint32_t)) +
                 Scratch::padded(N * sizeof(int64_t)) + Scratch::padded((N + 1) * sizeof(int64_t)) +
                 Scratch::padded(static_cast<size_t>(scan_scratch_elems(total + 1)) * sizeof(int64_t)) +
                 Scratch::padded(N * sizeof(int32_t));
    }
    if (std::all_of(totals.begin(), totals.end(), [](int64_t t) { return t == 0; })) return HETA_OK; // nothing for the device
    hipStream_t st = as_stream(hip_stream);
    Scratch scratch;
    heta_status e;
    {
        // All sets in one sort when the set index fits above the ids in a 32-bit key: set g's ids then occupy
        // exactly [base[g], base[g+1]) of the sorted array, and one pass of every stage serves all sets.
        int id_bits = 1, set_bits = 0;
        int64_t N = 0;
        for (int32_t gidx = 0; gidx < n_groups; ++gidx) {
            while ((int64_t(1) << id_bits) < id_limit[gidx]) ++id_bits;
            N += totals[gidx];
        }
        while ((1 << set_bits) < n_groups) ++set_bits;
        const int32_t n_lists = group_ptr[n_groups];
        if (n_groups <= kFusedItems && n_lists <= kFusedLists && id_bits + set_bits <= 32 && id_bits <= 31 && N < (int64_t(1) << 31)) {
            FusedLists fl{};
            FusedGroups fg{};
            fl.n_lists = n_lists;
            fl.shift = fg.shift = id_bits;
            fg.n = n_groups;
            int64_t off = 0, len_max = 0;
            int32_t *local_first = nullptr;
            bool contiguous = true; // the lists' local arrays laid end to end in the same order: written in place
            for (int32_t gidx = 0; gidx < n_groups; ++gidx) {
                fg.base[gidx] = off;
                fg.uniq[gidx] = unique_ids[gidx];
                for (int32_t l = group_ptr[gidx]; l < group_ptr[gidx + 1]; ++l) {
                    fl.ids[l] = lists[l];
                    fl.len[l] = lens[l];
                    fl.off[l] = off;
                    fl.limit[l] = id_limit[gidx];
                    fl.group[l] = static_cast<uint32_t>(gidx);
                    if (lens[l] > 0) {
                        if (!local_first) local_first = local[l];
                        contiguous = contiguous && local[l] == local_first + off;
                    }
                    off += lens[l];
                    len_max = std::max(len_max, lens[l]);
                }
            }
            fg.base[n_groups] = off;
            const size_t Ns = static_cast<size_t>(N), n_hist = static_cast<size_t>(sort_hist_elems(N));
            const size_t fused_bytes =
                Scratch::padded(static_cast<size_t>(n_groups) * sizeof(int)) + 4 * Scratch::padded(Ns * sizeof(uint32_t)) +
                2 * Scratch::padded(n_hist * sizeof(uint32_t)) +
                Scratch::padded(static_cast<size_t>(scan_scratch_elems(static_cast<int64_t>(n_hist))) * sizeof(uint32_t)) +
                Scratch::padded(Ns * sizeof(int64_t)) + Scratch::padded((Ns + 1) * sizeof(int64_t)) +
                Scratch::padded(static_cast<size_t>(scan_scratch_elems(N + 1)) * sizeof(int64_t)) + Scratch::padded(Ns * sizeof(int32_t)) +
                Scratch::padded(static_cast<size_t>(n_groups) * sizeof(int64_t));
            if ((e = scratch.alloc(fused_bytes)) != HETA_OK || (e = slots_reserve(2 * static_cast<size_t>(n_groups))) != HETA_OK) return e;
            int *bad = scratch.take<int>(static_cast<size_t>(n_groups));
            uint32_t *k0 = scratch.take<uint32_t>(Ns), *v0 = scratch.take<uint32_t>(Ns), *k1 = scratch.take<uint32_t>(Ns),
                     *v1 = scratch.take<uint32_t>(Ns), *hist = scratch.take<uint32_t>(n_hist), *offs = scratch.take<uint32_t>(n_hist);
            uint32_t *tsum32 = scratch.take<uint32_t>(static_cast<size_t>(scan_scratch_elems(static_cast<int64_t>(n_hist))));
            int64_t *head = scratch.take<int64_t>(Ns), *before = scratch.take<int64_t>(Ns + 1);
            int64_t *tsum64 = scratch.take<int64_t>(static_cast<size_t>(scan_scratch_elems(N + 1)));
            int32_t *local_scratch = scratch.take<int32_t>(Ns);
            int64_t *counts = scratch.take<int64_t>(static_cast<size_t>(n_groups));
            int32_t *local_all = contiguous ? local_first : local_scratch;
            HETA_HIP(hipMemsetAsync(bad, 0, static_cast<size_t>(n_groups) * sizeof(int), st));
            hipLaunchKernelGGL(gather_keys_multi_kernel, dim3((unsigned)((len_max + 255) / 256), (unsigned)n_lists), dim3(256), 0, st, fl,
                               k0, v0, bad);
            HETA_LAUNCH_CHECK("gather_keys_multi_kernel");
            uint32_t *ks = nullptr, *vs = nullptr;
            const int64_t key_limit = static_cast<int64_t>(n_groups) << id_bits;
            if ((e = device_sort_pairs_u32_async(k0, v0, k1, v1, N, key_limit, &ks, &vs, hist, offs, tsum32, st)) != HETA_OK) return e;
            const unsigned blocks = (unsigned)((N + 255) / 256);
            hipLaunchKernelGGL(head_flag_kernel, dim3(blocks), dim3(256), 0, st, ks, N, head);
            HETA_LAUNCH_CHECK("head_flag_kernel");
            if ((e = device_exclusive_scan_i64_async(head, N, before, N + 1, tsum64, st)) != HETA_OK) return e;
            hipLaunchKernelGGL(unique_scatter_multi_kernel, dim3(blocks), dim3(256), 0, st, fg, ks, vs, head, before, N, local_all);
            HETA_LAUNCH_CHECK("unique_scatter_multi_kernel");
            hipLaunchKernelGGL(group_counts_kernel, dim3(1), dim3(64), 0, st, fg, before, counts);
            HETA_LAUNCH_CHECK("group_counts_kernel");
            if (!contiguous)
                for (int32_t l = 0; l < n_lists; ++l)
                    if (lens[l] > 0)
                        HETA_HIP(hipMemcpyAsync(local[l], local_all + fl.off[l], static_cast<size_t>(lens[l]) * sizeof(int32_t),
                                                hipMemcpyDeviceToDevice, st));
            int64_t *h_counts = reinterpret_cast<int64_t *>(t_slots.p);
            int *h_bad = reinterpret_cast<int *>(t_slots.p + n_groups);
            HETA_HIP(hipMemcpyAsync(h_counts, counts, static_cast<size_t>(n_groups) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
            HETA_HIP(hipMemcpyAsync(h_bad, bad, static_cast<size_t>(n_groups) * sizeof(int), hipMemcpyDeviceToHost, st));
            HETA_HIP(hipStreamSynchronize(st));
            for (int32_t gidx = 0; gidx < n_groups; ++gidx)
                if (h_bad[gidx])
                    return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: an id lies outside [0, %lld)", (long long)id_limit[gidx]);
            for (int32_t gidx = 0; gidx < n_groups; ++gidx) n_unique[gidx] = h_counts[gidx];
            return HETA_OK;
        }
    }
    if ((e = scratch.alloc(bytes)) != HETA_OK || (e = slots_reserve(static_cast<size_t>(n_groups))) != HETA_OK) return e;
    int *bad = scratch.take<int>(static_cast<size_t>(n_groups));
    HETA_HIP(hipMemsetAsync(bad, 0, static_cast<size_t>(n_groups) * sizeof(int), st));
    // per group gather -> sort -> head flags -> scan -> scatter -> copies, all asynchronous; one synchronisation for the batch
    for (int32_t gidx = 0; gidx < n_groups; ++gidx) {
        t_slots.p[gidx].count = 0;
        t_slots.p[gidx].bad = 0;
        const int64_t total = totals[gidx];
        if (total == 0) continue;
        const size_t N = static_cast<size_t>(total), n_hist = static_cast<size_t>(sort_hist_elems(total));
        uint32_t *k0 = scratch.take<uint32_t>(N), *v0 = scratch.take<uint32_t>(N), *k1 = scratch.take<uint32_t>(N),
                 *v1 = scratch.take<uint32_t>(N), *hist = scratch.take<uint32_t>(n_hist), *offs = scratch.take<uint32_t>(n_hist);
        uint32_t *tsum32 = scratch.take<uint32_t>(static_cast<size_t>(scan_scratch_elems(static_cast<int64_t>(n_hist))));
        int64_t *head = scratch.take<int64_t>(N), *before = scratch.take<int64_t>(N + 1);
        int64_t *tsum64 = scratch.take<int64_t>(static_cast<size_t>(scan_scratch_elems(total + 1)));
        int32_t *local_all = scratch.take<int32_t>(N);
        int64_t off = 0;
        for (int32_t l = group_ptr[gidx]; l < group_ptr[gidx + 1]; ++l) {
            if (lens[l] == 0) continue;
            hipLaunchKernelGGL(gather_keys_kernel, dim3((unsigned)((lens[l] + 255) / 256)), dim3(256), 0, st, lists[l], lens[l], off,
                               id_limit[gidx], k0, v0, bad + gidx);
            HETA_LAUNCH_CHECK("gather_keys_kernel");
            off += lens[l];
        }
        // an id outside the range is reported after the synchronisation; until then it is only a key like any other
        uint32_t *ks = nullptr, *vs = nullptr;
        if ((e = device_sort_pairs_u32_async(k0, v0, k1, v1, total, id_limit[gidx], &ks, &vs, hist, offs, tsum32, st)) != HETA_OK)
            return e;
        const unsigned blocks = (unsigned)((total + 255) / 256);
        hipLaunchKernelGGL(head_flag_kernel, dim3(blocks), dim3(256), 0, st, ks, total, head);
        HETA_LAUNCH_CHECK("head_flag_kernel");
        if ((e = device_exclusive_scan_i64_async(head, total, before, total + 1, tsum64, st)) != HETA_OK) return e;
        hipLaunchKernelGGL(unique_scatter_kernel, dim3(blocks), dim3(256), 0, st, ks, vs, head, before, total, unique_ids[gidx],
                           local_all);
        HETA_LAUNCH_CHECK("unique_scatter_kernel");
        off = 0;
        for (int32_t l = group_ptr[gidx]; l < group_ptr[gidx + 1]; ++l) {
            if (lens[l] == 0) continue;
            HETA_HIP(hipMemcpyAsync(local[l], local_all + off, static_cast<size_t>(lens[l]) * sizeof(int32_t),
                                    hipMemcpyDeviceToDevice, st));
            off += lens[l];
        }
        HETA_HIP(hipMemcpyAsync(&t_slots.p[gidx].bad, bad + gidx, sizeof(int), hipMemcpyDeviceToHost, st));
        HETA_HIP(hipMemcpyAsync(&t_slots.p[gidx].count, before + total, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    }
    HETA_HIP(hipStreamSynchronize(st));
    for (int32_t gidx = 0; gidx < n_groups; ++gidx)
        if (t_slots.p[gidx].bad)
            return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: an id lies outside [0, %lld)", (long long)id_limit[gidx]);
    for (int32_t gidx = 0; gidx < n_groups; ++gidx) n_unique[gidx] = t_slots.p[gidx].count;
    return HETA_OK;
}

// No exception crosses the boundary: host containers may throw std::bad_alloc.
heta_status heta_unique_relabel_batch(int32_t n_groups, const int32_t *group_ptr, const int64_t *const *lists,
                                      const int64_t *lens, const int64_t *id_limit, int64_t *const *unique_ids,
                                      int64_t *n_unique, int32_t *const *local, void *hip_stream)
{
    try {
        return heta_unique_relabel_batch_impl(n_groups, group_ptr, lists, lens, id_limit, unique_ids, n_unique, local, hip_stream);
    } catch (const std::bad_alloc &) {
        return fail(HETA_ERR_OOM, "heta_unique_relabel_batch: host allocation failed");
    } catch (...) {
        return fail(HETA_ERR_DEVICE, "heta_unique_relabel_batch: unexpected exception");
    }
}

heta_status heta_unique_relabel(int32_t n_lists, const int64_t *const *lists, const int64_t *lens, int64_t id_limit,
                                int64_t *unique_ids, int64_t *n_unique, int32_t *const *local, void *hip_stream)
{
    if (n_lists < 0 || !n_unique) return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null argument");
    const int32_t group_ptr[2] = {0, n_lists};
    return heta_unique_relabel_batch(1, group_ptr, lists, lens, &id_limit, &unique_ids, n_unique, local, hip_stream);
}

} // extern "C"
