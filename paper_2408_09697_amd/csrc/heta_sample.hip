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

__global__ void __launch_bounds__(256) sample_count_kernel(const int64_t *ptr, int64_t n_rows, const int64_t *dst_ids,
                                                           int64_t n, int fanout, int64_t *cnt, int *bad)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t v = dst_ids[i];
    if (!id_ok(v, n_rows)) {
        *bad = 1; // every writer stores the same value
        cnt[i] = 0;
        return;
    }
    const int64_t deg = ptr[v + 1] - ptr[v];
    cnt[i] = deg < fanout ? deg : fanout;
}

__global__ void __launch_bounds__(256) sample_fill_kernel(const int64_t *ptr, const int32_t *idx, int64_t n_rows,
                                                          const int64_t *dst_ids, int64_t n, int fanout,
                                                          unsigned long long seed, const int64_t *rowptr, int64_t *out)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (i >= n) return; // uniform per wavefront
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

// scratch of one call, from the recycling pool (released idle: every entry point below synchronises its
// stream before it returns, and the destructor waits for the device in case an error path did not)
template <typename T> struct DevBuf {
    T *p = nullptr;
    ~DevBuf()
    {
        if (!p) return;
        (void)hipDeviceSynchronize(); // a no-op wait after the entry point's own synchronisation; covers error paths
        scratch_free(p);
    }
    heta_status alloc(size_t n)
    {
        hipError_t e = scratch_alloc(reinterpret_cast<void **>(&p), std::max<size_t>(n, 1) * sizeof(T));
        if (e != hipSuccess)
            return fail(e == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE, "allocation of sampler scratch failed: %s",
                        hipGetErrorString(e));
        return HETA_OK;
    }
};

} // namespace

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_sample_neighbors(const heta_graph *g, int32_t rel, const int64_t *dst_ids, int64_t n_dst, int32_t fanout,
                                  uint64_t seed, int64_t *rowptr, int64_t *src_ids, int64_t *n_sampled, void *hip_stream)
{
    if (!g || !rowptr || !n_sampled || (n_dst > 0 && (!dst_ids || !src_ids)))
        return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: null argument");
    if (rel < 0 || rel >= (int32_t)g->rels.size())
        return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: relation %d out of range", rel);
    if (n_dst < 0 || fanout < 1 || fanout > kMaxFanout)
        return fail(HETA_ERR_SHAPE, "heta_sample_neighbors: need n_dst >= 0 and 1 <= fanout <= %d", kMaxFanout);
    const Relation &r = g->rels[rel];
    hipStream_t st = as_stream(hip_stream);
    *n_sampled = 0;
    if (n_dst == 0) {
        HETA_HIP(hipMemsetAsync(rowptr, 0, sizeof(int64_t), st));
        HETA_HIP(hipStreamSynchronize(st));
        return HETA_OK;
    }
    // count -> scan -> fill -> counts to the host, all asynchronous; one synchronisation at the end
    DevBuf<int64_t> cnt, tsum;
    DevBuf<int> bad;
    heta_status e;
    if ((e = cnt.alloc(static_cast<size_t>(n_dst))) != HETA_OK) return e;
    if ((e = tsum.alloc(static_cast<size_t>(scan_scratch_elems(n_dst + 1)))) != HETA_OK) return e;
    if ((e = bad.alloc(1)) != HETA_OK) return e;
    HETA_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), st));
    hipLaunchKernelGGL(sample_count_kernel, dim3((unsigned)((n_dst + 255) / 256)), dim3(256), 0, st, r.csr.d_ptr, r.n_dst, dst_ids,
                       n_dst, (int)fanout, cnt.p, bad.p);
    HETA_LAUNCH_CHECK("sample_count_kernel");
    if ((e = device_exclusive_scan_i64_async(cnt.p, n_dst, rowptr, n_dst + 1, tsum.p, st)) != HETA_OK) return e;
    hipLaunchKernelGGL(sample_fill_kernel, dim3((unsigned)((n_dst + 3) / 4)), dim3(256), 0, st, r.csr.d_ptr, r.csr.d_idx, r.n_dst,
                       dst_ids, n_dst, (int)fanout, (unsigned long long)seed, rowptr, src_ids);
    HETA_LAUNCH_CHECK("sample_fill_kernel");
    int h_bad = 0;
    HETA_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HETA_HIP(hipMemcpyAsync(n_sampled, rowptr + n_dst, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    HETA_HIP(hipStreamSynchronize(st));
    if (h_bad) {
        *n_sampled = 0;
        return fail(HETA_ERR_INVALID_ARG, "heta_sample_neighbors: a destination id lies outside [0, %lld)", (long long)r.n_dst);
    }
    return HETA_OK;
}

heta_status heta_unique_relabel(int32_t n_lists, const int64_t *const *lists, const int64_t *lens, int64_t id_limit,
                                int64_t *unique_ids, int64_t *n_unique, int32_t *const *local, void *hip_stream)
{
    if (n_lists < 0 || (n_lists > 0 && (!lists || !lens || !local)) || !n_unique)
        return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null argument");
    if (id_limit < 0 || id_limit > (int64_t(1) << 31))
        return fail(HETA_ERR_SHAPE, "heta_unique_relabel: id_limit outside [0, 2^31]");
    int64_t total = 0;
    for (int32_t l = 0; l < n_lists; ++l) {
        if (lens[l] < 0 || (lens[l] > 0 && (!lists[l] || !local[l])))
            return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: list %d is null or has a negative length", l);
        total += lens[l];
    }
    *n_unique = 0;
    if (total == 0) return HETA_OK;
    if (total >= (int64_t(1) << 31)) return fail(HETA_ERR_UNSUPPORTED, "heta_unique_relabel: more than 2^31 ids");
    if (!unique_ids) return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: null unique_ids");
    hipStream_t st = as_stream(hip_stream);
    // gather -> sort -> head flags -> scan -> scatter -> copies, all asynchronous; one synchronisation at the end
    DevBuf<uint32_t> k0, v0, k1, v1, hist, offs, tsum32;
    DevBuf<int64_t> head, before, tsum64;
    DevBuf<int32_t> local_all;
    DevBuf<int> bad;
    heta_status e;
    const size_t N = static_cast<size_t>(total);
    const size_t n_hist = static_cast<size_t>(sort_hist_elems(total));
    if ((e = k0.alloc(N)) != HETA_OK || (e = v0.alloc(N)) != HETA_OK || (e = k1.alloc(N)) != HETA_OK ||
        (e = v1.alloc(N)) != HETA_OK || (e = hist.alloc(n_hist)) != HETA_OK || (e = offs.alloc(n_hist)) != HETA_OK ||
        (e = tsum32.alloc(static_cast<size_t>(scan_scratch_elems(static_cast<int64_t>(n_hist))))) != HETA_OK ||
        (e = head.alloc(N)) != HETA_OK || (e = before.alloc(N + 1)) != HETA_OK ||
        (e = tsum64.alloc(static_cast<size_t>(scan_scratch_elems(total + 1)))) != HETA_OK ||
        (e = local_all.alloc(N)) != HETA_OK || (e = bad.alloc(1)) != HETA_OK)
        return e;
    HETA_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), st));
    int64_t off = 0;
    for (int32_t l = 0; l < n_lists; ++l) {
        if (lens[l] == 0) continue;
        hipLaunchKernelGGL(gather_keys_kernel, dim3((unsigned)((lens[l] + 255) / 256)), dim3(256), 0, st, lists[l], lens[l], off,
                           id_limit, k0.p, v0.p, bad.p);
        HETA_LAUNCH_CHECK("gather_keys_kernel");
        off += lens[l];
    }
    // an id outside the range is reported after the synchronisation; until then it is only a key like any other
    uint32_t *ks = nullptr, *vs = nullptr;
    if ((e = device_sort_pairs_u32_async(k0.p, v0.p, k1.p, v1.p, total, id_limit, &ks, &vs, hist.p, offs.p, tsum32.p, st)) != HETA_OK)
        return e;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(head_flag_kernel, dim3(blocks), dim3(256), 0, st, ks, total, head.p);
    HETA_LAUNCH_CHECK("head_flag_kernel");
    if ((e = device_exclusive_scan_i64_async(head.p, total, before.p, total + 1, tsum64.p, st)) != HETA_OK) return e;
    hipLaunchKernelGGL(unique_scatter_kernel, dim3(blocks), dim3(256), 0, st, ks, vs, head.p, before.p, total, unique_ids,
                       local_all.p);
    HETA_LAUNCH_CHECK("unique_scatter_kernel");
    off = 0;
    for (int32_t l = 0; l < n_lists; ++l) {
        if (lens[l] == 0) continue;
        HETA_HIP(hipMemcpyAsync(local[l], local_all.p + off, static_cast<size_t>(lens[l]) * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        off += lens[l];
    }
    int h_bad = 0;
    HETA_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HETA_HIP(hipMemcpyAsync(n_unique, before.p + total, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    HETA_HIP(hipStreamSynchronize(st));
    if (h_bad) {
        *n_unique = 0;
        return fail(HETA_ERR_INVALID_ARG, "heta_unique_relabel: an id lies outside [0, %lld)", (long long)id_limit);
    }
    return HETA_OK;
}

} // extern "C"
