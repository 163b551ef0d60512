// Graph ingest on the device: everything index-shaped that the aggregation kernels need is
// derived from a relation's CSR (one mono-relation subgraph, Section 2.1 of the paper) by the
// kernels of this file - validation, in-degrees, the stable CSR -> CSC transpose, and per
// direction the degree-sorted row schedule with its schedule-ordered copy of the adjacency.
//
// Building blocks (all deterministic: integer atomics only count, every placement is by rank):
//   - a device-wide exclusive scan (tile scan, scan of the tile totals, add-back);
//   - a stable least-significant-digit radix sort of (key, value) pairs, 8 bits per pass:
//     per-tile digit histogram, scan over (digit, tile), then a scatter in which a key's rank
//     among equal digits is found with wavefront ballots (lanes holding the same digit) and
//     per-wavefront counters in LDS - no comparison of values, no dependence on timing;
//   - the transpose is that sort applied to (source id, destination row) pairs taken in CSR
//     order: stability keeps a column's entries in ascending original edge position;
//   - the schedule is the same sort applied to (512 - min(degree, 512), row).
#include <algorithm>
#include <vector>

#include "heta_internal.h"

namespace heta {

namespace {

constexpr int kScanItems = 8;                 // per thread
constexpr int kScanTile = 256 * kScanItems;   // per workgroup
constexpr int kSortRounds = 16;               // keys per thread
constexpr int kSortTile = 256 * kSortRounds;  // keys per workgroup

// Releases its device blocks when it goes out of scope (scratch of one ingest).  The blocks come from the
// recycling pool, which needs them idle on release: the destructor waits for the device first.
struct Scratch {
    std::vector<void *> blocks;
    ~Scratch()
    {
        if (blocks.empty()) return;
        (void)hipDeviceSynchronize();
        for (void *b : blocks) scratch_free(b);
    }
    template <typename T> heta_status get(T **out, size_t n)
    {
        void *p = nullptr;
        hipError_t e = scratch_alloc(&p, std::max<size_t>(n, 1) * sizeof(T));
        if (e != hipSuccess)
            return fail(e == hipErrorOutOfMemory ? HETA_ERR_OOM : HETA_ERR_DEVICE, "allocation of ingest scratch failed: %s",
                        hipGetErrorString(e));
        blocks.push_back(p);
        *out = static_cast<T *>(p);
        return HETA_OK;
    }
};

// ---- exclusive scan: out[i] = in[0] + ... + in[i-1] for i in [0, n_out), in[j] = 0 for j >= n_in ------
template <typename TI, typename TO>
__device__ __forceinline__ void scan_tile_body(const TI *in, int64_t n_in, TO *out, int64_t n_out, TO *tile_sums)
{
    __shared__ TO wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanTile + static_cast<int64_t>(tid) * kScanItems;
    TO v[kScanItems];
    TO sum = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = (base + i < n_in) ? static_cast<TO>(in[base + i]) : TO(0);
        sum += v[i];
    }
    TO incl = sum; // inclusive scan of the per-thread sums inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const TO up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    TO before = incl - sum;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < n_out) out[base + i] = before;
        before += v[i];
    }
    if (tid == 255) tile_sums[blockIdx.x] = before;
}
template <typename TI, typename TO>
__global__ void __launch_bounds__(256) scan_tile_kernel(const TI *in, int64_t n_in, TO *out, int64_t n_out, TO *tile_sums)
{
    scan_tile_body<TI, TO>(in, n_in, out, n_out, tile_sums);
}
// two scans of equal length in one launch set: blockIdx.y picks the array (tile sums of the second after the first's)
template <typename T> struct ScanPair {
    const T *in[2];
    T *out[2];
};
template <typename T>
__global__ void __launch_bounds__(256) scan_tile_pair_kernel(ScanPair<T> a, int64_t n_in, int64_t n_out, T *tile_sums, int64_t tiles)
{
    scan_tile_body<T, T>(a.in[blockIdx.y], n_in, a.out[blockIdx.y], n_out, tile_sums + blockIdx.y * tiles);
}

template <typename TO> __device__ __forceinline__ void scan_sums_body(TO *sums, int64_t n)
{
    __shared__ TO wave_tot[4];
    __shared__ TO carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 256) {
        const TO x = (base + tid < n) ? sums[base + tid] : TO(0);
        TO incl = x;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const TO up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        TO before = carry_s + incl - x;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (base + tid < n) sums[base + tid] = before;
        __syncthreads();
        if (tid == 255) carry_s = before + x;
        __syncthreads();
    }
}

template <typename TO> __global__ void __launch_bounds__(256) scan_sums_kernel(TO *sums, int64_t n) { scan_sums_body<TO>(sums, n); }
template <typename T> __global__ void __launch_bounds__(256) scan_sums_pair_kernel(T *sums, int64_t n) { scan_sums_body<T>(sums + blockIdx.x * n, n); }

template <typename TO> __global__ void __launch_bounds__(256) scan_add_kernel(TO *out, int64_t n, const TO *tile_sums)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) out[i] += tile_sums[i / kScanTile];
}
template <typename T> __global__ void __launch_bounds__(256) scan_add_pair_kernel(ScanPair<T> a, int64_t n, const T *tile_sums, int64_t tiles)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) a.out[blockIdx.y][i] += tile_sums[blockIdx.y * tiles + i / kScanTile];
}

// The whole scan by one workgroup of 1024 threads, 8192 elements per round with a running carry: for the
// short arrays of a sampled block (digit histograms of a sort pass, a few thousand rows) one launch instead
// of three dependent ones.
constexpr int kScanSingleMax = 4 * 8192;
template <typename TI, typename TO>
__device__ __forceinline__ void scan_single_body(const TI *in, int64_t n_in, TO *out, int64_t n_out)
{
    __shared__ TO wave_tot[16];
    __shared__ TO carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int64_t round0 = 0; round0 < n_out; round0 += 1024 * kScanItems) {
        const int64_t base = round0 + static_cast<int64_t>(tid) * kScanItems;
        TO v[kScanItems];
        TO sum = 0;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            v[i] = (base + i < n_in) ? static_cast<TO>(in[base + i]) : TO(0);
            sum += v[i];
        }
        TO incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const TO up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        TO before = carry_s + incl - sum;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            if (base + i < n_out) out[base + i] = before;
            before += v[i];
        }
        __syncthreads();
        if (tid == 1023) carry_s = before;
        __syncthreads();
    }
}

template <typename TI, typename TO>
__global__ void __launch_bounds__(1024) scan_single_kernel(const TI *in, int64_t n_in, TO *out, int64_t n_out)
{
    scan_single_body<TI, TO>(in, n_in, out, n_out);
}
template <typename T> __global__ void __launch_bounds__(1024) scan_single_pair_kernel(ScanPair<T> a, int64_t n_in, int64_t n_out)
{
    scan_single_body<T, T>(a.in[blockIdx.x], n_in, a.out[blockIdx.x], n_out);
}

// tile_sums: scratch of (n_out + kScanTile - 1) / kScanTile elements; asynchronous on st
template <typename TI, typename TO>
heta_status exclusive_scan_with(const TI *in, int64_t n_in, TO *out, int64_t n_out, TO *tile_sums, hipStream_t st)
{
    if (n_out <= 0) return HETA_OK;
    const int64_t tiles = (n_out + kScanTile - 1) / kScanTile;
    if (tiles > 1 && n_out <= kScanSingleMax) {
        hipLaunchKernelGGL((scan_single_kernel<TI, TO>), dim3(1), dim3(1024), 0, st, in, n_in, out, n_out);
        HETA_LAUNCH_CHECK("scan_single_kernel");
        return HETA_OK;
    }
    hipLaunchKernelGGL((scan_tile_kernel<TI, TO>), dim3((unsigned)tiles), dim3(256), 0, st, in, n_in, out, n_out, tile_sums);
    HETA_LAUNCH_CHECK("scan_tile_kernel");
    if (tiles > 1) {
        hipLaunchKernelGGL((scan_sums_kernel<TO>), dim3(1), dim3(256), 0, st, tile_sums, tiles);
        HETA_LAUNCH_CHECK("scan_sums_kernel");
        hipLaunchKernelGGL((scan_add_kernel<TO>), dim3((unsigned)((n_out + 255) / 256)), dim3(256), 0, st, out, n_out, tile_sums);
        HETA_LAUNCH_CHECK("scan_add_kernel");
    }
    return HETA_OK;
}

template <typename TI, typename TO>
heta_status exclusive_scan(const TI *in, int64_t n_in, TO *out, int64_t n_out, Scratch &scr, hipStream_t st)
{
    if (n_out <= 0) return HETA_OK;
    TO *tile_sums = nullptr;
    heta_status e = scr.get(&tile_sums, static_cast<size_t>((n_out + kScanTile - 1) / kScanTile));
    if (e != HETA_OK) return e;
    return exclusive_scan_with<TI, TO>(in, n_in, out, n_out, tile_sums, st);
}

// ---- stable LSD radix sort of (key, value) pairs ------------------------------------------------------
// RB = bits per pass (8 or 9); hist[digit * n_tiles + tile] = number of keys of the tile with that digit
template <int RB>
__global__ void __launch_bounds__(256) sort_hist_kernel(const uint32_t *keys, int64_t n, int shift, uint32_t *hist, int64_t n_tiles)
{
    constexpr int BINS = 1 << RB;
    __shared__ uint32_t cnt[BINS];
#pragma unroll
    for (int b = threadIdx.x; b < BINS; b += 256) cnt[b] = 0;
    __syncthreads();
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kSortTile;
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = base + r * 256 + threadIdx.x;
        if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & (BINS - 1)], 1u); // LDS integer counter: order-independent
    }
    __syncthreads();
#pragma unroll
    for (int b = threadIdx.x; b < BINS; b += 256) hist[static_cast<int64_t>(b) * n_tiles + blockIdx.x] = cnt[b];
}

// offs = exclusive scan of hist over (digit, tile); every key goes to offs[digit][tile] + its rank
// among the tile's keys of the same digit, ranks taken in index order (stable).
template <int RB>
__global__ void __launch_bounds__(256) sort_scatter_kernel(const uint32_t *keys, const uint32_t *vals, int64_t n, int shift,
                                                            const uint32_t *offs, int64_t n_tiles, uint32_t *keys_out,
                                                            uint32_t *vals_out)
{
    // A step places kSortStep x 256 consecutive keys: sub-round q holds the keys base + (step * kSortStep + q) * 256 + tid,
    // so index order is (q, wavefront, lane).  Three barriers per step instead of per 256 keys.
    constexpr int kSortStep = 4, BINS = 1 << RB;
    static_assert(kSortRounds % kSortStep == 0, "a tile is a whole number of steps");
    __shared__ uint32_t bin_base[BINS];               // next free output slot of each digit for this tile
    __shared__ uint32_t wave_cnt[kSortStep][4][BINS]; // keys of each digit per (sub-round, wavefront) in the current step
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int b = tid; b < BINS; b += 256) {
        bin_base[b] = offs[static_cast<int64_t>(b) * n_tiles + blockIdx.x];
#pragma unroll
        for (int q = 0; q < kSortStep; ++q)
#pragma unroll
            for (int w = 0; w < 4; ++w) wave_cnt[q][w][b] = 0;
    }
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kSortTile;
    // every round's key and value are loaded before the first step: one memory latency per tile instead of one
    // per step (the steps are chained through barriers, so a load inside a step is never in flight with the next)
    uint32_t key_r[kSortRounds], val_r[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = base + r * 256 + tid;
        key_r[r] = i < n ? keys[i] : 0u;
        val_r[r] = i < n ? vals[i] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int r0 = 0; r0 < kSortRounds; r0 += kSortStep) {
        uint32_t rank[kSortStep];
#pragma unroll
        for (int q = 0; q < kSortStep; ++q) {
            const bool valid = base + (r0 + q) * 256 + tid < n;
            const uint32_t d = (key_r[r0 + q] >> shift) & (BINS - 1);
            // lanes of this wavefront holding the same digit in this sub-round
            uint64_t peers = __ballot(valid);
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                const bool bit = (d >> b) & 1u;
                const uint64_t bal = __ballot(bit);
                peers &= bit ? bal : ~bal;
            }
            rank[q] = __popcll(peers & ((uint64_t(1) << lane) - 1));
            if (valid && rank[q] == 0) wave_cnt[q][wave][d] = __popcll(peers);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kSortStep; ++q) {
            if (base + (r0 + q) * 256 + tid < n) {
                const uint32_t key = key_r[r0 + q], d = (key >> shift) & (BINS - 1);
                uint32_t pos = bin_base[d] + rank[q];
#pragma unroll
                for (int qq = 0; qq < q; ++qq)
#pragma unroll
                    for (int w = 0; w < 4; ++w) pos += wave_cnt[qq][w][d];
                for (int w = 0; w < wave; ++w) pos += wave_cnt[q][w][d];
                keys_out[pos] = key;
                vals_out[pos] = val_r[r0 + q];
            }
        }
        __syncthreads();
#pragma unroll
        for (int b = tid; b < BINS; b += 256) {
            uint32_t add = 0;
#pragma unroll
            for (int q = 0; q < kSortStep; ++q)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    add += wave_cnt[q][w][b];
                    wave_cnt[q][w][b] = 0;
                }
            bin_base[b] += add;
        }
        __syncthreads();
    }
}

// Sorts n pairs by the low `bits` bits of the key.  (keys, vals) and (keys_tmp, vals_tmp) are
// ping-pong buffers; *keys_res / *vals_res point at whichever holds the result.
// hist, offs: scratch of 512 * n_tiles elements each (n_tiles = (n + kSortTile - 1) / kSortTile); tile_sums: scratch
// for a scan over 512 * n_tiles elements; asynchronous on st
heta_status radix_sort_pairs_with(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n, int bits,
                                  uint32_t **keys_res, uint32_t **vals_res, uint32_t *hist, uint32_t *offs, uint32_t *tile_sums,
                                  hipStream_t st)
{
    *keys_res = keys;
    *vals_res = vals;
    if (n <= 1 || bits <= 0) return HETA_OK;
    const int64_t n_tiles = (n + kSortTile - 1) / kSortTile;
    heta_status e;
    uint32_t *ki = keys, *vi = vals, *ko = keys_tmp, *vo = vals_tmp;
    // 9 bits per pass where that saves a pass (17-18 or 25-27 key bits): a pass is three dependent launches
    const int rb = (bits + 8) / 9 < (bits + 7) / 8 ? 9 : 8;
    const int64_t bins = int64_t(1) << rb;
    for (int shift = 0; shift < bits; shift += rb) {
        if (rb == 9) hipLaunchKernelGGL(sort_hist_kernel<9>, dim3((unsigned)n_tiles), dim3(256), 0, st, ki, n, shift, hist, n_tiles);
        else hipLaunchKernelGGL(sort_hist_kernel<8>, dim3((unsigned)n_tiles), dim3(256), 0, st, ki, n, shift, hist, n_tiles);
        HETA_LAUNCH_CHECK("sort_hist_kernel");
        if ((e = exclusive_scan_with<uint32_t, uint32_t>(hist, bins * n_tiles, offs, bins * n_tiles, tile_sums, st)) != HETA_OK) return e;
        if (rb == 9) hipLaunchKernelGGL(sort_scatter_kernel<9>, dim3((unsigned)n_tiles), dim3(256), 0, st, ki, vi, n, shift, offs, n_tiles, ko, vo);
        else hipLaunchKernelGGL(sort_scatter_kernel<8>, dim3((unsigned)n_tiles), dim3(256), 0, st, ki, vi, n, shift, offs, n_tiles, ko, vo);
        HETA_LAUNCH_CHECK("sort_scatter_kernel");
        std::swap(ki, ko);
        std::swap(vi, vo);
    }
    *keys_res = ki;
    *vals_res = vi;
    return HETA_OK;
}

heta_status radix_sort_pairs(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n, int bits,
                             uint32_t **keys_res, uint32_t **vals_res, Scratch &scr, hipStream_t st)
{
    *keys_res = keys;
    *vals_res = vals;
    if (n <= 1 || bits <= 0) return HETA_OK;
    const int64_t n_tiles = (n + kSortTile - 1) / kSortTile;
    uint32_t *hist = nullptr, *offs = nullptr, *tile_sums = nullptr;
    heta_status e;
    if ((e = scr.get(&hist, static_cast<size_t>(512 * n_tiles))) != HETA_OK) return e;
    if ((e = scr.get(&offs, static_cast<size_t>(512 * n_tiles))) != HETA_OK) return e;
    if ((e = scr.get(&tile_sums, static_cast<size_t>((512 * n_tiles + kScanTile - 1) / kScanTile))) != HETA_OK) return e;
    return radix_sort_pairs_with(keys, vals, keys_tmp, vals_tmp, n, bits, keys_res, vals_res, hist, offs, tile_sums, st);
}

// ---- validation of a device CSR ---------------------------------------------------------------------------
// err[0] = smallest (kind << 56 | index) over all violations, kinds in the order the host validator reports them
enum : unsigned long long { kErrPtr0 = 1, kErrDecrease = 2, kErrTotal = 3, kErrCol = 4, kErrNone = ~0ull };

__global__ void __launch_bounds__(256) validate_ptr_kernel(const int64_t *ptr, int64_t n_rows, int64_t n_edges,
                                                           unsigned long long *err)
{
    const int64_t v = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (v == 0 && ptr[0] != 0) atomicMin(err, (kErrPtr0 << 56));
    if (v < n_rows && ptr[v + 1] < ptr[v]) atomicMin(err, (kErrDecrease << 56) | static_cast<unsigned long long>(v));
    if (v == n_rows && ptr[n_rows] != n_edges) atomicMin(err, (kErrTotal << 56));
}

__global__ void __launch_bounds__(256) validate_col_kernel(const int32_t *col, int64_t n_edges, int64_t n_src,
                                                           unsigned long long *err)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e < n_edges && (col[e] < 0 || col[e] >= n_src)) atomicMin(err, (kErrCol << 56) | static_cast<unsigned long long>(e));
}

// ---- degrees, sort keys, degree histogram -------------------------------------------------------------------
// key[r] = kHubMinDeg - min(deg, kHubMinDeg) (ascending key = descending capped degree), val[r] = r;
// hist[k] / hist[kDegHist + k] = rows / edges in rows whose capped degree is k; inv_deg optional.
__global__ void __launch_bounds__(256) degree_key_kernel(const int64_t *ptr, int64_t n_rows, uint32_t *key, uint32_t *val,
                                                         unsigned long long *hist, float *inv_deg)
{
    __shared__ unsigned int rows_s[kDegHist];
    __shared__ unsigned long long edges_s[kDegHist];
    for (int k = threadIdx.x; k < kDegHist; k += 256) {
        rows_s[k] = 0;
        edges_s[k] = 0;
    }
    __syncthreads();
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (r < n_rows) {
        const int64_t deg = ptr[r + 1] - ptr[r];
        const int capped = static_cast<int>(min(deg, static_cast<int64_t>(kHubMinDeg)));
        key[r] = static_cast<uint32_t>(kHubMinDeg - capped);
        val[r] = static_cast<uint32_t>(r);
        if (inv_deg) inv_deg[r] = deg > 0 ? 1.0f / static_cast<float>(deg) : 0.0f;
        atomicAdd(&rows_s[capped], 1u);
        atomicAdd(&edges_s[capped], static_cast<unsigned long long>(deg));
    }
    __syncthreads();
    for (int k = threadIdx.x; k < kDegHist; k += 256) {
        if (rows_s[k]) {
            atomicAdd(&hist[k], static_cast<unsigned long long>(rows_s[k]));
            atomicAdd(&hist[kDegHist + k], edges_s[k]);
        }
    }
}

// sdeg[q] = degree of the row at schedule position q
__global__ void __launch_bounds__(256) sched_degree_kernel(const int64_t *ptr, const int32_t *perm, int64_t n_rows, int64_t *sdeg)
{
    const int64_t q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (q < n_rows) {
        const int64_t r = perm[q];
        sdeg[q] = ptr[r + 1] - ptr[r];
    }
}

// largest i in [0, n) with a[i] <= x, for non-decreasing a with a[0] <= x
__device__ __forceinline__ int64_t last_le(const int64_t *a, int64_t n, int64_t x)
{
    int64_t lo = 0, hi = n; // answer in [lo, hi)
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (a[mid] <= x) lo = mid;
        else hi = mid;
    }
    return lo;
}

// sidx[e'] = idx[ptr[perm[q]] + (e' - sptr[q])] for the schedule position q that owns e'
__global__ void __launch_bounds__(256) sched_fill_kernel(const int64_t *ptr, const int32_t *idx, const int32_t *perm,
                                                         const int64_t *sptr, int64_t n_rows, int64_t n_edges, int32_t *sidx)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= n_edges) return;
    const int64_t q = last_le(sptr, n_rows, e); // sptr[q] <= e < sptr[q + 1] (empty rows share offsets: the last one wins, and it is the owner)
    sidx[e] = idx[ptr[perm[q]] + (e - sptr[q])];
}

// value of edge e in CSR order = its destination row
__global__ void __launch_bounds__(256) edge_row_kernel(const int64_t *ptr, int64_t n_rows, int64_t n_edges, const int32_t *col,
                                                       uint32_t *key, uint32_t *val)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= n_edges) return;
    key[e] = static_cast<uint32_t>(col[e]);
    val[e] = static_cast<uint32_t>(last_le(ptr, n_rows, e));
}

// colptr[u] = number of sorted keys below u, u in [0, n_src]
__global__ void __launch_bounds__(256) colptr_kernel(const uint32_t *sorted_keys, int64_t n_edges, int64_t n_src, int64_t *colptr)
{
    const int64_t u = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (u > n_src) return;
    int64_t lo = 0, hi = n_edges; // first position whose key is >= u
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (sorted_keys[mid] < static_cast<uint32_t>(u)) lo = mid + 1;
        else hi = mid;
    }
    colptr[u] = lo;
}

// hub rows are the first n_hub schedule positions: their chunk counts, then the chunk descriptors
__global__ void __launch_bounds__(256) hub_count_kernel(const int64_t *sptr, int64_t n_hub, int64_t *n_chunks)
{
    const int64_t h = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (h < n_hub) n_chunks[h] = (sptr[h + 1] - sptr[h] + kHubChunk - 1) / kHubChunk;
}

__global__ void __launch_bounds__(256) hub_fill_kernel(const int64_t *sptr, const int64_t *chunk_ptr, HubChunk *chunks)
{
    const int64_t h = blockIdx.x;
    const int64_t e0 = sptr[h], e1 = sptr[h + 1], c0 = chunk_ptr[h], nc = chunk_ptr[h + 1] - c0;
    for (int64_t c = threadIdx.x; c < nc; c += 256) {
        HubChunk d;
        d.e0 = e0 + c * kHubChunk;
        d.len = static_cast<int32_t>(min(static_cast<int64_t>(kHubChunk), e1 - d.e0));
        d.slot = static_cast<int32_t>(c0 + c);
        chunks[c0 + c] = d;
    }
}

template <typename T> heta_status dev_alloc(T **p, size_t n)
{
    *p = nullptr;
    HETA_HIP(hipMalloc(reinterpret_cast<void **>(p), std::max<size_t>(n, 1) * sizeof(T)));
    return HETA_OK;
}

int bits_for(int64_t n) // bits needed for values in [0, n)
{
    int b = 1;
    while ((int64_t(1) << b) < n) ++b;
    return b;
}

} // namespace

// Fills s from its device pointer array and neighbour array (s.d_ptr, s.d_idx already set, owned by s).
heta_status build_schedule_on_device(Schedule &s, float *inv_deg, hipStream_t st)
{
    const int64_t n = s.n_rows, E = s.n_edges;
    Scratch scr;
    heta_status e;
    uint32_t *key = nullptr, *val = nullptr, *key2 = nullptr, *val2 = nullptr;
    unsigned long long *hist = nullptr;
    int64_t *sdeg = nullptr;
    if ((e = scr.get(&key, n)) != HETA_OK || (e = scr.get(&val, n)) != HETA_OK || (e = scr.get(&key2, n)) != HETA_OK ||
        (e = scr.get(&val2, n)) != HETA_OK || (e = scr.get(&hist, 2 * kDegHist)) != HETA_OK || (e = scr.get(&sdeg, n)) != HETA_OK)
        return e;
    HETA_HIP(hipMemsetAsync(hist, 0, 2 * kDegHist * sizeof(unsigned long long), st));
    if ((e = dev_alloc(&s.d_perm, n)) != HETA_OK || (e = dev_alloc(&s.d_sptr, n + 1)) != HETA_OK ||
        (e = dev_alloc(&s.d_sidx, E)) != HETA_OK)
        return e;
    const unsigned row_blocks = static_cast<unsigned>((n + 255) / 256);
    uint32_t *ks = key, *vs = val;
    if (n > 0) {
        hipLaunchKernelGGL(degree_key_kernel, dim3(row_blocks), dim3(256), 0, st, s.d_ptr, n, key, val, hist, inv_deg);
        HETA_LAUNCH_CHECK("degree_key_kernel");
        if ((e = radix_sort_pairs(key, val, key2, val2, n, bits_for(kHubMinDeg + 1), &ks, &vs, scr, st)) != HETA_OK) return e;
        HETA_HIP(hipMemcpyAsync(s.d_perm, vs, n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        hipLaunchKernelGGL(sched_degree_kernel, dim3(row_blocks), dim3(256), 0, st, s.d_ptr, s.d_perm, n, sdeg);
        HETA_LAUNCH_CHECK("sched_degree_kernel");
    }
    if ((e = exclusive_scan<int64_t, int64_t>(sdeg, n, s.d_sptr, n + 1, scr, st)) != HETA_OK) return e;
    if (E > 0) {
        hipLaunchKernelGGL(sched_fill_kernel, dim3((unsigned)((E + 255) / 256)), dim3(256), 0, st, s.d_ptr, s.d_idx, s.d_perm,
                           s.d_sptr, n, E, s.d_sidx);
        HETA_LAUNCH_CHECK("sched_fill_kernel");
    }
    // the degree histogram decides every launch shape later: bring it to the host
    std::vector<unsigned long long> h(2 * kDegHist);
    HETA_HIP(hipMemcpyAsync(h.data(), hist, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    HETA_HIP(hipStreamSynchronize(st));
    int64_t rows = 0, edges = 0;
    for (int k = kHubMinDeg; k >= 0; --k) {
        rows += static_cast<int64_t>(h[k]);
        edges += static_cast<int64_t>(h[kDegHist + k]);
        s.rows_with_deg_ge[k] = rows;
        s.edges_with_deg_ge[k] = edges;
    }
    s.n_hub_rows = s.rows_with_deg_ge[kHubMinDeg];
    s.n_hub_chunks = 0;
    if ((e = dev_alloc(&s.d_hub_chunk_ptr, s.n_hub_rows + 1)) != HETA_OK) return e;
    if (s.n_hub_rows > 0) {
        int64_t *cnt = nullptr;
        if ((e = scr.get(&cnt, s.n_hub_rows)) != HETA_OK) return e;
        hipLaunchKernelGGL(hub_count_kernel, dim3((unsigned)((s.n_hub_rows + 255) / 256)), dim3(256), 0, st, s.d_sptr, s.n_hub_rows, cnt);
        HETA_LAUNCH_CHECK("hub_count_kernel");
        if ((e = exclusive_scan<int64_t, int64_t>(cnt, s.n_hub_rows, s.d_hub_chunk_ptr, s.n_hub_rows + 1, scr, st)) != HETA_OK) return e;
        HETA_HIP(hipMemcpyAsync(&s.n_hub_chunks, s.d_hub_chunk_ptr + s.n_hub_rows, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        HETA_HIP(hipStreamSynchronize(st));
        if (s.n_hub_chunks >= (int64_t(1) << 31)) return fail(HETA_ERR_UNSUPPORTED, "too many hub chunks (%lld)", (long long)s.n_hub_chunks);
    } else {
        HETA_HIP(hipMemsetAsync(s.d_hub_chunk_ptr, 0, sizeof(int64_t), st));
    }
    if ((e = dev_alloc(&s.d_hub_chunks, s.n_hub_chunks)) != HETA_OK) return e;
    if (s.n_hub_rows > 0) {
        hipLaunchKernelGGL(hub_fill_kernel, dim3((unsigned)s.n_hub_rows), dim3(256), 0, st, s.d_sptr, s.d_hub_chunk_ptr, s.d_hub_chunks);
        HETA_LAUNCH_CHECK("hub_fill_kernel");
    }
    HETA_HIP(hipStreamSynchronize(st)); // scratch is released on return
    return HETA_OK;
}

// Checks a CSR that already lies on the device; the messages match the host validator's.
heta_status validate_csr_on_device(int32_t index, const int64_t *d_ptr, const int32_t *d_col, int64_t n_dst, int64_t n_src,
                                   int64_t E, hipStream_t st)
{
    Scratch scr;
    unsigned long long *err = nullptr;
    heta_status e = scr.get(&err, 1);
    if (e != HETA_OK) return e;
    HETA_HIP(hipMemsetAsync(err, 0xff, sizeof(unsigned long long), st));
    hipLaunchKernelGGL(validate_ptr_kernel, dim3((unsigned)((n_dst + 1 + 255) / 256)), dim3(256), 0, st, d_ptr, n_dst, E, err);
    HETA_LAUNCH_CHECK("validate_ptr_kernel");
    unsigned long long h = kErrNone;
    HETA_HIP(hipMemcpyAsync(&h, err, sizeof h, hipMemcpyDeviceToHost, st));
    HETA_HIP(hipStreamSynchronize(st));
    if (h == kErrNone && E > 0) { // the column check relies on E = rowptr[n_dst], just confirmed
        hipLaunchKernelGGL(validate_col_kernel, dim3((unsigned)((E + 255) / 256)), dim3(256), 0, st, d_col, E, n_src, err);
        HETA_LAUNCH_CHECK("validate_col_kernel");
        HETA_HIP(hipMemcpyAsync(&h, err, sizeof h, hipMemcpyDeviceToHost, st));
        HETA_HIP(hipStreamSynchronize(st));
    }
    if (h == kErrNone) return HETA_OK;
    const unsigned long long kind = h >> 56, at = h & ((1ull << 56) - 1);
    if (kind == kErrPtr0) return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr[0] is not 0", index);
    if (kind == kErrDecrease) return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr decreases at row %llu", index, at);
    if (kind == kErrTotal) return fail(HETA_ERR_BAD_CSR, "relation %d: rowptr[n_dst] differs from num_edges = %lld", index, (long long)E);
    return fail(HETA_ERR_BAD_CSR, "relation %d: col[%llu] outside [0, %lld)", index, at, (long long)n_src);
}

// Builds the transposed adjacency of a device CSR: csc.d_ptr [n_src + 1], csc.d_idx [E] (allocated here).
heta_status transpose_on_device(const Schedule &csr, int64_t n_src, Schedule &csc, hipStream_t st)
{
    const int64_t E = csr.n_edges, n_dst = csr.n_rows;
    csc.n_rows = n_src;
    csc.n_edges = E;
    heta_status e;
    if ((e = dev_alloc(&csc.d_ptr, n_src + 1)) != HETA_OK || (e = dev_alloc(&csc.d_idx, E)) != HETA_OK) return e;
    if (E == 0) {
        HETA_HIP(hipMemsetAsync(csc.d_ptr, 0, (n_src + 1) * sizeof(int64_t), st));
        return HETA_OK;
    }
    Scratch scr;
    uint32_t *key = nullptr, *val = nullptr, *key2 = nullptr, *val2 = nullptr, *ks = nullptr, *vs = nullptr;
    if ((e = scr.get(&key, E)) != HETA_OK || (e = scr.get(&val, E)) != HETA_OK || (e = scr.get(&key2, E)) != HETA_OK ||
        (e = scr.get(&val2, E)) != HETA_OK)
        return e;
    hipLaunchKernelGGL(edge_row_kernel, dim3((unsigned)((E + 255) / 256)), dim3(256), 0, st, csr.d_ptr, n_dst, E, csr.d_idx, key, val);
    HETA_LAUNCH_CHECK("edge_row_kernel");
    if ((e = radix_sort_pairs(key, val, key2, val2, E, bits_for(n_src), &ks, &vs, scr, st)) != HETA_OK) return e;
    hipLaunchKernelGGL(colptr_kernel, dim3((unsigned)((n_src + 1 + 255) / 256)), dim3(256), 0, st, ks, E, n_src, csc.d_ptr);
    HETA_LAUNCH_CHECK("colptr_kernel");
    HETA_HIP(hipMemcpyAsync(csc.d_idx, vs, E * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    HETA_HIP(hipStreamSynchronize(st)); // scratch is released on return
    return HETA_OK;
}

// ---- the scan and the sort for other translation units (the neighbour sampler) ---------------------------
// Asynchronous forms with caller-provided scratch (sizes from the two helpers, in elements):
int64_t scan_scratch_elems(int64_t n_out) { return (n_out + kScanTile - 1) / kScanTile; }
int64_t sort_hist_elems(int64_t n) { return 512 * ((n + kSortTile - 1) / kSortTile); }

heta_status device_exclusive_scan_i64_async(const int64_t *in, int64_t n_in, int64_t *out, int64_t n_out, int64_t *tile_sums,
                                            hipStream_t st)
{
    return exclusive_scan_with<int64_t, int64_t>(in, n_in, out, n_out, tile_sums, st);
}

// outA / outB = exclusive scans of inA / inB (n_in inputs, n_out outputs each) in one launch set;
// tile_sums: 2 x scan_scratch_elems(n_out) elements
heta_status device_exclusive_scan2_i64_async(const int64_t *inA, const int64_t *inB, int64_t n_in, int64_t *outA, int64_t *outB,
                                             int64_t n_out, int64_t *tile_sums, hipStream_t st)
{
    if (n_out <= 0) return HETA_OK;
    const int64_t tiles = (n_out + kScanTile - 1) / kScanTile;
    ScanPair<int64_t> a{{inA, inB}, {outA, outB}};
    if (tiles == 1 || n_out <= kScanSingleMax) {
        hipLaunchKernelGGL((scan_single_pair_kernel<int64_t>), dim3(2), dim3(1024), 0, st, a, n_in, n_out);
        HETA_LAUNCH_CHECK("scan_single_kernel");
        return HETA_OK;
    }
    hipLaunchKernelGGL((scan_tile_pair_kernel<int64_t>), dim3((unsigned)tiles, 2), dim3(256), 0, st, a, n_in, n_out, tile_sums, tiles);
    HETA_LAUNCH_CHECK("scan_tile_kernel");
    hipLaunchKernelGGL((scan_sums_pair_kernel<int64_t>), dim3(2), dim3(256), 0, st, tile_sums, tiles);
    HETA_LAUNCH_CHECK("scan_sums_kernel");
    hipLaunchKernelGGL((scan_add_pair_kernel<int64_t>), dim3((unsigned)((n_out + 255) / 256), 2), dim3(256), 0, st, a, n_out, tile_sums, tiles);
    HETA_LAUNCH_CHECK("scan_add_kernel");
    return HETA_OK;
}

heta_status device_sort_pairs_u32_async(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n,
                                        int64_t key_limit, uint32_t **keys_res, uint32_t **vals_res, uint32_t *hist, uint32_t *offs,
                                        uint32_t *tile_sums, hipStream_t st)
{
    return radix_sort_pairs_with(keys, vals, keys_tmp, vals_tmp, n, bits_for(key_limit), keys_res, vals_res, hist, offs, tile_sums, st);
}

// The synchronous forms are complete (stream synchronised) when they return, because their scratch is released on return.
heta_status device_exclusive_scan_i64(const int64_t *in, int64_t n_in, int64_t *out, int64_t n_out, hipStream_t st)
{
    Scratch scr;
    heta_status e = exclusive_scan<int64_t, int64_t>(in, n_in, out, n_out, scr, st);
    if (e != HETA_OK) return e;
    HETA_HIP(hipStreamSynchronize(st));
    return HETA_OK;
}

heta_status device_sort_pairs_u32(uint32_t *keys, uint32_t *vals, uint32_t *keys_tmp, uint32_t *vals_tmp, int64_t n,
                                  int64_t key_limit, uint32_t **keys_res, uint32_t **vals_res, hipStream_t st)
{
    Scratch scr;
    heta_status e = radix_sort_pairs(keys, vals, keys_tmp, vals_tmp, n, bits_for(key_limit), keys_res, vals_res, scr, st);
    if (e != HETA_OK) return e;
    HETA_HIP(hipStreamSynchronize(st));
    return HETA_OK;
}

} // namespace heta
