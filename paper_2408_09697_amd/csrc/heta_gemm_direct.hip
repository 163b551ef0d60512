// The projection's fast path: C[M,N] (+)= A[M,K] . B[K,N] with operand tiles copied from global
// memory straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS store
// instructions) through a ring of ST stages, one workgroup barrier per k-tile.
//
// Same contract as gemm_kernel (per-relation weight matrices of an R-GCN-style AGG_r,
// Section 2.1 of the paper; Eq. 1 as one k-concatenated contraction; the backward products of
// Algorithm 1's local backpropagation) and the same output tile shape (128 x 64*WN per
// workgroup, 64 x 64 per wavefront as 2 x 2 MFMA 32x32 accumulators).  What differs:
//   - an operand that needs no conversion (its storage type is the MFMA input type) is loaded
//     "direct": every wavefront instruction moves 64 consecutive 16-byte chunks to 1 KB of
//     consecutive LDS, so the LDS image of a tile is dictated by which chunk a lane asks for.
//       k-contiguous operand (element (r,k) at base[r*ld + k]): LDS row r holds the tile's k
//         range of row r, its 16-byte chunks permuted by an XOR with a function of r so that the
//         128-bit fragment reads of neighbouring rows fall on distinct banks (no padding);
//       r-contiguous fp32 operand (element (r,k) at base[k*ld + r]): LDS row k, as in memory;
//         fragments are 32-bit reads with lanes along r.
//     Rows / chunks beyond the matrix are clamped to the last valid one (the duplicated data
//     only reaches outputs that are never stored); a ragged last k-tile is masked in registers.
//   - an operand that must be converted (fp32 -> bf16) or pair-interleaved (r-contiguous bf16)
//     keeps the register-staged loader, double-buffered in LDS;
//   - on this chip vector-ALU instructions and fp32 MFMAs do not overlap within a SIMD, so the
//     k loop is written to need almost none: tile addresses are a scalar base plus per-lane
//     offsets that stay fixed for a segment, the loop is unrolled over the ring so that LDS
//     addresses are immediates, and the tile bookkeeping is 32-bit scalar arithmetic;
//   - register use stays below 128 per lane, so two 512-thread workgroups share a CU and one's
//     prologue / epilogue hides behind the other's MFMAs;
//   - workgroup ids are mapped so that the tiles sharing an operand (the segments of a batch,
//     the column tiles of one row block) run back to back on the same XCD, i.e. behind the
//     same L2.
#include <algorithm>
#include <type_traits>

#include "heta_gemm.h"

namespace heta {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// s_waitcnt: at most N vector-memory operations outstanding and, optionally, no LDS operation
// (gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14, lgkmcnt in bits 11:8; expcnt
// left at "no wait").
template <int N, bool LDS_DONE> __device__ __forceinline__ void wait_counters()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | ((LDS_DONE ? 0 : 15) << 8) | ((N >> 4) << 14));
}

// One 16-byte chunk per lane from global memory into LDS: lane l reads base + offset_l and its
// chunk lands at lds_byte_addr + 16*l (base and lds_byte_addr are wavefront-uniform and travel in
// scalar registers / M0, so advancing a tile costs no vector instruction).  Written as inline
// assembly so that the compiler's wait-count insertion does not treat every later LDS read as
// dependent on it (which would drain the whole prefetch ring); the kernel orders these loads
// against their readers itself, with wait_counters() and the workgroup barrier.
__device__ __forceinline__ void load_chunk_to_lds(const void *base, uint32_t offset, uint32_t lds_byte_addr)
{
    asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(offset), "s"(base), "{m0}"(lds_byte_addr) : "memory");
}

// Workgroup barrier that the compiler may not move memory operations across, without the
// "wait for every outstanding load" a fence would add.
__device__ __forceinline__ void barrier_no_drain() { asm volatile("s_barrier" ::: "memory"); }

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)p));
}

// Chunk permutation of a k-contiguous LDS row: chunk c of row r sits at position c ^ swz(r).
// Chosen so that 8 (32 banks) as well as 16 (64 banks) consecutive rows reading the same chunk
// index cover every 16-byte bank group once.
template <int CPR> __device__ __forceinline__ int swz(int r)
{
    if (CPR == 8) return ((r >> 1) + 4 * (r & 1)) & 7;
    if (CPR == 4) return ((r >> 1) + (r >> 3)) & 3;
    if (CPR == 2) return (r >> 2) & 1;
    return 0;
}

// Direct loader of one operand.  T = storage = MFMA input type.  The address of a lane's chunk is
// (uniform tile base) + (per-lane 32-bit byte offset); the offsets are fixed for a segment, the
// base advances by one k-tile per issue().  Rows / chunks along r beyond the matrix are clamped
// into it when the offsets are set up; along k only the last, ragged tile of a segment can reach
// beyond the matrix and gets offsets of its own.
template <typename T, bool RC, int ROWS, int BK, int NW>
struct DirectLoader {
    static constexpr int E = 16 / (int)sizeof(T);        // elements per chunk
    static constexpr int CPR = RC ? ROWS / E : BK / E;   // chunks per LDS row
    static constexpr int NROW = RC ? BK : ROWS;          // LDS rows per tile
    static constexpr int CHUNKS = NROW * CPR;
    static constexpr int NI = CHUNKS / (64 * NW);        // load instructions per wavefront and tile
    static constexpr int STAGE_ELEMS = CHUNKS * E;
    static_assert(CHUNKS % (64 * NW) == 0, "tile must be a whole number of wavefront loads");
    static_assert(!RC || sizeof(T) == 4, "r-contiguous direct loads are fp32 only");

    const char *tile;     // uniform: address of element (r0, k of the next tile)
    uint32_t off[NI];     // per lane: byte offset of its chunk from `tile`
    uint32_t ld_bytes;    // uniform
    int64_t step;         // uniform: bytes from one k-tile to the next
    int r_room;           // KC: valid rows from r0 on, minus 1 ; RC: valid chunks along r from r0 on, minus 1

    __device__ __forceinline__ static int row_of(int i, int wave, int lane) { return ((i * NW + wave) * 64 + lane) / CPR; }
    __device__ __forceinline__ static int pos_of(int i, int wave, int lane)
    {
        const int q = (i * NW + wave) * 64 + lane;
        return RC ? q % CPR : (q % CPR) ^ swz<CPR>(q / CPR);
    }

    // r0: first r of the tile; r_total: extent of the matrix along r; k0: first k
    __device__ __forceinline__ void init(const T *b, int64_t ld, int64_t r0, int64_t r_total, int64_t k0, int wave, int lane)
    {
        ld_bytes = static_cast<uint32_t>(ld * (int64_t)sizeof(T));
        step = RC ? static_cast<int64_t>(BK) * ld_bytes : static_cast<int64_t>(BK) * (int64_t)sizeof(T);
        tile = reinterpret_cast<const char *>(b) + (RC ? k0 * ld + r0 : r0 * ld + k0) * (int64_t)sizeof(T);
        r_room = RC ? static_cast<int>(min(static_cast<int64_t>(CPR), ld / E - r0 / E)) - 1
                    : static_cast<int>(min(static_cast<int64_t>(ROWS), r_total - r0)) - 1;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int lr = row_of(i, wave, lane), pos = pos_of(i, wave, lane);
            if (RC) off[i] = static_cast<uint32_t>(lr) * ld_bytes + static_cast<uint32_t>(min(pos, r_room)) * 16u;
            else off[i] = static_cast<uint32_t>(min(lr, r_room)) * ld_bytes + static_cast<uint32_t>(pos) * 16u;
        }
    }

    // issues the loads of the next k-tile into the stage at LDS byte address `lds` and advances
    __device__ __forceinline__ void issue(uint32_t lds, int wave)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) load_chunk_to_lds(tile, off[i], lds + (i * NW + wave) * 1024);
        tile += step;
    }

    // The same for a last tile with only kv < BK valid k-values; nothing beyond the matrix is
    // touched: KC chunk columns are clamped to the last chunk that starts inside the row
    // (k_room = elements from the tile's first k to the end of the row's leading dimension),
    // RC rows are clamped to the last valid k.
    __device__ __forceinline__ void issue_ragged(uint32_t lds, int wave, int lane, int kv, int64_t k_room)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int lr = row_of(i, wave, lane), pos = pos_of(i, wave, lane);
            uint32_t o;
            if (RC) o = static_cast<uint32_t>(min(lr, kv - 1)) * ld_bytes + static_cast<uint32_t>(min(pos, r_room)) * 16u;
            else o = static_cast<uint32_t>(min(lr, r_room)) * ld_bytes +
                     static_cast<uint32_t>(min(static_cast<int64_t>(pos), k_room / E - 1)) * 16u;
            load_chunk_to_lds(tile, o, lds + (i * NW + wave) * 1024);
        }
        tile += step;
    }
};

// stands in for the loader an operand does not use
struct NoLoader {
    static constexpr int NI = 0, STAGE_ELEMS = 0;
    template <typename... X> __device__ __forceinline__ void init(X...) {}
    template <typename... X> __device__ __forceinline__ void issue(X...) {}
    template <typename... X> __device__ __forceinline__ void issue_ragged(X...) {}
    template <typename... X> __device__ __forceinline__ void load(X...) {}
    template <typename... X> __device__ __forceinline__ void store(X...) const {}
};

// fragment readers of the direct layouts (same lane -> k assignment as frag_f32 / frag_bf16)
template <bool RC, int ROWS, int BK>
__device__ __forceinline__ void dfrag_f32(const float *tile, int r, int kk, int half, float f[4])
{
    if (RC) {
#pragma unroll
        for (int t = 0; t < 4; ++t) f[t] = tile[(kk + 4 * half + t) * ROWS + r];
    } else {
        constexpr int CPR = BK / 4;
        const int c = (kk / 4 + half) ^ swz<CPR>(r);
        const float4 v = *reinterpret_cast<const float4 *>(&tile[(r * CPR + c) * 4]);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
}

template <int BK> __device__ __forceinline__ uint4 dfrag_bf16(const bf16_t *tile, int r, int kk, int half)
{
    constexpr int CPR = BK / 8;
    const int c = (kk / 8 + half) ^ swz<CPR>(r);
    return *reinterpret_cast<const uint4 *>(&tile[(r * CPR + c) * 8]);
}

// bf16 fragment of a k-contiguous operand that is stored (and was loaded) as fp32: the eight
// k-values of a lane are two 16-byte chunks of its LDS row, rounded to bf16 (nearest even, the
// hardware's packed convert) on the way to the MFMA
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const floatx2_t f = {lo, hi};
    const bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&h);
}
template <int BK> __device__ __forceinline__ uint4 dfrag_bf16_from_f32(const float *tile, int r, int kk, int half)
{
    constexpr int CPR = BK / 4;
    const int c0 = kk / 4 + 2 * half, sw = swz<CPR>(r);
    const float4 lo = *reinterpret_cast<const float4 *>(&tile[(r * CPR + (c0 ^ sw)) * 4]);
    const float4 hi = *reinterpret_cast<const float4 *>(&tile[(r * CPR + ((c0 + 1) ^ sw)) * 4]);
    return make_uint4(pack_bf16(lo.x, lo.y), pack_bf16(lo.z, lo.w), pack_bf16(hi.x, hi.y), pack_bf16(hi.z, hi.w));
}

// zeroes the k-values of a bf16 fragment (8 consecutive k from k_first) that are >= kv
__device__ __forceinline__ uint4 mask_bf16(uint4 v, int k_first, int kv)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = k_first + 2 * j;
        if (k >= kv) w[j] = 0u;
        else if (k + 1 >= kv) w[j] &= 0xffffu;
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The sequence of k-tiles a workgroup walks: the k range of its split in every segment it owns.
// All of it is wavefront-uniform 32-bit arithmetic (k extents are below 2^31).
template <int BK> struct TileSeq {
    int s, s_end;        // current segment, end of the segment range
    int k, k_end;        // first k of the next tile, end of this split's k range in segment s
    int kb, k_per_split; // first k of the split, length of a split
    __device__ __forceinline__ bool seek(const GemmParams &p) // first segment from s on with work
    {
        for (; s < s_end; ++s) {
            k_end = static_cast<int>(min(p.seg[s].K, static_cast<int64_t>(kb) + k_per_split));
            if (kb < k_end) {
                k = kb;
                return true;
            }
        }
        return false;
    }
    __device__ __forceinline__ int valid() const { return min(BK, k_end - k); } // k-values of the next tile
    // steps over one tile; true when the segment (its split range) is exhausted
    __device__ __forceinline__ bool advance()
    {
        k += BK;
        return k >= k_end;
    }
};

template <typename CT, typename SA_T, bool A_RC, bool A_DIRECT, typename SB_T, bool B_RC, bool B_DIRECT, int WN, int BK,
          int ST, int OCC>
__global__ void __launch_bounds__(128 * WN, OCC) gemm_direct_kernel(GemmParams p)
{
    constexpr int NT = 128 * WN, NW = 2 * WN, BN = 64 * WN;
    // a direct operand lies in LDS in its storage type (fp32 storage under bf16 compute is converted
    // when fragments are read); a staged operand lies there in the compute type
    using DA = std::conditional_t<A_DIRECT, DirectLoader<SA_T, A_RC && A_DIRECT, BM, BK, NW>, NoLoader>;
    using DB = std::conditional_t<B_DIRECT, DirectLoader<SB_T, B_RC && B_DIRECT, BN, BK, NW>, NoLoader>;
    using SA = std::conditional_t<A_DIRECT, NoLoader, TileLoader<SA_T, CT, A_RC, BM, NT, true, BK>>;
    using SB = std::conditional_t<B_DIRECT, NoLoader, TileLoader<SB_T, CT, B_RC, BN, NT, true, BK>>;
    constexpr bool ANY_STAGED = !A_DIRECT || !B_DIRECT;
    // bytes of one LDS stage / buffer of each operand
    constexpr int A_STRIDE = A_DIRECT ? DA::STAGE_ELEMS * (int)sizeof(SA_T) : LdsTile<CT, A_RC, BM, BK>::elems * (int)sizeof(CT);
    constexpr int B_STRIDE = B_DIRECT ? DB::STAGE_ELEMS * (int)sizeof(SB_T) : LdsTile<CT, B_RC, BN, BK>::elems * (int)sizeof(CT);
    constexpr int A_BYTES = (A_DIRECT ? ST : 2) * A_STRIDE, B_BYTES = (B_DIRECT ? ST : 2) * B_STRIDE;
    constexpr int LD_PER_TILE = (A_DIRECT ? DA::NI : 0) + (B_DIRECT ? DB::NI : 0);
    static_assert(A_DIRECT || B_DIRECT, "at least one operand is loaded directly");
    static_assert(ST >= 2 && (ST - 2) * LD_PER_TILE < 64, "vmcnt range");
    __shared__ __attribute__((aligned(1024))) char As[A_BYTES];
    __shared__ __attribute__((aligned(1024))) char Bs[B_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    const int64_t xcd = blockIdx.x % 8, j = blockIdx.x / 8;
    const int64_t in_idx = j % inner, outer = (j / inner) * 8 + xcd;
    if (outer >= n_outer) return;
    const int s0 = p.batch ? static_cast<int>(in_idx % n_batch) : 0;
    const int64_t rest = in_idx / n_batch;
    const int64_t n0 = (rest % p.nt) * BN;
    const int64_t m0 = (p.partial ? rest / p.nt : outer) * BM;
    const int64_t split = p.partial ? outer : 0;
    const GemmSeg &out_seg = p.seg[s0];
    if (m0 >= out_seg.M || n0 >= out_seg.N) return; // uniform per workgroup
    const int rows_a = static_cast<int>(min(out_seg.M - m0, static_cast<int64_t>(BM)));
    const int rows_b = static_cast<int>(min(out_seg.N - n0, static_cast<int64_t>(BN)));

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;

    DA da;
    DB db;
    SA sa;
    SB sb;

    // issue side (direct loads, ST-1 tiles ahead), staged side (one tile ahead), consume side
    TileSeq<BK> I{s0, p.batch ? s0 + 1 : p.n_seg, 0, 0, static_cast<int>(split * p.k_per_split),
                  static_cast<int>(min(p.k_per_split, static_cast<int64_t>(0x7fffffff)))};
    TileSeq<BK> L = I, C = I;
    auto init_direct = [&]() {
        const GemmSeg &g = p.seg[I.s];
        if constexpr (A_DIRECT) da.init(static_cast<const SA_T *>(g.A), g.lda, m0, g.M, I.k, wave, lane);
        if constexpr (B_DIRECT) db.init(static_cast<const SB_T *>(g.B), g.ldb, n0, g.N, I.k, wave, lane);
    };
    auto init_staged = [&]() {
        const GemmSeg &g = p.seg[L.s];
        if constexpr (!A_DIRECT) sa.init(static_cast<const SA_T *>(g.A), g.lda, m0, L.k, tid);
        if constexpr (!B_DIRECT) sb.init(static_cast<const SB_T *>(g.B), g.ldb, n0, L.k, tid);
    };
    bool i_ok = I.seek(p);
    if (i_ok) init_direct();
    bool l_ok = ANY_STAGED && L.seek(p);
    if (l_ok) init_staged();
    bool c_ok = C.seek(p);
    int ahead = 0; // direct tiles issued and not yet consumed

    const uint32_t a_lds = lds_address(As), b_lds = lds_address(Bs);
    auto issue_direct = [&](int st) { // st: ring stage the tile goes to
        const int kv = I.valid();
        if (kv == BK) {
            if constexpr (A_DIRECT) da.issue(a_lds + st * A_STRIDE, wave);
            if constexpr (B_DIRECT) db.issue(b_lds + st * B_STRIDE, wave);
        } else {
            const GemmSeg &g = p.seg[I.s];
            if constexpr (A_DIRECT) da.issue_ragged(a_lds + st * A_STRIDE, wave, lane, kv, g.lda - I.k);
            if constexpr (B_DIRECT) db.issue_ragged(b_lds + st * B_STRIDE, wave, lane, kv, g.ldb - I.k);
        }
        ++ahead;
        if (I.advance()) {
            ++I.s;
            i_ok = I.seek(p);
            if (i_ok) init_direct();
        }
    };
    auto load_staged = [&]() {
        const int k_left = L.valid();
        if constexpr (!A_DIRECT) sa.load(rows_a, k_left, tid);
        if constexpr (!B_DIRECT) sb.load(rows_b, k_left, tid);
        if (L.advance()) {
            ++L.s;
            l_ok = L.seek(p);
            if (l_ok) init_staged();
        }
    };

    if constexpr (ANY_STAGED) {
        if (l_ok) load_staged();
    }
#pragma unroll
    for (int q = 0; q < ST - 1; ++q)
        if (i_ok) issue_direct(q);

    int sbuf = 0; // LDS buffer of the staged operand's current tile
    while (c_ok) {
#pragma unroll
        for (int st = 0; st < ST; ++st) { // st: ring stage of the tile consumed in this step (compile-time)
            if (!c_ok) break;
            // registers of this tile's staged operand -> its LDS buffer (last read two tiles ago)
            if constexpr (!A_DIRECT) sa.store(reinterpret_cast<CT *>(As + sbuf * A_STRIDE), tid);
            if constexpr (!B_DIRECT) sb.store(reinterpret_cast<CT *>(Bs + sbuf * B_STRIDE), tid);
            // this tile's direct loads have landed once at most the younger tiles' loads are
            // outstanding (and the staged stores above have reached LDS)
            if (ahead - 1 >= ST - 2) wait_counters<(ST - 2) * LD_PER_TILE, true>();
            else wait_counters<0, true>();
            barrier_no_drain(); // every wavefront's part of the tile is in LDS; the previous tile's stage is free
            if constexpr (ANY_STAGED) {
                if (l_ok) load_staged();
            }
            if (i_ok) issue_direct((st + ST - 1) % ST);

            const char *At = As + (A_DIRECT ? st : sbuf) * A_STRIDE;
            const char *Bt = Bs + (B_DIRECT ? st : sbuf) * B_STRIDE;
            const int kv = C.valid();
            const bool ragged = kv < BK;
            if constexpr (sizeof(CT) == 4) {
#pragma unroll
                for (int kk = 0; kk < BK; kk += 8) {
                    float a[2][4], b[2][4];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        if constexpr (A_DIRECT) dfrag_f32<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half, a[i]);
                        else frag_f32<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half, a[i]);
                    }
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        if constexpr (B_DIRECT) dfrag_f32<B_RC, BN, BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, b[jj]);
                        else frag_f32<B_RC, BN, BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, b[jj]);
                    }
                    if (ragged) {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (kk + 4 * half + t >= kv) {
                                a[0][t] = a[1][t] = 0.f;
                                b[0][t] = b[1][t] = 0.f;
                            }
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int jj = 0; jj < 2; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[jj][t], acc[i][jj], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < BK; kk += 16) {
                    union Frag { uint4 u; bf16x8 v; } a[2], b[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        if constexpr (A_DIRECT && sizeof(SA_T) == 4)
                            a[i].u = dfrag_bf16_from_f32<BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half);
                        else if constexpr (A_DIRECT) a[i].u = dfrag_bf16<BK>(reinterpret_cast<const bf16_t *>(At), wm + i * 32 + l32, kk, half);
                        else a[i].u = frag_bf16<A_RC, BM, BK>(reinterpret_cast<const bf16_t *>(At), wm + i * 32 + l32, kk, half);
                    }
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        if constexpr (B_DIRECT && sizeof(SB_T) == 4)
                            b[jj].u = dfrag_bf16_from_f32<BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half);
                        else if constexpr (B_DIRECT) b[jj].u = dfrag_bf16<BK>(reinterpret_cast<const bf16_t *>(Bt), wn + jj * 32 + l32, kk, half);
                        else b[jj].u = frag_bf16<B_RC, BN, BK>(reinterpret_cast<const bf16_t *>(Bt), wn + jj * 32 + l32, kk, half);
                    }
                    if (ragged) {
#pragma unroll
                        for (int i = 0; i < 2; ++i) {
                            a[i].u = mask_bf16(a[i].u, kk + 8 * half, kv);
                            b[i].u = mask_bf16(b[i].u, kk + 8 * half, kv);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj)
                            acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[jj].v, acc[i][jj], 0, 0, 0);
                }
            }
            --ahead;
            sbuf ^= 1;
            if (C.advance()) {
                ++C.s;
                c_ok = C.seek(p);
            }
        }
    }

    // epilogue: accumulator register v of lane (half, l32) is C[8*(v/4) + 4*half + v%4][l32] of its 32x32 tile;
    // a store instruction writes two 128-byte row segments (32-bit stores with lanes along the row:
    // 128-bit stores of a transposed accumulator, 32 bytes in each of 32 rows, measured slower)
    float *Cp = out_seg.C + (p.partial ? split * out_seg.M * out_seg.ldc : 0);
    const bool direct = !p.partial;
    const bool plain = !direct || (!p.row_scale && p.beta == 0.f && !p.relu);
    const bool interior = rows_a == BM && rows_b == BN;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int nl = wn + jj * 32 + l32;
            float *col = Cp + (m0 + wm + i * 32 + 4 * half) * out_seg.ldc + n0 + nl;
            if (p.out_bf16) { // bf16 output: same element mapping, 16-bit stores
                if (nl >= rows_b) continue;
                bf16_t *hcol = reinterpret_cast<bf16_t *>(out_seg.C) + (m0 + wm + i * 32 + 4 * half) * out_seg.ldc + n0 + nl;
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (wm + i * 32 + 8 * (v / 4) + 4 * half + (v % 4) < rows_a)
                        hcol[(8 * (v / 4) + (v % 4)) * out_seg.ldc] = to_bf16(acc[i][jj][v]);
                continue;
            }
            if (interior && plain) {
#pragma unroll
                for (int v = 0; v < 16; ++v) col[(8 * (v / 4) + (v % 4)) * out_seg.ldc] = acc[i][jj][v];
                continue;
            }
            if (nl >= rows_b) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int ml = wm + i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (ml >= rows_a) continue;
                float val = acc[i][jj][v];
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

// ---- host side -------------------------------------------------------------------------------------

template <typename CT, typename SA_T, bool A_RC, bool A_DIRECT, typename SB_T, bool B_RC, bool B_DIRECT, int WN, int BK,
          int ST, int OCC>
static heta_status launch_direct(GemmParams &p, hipStream_t st, const char *name, double bytes, double flops)
{
    constexpr int BN = 64 * WN;
    int64_t mt = 0, nt = 0;
    for (int s = 0; s < p.n_seg; ++s) {
        mt = std::max(mt, (p.seg[s].M + BM - 1) / BM);
        nt = std::max(nt, (p.seg[s].N + BN - 1) / BN);
    }
    p.mt = mt;
    p.nt = nt;
    const int64_t inner = nt * (p.batch ? p.n_seg : 1) * (p.partial ? mt : 1);
    const int64_t outer = p.partial ? std::max(1, p.n_split) : mt;
    const int64_t blocks = (outer + 7) / 8 * 8 * inner;
    if (blocks <= 0) return HETA_OK;
    if (blocks > 0x7fffffff) return fail(HETA_ERR_UNSUPPORTED, "projection: matrix too large for one launch");
    ProfScope prof(name, st, bytes, flops);
    hipLaunchKernelGGL((gemm_direct_kernel<CT, SA_T, A_RC, A_DIRECT, SB_T, B_RC, B_DIRECT, WN, BK, ST, OCC>),
                       dim3((unsigned)blocks), dim3(128 * WN), 0, st, p);
    HETA_LAUNCH_CHECK("gemm_direct_kernel");
    return HETA_OK;
}

heta_status launch_gemm_direct(GemmParams &p, heta_dtype a_dt, heta_dtype b_dt, bool a_rc, bool b_rc, hipStream_t st,
                               const char *name, double bytes, double flops, bool *handled)
{
    *handled = false;
    if (p.n_split < 1) p.n_split = 1;
    int64_t n_max = 0;
    for (int s = 0; s < p.n_seg; ++s) {
        const GemmSeg &g = p.seg[s];
        // 16-byte rows on both operands; r-contiguous operands are read in whole chunks along r
        if (!aligned16(g.A) || !aligned16(g.B)) return HETA_OK;
        const int64_t a_row = g.lda * (int64_t)dtype_size(a_dt), b_row = g.ldb * (int64_t)dtype_size(b_dt);
        if (a_row % 16 || b_row % 16) return HETA_OK;
        if (g.M < 1 || g.N < 1 || g.K < 1) return HETA_OK;
        // per-lane offsets within a tile are 32-bit; k extents are walked in 32-bit arithmetic
        if (a_row * 256 >= (int64_t(1) << 31) || b_row * 256 >= (int64_t(1) << 31) || g.K >= (int64_t(1) << 31) - 256)
            return HETA_OK;
        n_max = std::max(n_max, g.N);
    }
    if (p.n_split > 1 && p.k_per_split * p.n_split >= (int64_t(1) << 31) - 256) return HETA_OK;
    bool wide = n_max > 128;
    if (wide) {
        // A launch that gives a workgroup to half the CUs at most (the projections of a sampled mini-batch
        // block) is bound by the matrix pipe of the few CUs it runs on: a 128 x 256 tile keeps two wavefronts
        // per SIMD busy for 32 MFMAs each per k-step.  128 x 128 tiles put the same work on twice the CUs.
        int64_t mt = 0, nt = 0;
        for (int s = 0; s < p.n_seg; ++s) {
            mt = std::max(mt, (p.seg[s].M + BM - 1) / BM);
            nt = std::max(nt, (p.seg[s].N + 255) / 256);
        }
        const int64_t inner = nt * (p.batch ? p.n_seg : 1) * (p.partial ? mt : 1);
        const int64_t outer = p.partial ? std::max(1, p.n_split) : mt;
        if (outer * inner <= 128) wide = false;
    }
    *handled = true;
    if (a_dt == HETA_F32 && b_dt == HETA_F32) {
#define HETA_D32(ARC, BRC)                                                                                          \
    return wide ? launch_direct<float, float, ARC, true, float, BRC, true, 4, 16, 3, 4>(p, st, name, bytes, flops)   \
                : launch_direct<float, float, ARC, true, float, BRC, true, 2, 16, 3, 3>(p, st, name, bytes, flops)
        if (!a_rc && b_rc) { HETA_D32(false, true); }
        if (!a_rc && !b_rc) { HETA_D32(false, false); }
        if (a_rc && b_rc) { HETA_D32(true, true); }
#undef HETA_D32
    }
    if (a_dt == HETA_BF16 && b_dt == HETA_BF16 && !a_rc && b_rc) { // forward: M_r (bf16) x W_r (bf16, n-contiguous)
        return wide ? launch_direct<bf16_t, bf16_t, false, true, bf16_t, true, false, 4, 32, 3, 4>(p, st, name, bytes, flops)
                    : launch_direct<bf16_t, bf16_t, false, true, bf16_t, true, false, 2, 32, 3, 2>(p, st, name, bytes, flops);
    }
    if (a_dt == HETA_F32 && b_dt == HETA_BF16 && !a_rc && !b_rc) { // backward: G (fp32, rounded at the MFMA) x W_r^T (bf16, k-contiguous)
        // (256 output columns: the fp32 tiles of a direct A would leave LDS room for one workgroup per CU only,
        // so A goes through the register stage there)
        return wide ? launch_direct<bf16_t, float, false, false, bf16_t, false, true, 4, 32, 3, 4>(p, st, name, bytes, flops)
                    : launch_direct<bf16_t, float, false, true, bf16_t, false, true, 2, 32, 3, 2>(p, st, name, bytes, flops);
    }
    if (a_dt == HETA_BF16 && b_dt == HETA_BF16 && !a_rc && !b_rc) { // both k-contiguous bf16 (forward with a packed W_r^T)
        return wide ? launch_direct<bf16_t, bf16_t, false, true, bf16_t, false, true, 4, 32, 3, 4>(p, st, name, bytes, flops)
                    : launch_direct<bf16_t, bf16_t, false, true, bf16_t, false, true, 2, 32, 3, 3>(p, st, name, bytes, flops);
    }
    *handled = false;
    return HETA_OK;
}

} // namespace heta
