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
//       r-contiguous operand (element (r,k) at base[k*ld + r]): LDS row k, as in memory; fp32 compute
//         reads fragments with 32-bit loads, lanes along r; under bf16 compute (the weight gradient,
//         whose two operands both lie with the contraction index outermost) a lane gathers its eight
//         consecutive k-values with eight 16-bit loads (bf16 storage) or eight 32-bit loads and
//         packed converts (fp32 storage).  That costs four times the LDS instructions of a
//         k-contiguous fragment, which a product bound by HBM (two short operand rows per graph row
//         against 2*d_in*d_out flops) can afford; in exchange no operand passes through registers.
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
    // load instructions per wavefront and tile.  Every wavefront issues the same number (the kernel counts
    // outstanding loads per wavefront); when the tile is not a whole number of workgroup-wide loads the
    // surplus slots wrap around and fetch chunks a second time into the same LDS place (same bytes).
    static constexpr int NI = (CHUNKS + 64 * NW - 1) / (64 * NW);
    static constexpr int STAGE_ELEMS = CHUNKS * E;
    static_assert(CHUNKS % 64 == 0, "tile must be a whole number of wavefront loads");

    const char *tile;     // uniform: address of element (r0, k of the next tile)
    uint32_t off[NI];     // per lane: byte offset of its chunk from `tile`
    uint32_t ld_bytes;    // uniform
    int64_t step;         // uniform: bytes from one k-tile to the next
    int r_room;           // KC: valid rows from r0 on, minus 1 ; RC: valid chunks along r from r0 on, minus 1

    // the 64-chunk slot that instruction i of this wavefront fills
    __device__ __forceinline__ static int slot_of(int i, int wave) { return (i * NW + wave) % (CHUNKS / 64); }
    __device__ __forceinline__ static int row_of(int i, int wave, int lane) { return (slot_of(i, wave) * 64 + lane) / CPR; }
    __device__ __forceinline__ static int pos_of(int i, int wave, int lane)
    {
        const int q = slot_of(i, wave) * 64 + lane;
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
        for (int i = 0; i < NI; ++i) load_chunk_to_lds(tile, off[i], lds + slot_of(i, wave) * 1024);
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
            load_chunk_to_lds(tile, o, lds + slot_of(i, wave) * 1024);
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

// bf16 fragment of an r-contiguous bf16 operand lying in LDS as in memory (row k holds ROWS elements):
// the lane's eight k-values kk + 8*half + 0..7 of its row r, one 16-bit read each
template <int ROWS> __device__ __forceinline__ uint4 dfrag_bf16_rc(const bf16_t *tile, int r, int kk, int half)
{
    const bf16_t *p = tile + (kk + 8 * half) * ROWS + r;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        w[j] = static_cast<uint32_t>(p[(2 * j) * ROWS]) | (static_cast<uint32_t>(p[(2 * j + 1) * ROWS]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// the same for an r-contiguous fp32 operand: eight 32-bit reads, rounded to bf16 in pairs.  With SPLIT
// the fragment `lo` receives what the rounding left (x - bf16(x), itself rounded to bf16): fed as a
// second MFMA term it restores 16 significant bits of the operand.
template <int ROWS, bool SPLIT>
__device__ __forceinline__ uint4 dfrag_bf16_rc_from_f32(const float *tile, int r, int kk, int half, uint4 *lo)
{
    const float *p = tile + (kk + 8 * half) * ROWS + r;
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = p[j * ROWS];
    uint32_t w[4], wl[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        w[j] = pack_bf16(x[2 * j], x[2 * j + 1]);
        if (SPLIT) {
            const float ra = x[2 * j] - __uint_as_float(w[j] << 16);
            const float rb = x[2 * j + 1] - __uint_as_float(w[j] & 0xffff0000u);
            wl[j] = pack_bf16(ra, rb);
        }
    }
    if (SPLIT) *lo = make_uint4(wl[0], wl[1], wl[2], wl[3]);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// fp32 products on the bf16 matrix pipe.  x = h + m + l with three bf16 terms (h = bf16(x), m = bf16(x - h),
// l = bf16(x - h - m); both differences are exact in fp32), so |x - (h + m + l)| <= 2^-27 |x|.  A product a b
// is fed as the six terms ah bh, ah bm, am bh, am bm, ah bl, al bh (each a product of two 8-bit significands,
// exact in the fp32 accumulator's input); the three terms left out are below 2^-25 |a b|, less than the
// rounding of one fp32 multiplication.  Six bf16 MFMAs of 16 k-values cost 6 x 8 passes where the fp32 MFMA
// needs 8 x 16 for the same 16 k-values.
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t &h, uint32_t &m, uint32_t &l)
{
    h = pack_bf16(x0, x1);
    const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xffff0000u);
    m = pack_bf16(r0, r1);
    const float s0 = r0 - __uint_as_float(m << 16), s1 = r1 - __uint_as_float(m & 0xffff0000u);
    l = pack_bf16(s0, s1);
}

// The lane's eight k-values kk + 8*half + 0..7 of row r of an fp32 operand lying in LDS (k-contiguous with
// swizzled chunks, or r-contiguous as in memory): the LDS reads only.
template <bool RC, int ROWS, int BK>
__device__ __forceinline__ void dfrag_load8(const float *tile, int r, int kk, int half, float x[8])
{
    if constexpr (RC) {
        const float *p = tile + (kk + 8 * half) * ROWS + r;
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = p[j * ROWS];
    } else {
        constexpr int CPR = BK / 4;
        const int c0 = kk / 4 + 2 * half, sw = swz<CPR>(r);
        const float4 lo = *reinterpret_cast<const float4 *>(&tile[(r * CPR + (c0 ^ sw)) * 4]);
        const float4 hi = *reinterpret_cast<const float4 *>(&tile[(r * CPR + ((c0 + 1) ^ sw)) * 4]);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w; x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    }
}

// Eight k-values (the first is k0 of its tile) as three bf16 fragments; with MASKED, k-values from kv on
// count as zero (branch-free: the caller's code stays one scheduling region).
template <bool MASKED> __device__ __forceinline__ void split3_frag(const float x[8], int k0, int kv, uint4 out[3])
{
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float x0 = x[2 * j], x1 = x[2 * j + 1];
        if constexpr (MASKED) {
            x0 = k0 + 2 * j < kv ? x0 : 0.f;
            x1 = k0 + 2 * j + 1 < kv ? x1 : 0.f;
        }
        split3_pair(x0, x1, h[j], m[j], l[j]);
    }
    out[0] = make_uint4(h[0], h[1], h[2], h[3]);
    out[1] = make_uint4(m[0], m[1], m[2], m[3]);
    out[2] = make_uint4(l[0], l[1], l[2], l[3]);
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

// The splitting of one fragment (8 k-values of a lane) in pieces, so that a k-step can place them between its
// MFMAs: hp / mp / lp pack the leading, middle and last term of a pair of values, r1 / r2 leave the residuals.
struct X3Frag {
    float x[8];      // the values, then their residuals
    uint32_t h[4], m[4], l[4];
    __device__ __forceinline__ void hp(int j) { h[j] = pack_bf16(x[2 * j], x[2 * j + 1]); }
    __device__ __forceinline__ void r1(int j)
    {
        x[2 * j] -= __uint_as_float(h[j] << 16);
        x[2 * j + 1] -= __uint_as_float(h[j] & 0xffff0000u);
    }
    __device__ __forceinline__ void mp(int j) { m[j] = pack_bf16(x[2 * j], x[2 * j + 1]); }
    __device__ __forceinline__ void r2(int j)
    {
        x[2 * j] -= __uint_as_float(m[j] << 16);
        x[2 * j + 1] -= __uint_as_float(m[j] & 0xffff0000u);
    }
    __device__ __forceinline__ void lp(int j) { l[j] = pack_bf16(x[2 * j], x[2 * j + 1]); }
    __device__ __forceinline__ bf16x8 term(int t) const
    {
        union { uint4 u; bf16x8 v; } f;
        const uint32_t *w = t == 0 ? h : (t == 1 ? m : l);
        f.u = make_uint4(w[0], w[1], w[2], w[3]);
        return f.v;
    }
};

// Loader of an operand that lies in memory as three bf16 terms (pack_split3_weights): a stage holds, for each
// term and each of the tile's two k-octets, the BN columns' 16-byte chunks (8 k-values) side by side, so a
// fragment read (lane = column, half = octet) is one conflict-free 128-bit load per term and a wavefront load
// instruction copies 64 neighbouring columns' chunks, 1 KB that is contiguous in memory too.  The packed
// operand is zero beyond K and N, so no tile needs clamping or masking on this side.
template <int BN, int NW> struct Split3Loader {
    static constexpr int SLOTS = 3 * 2 * (BN / 64);
    static constexpr int NI = (SLOTS + NW - 1) / NW;
    static constexpr int STAGE_BYTES = SLOTS * 1024;
    const char *tile;    // uniform: the chunk of term 0, the next tile's first octet, column n0
    uint32_t off;        // per lane
    int64_t plane, oct;  // uniform: bytes from term to term, from octet to octet
    __device__ __forceinline__ void init(const void *b3, int ko, int n_pad, int64_t n0, int64_t k0, int lane)
    {
        oct = static_cast<int64_t>(n_pad) * 16;
        plane = ko * oct;
        tile = static_cast<const char *>(b3) + (k0 / 8) * oct + n0 * 16;
        off = static_cast<uint32_t>(lane) * 16u;
    }
    __device__ __forceinline__ void issue(uint32_t lds, int wave)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int slot = (i * NW + wave) % SLOTS; // surplus slots repeat earlier ones (same bytes, same place)
            const int t = slot / (2 * (BN / 64)), o = (slot / (BN / 64)) % 2, hn = slot % (BN / 64);
            load_chunk_to_lds(tile + t * plane + o * oct + hn * 1024, off, lds + slot * 1024);
        }
        tile += 2 * oct;
    }
    // term t of the 8 k-values of octet `half` of column c, of the stage at `stage`
    __device__ __forceinline__ static uint4 frag(const char *stage, int t, int half, int c)
    {
        return *reinterpret_cast<const uint4 *>(stage + ((t * 2 + half) * BN + c) * 16);
    }
};

// One whole k-step (16 k-values, none masked) of a wavefront's 2 x 2 accumulators with B already in three
// terms: only A's two fragments are split (88 vector instructions), and the order is pinned with scheduling
// barriers so that the splitting runs between the twelve MFMAs that need A's leading term alone; the twelve
// that need its m and l terms follow.  Terms of one accumulator are added leading term first.
template <bool A_RC, int BM, int BN, int BK>
__device__ __forceinline__ void x3_step_2x2_presplit(const float *At, const char *Bt, int ra, int cb, int half, floatx16 (&acc)[2][2])
{
    X3Frag a[2];
    dfrag_load8<A_RC, BM, BK>(At, ra, 0, half, a[0].x);
    dfrag_load8<A_RC, BM, BK>(At, ra + 32, 0, half, a[1].x);
    union BF { uint4 u; bf16x8 v; } b[2][3];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j][t].u = Split3Loader<BN, 4>::frag(Bt, t, half, cb + 32 * j);
#define X3_PIN __builtin_amdgcn_sched_barrier(0)
#define X3_MM(TA_, I_, TB_, J_)                                                                                        \
    X3_PIN;                                                                                                            \
    acc[I_][J_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[I_].term(TA_), b[J_][TB_].v, acc[I_][J_], 0, 0, 0);       \
    X3_PIN
#define X3_ALL(F_, OP_) F_.OP_(0); F_.OP_(1); F_.OP_(2); F_.OP_(3)
#define X3_LO(F_, OP_) F_.OP_(0); F_.OP_(1)
#define X3_HI(F_, OP_) F_.OP_(2); F_.OP_(3)
    X3_ALL(a[0], hp); X3_ALL(a[1], hp);
    X3_MM(0, 0, 0, 0); X3_LO(a[0], r1);
    X3_MM(0, 0, 0, 1); X3_HI(a[0], r1);
    X3_MM(0, 1, 0, 0); X3_ALL(a[0], mp); X3_LO(a[1], r1);
    X3_MM(0, 1, 0, 1); X3_HI(a[1], r1);
    X3_MM(0, 0, 1, 0); X3_ALL(a[1], mp); X3_LO(a[0], r2);
    X3_MM(0, 0, 1, 1); X3_HI(a[0], r2);
    X3_MM(0, 1, 1, 0); X3_ALL(a[0], lp); X3_LO(a[1], r2);
    X3_MM(0, 1, 1, 1); X3_HI(a[1], r2);
    X3_MM(0, 0, 2, 0); X3_ALL(a[1], lp);
    X3_MM(0, 0, 2, 1); X3_MM(0, 1, 2, 0); X3_MM(0, 1, 2, 1);
    X3_MM(1, 0, 0, 0); X3_MM(1, 0, 0, 1); X3_MM(1, 1, 0, 0); X3_MM(1, 1, 0, 1);
    X3_MM(1, 0, 1, 0); X3_MM(1, 0, 1, 1); X3_MM(1, 1, 1, 0); X3_MM(1, 1, 1, 1);
    X3_MM(2, 0, 0, 0); X3_MM(2, 0, 0, 1); X3_MM(2, 1, 0, 0); X3_MM(2, 1, 0, 1);
#undef X3_PIN
#undef X3_MM
#undef X3_ALL
#undef X3_LO
#undef X3_HI
}

// Writes the three-term form of one B operand: one thread per (k-octet, column).
__global__ void __launch_bounds__(256) pack_split3_kernel(const float *W, int64_t ldw, int K, int N, int trans, uint4 *out, int ko, int n_pad)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int n = static_cast<int>(idx % n_pad), o = static_cast<int>(idx / n_pad);
    if (o >= ko) return;
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float x[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = o * 8 + 2 * j + e;
            x[e] = (k < K && n < N) ? (trans ? W[static_cast<int64_t>(n) * ldw + k] : W[static_cast<int64_t>(k) * ldw + n]) : 0.f;
        }
        split3_pair(x[0], x[1], h[j], m[j], l[j]);
    }
    const int64_t plane = static_cast<int64_t>(ko) * n_pad, at = static_cast<int64_t>(o) * n_pad + n;
    out[at] = make_uint4(h[0], h[1], h[2], h[3]);
    out[plane + at] = make_uint4(m[0], m[1], m[2], m[3]);
    out[2 * plane + at] = make_uint4(l[0], l[1], l[2], l[3]);
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

// ---- epilogue ---------------------------------------------------------------------------------------
template <int MI, int NJ>
__device__ __forceinline__ void store_tile(const GemmParams &p, const GemmSeg &out_seg, float *strips, floatx16 (&acc)[MI][NJ],
                                           int wave, int lane, int wm, int wn, int64_t m0, int64_t n0, int rows_a, int rows_b,
                                           int64_t split)
{
    // Epilogue through LDS.  Accumulator register v of lane (half, l32) is C[8*(v/4) + 4*half + v%4][l32] of
    // its 32 x 32 tile: written out as it lies, a store instruction would touch 32 x 4 (or 32 x 2) bytes in
    // each of two rows.  Instead every wavefront passes its 64 x 64 block through a private LDS strip, 8 rows
    // x 64 columns at a time (the ring stages are free once every wavefront has left the k loop), and reads
    // it back with a lane owning 4 consecutive columns: a store instruction then writes whole 256-byte
    // (fp32) or 128-byte (bf16) row segments of 4 rows, and the accumulate / scale / activation forms read
    // and write the same 16-byte pieces.
    constexpr int EW = 32 * NJ;    // columns of a wavefront's block
    constexpr int EPP = EW + 4;    // strip pitch in floats (rows 4 apart fall on different banks)
    constexpr int PIECES = 8 * NJ; // 16-byte pieces per strip row
    const int half = lane >> 5, l32 = lane & 31;
    float *ep = strips + wave * (8 * EPP);
    float *Cp = out_seg.C + (p.partial ? split * out_seg.M * out_seg.ldc : 0);
    bf16_t *Hp = reinterpret_cast<bf16_t *>(out_seg.C);
    const bool direct = !p.partial;
    const bool fused = direct && (p.row_scale || p.beta != 0.f || p.relu);
    // 16-byte pieces (4 fp32 or 8 bf16 columns) need rows that keep that alignment
    const bool vec_out = p.out_bf16 ? ((out_seg.ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(Hp) & 15u) == 0)
                                    : ((out_seg.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(Cp) & 15u) == 0);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj)
#pragma unroll
                for (int t = 0; t < 4; ++t) ep[(4 * half + t) * EPP + jj * 32 + l32] = acc[i][jj][4 * q + t];
            if (p.out_bf16) { // 8 rows x 4 NJ pieces of 8 columns: 16-byte stores, 128-byte row segments for NJ = 2
#pragma unroll
                for (int h = 0; h < (NJ + 1) / 2; ++h) {
                    const int piece = h * 64 + lane;
                    if (piece >= 32 * NJ) continue;
                    const int row_l = piece / (4 * NJ), c8 = (piece % (4 * NJ)) * 8;
                    const float4 lo4 = *reinterpret_cast<const float4 *>(&ep[row_l * EPP + c8]);
                    const float4 hi4 = *reinterpret_cast<const float4 *>(&ep[row_l * EPP + c8 + 4]);
                    const int ml = wm + i * 32 + 8 * q + row_l, nl = wn + c8;
                    if (ml >= rows_a || nl >= rows_b) continue;
                    const int64_t off = (m0 + ml) * out_seg.ldc + n0 + nl;
                    if (vec_out && nl + 8 <= rows_b) {
                        *reinterpret_cast<uint4 *>(Hp + off) = make_uint4(pack_bf16(lo4.x, lo4.y), pack_bf16(lo4.z, lo4.w),
                                                                          pack_bf16(hi4.x, hi4.y), pack_bf16(hi4.z, hi4.w));
                    } else {
                        const float v[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (nl + e < rows_b) Hp[off + e] = to_bf16(v[e]);
                    }
                }
                continue;
            }
#pragma unroll
            for (int h = 0; h < NJ; ++h) { // the strip's 8 x PIECES pieces, 64 per pass
                const int piece = h * 64 + lane;
                const int row_l = piece / PIECES, c4 = (piece % PIECES) * 4;
                const float4 v4 = *reinterpret_cast<const float4 *>(&ep[row_l * EPP + c4]);
                const int ml = wm + i * 32 + 8 * q + row_l, nl = wn + c4;
                if (ml >= rows_a || nl >= rows_b) continue;
                float v[4] = {v4.x, v4.y, v4.z, v4.w};
                const int64_t off = (m0 + ml) * out_seg.ldc + n0 + nl;
                float *o = Cp + off;
                const bool whole = vec_out && nl + 4 <= rows_b;
                if (fused) {
                    const float sc = p.row_scale ? p.row_scale[m0 + ml] : 1.f;
                    float old[4] = {0.f, 0.f, 0.f, 0.f};
                    if (p.beta != 0.f) {
                        if (whole) {
                            const float4 o4 = *reinterpret_cast<const float4 *>(o);
                            old[0] = o4.x; old[1] = o4.y; old[2] = o4.z; old[3] = o4.w;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (nl + e < rows_b) old[e] = o[e];
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float x = v[e] * sc;
                        if (p.beta != 0.f) x += p.beta * old[e];
                        if (p.relu) x = fmaxf(x, 0.f);
                        v[e] = x;
                    }
                }
                if (whole) {
                    *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (nl + e < rows_b) o[e] = v[e];
                }
            }
        }
}

template <bool W3, bool B_DIRECT, typename DB, typename SB_T, typename Staged, typename CT> constexpr int b_stage_bytes()
{
    if constexpr (W3) return DB::STAGE_BYTES;
    else if constexpr (B_DIRECT) return DB::STAGE_ELEMS * (int)sizeof(SB_T);
    else return Staged::elems * (int)sizeof(CT);
}

// Shape of the output tile: WMW x WN wavefronts, each holding MI x NJ MFMA 32 x 32 accumulators; the
// tile is (32 MI WMW) x (32 NJ WN).  The default 2 x 2 blocks per wavefront with 2 x WN wavefronts is the
// 128 x (64 WN) tile; tall tiles (MI = 5, NJ = 1: 320 x 128) let a weight gradient whose input is wider than
// 128 columns read its large gradient operand once, wide ones (MI = 1, NJ = 5: 128 x 320) do the same for a
// product with more than 256 output columns and its input rows.  Where the k loop is long, both grow along their
// second side too (MI x NJ = 5 x 2 or 4 x 2: 320 x 256 / 256 x 256; 2 x 5: 256 x 320), one workgroup per CU: fewer
// operand bytes loaded per MFMA.
template <typename CT, typename SA_T, bool A_RC, bool A_DIRECT, typename SB_T, bool B_RC, bool B_DIRECT, int WN, int BK,
          int ST, int OCC, bool B_SPLIT = false, int MI = 2, int NJ = 2, int WMW = 2, int X3 = 0>
__global__ void __launch_bounds__(64 * WMW * WN, OCC) gemm_direct_kernel(GemmParams p)
{
    constexpr int NW = WMW * WN, NT = 64 * NW, BN = 32 * NJ * WN, BM = 32 * MI * WMW; // BM shadows the default tile height
    // a direct operand lies in LDS in its storage type (fp32 storage under bf16 compute is converted
    // when fragments are read); a staged operand lies there in the compute type
    using DA = std::conditional_t<A_DIRECT, DirectLoader<SA_T, A_RC && A_DIRECT, BM, BK, NW>, NoLoader>;
    // X3: fp32 operands as three bf16 terms each - 1: both split when their fragments are read, 2: B comes pre-split
    constexpr bool W3 = X3 == 2;
    using DB = std::conditional_t<W3, Split3Loader<BN, NW>, std::conditional_t<B_DIRECT, DirectLoader<SB_T, B_RC && B_DIRECT, BN, BK, NW>, NoLoader>>;
    using SA = std::conditional_t<A_DIRECT, NoLoader, TileLoader<SA_T, CT, A_RC, BM, NT, true, BK>>;
    using SB = std::conditional_t<B_DIRECT, NoLoader, TileLoader<SB_T, CT, B_RC, BN, NT, true, BK>>;
    constexpr bool ANY_STAGED = !A_DIRECT || !B_DIRECT;
    // bytes of one LDS stage / buffer of each operand
    constexpr int A_STRIDE = A_DIRECT ? DA::STAGE_ELEMS * (int)sizeof(SA_T) : LdsTile<CT, A_RC, BM, BK>::elems * (int)sizeof(CT);
    constexpr int B_STRIDE = b_stage_bytes<W3, B_DIRECT, DB, SB_T, LdsTile<CT, B_RC, BN, BK>, CT>();
    constexpr int A_BYTES = (A_DIRECT ? ST : 2) * A_STRIDE, B_BYTES = (B_DIRECT ? ST : 2) * B_STRIDE;
    constexpr int LD_PER_TILE = (A_DIRECT ? DA::NI : 0) + (B_DIRECT ? DB::NI : 0);
    static_assert(A_DIRECT || B_DIRECT, "at least one operand is loaded directly");
    static_assert(!B_SPLIT || (B_DIRECT && B_RC && sizeof(SB_T) == 4 && sizeof(CT) == 2), "two-term feeding: direct r-contiguous fp32 B");
    static_assert(ST >= 2 && (ST - 2) * LD_PER_TILE < 64, "vmcnt range");
    static_assert(!X3 || (A_DIRECT && B_DIRECT && sizeof(SA_T) == 4 && sizeof(SB_T) == 4 && sizeof(CT) == 2 && !B_SPLIT),
                  "three-term feeding: both operands direct fp32, bf16 MFMA");
    static_assert(!W3 || (BK == 16 && MI == 2 && NJ == 2 && NW == 4 && !A_RC), "pre-split B: 128 x 128 tiles of 16 k-values");
    static_assert(A_BYTES % 1024 == 0, "stage addresses stay 1 KB aligned");
    __shared__ __attribute__((aligned(1024))) char ring[A_BYTES + B_BYTES];
    char *const As = ring, *const Bs = ring + A_BYTES;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave / WN) * (32 * MI), wn = (wave % WN) * (32 * NJ);
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

    floatx16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj)
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
        if constexpr (W3) db.init(g.B3, g.ko, g.n_pad, n0, I.k, lane);
        else if constexpr (B_DIRECT) db.init(static_cast<const SB_T *>(g.B), g.ldb, n0, g.N, I.k, wave, lane);
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
            if constexpr (W3) db.issue(b_lds + st * B_STRIDE, wave);
            else if constexpr (B_DIRECT) db.issue_ragged(b_lds + st * B_STRIDE, wave, lane, kv, g.ldb - I.k);
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
                    float a[MI][4], b[NJ][4];
#pragma unroll
                    for (int i = 0; i < MI; ++i) {
                        if constexpr (A_DIRECT) dfrag_f32<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half, a[i]);
                        else frag_f32<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half, a[i]);
                    }
#pragma unroll
                    for (int jj = 0; jj < NJ; ++jj) {
                        if constexpr (B_DIRECT) dfrag_f32<B_RC, BN, BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, b[jj]);
                        else frag_f32<B_RC, BN, BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, b[jj]);
                    }
                    if (ragged) {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (kk + 4 * half + t >= kv) {
#pragma unroll
                                for (int i = 0; i < MI; ++i) a[i][t] = 0.f;
#pragma unroll
                                for (int jj = 0; jj < NJ; ++jj) b[jj][t] = 0.f;
                            }
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int i = 0; i < MI; ++i)
#pragma unroll
                            for (int jj = 0; jj < NJ; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t], b[jj][t], acc[i][jj], 0, 0, 0);
                }
            } else if constexpr (W3) {
                // fp32 A split as its fragments are read, B read as the three terms it was packed into
                if (!ragged) {
                    x3_step_2x2_presplit<A_RC, BM, BN, BK>(reinterpret_cast<const float *>(At), Bt, wm + l32, wn + l32, half, acc);
                } else {
                    union Frag { uint4 u; bf16x8 v; };
                    uint4 a3[2][3];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        float x[8];
                        dfrag_load8<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, 0, half, x);
                        split3_frag<true>(x, 8 * half, kv, a3[i]);
                    }
                    constexpr int TA[6] = {0, 0, 0, 1, 1, 2}, TB[6] = {0, 1, 2, 0, 1, 0}; // the order of x3_step_2x2_presplit
#pragma unroll
                    for (int q = 0; q < 6; ++q)
#pragma unroll
                        for (int i = 0; i < 2; ++i)
#pragma unroll
                            for (int jj = 0; jj < 2; ++jj) {
                                Frag fa, fb;
                                fa.u = a3[i][TA[q]];
                                fb.u = DB::frag(Bt, TB[q], half, wn + jj * 32 + l32);
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, fb.v, acc[i][jj], 0, 0, 0);
                            }
                }
            } else if constexpr (X3 != 0) {
                // fp32 operands, every product as six bf16 terms (split3_pair)
#pragma unroll
                for (int kk = 0; kk < BK; kk += 16) {
                    union Frag { uint4 u; bf16x8 v; };
                    uint4 a3[MI][3], b3[NJ][3];
#pragma unroll
                    for (int i = 0; i < MI; ++i) {
                        float x[8];
                        dfrag_load8<A_RC, BM, BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half, x);
                        if (ragged) split3_frag<true>(x, kk + 8 * half, kv, a3[i]);
                        else split3_frag<false>(x, kk + 8 * half, kv, a3[i]);
                    }
#pragma unroll
                    for (int jj = 0; jj < NJ; ++jj) {
                        float x[8];
                        dfrag_load8<B_RC, BN, BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, x);
                        if (ragged) split3_frag<true>(x, kk + 8 * half, kv, b3[jj]);
                        else split3_frag<false>(x, kk + 8 * half, kv, b3[jj]);
                    }
                    constexpr int TA[6] = {2, 0, 1, 1, 0, 0}, TB[6] = {0, 2, 1, 0, 1, 0}; // smallest products first
#pragma unroll
                    for (int q = 0; q < 6; ++q)
#pragma unroll
                        for (int i = 0; i < MI; ++i)
#pragma unroll
                            for (int jj = 0; jj < NJ; ++jj) {
                                Frag fa, fb;
                                fa.u = a3[i][TA[q]];
                                fb.u = b3[jj][TB[q]];
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, fb.v, acc[i][jj], 0, 0, 0);
                            }
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < BK; kk += 16) {
                    union Frag { uint4 u; bf16x8 v; } a[MI], b[NJ], bl[NJ];
#pragma unroll
                    for (int i = 0; i < MI; ++i) {
                        if constexpr (A_DIRECT && A_RC && sizeof(SA_T) == 2)
                            a[i].u = dfrag_bf16_rc<BM>(reinterpret_cast<const bf16_t *>(At), wm + i * 32 + l32, kk, half);
                        else if constexpr (A_DIRECT && sizeof(SA_T) == 4)
                            a[i].u = dfrag_bf16_from_f32<BK>(reinterpret_cast<const float *>(At), wm + i * 32 + l32, kk, half);
                        else if constexpr (A_DIRECT) a[i].u = dfrag_bf16<BK>(reinterpret_cast<const bf16_t *>(At), wm + i * 32 + l32, kk, half);
                        else a[i].u = frag_bf16<A_RC, BM, BK>(reinterpret_cast<const bf16_t *>(At), wm + i * 32 + l32, kk, half);
                    }
#pragma unroll
                    for (int jj = 0; jj < NJ; ++jj) {
                        if constexpr (B_DIRECT && B_RC && sizeof(SB_T) == 4)
                            b[jj].u = dfrag_bf16_rc_from_f32<BN, B_SPLIT>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half, &bl[jj].u);
                        else if constexpr (B_DIRECT && B_RC)
                            b[jj].u = dfrag_bf16_rc<BN>(reinterpret_cast<const bf16_t *>(Bt), wn + jj * 32 + l32, kk, half);
                        else if constexpr (B_DIRECT && sizeof(SB_T) == 4)
                            b[jj].u = dfrag_bf16_from_f32<BK>(reinterpret_cast<const float *>(Bt), wn + jj * 32 + l32, kk, half);
                        else if constexpr (B_DIRECT) b[jj].u = dfrag_bf16<BK>(reinterpret_cast<const bf16_t *>(Bt), wn + jj * 32 + l32, kk, half);
                        else b[jj].u = frag_bf16<B_RC, BN, BK>(reinterpret_cast<const bf16_t *>(Bt), wn + jj * 32 + l32, kk, half);
                    }
                    if (ragged) {
#pragma unroll
                        for (int i = 0; i < MI; ++i) a[i].u = mask_bf16(a[i].u, kk + 8 * half, kv);
#pragma unroll
                        for (int jj = 0; jj < NJ; ++jj) {
                            b[jj].u = mask_bf16(b[jj].u, kk + 8 * half, kv);
                            if constexpr (B_SPLIT) bl[jj].u = mask_bf16(bl[jj].u, kk + 8 * half, kv);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int jj = 0; jj < NJ; ++jj)
                            acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, b[jj].v, acc[i][jj], 0, 0, 0);
                    if constexpr (B_SPLIT) {
#pragma unroll
                        for (int i = 0; i < MI; ++i)
#pragma unroll
                            for (int jj = 0; jj < NJ; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i].v, bl[jj].v, acc[i][jj], 0, 0, 0);
                    }
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

    barrier_no_drain();     // every wavefront's last fragment reads are done (they fed its last MFMAs)
    static_assert(A_BYTES + B_BYTES >= NW * 8 * (32 * NJ + 4) * 4, "the epilogue strips overlay the ring");
    store_tile<MI, NJ>(p, out_seg, reinterpret_cast<float *>(ring), acc, wave, lane, wm, wn, m0, n0, rows_a, rows_b, split);
}

// ---- host side -------------------------------------------------------------------------------------

template <typename CT, typename SA_T, bool A_RC, bool A_DIRECT, typename SB_T, bool B_RC, bool B_DIRECT, int WN, int BK,
          int ST, int OCC, bool B_SPLIT = false, int MI = 2, int NJ = 2, int WMW = 2, int X3 = 0>
static heta_status launch_direct(GemmParams &p, hipStream_t st, const char *name, double bytes, double flops)
{
    constexpr int BN = 32 * NJ * WN, BM = 32 * MI * WMW;
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
    hipLaunchKernelGGL((gemm_direct_kernel<CT, SA_T, A_RC, A_DIRECT, SB_T, B_RC, B_DIRECT, WN, BK, ST, OCC, B_SPLIT, MI, NJ, WMW, X3>),
                       dim3((unsigned)blocks), dim3(64 * WMW * WN), 0, st, p);
    HETA_LAUNCH_CHECK("gemm_direct_kernel");
    return HETA_OK;
}

// test switch: fp32 products on the fp32 MFMA (32x32x2) instead of as six bf16 terms
bool g_f32_native = false;

bool gemm_direct_small(const GemmParams &p)
{
    if (p.partial) return false;
    int64_t mt = 0, nt = 0;
    for (int s = 0; s < p.n_seg; ++s) {
        mt = std::max(mt, (p.seg[s].M + 127) / 128);
        nt = std::max(nt, (p.seg[s].N + 127) / 128);
    }
    return mt * nt * (p.batch ? p.n_seg : 1) <= 96;
}

static int64_t split3_octets(int64_t K) { return (K + 15) / 16 * 2; }
static int64_t split3_columns(int64_t N) { return (N + 127) / 128 * 128; }
size_t split3_weight_bytes(int64_t K, int64_t N) { return static_cast<size_t>(3 * split3_octets(K) * split3_columns(N) * 16); }

heta_status pack_split3_weights(const float *W, int64_t ldw, int64_t K, int64_t N, int trans, void *out, GemmSeg *seg, hipStream_t st)
{
    const int64_t ko = split3_octets(K), n_pad = split3_columns(N);
    if (K >= (int64_t(1) << 30) || N >= (int64_t(1) << 30) || ko * n_pad >= (int64_t(1) << 31))
        return fail(HETA_ERR_UNSUPPORTED, "projection: weight matrix too large to pack");
    hipLaunchKernelGGL(pack_split3_kernel, dim3((unsigned)((ko * n_pad + 255) / 256)), dim3(256), 0, st, W, ldw, static_cast<int>(K),
                       static_cast<int>(N), trans, static_cast<uint4 *>(out), static_cast<int>(ko), static_cast<int>(n_pad));
    HETA_LAUNCH_CHECK("pack_split3_kernel");
    seg->B3 = out;
    seg->ko = static_cast<int32_t>(ko);
    seg->n_pad = static_cast<int32_t>(n_pad);
    return HETA_OK;
}

// rows of the output tile a weight gradient with more than 128 input and output columns takes: 320 or 256,
// whichever pads the input columns (the tile rows) less over all segments
int wgrad_tile_rows(const GemmParams &p)
{
    int64_t pad320 = 0, pad256 = 0;
    for (int s = 0; s < p.n_seg; ++s) {
        pad320 += (p.seg[s].M + 319) / 320 * 320;
        pad256 += (p.seg[s].M + 255) / 256 * 256;
    }
    return pad256 < pad320 ? 256 : 320;
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
    if (a_dt == HETA_BF16 && b_dt == HETA_F32 && a_rc && b_rc) {
        // The weight gradient with bf16 inputs: both operands lie with the graph rows (the contraction index)
        // outermost and stream into LDS as they are, 16 graph rows per stage, four stages; 128 x 128 output tiles
        // (256 threads, three workgroups per CU); the fp32 gradient operand is rounded, or split into two bf16
        // terms, when its fragments are read.
        *handled = true;
        int64_t m_max = 0;
        for (int s = 0; s < p.n_seg; ++s) m_max = std::max(m_max, p.seg[s].M);
        if (m_max > 128 && n_max > 128) {
            // inputs wider than 128 columns and more than 128 output columns: 320 x 256 tiles (8 wavefronts of 5 x 2
            // accumulators, one workgroup per CU), or 256 x 256 (4 x 2) when that covers the input columns with less
            // padding.  Per MFMA the workgroup loads two thirds of what a 320 x 128 tile loads, and these launches are
            // bound by the loads a CU can keep in flight: 1.52 -> 0.93 ms on 6 x (500 k x 300)^T (500 k x 256).
            if (wgrad_tile_rows(p) == 256)
                return p.split_b ? launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 1, true, 4, 2, 2>(p, st, name, bytes, flops)
                                 : launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 1, false, 4, 2, 2>(p, st, name, bytes, flops);
            return p.split_b ? launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 1, true, 5, 2, 2>(p, st, name, bytes, flops)
                             : launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 1, false, 5, 2, 2>(p, st, name, bytes, flops);
        }
        if (m_max > 128) {
            // inputs wider than 128 columns: 320 x 128 tiles (8 wavefronts of 5 x 1 accumulators), so that up to 320
            // input columns share one pass over the gradient operand, which is the larger of the two
            return p.split_b ? launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 2, true, 5, 1, 2>(p, st, name, bytes, flops)
                             : launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 2, false, 5, 1, 2>(p, st, name, bytes, flops);
        }
        // more than 128 output columns: 128 x 256 tiles (eight wavefronts, two workgroups per CU), so that the gradient
        // rows, the larger operand, are loaded by one workgroup per segment instead of two.  These launches are bound by
        // the load instructions a CU can have in flight, not by HBM bytes: 0.37 -> 0.30 ms on 3 x (700 k x 128)^T (700 k x 256).
        if (n_max > 128)
            return p.split_b ? launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 4, true>(p, st, name, bytes, flops)
                             : launch_direct<bf16_t, bf16_t, true, true, float, true, true, 4, 16, 4, 4, false>(p, st, name, bytes, flops);
        return p.split_b ? launch_direct<bf16_t, bf16_t, true, true, float, true, true, 2, 16, 4, 3, true>(p, st, name, bytes, flops)
                         : launch_direct<bf16_t, bf16_t, true, true, float, true, true, 2, 16, 4, 3, false>(p, st, name, bytes, flops);
    }
    bool wide = n_max > 128;
    if (wide) {
        // A launch of at most one and a half 128 x 256 tiles per CU (the projections of a sampled mini-batch
        // block) runs as one uneven round of workgroups, each a serial chain of k-steps with nothing beside it
        // on its CU: 128 x 128 tiles put the same work on twice the workgroups, two or three to a CU.
        int64_t mt = 0, nt = 0;
        for (int s = 0; s < p.n_seg; ++s) {
            mt = std::max(mt, (p.seg[s].M + BM - 1) / BM);
            nt = std::max(nt, (p.seg[s].N + 255) / 256);
        }
        const int64_t inner = nt * (p.batch ? p.n_seg : 1) * (p.partial ? mt : 1);
        const int64_t outer = p.partial ? std::max(1, p.n_split) : mt;
        if (outer * inner <= 384) wide = false;
    }
    // Fewer than a hundred 128 x 128 tiles (the projections of a sampled mini-batch block: a few thousand rows):
    // every tile is a serial chain of MFMAs on one CU while most CUs idle.  64 x 64 tiles (four wavefronts of one
    // accumulator each) cut the chain to a quarter and put four times as many CUs to work.
    const bool small = gemm_direct_small(p);
    *handled = true;
    if (a_dt == HETA_F32 && b_dt == HETA_F32 && !g_f32_native && !a_rc && !small && !p.partial) {
        // B already packed as three bf16 terms by the caller (the weights of a forward or input-gradient product):
        // half the splitting arithmetic leaves the k loop.  12 KB of B per stage: two workgroups per CU.
        bool packed = true;
        for (int s = 0; s < p.n_seg; ++s) packed = packed && p.seg[s].B3 != nullptr;
        if (packed) return launch_direct<bf16_t, float, false, true, float, false, true, 2, 16, 3, 2, false, 2, 2, 2, 2>(p, st, name, bytes, flops);
    }
    if (a_dt == HETA_F32 && b_dt == HETA_F32 && !g_f32_native) {
        // fp32 operands, fp32-exact products as six bf16 MFMA terms each (see split3_pair), fp32 accumulation
        // 128 x 128 tiles (four wavefronts, three workgroups per CU) also where the output is wider: the
        // 128 x 256 tile's eight wavefronts need more than the 128 registers that two workgroups per CU allow,
        // and with one workgroup per CU nothing runs under its barriers (measured: 0.93 against 1.05 ms)
#define HETA_X32(ARC, BRC)                                                                                                        \
    return small ? launch_direct<bf16_t, float, ARC, true, float, BRC, true, 2, 16, 3, 4, false, 1, 1, 2, 1>(p, st, name, bytes, flops) \
                 : launch_direct<bf16_t, float, ARC, true, float, BRC, true, 2, 16, 3, 3, false, 2, 2, 2, 1>(p, st, name, bytes, flops)
        if (!a_rc && b_rc) { HETA_X32(false, true); }
        if (!a_rc && !b_rc) { HETA_X32(false, false); }
        if (a_rc && b_rc) { HETA_X32(true, true); }
#undef HETA_X32
    }
    if (small) {
        if (a_dt == HETA_F32 && b_dt == HETA_F32 && !a_rc)
            return b_rc ? launch_direct<float, float, false, true, float, true, true, 2, 16, 3, 4, false, 1, 1, 2>(p, st, name, bytes, flops)
                        : launch_direct<float, float, false, true, float, false, true, 2, 16, 3, 4, false, 1, 1, 2>(p, st, name, bytes, flops);
        if (a_dt == HETA_BF16 && b_dt == HETA_BF16 && !a_rc && b_rc)
            return launch_direct<bf16_t, bf16_t, false, true, bf16_t, true, true, 2, 32, 3, 4, false, 1, 1, 2>(p, st, name, bytes, flops);
        if (a_dt == HETA_F32 && b_dt == HETA_BF16 && !a_rc && !b_rc)
            return launch_direct<bf16_t, float, false, true, bf16_t, false, true, 2, 32, 3, 4, false, 1, 1, 2>(p, st, name, bytes, flops);
    }
    if (a_dt == HETA_F32 && b_dt == HETA_F32) {
#define HETA_D32(ARC, BRC)                                                                                          \
    return wide ? launch_direct<float, float, ARC, true, float, BRC, true, 4, 16, 3, 4>(p, st, name, bytes, flops)   \
                : launch_direct<float, float, ARC, true, float, BRC, true, 2, 16, 3, 3>(p, st, name, bytes, flops)
        if (!a_rc && b_rc) { HETA_D32(false, true); }
        if (!a_rc && !b_rc) { HETA_D32(false, false); }
        if (a_rc && b_rc) { HETA_D32(true, true); }
#undef HETA_D32
    }
    if (a_dt == HETA_BF16 && b_dt == HETA_BF16 && !a_rc && b_rc) { // forward: M_r (bf16) x W_r (bf16, n-contiguous, as it lies in memory)
        return wide ? launch_direct<bf16_t, bf16_t, false, true, bf16_t, true, true, 4, 32, 3, 4>(p, st, name, bytes, flops)
                    : launch_direct<bf16_t, bf16_t, false, true, bf16_t, true, true, 2, 32, 3, 3>(p, st, name, bytes, flops);
    }
    if (a_dt == HETA_F32 && b_dt == HETA_BF16 && !a_rc && !b_rc) { // backward: G (fp32, rounded at the MFMA) x W_r^T (bf16, k-contiguous)
        // (256 output columns: 16 k-values per stage keep the fp32 tiles of A small enough for two workgroups per CU)
        if (n_max > 256 && n_max <= 320) {
            // 320 output columns in one tile (wavefronts of MI x 5 accumulators): the fp32 rows of A are read once.  256 rows
            // per tile (one workgroup per CU) where the launch still fills the chip several times: W_r^T, re-read by every
            // workgroup, is then loaded once per 256 rows (1.25 -> 0.92 ms on 6 x (500 k x 256)(256 x 300)); else 128 rows.
            int64_t m_all = 0;
            for (int s = 0; s < p.n_seg; ++s) m_all = std::max(m_all, p.seg[s].M);
            if (m_all >= 256 * 1024)
                return launch_direct<bf16_t, float, false, true, bf16_t, false, true, 2, 16, 4, 1, false, 2, 5, 4>(p, st, name, bytes, flops);
            return launch_direct<bf16_t, float, false, true, bf16_t, false, true, 2, 16, 4, 2, false, 1, 5, 4>(p, st, name, bytes, flops);
        }
        return wide ? launch_direct<bf16_t, float, false, true, bf16_t, false, true, 4, 16, 4, 4>(p, st, name, bytes, flops)
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
