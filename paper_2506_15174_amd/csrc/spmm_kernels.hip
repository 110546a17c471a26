// gfx950 executor: C <- A x B over the chunked, schedule-ordered arrays built by
// the inspector (paper Section 3.3 "Sparse Coarsen", Listings 5-7, re-derived
// for wave64 and for the memory paths of a CDNA4 compute unit).
//
// One wave executes one row group; 8 waves form a workgroup, and the register
// budget of an instance (128 / 80 / 64 VGPRs for 2 / 4 / 8 slices) lets two to
// four workgroups share a compute unit.
//
//   * Lanes run along j, the columns of B and C (the paper's map(j, .),
//     Listing 5).  A vector load costs the compute unit's address path the same
//     ~16 cycles whether a lane asks for 4, 8 or 16 bytes, so every lane asks for
//     16 (four columns).  A column tile of 128 / 64 / 32 columns then needs only
//     32 / 16 / 8 lanes, and the wave is cut into S = 2 / 4 / 8 *slices* that work
//     on different enumerated columns of the same chunk (the paper's map(k, .)
//     inside a warp, Section 3.3.1); their partial tiles are added across lanes
//     when a panel ends (the warp-level reduction of Section 3.3.2).
//   * The UFI x 4 accumulators of a panel stay in VGPRs across all chunks of the
//     panel (the paper's register tile, Listing 6).
//   * A chunk is UFKT = 8 (16, 32, 64 in plans made for narrow B) enumerated
//     columns of one nonzero pattern (or leftovers of several patterns under the
//     union of their patterns, with zeros where a column lacks a row).  Its column
//     indices and values are staged through LDS, a window of the group's stream at
//     a time, with coalesced 16-byte loads (the scalar data path tops out far below
//     what the stream needs); a slice reads its own slots back with one broadcast
//     LDS read per row of the pattern.  The one-word chunk header comes from the
//     same window: its pattern selects, with wave-uniform branches,
//     which of the UFI row blocks run, so no lane ever tests a sparsity condition
//     (Section 3.2.2: enumerated blocks carry no conditionals).  No scalar load
//     sits inside the chunk loop, so its LDS waits are counted, not drained.
//   * The chunk loop is software-pipelined D chunks deep (the paper's
//     unroll(k, UFk) for loads in flight, Section 3.3.2): while chunk c is
//     multiplied the B rows of chunks c+1 .. c+D-1 are in flight.
//   * Pieces of a panel that was too heavy for one wave sit in one workgroup:
//     they park their partial tiles in LDS, meet at one barrier and one wave per
//     tile row adds the pieces in piece order (the write-after-write hazard of
//     Section 3.3.2, solved without atomics and with a fixed summation order).
//     A panel too heavy even for one workgroup is cut across several: each parks
//     the sum of its pieces in a scratch slot and spmm_cross_combine_kernel, a
//     second launch, adds the slots in workgroup order.
//   * A plan cut along K (a column tile of B larger than one XCD's L2) holds every
//     row once per column range; workgroup b of the launch works on range
//     b mod k_slices, so that the XCDs, which receive the workgroups in turn, each
//     gather from one range of B.  The kernel is the same: it writes the ranges'
//     partial rows of C to a buffer and spmm_kslice_combine_kernel adds them in
//     range order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "spmm_format.h"
#include "spmm_kernels.h"

using namespace spmm_fmt;

namespace {

// Scalar (wave-uniform) view of read-only plan memory: loads through this
// address space are issued as s_load_* when the address is uniform.
typedef const uint32_t __attribute__((address_space(4))) cword_t;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int VW> struct Vec;
template <> struct Vec<1> {
    typedef float type;
    static __device__ __forceinline__ type zero() { return 0.0f; }
};
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <> struct Vec<4> {
    typedef f32x4_t type;
    static __device__ __forceinline__ type zero() { return type{0.f, 0.f, 0.f, 0.f}; }
};

__device__ __forceinline__ void fma_acc(float &acc, float a, float b) { acc = __builtin_fmaf(a, b, acc); }
__device__ __forceinline__ void fma_acc(f32x4_t &acc, float a, const f32x4_t &b)
{
    acc[0] = __builtin_fmaf(a, b[0], acc[0]);
    acc[1] = __builtin_fmaf(a, b[1], acc[1]);
    acc[2] = __builtin_fmaf(a, b[2], acc[2]);
    acc[3] = __builtin_fmaf(a, b[3], acc[3]);
}
// Stores of a lane's columns to C: rows of C are only 4-byte aligned in general, and
// the last lane of a tile may own fewer than four columns.
typedef float f32x4_unaligned_t __attribute__((ext_vector_type(4), aligned(4)));
__device__ __forceinline__ void store_cols(float *p, float v, int) { *p = v; }
__device__ __forceinline__ void store_cols(float *p, const f32x4_t &v, int valid)
{
    if (valid >= 4) {
        *reinterpret_cast<f32x4_unaligned_t *>(p) = v;
    } else {
        p[0] = v[0];
        if (valid > 1) p[1] = v[1];
        if (valid > 2) p[2] = v[2];
    }
}
__device__ __forceinline__ void add_to(float &a, float b) { a += b; }
__device__ __forceinline__ void add_to(f32x4_t &a, const f32x4_t &b) { a += b; }
template <int MASK> __device__ __forceinline__ void add_across(float &a) { a += __shfl_xor(a, MASK); }
template <int MASK> __device__ __forceinline__ void add_across(f32x4_t &a)
{
    a[0] += __shfl_xor(a[0], MASK);
    a[1] += __shfl_xor(a[1], MASK);
    a[2] += __shfl_xor(a[2], MASK);
    a[3] += __shfl_xor(a[3], MASK);
}

// In-place addition of the slices' partial tiles across lanes.  A wave of S slices holds,
// per tile row, four accumulators x0 .. x3 per lane (columns 4 sl + v of the tile, sl the
// lane's place inside its slice of 64 / S lanes); the sum over the slices of column
// 4 sl + v is wanted.  Slices are lane groups, so the sum runs over the lane bits above the
// slice width:
//   * bits inside a row of 16 lanes (8 and more slices): x += x rotated by 8 (4, 2, 1)
//     lanes within the row, one DPP add per stage and register; every lane of a residue
//     class then holds the class's sum;
//   * bit 4 (four and more slices): the row swap (odd rows of one register against even
//     rows of another) followed by one add turns two registers into one whose lane rows
//     hold [a0 + a1, b0 + b1, a2 + a3, b2 + b3];
//   * bit 5: the half swap (upper half of one register against the lower half of another)
//     and one add turn two registers into one holding [a_lo + a_hi | b_lo + b_hi].
// Two registers become one per swap stage, so the adds halve from stage to stage and no
// stage needs a temporary per accumulator: the exchange through __shfl_xor cost 16 to 35
// registers on top of the tile and the B rows in flight, which is what capped the pipeline
// depth of the tall-panel instances.
// Result: four and more slices: `lo` of lane l is the sum of column 4 sl + l / 16 (sl = l % L
// for the lanes with l % 16 < L); two slices: `lo`, `hi` of lane l are the sums of columns
// 4 (l % 32) + 2 (l / 32) and the next one.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_unaligned_t __attribute__((ext_vector_type(2), aligned(4)));
__device__ __forceinline__ float swap32_add(float a, float b)
{
    const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap16_add(float a, float b)
{
    const u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <int ROR> __device__ __forceinline__ float ror_add(float a)
{
    return a + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(a), 0x120 | ROR, 0xF, 0xF, false));
}
template <int S> __device__ __forceinline__ void fold_row(const f32x4_t &x, float &lo, float &hi)
{
    float x0 = x[0], x1 = x[1], x2 = x[2], x3 = x[3];
    if constexpr (S >= 8) { x0 = ror_add<8>(x0); x1 = ror_add<8>(x1); x2 = ror_add<8>(x2); x3 = ror_add<8>(x3); }
    if constexpr (S >= 16) { x0 = ror_add<4>(x0); x1 = ror_add<4>(x1); x2 = ror_add<4>(x2); x3 = ror_add<4>(x3); }
    if constexpr (S >= 32) { x0 = ror_add<2>(x0); x1 = ror_add<2>(x1); x2 = ror_add<2>(x2); x3 = ror_add<2>(x3); }
    if constexpr (S >= 64) { x0 = ror_add<1>(x0); x1 = ror_add<1>(x1); x2 = ror_add<1>(x2); x3 = ror_add<1>(x3); }
    if constexpr (S >= 4) {
        const float a = swap16_add(x0, x1);   // lane rows: [x0, x1, x0, x1] summed over the row pairs
        const float b = swap16_add(x2, x3);   //            [x2, x3, x2, x3]
        lo = swap32_add(a, b);                // lane rows: [x0, x1 | x2, x3] summed over all slices
        hi = 0.0f;
    } else {
        lo = swap32_add(x0, x2);              // halves: [x0 | x2]
        hi = swap32_add(x1, x3);              //         [x1 | x3]
    }
}
// Tile column whose sum lane l holds after fold_row, and whether lane l is the one that stores it.
template <int S> __device__ __forceinline__ int fold_col(int l)
{
    if constexpr (S >= 4) return 4 * (l % (64 / S)) + l / 16;
    else return 4 * (l % 32) + 2 * (l / 32);
}
template <int S> __device__ __forceinline__ bool fold_owner(int l)
{
    if constexpr (S > 4) return (l % 16) < 64 / S;
    else return true;
}

// Source of B rows.  Narrow: a raw buffer descriptor over the column tile's
// bytes (hardware range check, 32-bit per-lane byte offset).  Wide: plain 64-bit
// addressing for B beyond the narrow limits.
//
// The loads are issued from inline assembly and their completion is awaited
// with explicit s_waitcnt vmcnt(n) (wait_for below): the compiler's own wait
// insertion treats every load that is still in flight at a loop back edge as if
// it were the newest one, which would drain the software pipeline once per trip.
// Vector memory operations complete in issue order, so "at most n younger
// operations outstanding" is a sufficient condition whatever else (stores of C,
// window staging) the compiler has in flight.
template <bool WIDE> struct BSource;

template <> struct BSource<false> {
    u32x4 rsrc;
    __device__ __forceinline__ void init(const float *B, uint32_t n_bytes)
    {
        const uint64_t p = reinterpret_cast<uint64_t>(B);
        rsrc[0] = (uint32_t)p;
        rsrc[1] = (uint32_t)(p >> 32) & 0xFFFFu;  // 48-bit base, stride 0
        rsrc[2] = n_bytes;                        // raw buffer: range in bytes
        rsrc[3] = 0x00020000u;                    // 32-bit data format, untyped
        // the descriptor must live in SGPRs
        rsrc[0] = __builtin_amdgcn_readfirstlane(rsrc[0]);
        rsrc[1] = __builtin_amdgcn_readfirstlane(rsrc[1]);
        rsrc[2] = __builtin_amdgcn_readfirstlane(rsrc[2]);
        rsrc[3] = __builtin_amdgcn_readfirstlane(rsrc[3]);
    }
    // byte offset of a lane's segment: row pitch and column index both below 2^24
    static __device__ __forceinline__ uint32_t offset(uint32_t col, uint32_t ld_bytes, uint32_t lane_off)
    {
        return __umul24(col, ld_bytes) + lane_off;
    }
    typedef uint32_t off_t;
    __device__ __forceinline__ void load(float &dst, uint32_t off) const
    {
        asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "=v"(dst) : "v"(off), "s"(rsrc));
    }
    __device__ __forceinline__ void load(f32x4_t &dst, uint32_t off) const
    {
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(off), "s"(rsrc));
    }
};

template <> struct BSource<true> {
    const char *base;
    __device__ __forceinline__ void init(const float *B, uint32_t) { base = reinterpret_cast<const char *>(B); }
    static __device__ __forceinline__ uint64_t offset(uint32_t col, uint32_t ld_bytes, uint32_t lane_off)
    {
        return (uint64_t)col * (uint64_t)ld_bytes + lane_off;
    }
    typedef uint64_t off_t;
    __device__ __forceinline__ void load(float &dst, uint64_t off) const
    {
        const char *p = base + off;
        asm volatile("global_load_dword %0, %1, off" : "=v"(dst) : "v"(p));
    }
    __device__ __forceinline__ void load(f32x4_t &dst, uint64_t off) const
    {
        const char *p = base + off;
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p));
    }
};

// Blocks until at most N vector memory operations younger than the Q loads of
// `b` are outstanding, and tells the compiler that `b` is defined from here on.
template <int N, typename T, int Q> __device__ __forceinline__ void wait_for(T (&b)[Q])
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    if constexpr (Q == 8)
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
                     : "n"(N));
    else if constexpr (Q == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]) : "n"(N));
    else if constexpr (Q == 2)
        asm volatile("s_waitcnt vmcnt(%2)" : "+v"(b[0]), "+v"(b[1]) : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(b[0]) : "n"(N));
}

// Q consecutive words of this wave's LDS window, starting at word `at`.
template <int Q> __device__ __forceinline__ void lds_read(uint32_t (&out)[Q], const uint32_t *win, uint32_t at)
{
    if constexpr (Q == 8) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(win + at);
        const uint4 hi = *reinterpret_cast<const uint4 *>(win + at + 4);
        out[0] = lo.x; out[1] = lo.y; out[2] = lo.z; out[3] = lo.w;
        out[4] = hi.x; out[5] = hi.y; out[6] = hi.z; out[7] = hi.w;
    } else if constexpr (Q == 4) {
        const uint4 v = *reinterpret_cast<const uint4 *>(win + at);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else if constexpr (Q == 2) {
        const uint2 v = *reinterpret_cast<const uint2 *>(win + at);
        out[0] = v.x; out[1] = v.y;
    } else {
        out[0] = win[at];
    }
}

// Word of a slice's value block for row r of a chunk with the given pattern whose
// blocks start at `at`: the block index is the number of pattern rows below r.
// Clamped to `limit` so that the request stays inside the wave's window for rows
// the pattern does not hold.
template <int UFKT> __device__ __forceinline__ uint32_t value_block(uint32_t at, uint32_t pattern, int r, uint32_t limit)
{
    const uint32_t w = at + (uint32_t)UFKT * (uint32_t)__builtin_popcount(pattern & ((1u << r) - 1u));
    return w < limit ? w : limit;
}

// UFI   rows per panel (1, 2, 4, 8): height of the register tile
// S     slices per wave (1, 2, 4, 8; 16, 32, 64 for narrow B); a slice has 64 / S lanes and UFKT / S column slots per chunk
// UFKT  enumerated columns per chunk of the plan (8; 16, 32, 64 in plans made for narrow B)
// VW    columns per lane (4 with 16-byte loads; 1 for the generic path, S == 1 only)
// D     chunks of B rows in flight per wave
// WIDE  64-bit addressing of B
// Waves per SIMD the register budget of an instance is sized for.  Narrow slices
// keep few B rows in flight per wave and walk a long dependent chain per chunk
// (header, row branches, LDS reads), so they need more resident waves to cover
// it: 8 (64 VGPRs) with eight slices, 6 (80 VGPRs) with four, 4 (128 VGPRs)
// with two.  The eight-row tile alone is 32 registers: 4 waves whatever the slices
// (sized for 6, the eight-slice instance spilled 68 registers and ran 10-28 % slower).
// Waves per SIMD an instance is compiled for (its register budget: 512 / waves).  Measured on
// the pruned-layer shapes with every depth forced: past two or three chunks in flight a deeper
// pipeline buys nothing (the memory path, not the number of requests a wave has outstanding,
// paces the gather), while every further resident wave hides more of the chunk's dependent
// chain (header, row branches, value reads).  So each instance takes the shallowest pipeline
// that keeps the loads flowing and the occupancy its tile allows: eight-row tiles 4 waves
// (6 on four slices), four-row tiles 4 waves on two slices and 8 otherwise, shorter tiles 6 to
// 8.  Wider chunks (UFKT > 8) give a slice two column slots per chunk: 6 waves (4 with eight
// rows); windows of 2048 words (UFKT >= 32) cap a compute unit at two workgroups.
// Every budget is one the instance fits without spilling (the build checks it): a spilled
// register could be the destination of a B row still in flight.  64-bit addressing costs a
// register more per column slot, so those instances get the budget of two waves fewer.
constexpr int waves_per_simd(int S, int UFI, int UFKT, bool WIDE)
{
    const int narrow = UFKT >= 32  ? 4
                       : UFKT == 16 ? (UFI > 4 ? 4 : 6)
                       : S == 1     ? 4
                       : UFI == 8   ? (S == 2 ? 4 : 6)
                       : UFI == 4   ? (S == 2 ? 4 : 8)
                       : UFI == 2   ? (S == 2 ? 6 : 8)
                                    : 8;
    return WIDE ? (narrow > 4 ? narrow - 2 : 2) : narrow;
}

// PROBE instances request and await every B row exactly as the product does but skip the
// value reads and the multiply-adds (C becomes all zeros): the time of such a launch is the
// on-chip gather ceiling of the plan's own index stream.
template <int UFI, int S, int VW, int D, bool WIDE, int UFKT = UFK, bool PROBE = false>
__global__ __launch_bounds__(64 * WAVES_PER_WG, (waves_per_simd(S, UFI, UFKT, WIDE))) void
spmm_chunks_kernel(const uint32_t *__restrict__ stream_g,
                   const uint32_t *__restrict__ wins_g, const uint32_t *__restrict__ items_g,
                   const uint32_t *__restrict__ rowmap_g, const float *__restrict__ B_all, uint32_t b_bytes_all,
                   float *__restrict__ C_all, int32_t ldn, int32_t ldc, int32_t width_all, int32_t tile_cols, uint32_t col_mask,
                   float *__restrict__ cross_sums, uint32_t n_cross_slots)
{
    // blockIdx.y: the column tile this workgroup computes (tiles of tile_cols columns of
    // the width_all columns of this launch; the last one may be narrower).  Workgroups
    // are started tile by tile, so a tile begins while the previous one drains.
    const int32_t col0 = (int32_t)blockIdx.y * tile_cols;
    const float *__restrict__ B = B_all + col0;
    float *__restrict__ C = C_all + col0;
    const int32_t width = width_all - col0 < tile_cols ? width_all - col0 : tile_cols;
    const uint32_t b_bytes = b_bytes_all > (uint32_t)col0 * 4u ? b_bytes_all - (uint32_t)col0 * 4u : 0u;

    typedef typename Vec<VW>::type vec_t;
    typedef typename BSource<WIDE>::off_t off_t;
    constexpr int L = 64 / S;    // lanes per slice
    constexpr int Q = UFKT / S;  // column slots per slice and chunk
    constexpr int WINW = win_words(UFKT);
    static_assert(UFKT % S == 0 && VW * L * UFI * 4 <= WINW * 4, "tile must fit the wave's window");
    static_assert(D <= lookahead(UFKT), "the inspector keeps so many chunks of column slots inside every window");

    // Per wave: the staged window of its stream; later the partial tile of a split panel.
    __shared__ __attribute__((aligned(16))) uint32_t lds[WAVES_PER_WG][WINW];

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const int slice = lane / L;
    const int sl = lane % L;
    cword_t *it = (cword_t *)(items_g) + ((size_t)blockIdx.x * WAVES_PER_WG + wave) * ITEM_WORDS;
    const uint32_t flags = it[IT_FLAGS];
    const uint32_t n_wins = it[IT_NWINS];
    uint32_t *win = lds[wave];

    // Column index of a column word.  The top byte may hold a slot pattern (shared
    // leftover chunks); the 24-bit multiply of the narrow path ignores it anyway.
    auto col_index = [&](uint32_t word) -> uint32_t { return WIDE ? (word & col_mask) : word; };

    // Lanes beyond the tile width compute on the tile's first columns and store
    // nothing: no divergent control flow in the hot loop, no out-of-range access.
    // The last active lane may own fewer than VW columns: it loads past the end of
    // its rows of B (the next row, or zeros past the end of B through the buffer
    // descriptor's range check) and stores only its own columns.
    const int valid = width - sl * VW;  // columns of C this lane owns (all VW when larger)
    const bool active = valid > 0;

    if (n_wins != 0) {
        uint32_t row = it[IT_ROW0];
        uint32_t rows_left = it[IT_NROWS];
        cword_t *wins = (cword_t *)(wins_g) + it[IT_WIN0];
        const uint32_t *stream = stream_g + (size_t)it[IT_STREAM0];
        const uint32_t ld_bytes = (uint32_t)ldn * 4u;
        const uint32_t lane_off = active ? (uint32_t)(sl * VW * 4) : 0u;
        const uint32_t slot0 = (uint32_t)(slice * Q);  // this slice's first column slot
        BSource<WIDE> src;
        src.init(B, b_bytes);

        vec_t acc[UFI];
#pragma unroll
        for (int r = 0; r < UFI; ++r) acc[r] = Vec<VW>::zero();

        uint32_t wd_next = it[IT_WIN_FIRST];
        for (uint32_t w = 0; w < n_wins; ++w) {
            const uint32_t wd = wd_next;
            if (w + 1 < n_wins) wd_next = wins[w + 1];  // in flight while this window is consumed
            const uint32_t wc = wd & 0xFFFFu;   // chunks in this window
            const uint32_t ww = wd >> 16;       // words in this window
            // ---- stage the window (the wave's LDS traffic is in order: no wait needed
            //      between these writes and the reads below)
            for (uint32_t i = (uint32_t)lane * 4u; i < ww; i += 256u)
                *reinterpret_cast<uint4 *>(win + i) = *reinterpret_cast<const uint4 *>(stream + i);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

            // ---- pipeline over the window's chunks.  Window layout: headers
            //      (padded to 8 words), UFKT column words per chunk, then the value
            //      blocks back to back.
            const uint32_t cols_base = ((wc + 7u) & ~7u) + slot0;
            uint32_t at_val = ((wc + 7u) & ~7u) + wc * (uint32_t)UFKT + slot0;  // values of the chunk multiplied next
            vec_t b[D][Q];
            off_t voff[Q];
#pragma unroll
            for (int j = 0; j < D - 1; ++j) {
                uint32_t cv[Q];
                lds_read<Q>(cv, win, cols_base + (uint32_t)(j * UFKT));
                const uint32_t ld_eff = (uint32_t)j < wc ? ld_bytes : 0u;
#pragma unroll
                for (int q = 0; q < Q; ++q) src.load(b[j][q], BSource<WIDE>::offset(col_index(cv[q]), ld_eff, lane_off));
            }
            {
                uint32_t cv[Q];
                lds_read<Q>(cv, win, cols_base + (uint32_t)((D - 1) * UFKT));
                const uint32_t ld_eff = (uint32_t)(D - 1) < wc ? ld_bytes : 0u;
#pragma unroll
                for (int q = 0; q < Q; ++q) voff[q] = BSource<WIDE>::offset(col_index(cv[q]), ld_eff, lane_off);
            }
            // last word a slice may start a value read at (blocks are requested for
            // every row of the tile; those of rows outside the pattern are clamped
            // into the window and never used)
            const uint32_t val_limit = (uint32_t)(WINW - UFKT) + slot0;
            uint32_t h_next = win[0];  // header of the chunk multiplied in the next step (same in all lanes)
            uint32_t c = 0;
            bool more = true;
            while (more) {
#pragma unroll
                for (int s = 0; s < D; ++s) {
                    // step for chunk c (c % D == s): voff holds the offsets of chunk c+D-1
#pragma unroll
                    for (int q = 0; q < Q; ++q) src.load(b[(s + D - 1) % D][q], voff[q]);
                    // columns of chunk c+D for the next step; a chunk past the window's
                    // end reads row 0 through a zero pitch (its columns are never used)
                    uint32_t cv[Q];
                    lds_read<Q>(cv, win, cols_base + (c + (uint32_t)D) * (uint32_t)UFKT);
                    const uint32_t ld_next = c + (uint32_t)D < wc ? ld_bytes : 0u;
                    const uint32_t h_now = __builtin_amdgcn_readfirstlane(h_next);
                    h_next = win[c + 1];

                    // the enumerated block of chunk c (paper Listing 7); its B rows are
                    // older than the (D - 1) * Q loads issued since
                    const uint32_t pattern = h_now & HDR_PATTERN_MASK;
                    if constexpr (PROBE) {
                        wait_for<(D - 1) * Q>(b[s]);
                    } else if constexpr (S <= 2 && UFI <= 4) {
                        // wide slices: request the value blocks of all UFI rows before
                        // the wait for the B rows (blocks of rows outside the pattern
                        // are never used), so the LDS latency hides behind it
                        uint32_t a[UFI][Q];
#pragma unroll
                        for (int r = 0; r < UFI; ++r) lds_read<Q>(a[r], win, value_block<UFKT>(at_val, pattern, r, val_limit));
                        at_val += (uint32_t)UFKT * (uint32_t)__builtin_popcount(pattern);
                        wait_for<(D - 1) * Q>(b[s]);
#pragma unroll
                        for (int r = 0; r < UFI; ++r) {
                            if (pattern & (1u << r)) {
#pragma unroll
                                for (int q = 0; q < Q; ++q) fma_acc(acc[r], __uint_as_float(a[r][q]), b[s][q]);
                            }
                        }
                    } else {
                        // narrow slices, tall panels, generic tiles: one LDS read per row
                        // of the pattern
                        wait_for<(D - 1) * Q>(b[s]);
#pragma unroll
                        for (int r = 0; r < UFI; ++r) {
                            if (pattern & (1u << r)) {
                                uint32_t a[Q];
                                lds_read<Q>(a, win, at_val);
#pragma unroll
                                for (int q = 0; q < Q; ++q) fma_acc(acc[r], __uint_as_float(a[q]), b[s][q]);
                                at_val += (uint32_t)UFKT;
                            }
                        }
                    }

#pragma unroll
                    for (int q = 0; q < Q; ++q) voff[q] = BSource<WIDE>::offset(col_index(cv[q]), ld_next, lane_off);

                    if (__builtin_expect((h_now & HDR_END_PANEL) != 0, 0)) {
                        const uint32_t rows_here = rows_left < (uint32_t)UFI ? rows_left : (uint32_t)UFI;
                        // The lane's place in the wave is worked out afresh here (an opaque lane
                        // count the compiler cannot hoist), so that no lane constant but the byte
                        // offset of the loads stays in a register across the chunk loop.
                        int lane_now;
                        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_now));
                        if constexpr (VW == 4 && S >= 2) {
                            // The slices' partial tiles are added across lanes in place (fold_row):
                            // afterwards lane l holds, per tile row, the sum of column fold_col(l)
                            // (two adjacent columns when the wave has two slices).
                            const int col = fold_col<S>(lane_now);
                            const bool owner = fold_owner<S>(lane_now);
                            cword_t *map = rowmap_g ? (cword_t *)(rowmap_g) + row : nullptr;
#pragma unroll
                            for (int r = 0; r < UFI; ++r) {
                                float lo, hi;
                                fold_row<S>(acc[r], lo, hi);
                                if (flags & FLAG_SPLIT) {
                                    // the window is dead by now (a piece ends with its panel)
                                    if (owner) {
                                        if constexpr (S == 2) *reinterpret_cast<float2 *>(win + r * L * VW + col) = float2{lo, hi};
                                        else win[r * L * VW + col] = __float_as_uint(lo);
                                    }
                                } else if ((uint32_t)r < rows_here && owner && col < width) {
                                    // rows sorted by length: the plan's row `row + r` is another row of C
                                    const size_t c_row = map ? (size_t)map[r] : (size_t)row + (size_t)r;
                                    float *dst = C + c_row * (size_t)ldc + col;
                                    if constexpr (S == 2) {
                                        if (col + 1 < width) *reinterpret_cast<f32x2_unaligned_t *>(dst) = f32x2_unaligned_t{lo, hi};
                                        else *dst = lo;
                                    } else {
                                        *dst = lo;
                                    }
                                }
                            }
                        } else {
                        // one column per lane, one slice: nothing to add across lanes
                        const int sl_now = lane_now % L;
                        const int valid_now = width - sl_now * VW;
                        if (lane_now < L) {   // slice 0 holds the sums
                            if (flags & FLAG_SPLIT) {
                                // the window is dead by now (a piece ends with its panel)
#pragma unroll
                                for (int r = 0; r < UFI; ++r)
                                    *reinterpret_cast<vec_t *>(win + (r * L + sl_now) * VW) = acc[r];
                            } else if (valid_now > 0) {
                                if (rowmap_g) {
                                    // rows sorted by length: the plan's row `row + r` is another row of C
                                    cword_t *map = (cword_t *)(rowmap_g) + row;
#pragma unroll
                                    for (int r = 0; r < UFI; ++r)
                                        if ((uint32_t)r < rows_here)
                                            store_cols(C + (size_t)map[r] * (size_t)ldc + sl_now * VW, acc[r], valid_now);
                                } else {
                                    float *c_panel = C + (size_t)row * (size_t)ldc + sl_now * VW;
#pragma unroll
                                    for (int r = 0; r < UFI; ++r)
                                        if ((uint32_t)r < rows_here) store_cols(c_panel + (size_t)r * ldc, acc[r], valid_now);
                                }
                            }
                        }
                        }
                        row += rows_here;
                        rows_left -= rows_here;
#pragma unroll
                        for (int r = 0; r < UFI; ++r) acc[r] = Vec<VW>::zero();
                    }
                    if (++c >= wc) {
                        more = false;
                        break;
                    }
                }
            }
            // The look-ahead loads of chunks past the window's end are still in
            // flight into registers the compiler considers free from here on.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            stream += ww;
        }
    }

    if (flags & FLAG_SYNC) {
        // Every wave of a block with split panels arrives here exactly once.
        __syncthreads();
        const uint32_t nseg = it[IT_RED_NSEG];
        const bool adds = nseg != 0 && slice == 0 && active;
        vec_t sum = Vec<VW>::zero();
        if (adds) {
            const uint32_t first = it[IT_RED_SLOT0];
            const uint32_t r = it[IT_RED_R];
            for (uint32_t p = 0; p < nseg; ++p)
                add_to(sum, *reinterpret_cast<const vec_t *>(&lds[first + p][(r * L + sl) * VW]));
        }
        if (!(flags & FLAG_CROSS)) {
            if (adds) store_cols(C + (size_t)it[IT_RED_ROW] * (size_t)ldc + sl * VW, sum, valid);
        } else if (adds) {
            // The panel is cut across several blocks: each parks the sums of its pieces in
            // its scratch slot; spmm_cross_combine_kernel, enqueued behind this launch, adds the
            // slots in block order and writes C.
            const size_t base = (size_t)blockIdx.y * n_cross_slots + it[IT_X_SLOT0] + it[IT_X_PART];
            float *slot = cross_sums + base * (size_t)(UFI * CROSS_ROW_FLOATS);
            *reinterpret_cast<vec_t *>(slot + it[IT_RED_R] * (uint32_t)CROSS_ROW_FLOATS + (uint32_t)(sl * VW)) = sum;
        }
    }
}

// Second step of panels cut across workgroups: block (x, y) adds, for panel x and column
// tile y of the launch before it, the sums its workgroups parked in their scratch slots, in
// workgroup order (so the result does not depend on how the launch was scheduled), and
// writes the panel's rows of C.  Thread t owns row t / 32 of the tile and its columns
// 4 (t % 32) .. + 3.  The kernel boundary makes the first step's stores visible: no fences,
// no counters, nothing to clear between launches.
__global__ __launch_bounds__(256) void
spmm_cross_combine_kernel(const uint32_t *__restrict__ table, const float *__restrict__ sums, uint32_t n_cross_slots,
                          int32_t ufi, float *__restrict__ C_all, int32_t ldc, int32_t width_all, int32_t tile_cols)
{
    const uint32_t *e = table + (size_t)blockIdx.x * CROSS_ENTRY_WORDS;
    const uint32_t slot0 = e[CE_SLOT0], nparts = e[CE_NPARTS], nrows = e[CE_NROWS];
    const uint32_t r = threadIdx.x / 32u;
    const int32_t c = (int32_t)(threadIdx.x % 32u) * 4;
    const int32_t col0 = (int32_t)blockIdx.y * tile_cols;
    const int32_t width = width_all - col0 < tile_cols ? width_all - col0 : tile_cols;
    if (r >= nrows || c >= width) return;
    const size_t slot_floats = (size_t)ufi * CROSS_ROW_FLOATS;
    const float *s = sums + ((size_t)blockIdx.y * n_cross_slots + slot0) * slot_floats + r * (uint32_t)CROSS_ROW_FLOATS + c;
    f32x4_t total = Vec<4>::zero();
    for (uint32_t p = 0; p < nparts; ++p) total += *reinterpret_cast<const f32x4_t *>(s + (size_t)p * slot_floats);
    store_cols(C_all + (size_t)e[CE_ROW0 + r] * (size_t)ldc + col0 + c, total, width - c);
}

// Last step of a plan cut along K: C = sum over the slices, in slice order, of the rows the
// main launch (and the step above) wrote to the slices' buffer: slice s of row i at row
// s * slice_rows + i, `ldp` floats per row.  Thread t of block b owns four columns of one row.
__global__ __launch_bounds__(256) void
spmm_kslice_combine_kernel(const float *__restrict__ sums, int32_t k_slices, uint32_t slice_rows, int32_t ldp,
                           float *__restrict__ C, int32_t ldc, uint32_t M, int32_t width)
{
    const uint32_t quads = (uint32_t)(width + 3) / 4u;
    const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const uint32_t row = (uint32_t)(t / quads);
    const int32_t c = (int32_t)(t % quads) * 4;
    if (row >= M) return;
    const float *p = sums + (size_t)row * (size_t)ldp + c;
    f32x4_t total = *reinterpret_cast<const f32x4_t *>(p);
    for (int32_t s = 1; s < k_slices; ++s)
        total += *reinterpret_cast<const f32x4_t *>(p + (size_t)s * (size_t)slice_rows * (size_t)ldp);
    store_cols(C + (size_t)row * (size_t)ldc + c, total, width - c);
}

template <int U, int S, int VW, int D, bool WIDE, int UFKT = UFK, bool PROBE = false>
void launch_instance(const spmm_launch_args &a, void *stream)
{
    hipLaunchKernelGGL((spmm_chunks_kernel<U, S, VW, D, WIDE, UFKT, PROBE>), dim3((unsigned)a.n_blocks, (unsigned)a.n_tiles),
                       dim3(64 * WAVES_PER_WG), a.lds_pad, (hipStream_t)stream, a.stream, a.wins, a.items, a.rowmap,
                       a.B, a.b_bytes, a.C, a.ldn, a.ldc, a.width, a.tile_cols, a.col_mask, a.cross_sums, a.n_cross_slots);
}

// One (height, slices) pair at the pipeline depth asked for.  DMAX is the depth the
// instance is tuned for (as deep as its register budget allows); a caller may ask for a
// shallower pipeline (1, 2, 3, 4, 8: the loads-in-flight axis of the paper's Figure 2),
// a deeper request runs at DMAX.  The 64-bit addressing kernels exist at DMAX only.
template <int U, int S, int VW, int DMAX, bool WIDE> void launch_depth(const spmm_launch_args &a, int depth, void *stream)
{
    if constexpr (!WIDE) {
        if (a.probe) return launch_instance<U, S, VW, DMAX, WIDE, UFK, true>(a, stream);
        if (depth == 1 && DMAX > 1) return launch_instance<U, S, VW, 1, WIDE>(a, stream);
        if (depth == 2 && DMAX > 2) return launch_instance<U, S, VW, 2, WIDE>(a, stream);
        if (depth == 3 && DMAX > 3) return launch_instance<U, S, VW, (DMAX > 3 ? 3 : DMAX), WIDE>(a, stream);
        if (depth == 4 && DMAX > 4) return launch_instance<U, S, VW, (DMAX > 4 ? 4 : DMAX), WIDE>(a, stream);
    }
    launch_instance<U, S, VW, DMAX, WIDE>(a, stream);
}

// Pipeline depths per height (D2, D4, D8 for 2, 4, 8 slices): the shallowest that keeps the
// loads flowing (see waves_per_simd); one column slot per slice (8 slices) needs more chunks
// in flight for the same number of requests.
template <int U, int D2, int D4, int D8> void launch_slices(const spmm_launch_args &a, int slices, bool wide, int depth, void *stream)
{
    switch (slices) {
    case 2: wide ? launch_depth<U, 2, 4, D2, true>(a, depth, stream) : launch_depth<U, 2, 4, D2, false>(a, depth, stream); break;
    case 4: wide ? launch_depth<U, 4, 4, D4, true>(a, depth, stream) : launch_depth<U, 4, 4, D4, false>(a, depth, stream); break;
    case 8: wide ? launch_depth<U, 8, 4, D8, true>(a, depth, stream) : launch_depth<U, 8, 4, D8, false>(a, depth, stream); break;
    default: wide ? launch_depth<U, 1, 1, 3, true>(a, depth, stream) : launch_depth<U, 1, 1, 3, false>(a, depth, stream); break;
    }
}

// Plans made for narrow B (chunks of 16, 32 or 64 columns): one instance per height and chunk
// width pair, at the tuned depth, 32-bit addressing only.  slices: 8 (tile of 32 columns,
// chunks of 16), 16 (16 columns, chunks of 32), 32 or 64 (8 or 4 columns, chunks of 64).
template <int U, int D> bool launch_narrow(const spmm_launch_args &a, int ufk, int slices, void *stream)
{
    if (a.probe && ufk == 16 && slices == 8) launch_instance<U, 8, 4, D, false, 16, true>(a, stream);
    else if (ufk == 16 && slices == 8) launch_instance<U, 8, 4, D, false, 16>(a, stream);
    else if (ufk == 32 && slices == 16) launch_instance<U, 16, 4, (D > 4 ? 4 : D), false, 32>(a, stream);
    else if (ufk == 64 && slices == 32) launch_instance<U, 32, 4, (D > 4 ? 4 : D), false, 64>(a, stream);
    else if (ufk == 64 && slices == 64) launch_instance<U, 64, 4, (D > 4 ? 4 : D), false, 64>(a, stream);
    else return false;
    return true;
}

}  // namespace

// The depth table (instances per height: 2, 4, 8 slices): kept in step with
// spmm_default_depth below.
int spmm_launch_chunks(const spmm_launch_args &a, int ufi, int ufk, int slices, bool wide, int depth, void *stream)
{
    if (a.n_blocks <= 0 || a.n_tiles <= 0) return 0;
    if (ufk != UFK) {
        bool ok = !wide;
        if (ok) {
            switch (ufi) {
            case 8: ok = launch_narrow<8, 4>(a, ufk, slices, stream); break;
            case 4: ok = launch_narrow<4, 3>(a, ufk, slices, stream); break;
            case 2: ok = launch_narrow<2, 4>(a, ufk, slices, stream); break;
            case 1: ok = launch_narrow<1, 4>(a, ufk, slices, stream); break;
            default: ok = false;
            }
        }
        if (!ok) return (int)hipErrorInvalidValue;
    } else
    switch (ufi) {
    case 8: launch_slices<8, 2, 3, 4>(a, slices, wide, depth, stream); break;
    case 4: launch_slices<4, 2, 3, 4>(a, slices, wide, depth, stream); break;
    case 2: launch_slices<2, 2, 2, 6>(a, slices, wide, depth, stream); break;
    case 1: launch_slices<1, 2, 2, 8>(a, slices, wide, depth, stream); break;
    default: return (int)hipErrorInvalidValue;
    }
    if (a.n_cross > 0)
        hipLaunchKernelGGL(spmm_cross_combine_kernel, dim3((unsigned)a.n_cross, (unsigned)a.n_tiles), dim3(256), 0,
                           (hipStream_t)stream, a.cross_table, a.cross_sums, a.n_cross_slots, (int32_t)ufi, a.C, a.ldc,
                           a.width, a.tile_cols);
    if (a.k_slices > 1) {
        const uint64_t threads = (uint64_t)a.M * (uint64_t)((a.width + 3) / 4);
        hipLaunchKernelGGL(spmm_kslice_combine_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                           (hipStream_t)stream, a.C, a.k_slices, (uint32_t)a.slice_rows, a.ldc, a.C_out, a.ldc_out,
                           (uint32_t)a.M, a.width);
    }
    return (int)hipGetLastError();
}

// Scratch memory that exists without any allocation call: a device array of the library's
// code object, for callers of spmm_execute_static.  In host code the array's name is only a
// handle for the runtime; its address on each device is asked for once and kept.
namespace {
static __device__ __align__(256) float scratch[SPMM_STATIC_SCRATCH_BYTES / sizeof(float)];
constexpr int MAX_DEVICES = 64;
float *scratch_on_device[MAX_DEVICES];
std::mutex scratch_lock;
}  // namespace

int spmm_static_scratch(float **ptr, size_t *bytes)
{
    *ptr = nullptr;
    *bytes = 0;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= MAX_DEVICES) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_on_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // this device's copy of the array
        if (e != hipSuccess || !p) return e != hipSuccess ? (int)e : (int)hipErrorInvalidSymbol;
        scratch_on_device[dev] = static_cast<float *>(p);
    }
    *ptr = scratch_on_device[dev];
    *bytes = SPMM_STATIC_SCRATCH_BYTES;
    return 0;
}

int spmm_default_depth(int ufi, int slices)
{
    static const int table[4][3] = {{2, 2, 8}, {2, 2, 6}, {2, 3, 4}, {2, 3, 4}};  // rows: height 1, 2, 4, 8
    const int u = ufi == 8 ? 3 : ufi == 4 ? 2 : ufi == 2 ? 1 : 0;
    return slices == 2 ? table[u][0] : slices == 4 ? table[u][1] : slices == 8 ? table[u][2] : 3;
}
