// gfx950 executor: C <- A x B over the chunked, schedule-ordered arrays built by
// the inspector (paper Section 3.3 "Sparse Coarsen", Listings 5-7, re-derived
// for wave64).
//
// Mapping (one wave = one row group, 4 independent waves per workgroup):
//   * lanes run along j, the columns of B and C (the paper's map(j, .),
//     Listing 5): lane l owns columns VW*l .. VW*l+VW-1 of the current column
//     tile, so one wave-wide load fetches a whole B row segment, coalesced;
//   * the UFI x VW accumulators of a panel stay in VGPRs across all chunks of
//     the panel (the paper's register tile, Listing 6) and are stored once;
//   * everything that describes A -- chunk headers, column indices, values -- is
//     identical for all lanes, so it is fetched with scalar loads into SGPRs; the
//     values feed v_fmac_f32 as scalar operands and the row offsets feed the
//     buffer loads as scalar offsets.  No lane ever tests a sparsity condition
//     (Section 3.2.2: enumerated blocks carry no conditionals): the pattern of a
//     chunk selects, with wave-uniform branches, which of the UFI row blocks run;
//   * a chunk is UFK enumerated columns of one pattern: UFK independent B loads
//     in flight, then popcount(pattern) x UFK x VW FMAs (the paper's
//     unroll(k, UFk)).  The loads of the next chunk are issued before the FMAs of
//     the current one, and the descriptors of the chunk after that are already on
//     their way, so a wave always has two chunks of B rows in flight.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spmm_format.h"
#include "spmm_kernels.h"

using namespace spmm_fmt;

namespace {

// Scalar (wave-uniform) view of read-only plan memory: loads through this
// address space are issued as s_load_* when the address is uniform.
typedef const uint32_t __attribute__((address_space(4))) cword_t;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int VW> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<2> { typedef float2 type; };

__device__ __forceinline__ void fma_acc(float &acc, float a, float b) { acc = __builtin_fmaf(a, b, acc); }
__device__ __forceinline__ void fma_acc(float2 &acc, float a, float2 b)
{
    acc.x = __builtin_fmaf(a, b.x, acc.x);
    acc.y = __builtin_fmaf(a, b.y, acc.y);
}
__device__ __forceinline__ void zero(float &v) { v = 0.0f; }
__device__ __forceinline__ void zero(float2 &v) { v.x = 0.0f; v.y = 0.0f; }
__device__ __forceinline__ void add_to(float &a, float b) { a += b; }
__device__ __forceinline__ void add_to(float2 &a, float2 b) { a.x += b.x; a.y += b.y; }

// Source of B rows.  Narrow: a raw buffer descriptor over the column tile's
// bytes (hardware range check, scalar row offset, per-lane byte offset).  Wide:
// plain 64-bit addressing for B larger than 4 GiB.
template <bool WIDE> struct BSource;

template <> struct BSource<false> {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t ld_bytes;
    uint32_t lane_off;
    __device__ __forceinline__ void init(const float *B, uint32_t ld_bytes_, uint32_t lane_off_, uint32_t n_bytes)
    {
        // word 3: 32-bit data format, raw (untyped, stride 0) addressing
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(B), 0, (int)n_bytes, 0x00020000);
        ld_bytes = ld_bytes_;
        lane_off = lane_off_;
    }
    __device__ __forceinline__ float load(uint32_t col, float) const
    {
        return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, col * ld_bytes, 0));
    }
    __device__ __forceinline__ float2 load(uint32_t col, float2) const
    {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, col * ld_bytes, 0);
        return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
    }
};

template <> struct BSource<true> {
    const char *base;
    uint32_t ld_bytes;
    uint32_t lane_off;
    __device__ __forceinline__ void init(const float *B, uint32_t ld_bytes_, uint32_t lane_off_, uint32_t)
    {
        base = reinterpret_cast<const char *>(B);
        ld_bytes = ld_bytes_;
        lane_off = lane_off_;
    }
    __device__ __forceinline__ float load(uint32_t col, float) const
    {
        return *reinterpret_cast<const float *>(base + (uint64_t)col * ld_bytes + lane_off);
    }
    __device__ __forceinline__ float2 load(uint32_t col, float2) const
    {
        return *reinterpret_cast<const float2 *>(base + (uint64_t)col * ld_bytes + lane_off);
    }
};

struct ChunkDesc {
    uint32_t hdr;
    uint32_t col[UFK];
};

__device__ __forceinline__ void fetch_desc(ChunkDesc &d, cword_t *hdrs, cword_t *cols, uint32_t c)
{
    d.hdr = hdrs[c];
#pragma unroll
    for (int u = 0; u < UFK; ++u) d.col[u] = cols[(size_t)c * UFK + u];
}

template <int VW, bool WIDE>
__device__ __forceinline__ void issue_b(typename Vec<VW>::type (&b)[UFK], const ChunkDesc &d,
                                        const BSource<WIDE> &src)
{
    typedef typename Vec<VW>::type vec_t;
#pragma unroll
    for (int u = 0; u < UFK; ++u) b[u] = src.load(d.col[u], vec_t());
}

// The enumerated block of one chunk (paper Listing 7): for every row r of the
// pattern, UFK FMAs per lane column with the row's values as scalar operands.
// Returns the number of value words the chunk owns.
template <int VW>
__device__ __forceinline__ uint32_t
fma_chunk(typename Vec<VW>::type (&acc)[UFI], const typename Vec<VW>::type (&b)[UFK], uint32_t hdr,
          cword_t *vals)
{
    const uint32_t pattern = hdr & HDR_PATTERN_MASK;
    // Value block of row r starts UFK * (set rows below r) words in.  All four
    // loads are issued up front (the blocks of absent rows are never used; the
    // array is padded so that they stay in range).
    uint32_t w[UFI][UFK];
#pragma unroll
    for (int r = 0; r < UFI; ++r) {
        const uint32_t below = __builtin_popcount(pattern & ((1u << r) - 1u));
#pragma unroll
        for (int u = 0; u < UFK; ++u) w[r][u] = vals[below * UFK + u];
    }
#pragma unroll
    for (int r = 0; r < UFI; ++r) {
        if (pattern & (1u << r)) {
#pragma unroll
            for (int u = 0; u < UFK; ++u) fma_acc(acc[r], __uint_as_float(w[r][u]), b[u]);
        }
    }
    return (uint32_t)__builtin_popcount(pattern) * UFK;
}

template <int VW>
__device__ __forceinline__ void store_row(float *__restrict__ row, int lane, typename Vec<VW>::type v)
{
    *reinterpret_cast<typename Vec<VW>::type *>(row + lane * VW) = v;
}

struct ItemCtx {
    uint32_t flags, ticket, nseg, slot0, seg;
};

// Writes the finished tile of one panel.  Whole panels store straight to C.  A
// piece of a split panel parks its partial tile in scratch and counts arrivals;
// the last piece to arrive adds all pieces in index order (deterministic) and
// writes C.  No wave ever waits for another.
template <int VW>
__device__ __forceinline__ void
finish_panel(typename Vec<VW>::type (&acc)[UFI], const ItemCtx &ctx, float *__restrict__ C, int32_t ldn,
             uint32_t row, uint32_t rows_here, int lane, bool active, float *__restrict__ scratch,
             uint32_t *__restrict__ tickets)
{
    typedef typename Vec<VW>::type vec_t;
    float *c_panel = C + (size_t)row * (size_t)ldn;
    if (!(ctx.flags & FLAG_SPLIT)) {
        if (active) {
#pragma unroll
            for (int r = 0; r < UFI; ++r)
                if ((uint32_t)r < rows_here) store_row<VW>(c_panel + (size_t)r * ldn, lane, acc[r]);
        }
        return;
    }
    float *mine = scratch + (size_t)(ctx.slot0 + ctx.seg) * SLOT_FLOATS;
#pragma unroll
    for (int r = 0; r < UFI; ++r) store_row<VW>(mine + r * SLOT_COLS, lane, acc[r]);
    __threadfence();
    uint32_t *ticket = tickets + ctx.ticket;
    uint32_t arrived = 0;
    if (lane == 0) arrived = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    if (arrived != ctx.nseg - 1) return;
    __threadfence();
#pragma unroll
    for (int r = 0; r < UFI; ++r) zero(acc[r]);
    for (uint32_t p = 0; p < ctx.nseg; ++p) {
        const float *part = scratch + (size_t)(ctx.slot0 + p) * SLOT_FLOATS;
#pragma unroll
        for (int r = 0; r < UFI; ++r)
            add_to(acc[r], *reinterpret_cast<const vec_t *>(part + r * SLOT_COLS + lane * VW));
    }
    if (active) {
#pragma unroll
        for (int r = 0; r < UFI; ++r)
            if ((uint32_t)r < rows_here) store_row<VW>(c_panel + (size_t)r * ldn, lane, acc[r]);
    }
    // Re-arm the counter for the next execute (ordered by the kernel boundary).
    if (lane == 0) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// VW   columns per lane (1: tiles of up to 64 columns, 2: tiles of up to 128)
// WIDE byte offsets into B need more than 32 bits
template <int VW, bool WIDE>
__global__ __launch_bounds__(64 * WAVES_PER_WG) void
spmm_chunks_kernel(const uint32_t *__restrict__ hdr_g, const uint32_t *__restrict__ cols_g,
                   const uint32_t *__restrict__ vals_g, const uint32_t *__restrict__ items_g,
                   int32_t n_items, const float *__restrict__ B, uint32_t b_bytes, float *__restrict__ C,
                   int32_t ldn, int32_t width, float *__restrict__ scratch, uint32_t *__restrict__ tickets)
{
    typedef typename Vec<VW>::type vec_t;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int item = (int)blockIdx.x * WAVES_PER_WG + wave;
    if (item >= n_items) return;
    const int lane = (int)(threadIdx.x & 63);

    cword_t *it = (cword_t *)(items_g) + (size_t)item * ITEM_WORDS;
    uint32_t row = it[IT_ROW0];
    uint32_t rows_left = it[IT_NROWS];
    const uint32_t chunk0 = it[IT_CHUNK0];
    const uint32_t n_chunks = it[IT_NCHUNKS];
    cword_t *vals = (cword_t *)(vals_g) + it[IT_VALS0];
    ItemCtx ctx;
    ctx.flags = it[IT_FLAGS];
    ctx.ticket = it[IT_TICKET];
    ctx.nseg = it[IT_NSEG];
    ctx.slot0 = it[IT_SLOT0];
    ctx.seg = it[IT_SEG];
    cword_t *hdrs = (cword_t *)(hdr_g) + chunk0;
    cword_t *cols = (cword_t *)(cols_g) + (size_t)chunk0 * UFK;

    // Lanes beyond the tile width compute on the tile's first columns and store
    // nothing: no divergent control flow in the hot loop, no out-of-range access.
    const bool active = lane * VW < width;
    BSource<WIDE> src;
    src.init(B, (uint32_t)ldn * 4u, active ? (uint32_t)(lane * VW * 4) : 0u, b_bytes);

    vec_t acc[UFI];
#pragma unroll
    for (int r = 0; r < UFI; ++r) zero(acc[r]);

    // Software pipeline over chunks c = 0 .. n_chunks-1:
    //   descriptors of chunk c+2 requested | B rows of chunk c+1 requested | FMAs of chunk c
    // Chunks past the group's end are the next group's (or the zero padding):
    // their B rows are fetched and dropped, which keeps the loop free of
    // conditional loads so the wait counts stay exact.
    vec_t b0[UFK], b1[UFK];
    ChunkDesc d0, d1, d2;
    fetch_desc(d0, hdrs, cols, 0);
    fetch_desc(d1, hdrs, cols, 1);
    issue_b<VW, WIDE>(b0, d0, src);

    for (uint32_t c = 0;;) {
        // ---- even step: chunk c lives in b0 / d0
        issue_b<VW, WIDE>(b1, d1, src);
        fetch_desc(d2, hdrs, cols, c + 2);
        vals += fma_chunk<VW>(acc, b0, d0.hdr, vals);
        if (d0.hdr & HDR_END_PANEL) {
            const uint32_t rows_here = rows_left < (uint32_t)UFI ? rows_left : (uint32_t)UFI;
            finish_panel<VW>(acc, ctx, C, ldn, row, rows_here, lane, active, scratch, tickets);
            row += rows_here;
            rows_left -= rows_here;
#pragma unroll
            for (int r = 0; r < UFI; ++r) zero(acc[r]);
        }
        if (++c >= n_chunks) break;
        // ---- odd step: chunk c lives in b1 / d1
        issue_b<VW, WIDE>(b0, d2, src);
        fetch_desc(d0, hdrs, cols, c + 2);
        vals += fma_chunk<VW>(acc, b1, d1.hdr, vals);
        if (d1.hdr & HDR_END_PANEL) {
            const uint32_t rows_here = rows_left < (uint32_t)UFI ? rows_left : (uint32_t)UFI;
            finish_panel<VW>(acc, ctx, C, ldn, row, rows_here, lane, active, scratch, tickets);
            row += rows_here;
            rows_left -= rows_here;
#pragma unroll
            for (int r = 0; r < UFI; ++r) zero(acc[r]);
        }
        if (++c >= n_chunks) break;
        d1 = d0;   // chunk c+1
        d0 = d2;   // chunk c
    }
}

}  // namespace

#define SPMM_LAUNCH(VW, WIDE)                                                                        \
    hipLaunchKernelGGL((spmm_chunks_kernel<VW, WIDE>), dim3(grid), dim3(64 * WAVES_PER_WG), 0,       \
                       (hipStream_t)stream, a.hdr, a.cols, a.vals, a.items, a.n_items, a.B,          \
                       a.b_bytes, a.C, a.ldn, a.width, a.scratch, a.tickets)

int spmm_launch_chunks(const spmm_launch_args &a, int vw, bool wide, void *stream)
{
    if (a.n_items <= 0) return 0;
    const unsigned grid = (unsigned)((a.n_items + WAVES_PER_WG - 1) / WAVES_PER_WG);
    if (vw == 2) {
        if (wide) SPMM_LAUNCH(2, true); else SPMM_LAUNCH(2, false);
    } else {
        if (wide) SPMM_LAUNCH(1, true); else SPMM_LAUNCH(1, false);
    }
    return (int)hipGetLastError();
}
