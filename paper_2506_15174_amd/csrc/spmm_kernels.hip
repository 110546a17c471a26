// gfx950 executor: C <- A x B over the chunked, schedule-ordered arrays built by
// the inspector (paper Section 3.3 "Sparse Coarsen", Listings 5-7, re-derived
// for wave64).
//
// Mapping (one wave = one row group, up to 16 waves per workgroup):
//   * lanes run along j, the columns of B and C (the paper's map(j, .),
//     Listing 5): lane l owns columns VW*l .. VW*l+VW-1 of the current column
//     tile, so one wave-wide load fetches a whole B row segment, coalesced;
//   * the UFI x VW accumulators of a panel stay in VGPRs across all chunks of
//     the panel (the paper's register tile, Listing 6) and are written once;
//   * everything that describes A -- chunk headers, column indices, values -- is
//     identical for all lanes, so it is fetched with scalar loads into SGPRs; the
//     values feed v_fmac_f32 as scalar operands and the row offsets feed the
//     buffer loads as scalar offsets.  No lane ever tests a sparsity condition
//     (Section 3.2.2: enumerated blocks carry no conditionals): the pattern of a
//     chunk selects, with wave-uniform branches, which of the UFI row blocks run;
//   * a chunk is UFK enumerated columns of one pattern: UFK independent B loads,
//     then popcount(pattern) x UFK x VW FMAs (the paper's unroll(k, UFk)).  The
//     loop is software-pipelined three chunks deep: while chunk c is multiplied,
//     the B rows of chunks c+1 and c+2 are in flight and the descriptors of
//     chunks c+3 and c+4 are on their way;
//   * pieces of a panel that was too heavy for one wave sit in the same
//     workgroup: they park their partial tiles in LDS, meet at one barrier and
//     one wave per tile row adds the pieces in piece order (the paper's
//     write-after-write hazard, Section 3.3.2, solved without atomics and with a
//     fixed summation order).
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
    uint32_t lane_off;
    __device__ __forceinline__ void init(const float *B, uint32_t lane_off_, uint32_t n_bytes)
    {
        // word 3: 32-bit data format, raw (untyped, stride 0) addressing
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(B), 0, (int)n_bytes, 0x00020000);
        lane_off = lane_off_;
    }
    __device__ __forceinline__ float load(uint32_t col, uint32_t ld_bytes, float) const
    {
        return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, col * ld_bytes, 0));
    }
    __device__ __forceinline__ float2 load(uint32_t col, uint32_t ld_bytes, float2) const
    {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, col * ld_bytes, 0);
        return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
    }
};

template <> struct BSource<true> {
    const char *base;
    uint32_t lane_off;
    __device__ __forceinline__ void init(const float *B, uint32_t lane_off_, uint32_t)
    {
        base = reinterpret_cast<const char *>(B);
        lane_off = lane_off_;
    }
    __device__ __forceinline__ float load(uint32_t col, uint32_t ld_bytes, float) const
    {
        return *reinterpret_cast<const float *>(base + (uint64_t)col * ld_bytes + lane_off);
    }
    __device__ __forceinline__ float2 load(uint32_t col, uint32_t ld_bytes, float2) const
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

// Requests the UFK B rows of one chunk.  ld_bytes is the row pitch, or 0 for a
// chunk past the group's end: then every slot reads row 0 (one cached line per
// lane group), so the loop needs no conditional loads and its wait counts stay
// exact.
template <int VW, bool WIDE>
__device__ __forceinline__ void issue_b(typename Vec<VW>::type (&b)[UFK], const ChunkDesc &d,
                                        const BSource<WIDE> &src, uint32_t ld_bytes)
{
    typedef typename Vec<VW>::type vec_t;
#pragma unroll
    for (int u = 0; u < UFK; ++u) b[u] = src.load(d.col[u], ld_bytes, vec_t());
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
#pragma unroll
    for (int r = 0; r < UFI; ++r) {
        if (pattern & (1u << r)) {
            // value block of row r: UFK words per set row below r
            const uint32_t below = __builtin_popcount(pattern & ((1u << r) - 1u));
            uint32_t w[UFK];
#pragma unroll
            for (int u = 0; u < UFK; ++u) w[u] = vals[below * UFK + u];
#pragma unroll
            for (int u = 0; u < UFK; ++u) fma_acc(acc[r], __uint_as_float(w[u]), b[u]);
        }
    }
    return (uint32_t)__builtin_popcount(pattern) * UFK;
}

template <int VW>
__device__ __forceinline__ void store_row(float *__restrict__ row, int lane, typename Vec<VW>::type v)
{
    *reinterpret_cast<typename Vec<VW>::type *>(row + lane * VW) = v;
}

// VW   columns per lane (1: tiles of up to 64 columns, 2: tiles of up to 128)
// WIDE byte offsets into B need more than 32 bits
template <int VW, bool WIDE>
__global__ __launch_bounds__(64 * WAVES_PER_WG) void
spmm_chunks_kernel(const uint32_t *__restrict__ hdr_g, const uint32_t *__restrict__ cols_g,
                   const uint32_t *__restrict__ vals_g, const uint32_t *__restrict__ items_g,
                   const float *__restrict__ B, uint32_t b_bytes, float *__restrict__ C, int32_t ldn,
                   int32_t width)
{
    typedef typename Vec<VW>::type vec_t;
    // Partial tiles of split panels, one per wave slot.
    __shared__ vec_t tiles[WAVES_PER_WG][UFI][64];

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    cword_t *it = (cword_t *)(items_g) + ((size_t)blockIdx.x * WAVES_PER_WG + wave) * ITEM_WORDS;
    const uint32_t flags = it[IT_FLAGS];
    const uint32_t n_chunks = it[IT_NCHUNKS];

    // Lanes beyond the tile width compute on the tile's first columns and store
    // nothing: no divergent control flow in the hot loop, no out-of-range access.
    const bool active = lane * VW < width;

    if (n_chunks != 0) {
        uint32_t row = it[IT_ROW0];
        uint32_t rows_left = it[IT_NROWS];
        const uint32_t chunk0 = it[IT_CHUNK0];
        cword_t *vals = (cword_t *)(vals_g) + it[IT_VALS0];
        cword_t *hdrs = (cword_t *)(hdr_g) + chunk0;
        cword_t *cols = (cword_t *)(cols_g) + (size_t)chunk0 * UFK;
        const uint32_t ld_bytes = (uint32_t)ldn * 4u;
        BSource<WIDE> src;
        src.init(B, active ? (uint32_t)(lane * VW * 4) : 0u, b_bytes);

        vec_t acc[UFI];
#pragma unroll
        for (int r = 0; r < UFI; ++r) zero(acc[r]);

        // Three-deep rings, all indexed by (chunk number mod 3):
        //   d[k % 3]  descriptor of chunk k, from its request until its B rows are requested
        //   b[k % 3]  B rows of chunk k, from their request until the chunk is multiplied
        //   h[k % 3]  header of chunk k, kept for the multiply step
        ChunkDesc d[3];
        vec_t b[3][UFK];
        uint32_t h[3];
        fetch_desc(d[0], hdrs, cols, 0);
        fetch_desc(d[1], hdrs, cols, 1);
        fetch_desc(d[2], hdrs, cols, 2);
        issue_b<VW, WIDE>(b[0], d[0], src, ld_bytes);
        h[0] = d[0].hdr;
        fetch_desc(d[0], hdrs, cols, 3);
        issue_b<VW, WIDE>(b[1], d[1], src, n_chunks > 1 ? ld_bytes : 0u);
        h[1] = d[1].hdr;

        uint32_t c = 0;
        bool more = true;
        while (more) {
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                // step for chunk c (c % 3 == s)
                issue_b<VW, WIDE>(b[(s + 2) % 3], d[(s + 2) % 3], src, c + 2 < n_chunks ? ld_bytes : 0u);
                h[(s + 2) % 3] = d[(s + 2) % 3].hdr;
                fetch_desc(d[(s + 1) % 3], hdrs, cols, c + 4);
                vals += fma_chunk<VW>(acc, b[s], h[s], vals);
                if (h[s] & HDR_END_PANEL) {
                    const uint32_t rows_here = rows_left < (uint32_t)UFI ? rows_left : (uint32_t)UFI;
                    if (flags & FLAG_SPLIT) {
#pragma unroll
                        for (int r = 0; r < UFI; ++r) tiles[wave][r][lane] = acc[r];
                    } else if (active) {
                        float *c_panel = C + (size_t)row * (size_t)ldn;
#pragma unroll
                        for (int r = 0; r < UFI; ++r)
                            if ((uint32_t)r < rows_here) store_row<VW>(c_panel + (size_t)r * ldn, lane, acc[r]);
                    }
                    row += rows_here;
                    rows_left -= rows_here;
#pragma unroll
                    for (int r = 0; r < UFI; ++r) zero(acc[r]);
                }
                if (++c >= n_chunks) {
                    more = false;
                    break;
                }
            }
        }
    }

    if (flags & FLAG_SYNC) {
        // Every wave of a block with split panels arrives here exactly once.
        __syncthreads();
        const uint32_t nseg = it[IT_RED_NSEG];
        if (nseg != 0 && active) {
            const uint32_t slot0 = it[IT_RED_SLOT0];
            const uint32_t r = it[IT_RED_R];
            vec_t sum;
            zero(sum);
            for (uint32_t p = 0; p < nseg; ++p) add_to(sum, tiles[slot0 + p][r][lane]);
            store_row<VW>(C + (size_t)it[IT_RED_ROW] * (size_t)ldn, lane, sum);
        }
    }
}

}  // namespace

#define SPMM_LAUNCH(VW, WIDE)                                                                         \
    hipLaunchKernelGGL((spmm_chunks_kernel<VW, WIDE>), dim3((unsigned)a.n_blocks),                    \
                       dim3(64 * WAVES_PER_WG), 0, (hipStream_t)stream, a.hdr, a.cols, a.vals,        \
                       a.items, a.B, a.b_bytes, a.C, a.ldn, a.width)

int spmm_launch_chunks(const spmm_launch_args &a, int vw, bool wide, void *stream)
{
    if (a.n_blocks <= 0) return 0;
    if (vw == 2) {
        if (wide) SPMM_LAUNCH(2, true); else SPMM_LAUNCH(2, false);
    } else {
        if (wide) SPMM_LAUNCH(1, true); else SPMM_LAUNCH(1, false);
    }
    return (int)hipGetLastError();
}
