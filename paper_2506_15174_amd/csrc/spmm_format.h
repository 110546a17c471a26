// Device format shared by the host inspector (spmm_plan.cpp) and the gfx950
// executor (spmm_kernels.hip).  Plain integers only.
//
// The format is this library's re-derivation of the paper's transformed matrix
// TA (Section 3.3 "Data transformation", Listing 7: ANNZ / NPP / RPP / Cols):
// the values are stored in the order the kernel consumes them, one column index
// is stored per *enumerated column* (a column of a panel of UFI rows together
// with its nonzero pattern, Section 3.2), and the enumerated columns of a panel
// that share a pattern are stored next to each other ("a list of pointers to the
// same pattern", Section 3.2.2).  Each such run is cut into *chunks* of at most
// UFK columns; a chunk is the unit the kernel keeps in flight (the paper's
// unroll(k, UFk), Section 3.3.2).  Where the paper launches one thread block per
// (panel, pattern) and meets in C with atomics, one wave here walks all chunks
// of its panels with the UFI x (columns per lane) tile held in registers.
#ifndef SPMM_FORMAT_H
#define SPMM_FORMAT_H

#include <stdint.h>

namespace spmm_fmt {

// Rows per panel: height of the register tile (the paper's UFi).
constexpr int UFI = 4;
constexpr int N_PATTERNS = (1 << UFI) - 1;  // 15 nonzero patterns (paper Section 2)

// Enumerated columns per chunk (the paper's UFk).
constexpr int UFK = 8;

// Three parallel arrays describe the chunks, in launch order of their groups:
//
//   hdr[c]            one word:  bits 0..3  pattern (rows of the panel that own a value
//                                           in every column of the chunk), 0 only for
//                                           the single chunk of a panel without nonzeros
//                                bits 4..7  count of real columns, 0..UFK
//                                bit  8     last chunk of its panel (store the tile)
//   cols[c*UFK + u]   column index of slot u; slots >= count repeat a valid column
//                     of the chunk (or 0) and carry zero values
//   vals              for chunk c, popcount(pattern) blocks of UFK floats, one block
//                     per set row in ascending row order, block[u] = value of that
//                     row in column slot u (zero in unused slots); chunks follow each
//                     other without gaps, so a chunk's block offset is the running
//                     sum of UFK * popcount(pattern)
constexpr uint32_t HDR_PATTERN_MASK = 0xFu;
constexpr int HDR_COUNT_SHIFT = 4;
constexpr uint32_t HDR_COUNT_MASK = 0xFu;
constexpr uint32_t HDR_END_PANEL = 1u << 8;

// Chunks (all zero) appended after the last real chunk so that the kernels'
// look-ahead of two chunks never leaves the arrays.
constexpr int CHUNK_TAIL_PAD = 4;
// Zero words appended to vals so that the four per-row block loads of a chunk
// stay inside the array whatever its pattern.
constexpr int VALS_TAIL_PAD = UFI * UFK;

// Work-item descriptor, one per row group, launch order.
constexpr int ITEM_WORDS = 16;
enum ItemField {
    IT_ROW0 = 0,    // first row
    IT_NROWS = 1,   // rows covered (whole panels; the last may be short)
    IT_CHUNK0 = 2,  // first chunk
    IT_NCHUNKS = 3, // chunks of the group (>= 1)
    IT_VALS0 = 4,   // first word of the group's values
    IT_FLAGS = 5,   // bit 0: piece of a split panel
    IT_TICKET = 6,  // split: index of the panel's arrival counter
    IT_NSEG = 7,    // split: pieces the panel was cut into
    IT_SLOT0 = 8,   // split: scratch slot of the panel's first piece
    IT_SEG = 9      // split: index of this piece
};
constexpr int FLAG_SPLIT = 1;

// Scratch slot of one piece: UFI rows x SLOT_COLS floats.
constexpr int SLOT_COLS = 128;
constexpr int SLOT_FLOATS = UFI * SLOT_COLS;

// Waves (= work items) per workgroup.
constexpr int WAVES_PER_WG = 4;

}  // namespace spmm_fmt
#endif
