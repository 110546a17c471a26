// Device format shared by the host inspector (spmm_plan.cpp) and the gfx950
// executor (spmm_kernels.hip).  Plain integers only.
//
// The format is this library's re-derivation of the paper's transformed matrix
// TA (Section 3.3 "Data transformation", Listing 7: ANNZ / NPP / RPP / Cols):
// the values are stored in the order the kernel consumes them, one column index
// is stored per *enumerated column* (a column of a panel of UFI rows together
// with its nonzero pattern, Section 3.2), and the enumerated columns of a panel
// that share a pattern are stored next to each other (the per-pattern column
// lists of Section 3.2.2).  Each such run is cut into *chunks* of at most
// UFK columns; a chunk is the unit the kernel keeps in flight (the paper's
// unroll(k, UFk), Section 3.3.2).  Where the paper launches one thread block per
// (panel, pattern) and meets in C with atomics, one wave here walks all chunks
// of its panels with the UFI x (columns per lane) tile held in registers.
#ifndef SPMM_FORMAT_H
#define SPMM_FORMAT_H

#include <stdint.h>

namespace spmm_fmt {

// Rows per panel: height of the register tile (the paper's UFi).  A plan uses
// 8, 4, 2 or 1; a panel of u rows has 2^u - 1 nonzero patterns (paper Section 2).
constexpr int MAX_UFI = 8;

// Enumerated columns per chunk (the paper's UFk): a property of the plan.  8 for B of more
// than 32 columns (or unknown width); plans made for narrower B take wider chunks, so that a
// wave cut into more slices (16 bytes of a B row need only one lane per four columns) still
// hands every slice two column slots per chunk: 16 for up to 32 columns of B, 32 for up to
// 16, 64 for up to 8.
constexpr int UFK = 8;
constexpr int MAX_UFK = 64;
constexpr bool valid_ufk(int u) { return u == 8 || u == 16 || u == 32 || u == 64; }

// A chunk is described by
//
//   header     one word:  bits 0..7   pattern (rows of the panel that own a value in
//                                     every column of the chunk), 0 only for the
//                                     single chunk of a panel without nonzeros
//                         bits 8..14  count of real columns, 0..ufk
//                         bit  15     last chunk of its panel (write the tile)
//   columns    ufk column words (slots >= count repeat a valid column of the chunk,
//              or 0, and carry zero values).  Bits 0..23 hold the column index.  The
//              leftovers of several patterns may share a chunk; its header then holds
//              the union of their patterns and a slot whose own pattern is smaller
//              keeps it in bits 24..31 (0 = the slot has the chunk's pattern).  Plans
//              of matrices with more than 2^24 columns never share chunks and use all
//              32 bits for the index.
//   values     for every set row of the pattern in ascending row order ufk value
//              words (float bits, value of that row in column slot u; zero in
//              unused slots and in slots whose own pattern lacks the row)
//
// The chunks of a row group are cut into *windows*, the unit a wave stages through
// LDS: as many consecutive chunks as fit win_words(ufk) words.  `stream` holds the
// windows back to back, each laid out as
//   [ headers of its chunks, zero-padded to a multiple of 8 words ]
//   [ columns of its chunks, ufk words each ]
//   [ values of its chunks, back to back ]
// so a chunk's header and columns sit at fixed strides and only its value offset
// is a running sum (ufk * popcount(pattern) per chunk).
//   wins[i]    one word per window: bits 0..15 chunks, bits 16..31 words
//   hdr[c]     host-side copy of all headers in launch order (introspection only)
constexpr uint32_t HDR_PATTERN_MASK = 0xFFu;
constexpr int HDR_COUNT_SHIFT = 8;
constexpr uint32_t HDR_COUNT_MASK = 0x7Fu;
constexpr uint32_t HDR_END_PANEL = 1u << 15;
constexpr int COL_PATTERN_SHIFT = 24;
constexpr uint32_t COL_INDEX_MASK = (1u << COL_PATTERN_SHIFT) - 1u;

// Words of LDS one wave owns (its window; later its partial tile): 1024 for chunks of 8 or
// 16 columns, 2048 for wider chunks (a chunk of 64 columns of an eight-row panel is 577 words).
constexpr int WIN_WORDS = 1024;
constexpr int MAX_WIN_WORDS = 2048;
constexpr int win_words(int ufk) { return ufk >= 32 ? MAX_WIN_WORDS : WIN_WORDS; }
// Deepest software pipeline of any kernel instance: column slots of up to this
// many chunks past a window's last chunk are read (and never used).
constexpr int LOOKAHEAD = 8;
constexpr int lookahead(int ufk) { return ufk > 8 ? 4 : LOOKAHEAD; }

// Headers (all zero) appended after the last real chunk so that the kernels'
// look-ahead never leaves the array.
constexpr int CHUNK_TAIL_PAD = 16;
// Zero words appended to the stream.
constexpr int STREAM_TAIL_PAD = 16;

// Waves per workgroup.  One wave executes one row group; a workgroup ("block")
// holds up to WAVES_PER_WG of them.  A panel too heavy for one wave is cut into
// at most WAVES_PER_WG pieces that sit in one block and meet in LDS.
constexpr int WAVES_PER_WG = 8;
// A block holds at most WAVES_PER_WG / ufi split panels, so that every
// (panel, row) sum after the barrier has a wave of its own.

// Wave-slot descriptor: WAVES_PER_WG per block, launch order.  In a plan cut along K a block
// holds groups of one column range only and block b of the launch belongs to range b mod k_slices.
constexpr int ITEM_WORDS = 16;
enum ItemField {
    IT_ROW0 = 0,      // first row of the plan (a plan cut along K: column range * slice_rows + row)
    IT_NROWS = 1,     // rows covered (whole panels; the last may be short)
    IT_CHUNK0 = 2,    // first chunk
    IT_NCHUNKS = 3,   // chunks of the group (0 for an idle slot)
    IT_STREAM0 = 4,   // first word of the group's records
    IT_FLAGS = 5,     // FLAG_* bits
    IT_RED_NSEG = 6,  // after the barrier: pieces to add (0 = this wave adds nothing)
    IT_RED_SLOT0 = 7, // ... wave slot of the first piece
    IT_RED_R = 8,     // ... row of the tile to add
    IT_RED_ROW = 9,   // ... row to write: of C, or of the ranges' buffer in a plan cut along K
    IT_WIN0 = 10,     // first window of the group
    IT_NWINS = 11,    // windows of the group (0 for an idle slot)
    IT_WIN_FIRST = 12,// copy of the first window's entry of the window table (saves a dependent load)
    IT_X_NPARTS = 13, // blocks that share this block's panel (FLAG_CROSS only)
    IT_X_SLOT0 = 14,  // ... scratch slot of the panel's first block
    IT_X_PART = 15    // ... this block's place among them
};
constexpr int FLAG_SPLIT = 1;  // the group is one piece of a split panel: its tile goes to LDS
constexpr int FLAG_IDLE = 2;   // no group in this wave slot
constexpr int FLAG_SYNC = 4;   // the block holds split panels: every wave meets at one barrier
constexpr int FLAG_CROSS = 8;  // the block holds WAVES_PER_WG pieces (or the last few) of a panel cut into more
                               // pieces than one block has waves: the blocks' sums meet in scratch memory
                               // and a second, small launch adds them

// A panel is cut across blocks when it is heavier than both WAVES_PER_WG group budgets
// and 1 / CROSS_SHARE of all entries (a quarter of a compute unit's share on 256 units):
// left in one block it would outlast the rest of the launch.  At most MAX_CROSS_PARTS blocks.
constexpr int CROSS_SHARE = 1024;
constexpr int MAX_CROSS_PARTS = 64;
// Floats per tile row of a scratch slot (the widest column tile); a slot holds ufi rows.
constexpr int CROSS_ROW_FLOATS = 128;
// Column tiles one launch of a plan with such panels may hold: the scratch is sized for them.
constexpr int CROSS_MAX_TILES = 4;
// Table of the panels cut across blocks (`cross`), one entry each: the combine step's input.
constexpr int CROSS_ENTRY_WORDS = 12;
enum CrossField {
    CE_SLOT0 = 0,   // scratch slot of the panel's first block
    CE_NPARTS = 1,  // blocks of the panel
    CE_NROWS = 2,   // rows of the panel
    CE_ROW0 = 4     // CE_ROW0 + r: row of C (of the ranges' buffer in a plan cut along K) that row r of the panel is
};

}  // namespace spmm_fmt
#endif
