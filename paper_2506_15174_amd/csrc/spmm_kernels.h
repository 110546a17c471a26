// Host-side launch interface of the gfx950 kernels (internal; the public C ABI
// is include/spmm.h).
#ifndef SPMM_KERNELS_H
#define SPMM_KERNELS_H

#include <stddef.h>
#include <stdint.h>

struct spmm_launch_args {
    const uint32_t *stream; // DEVICE staging windows: headers, column indices, value bits
    const uint32_t *wins;   // DEVICE window table
    const uint32_t *items;  // DEVICE wave-slot descriptors, 16 per block
    const uint32_t *rowmap = nullptr; // DEVICE row of C per row of the plan, or null (same rows)
    int32_t n_blocks;       // workgroups to launch
    const float *B;         // DEVICE first column of the launch's first column tile
    uint32_t b_bytes;       // bytes of B reachable from that pointer (narrow addressing only)
    float *C;               // DEVICE first column of the launch's first column tile (of the slices' buffer when k_slices > 1)
    int32_t ldn;            // leading dimension of B (= N)
    int32_t ldc;            // leading dimension of what C points to
    int32_t width;          // columns of this launch: n_tiles tiles of tile_cols, the last maybe narrower
    int32_t tile_cols;      // columns per tile (per blockIdx.y)
    int32_t n_tiles;        // column tiles of this launch (grid y)
    uint32_t col_mask;      // bits of a column word that hold the column index
    uint32_t lds_pad = 0;   // extra LDS bytes per workgroup (never touched): caps the workgroups per CU
    bool probe = false;     // launch the loads-only instance (32-bit addressing, tuned depth, chunks of 8 or 16)
    // Panels cut across workgroups (plans with n_cross > 0; else unused):
    float *cross_sums = nullptr;          // DEVICE n_tiles x n_cross_slots slots of ufi x 128 floats (scratch)
    const uint32_t *cross_table = nullptr;// DEVICE one entry per such panel: slots and rows of C
    uint32_t n_cross_slots = 0;
    int32_t n_cross = 0;
    // Plans cut along K (k_slices > 1; else unused): C above is the slices' buffer (k_slices x
    // slice_rows rows of ldc floats); a last launch adds the slices of the first M rows into C_out.
    int32_t k_slices = 1;
    int64_t slice_rows = 0, M = 0;
    float *C_out = nullptr;  // DEVICE first column of this launch in the caller's C
    int32_t ldc_out = 0;     // its leading dimension (= N)
};

// Enqueues one launch of n_tiles column tiles (plus the small launches that add the sums of
// panels cut across workgroups and of plans cut along K).  ufi = rows per panel of the plan (1, 2, 4, 8).
// slices = 2 / 4 / 8: four columns per lane (16-byte loads and stores at 4-byte alignment;
// the last lane of a tile may own fewer than four columns), tile of up to 128 / 64 / 32
// columns; slices = 1: one column per lane, tile of up to 64 columns.  wide = 64-bit
// addressing of B.  depth = chunks of B rows in flight (0 or anything deeper than the
// instance's tuned depth = the tuned depth).  Returns the hipError_t of the launch as int.
// ufk = columns per chunk of the plan: 8, or 16 / 32 / 64 with slices = 8 / 16 / 32 or 64 (tiles
// of 32 / 16 / 8 or 4 columns; 32-bit addressing and the tuned depth only).
int spmm_launch_chunks(const spmm_launch_args &a, int ufi, int ufk, int slices, bool wide, int depth, void *stream);

// Size of the library's statically allocated device scratch (one copy per device, held
// until the process ends).
#define SPMM_STATIC_SCRATCH_BYTES ((size_t)6 << 20)

// The current device's copy of that scratch: *ptr = its device address, *bytes = its size.
// The first call on a device asks the runtime for the address (no allocation: the array is
// part of the loaded code object); later calls return the kept value.  Returns a hipError_t.
int spmm_static_scratch(float **ptr, size_t *bytes);

// The pipeline depth an instance is tuned for.
int spmm_default_depth(int ufi, int slices);

#endif
