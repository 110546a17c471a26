// Host-side launch interface of the gfx950 kernels (internal; the public C ABI
// is include/spmm.h).
#ifndef SPMM_KERNELS_H
#define SPMM_KERNELS_H

#include <stdint.h>

struct spmm_launch_args {
    const uint32_t *hdr;    // DEVICE chunk headers
    const uint32_t *cols;   // DEVICE chunk column slots
    const uint32_t *vals;   // DEVICE chunk value blocks (float bits)
    const uint32_t *items;  // DEVICE wave-slot descriptors, 16 per block
    int32_t n_blocks;       // workgroups to launch
    const float *B;         // DEVICE first column of the column tile
    uint32_t b_bytes;       // bytes of B reachable from that pointer (narrow addressing only)
    float *C;               // DEVICE first column of the column tile
    int32_t ldn;            // leading dimension of B and C (= N)
    int32_t width;          // columns in this tile (<= 64 * vw)
};

// Enqueues one column tile.  vw = columns per lane (1 or 2); wide = byte offsets
// into B exceed 32 bits.  Returns the hipError_t of the launch as int.
int spmm_launch_chunks(const spmm_launch_args &a, int vw, bool wide, void *stream);

#endif
