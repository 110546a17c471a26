// Host inspector (internal): builds the schedule-ordered arrays of
// spmm_format.h from CSR.  No HIP here; spmm_api.cpp uploads the result.
#ifndef SPMM_PLAN_H
#define SPMM_PLAN_H

#include <stdint.h>
#include <vector>

struct HostPlan {
    int64_t M = 0, K = 0, nnz = 0;
    int32_t ufi = 0;           // rows per panel (8, 4, 2 or 1)
    int32_t ufk = 8;           // enumerated columns per chunk (8, 16, 32 or 64)
    int32_t group_nnz = 0;     // nonzero budget per row group
    int32_t group_panels = 0;  // panel cap per row group

    // Row groups in launch order, five int32 each (see include/spmm.h).
    std::vector<int32_t> groups;
    // Wave-slot descriptors, ITEM_WORDS per slot, WAVES_PER_WG slots per block.
    std::vector<uint32_t> items;
    int64_t n_blocks = 0;      // workgroups of one launch
    // Chunk headers, chunk records and staging windows (already padded for the
    // kernels' look-ahead), launch order.
    std::vector<uint32_t> hdr, stream, wins;
    int64_t n_chunks = 0;      // real chunks (without the padding)
    int64_t n_enum = 0;        // enumerated columns (real column slots)
    int64_t n_split = 0;       // groups that are pieces of split panels
    int64_t n_cross = 0;       // panels cut across several blocks
    int64_t n_cross_slots = 0; // blocks of such panels: scratch slots of ufi x CROSS_ROW_FLOATS floats per column tile
    std::vector<uint32_t> cross; // CROSS_ENTRY_WORDS per such panel (spmm_format.h)
    // Rows sorted by length (skewed matrices): rowmap[i] = row of A and C that the
    // plan's row i stands for.  Empty = the plan's rows are the matrix's rows.
    std::vector<uint32_t> rowmap;
    // Plans cut along K (k_slices > 1): the plan's rows are k_slices copies of the matrix's
    // rows, copy s holding the entries whose columns fall into [s * slice_cols, (s + 1) *
    // slice_cols); every copy is padded to slice_rows rows (a multiple of the tallest panel),
    // so plan row s * slice_rows + i stands for slice s of row i (of row rowmap[...] when sorted).
    // The executor writes the slices' sums to a buffer of k_slices * slice_rows rows and a
    // second launch adds them into C.  rowmap then has plan_rows entries and holds rows of
    // that buffer.  k_slices == 1: plan_rows == M, slice_rows == M, slice_cols == K.
    int32_t k_slices = 1;
    int64_t slice_rows = 0, slice_cols = 0, plan_rows = 0;
};

struct InspectorOptions {
    int32_t group_nnz = 0;     // 0 = choose
    int32_t group_panels = 0;  // 0 = choose
    int32_t ufi = 0;           // 0 = choose; else 1, 2, 4 or 8
    int32_t n_hint = 0;        // B columns the plan is meant for; 0 = unknown
    int32_t sort_rows = 0;     // 0 = choose; > 0 = sort rows by length; < 0 = keep the row order
    int32_t threads = 0;       // 0 = choose; else host threads of the enumeration (1..64)
    int32_t cross = 0;         // 0 = choose whether panels may be cut across blocks; < 0 = never; > 0 = always
    int32_t ufk = 0;           // 0 = choose; else columns per chunk: 8, 16, 32 or 64
    int32_t kslices = 0;       // 0 = choose; 1 = never cut along K; 2, 4 or 8 = so many slices
};

// Status codes follow spmm_status_t (0 ok, 1 invalid argument, 2 invalid CSR,
// 3 allocation failure, 5 unsupported size).
int spmm_inspect(int64_t M, int64_t K, const int32_t *row_ptr, const int32_t *col_idx,
                 const float *vals, const InspectorOptions &opts, HostPlan &out);

#endif
