/*
 * spmm.h -- C ABI of the MI355X (gfx950) sparse-times-dense library.
 *
 * Computes C = A x B in fp32 where A (M x K) is an unstructured-sparse weight
 * matrix handed over once in CSR, B (K x N) is a dense row-major activation
 * matrix and C (M x N) is dense row-major (paper: Section 1, second paragraph
 * and Section 2, first paragraph, for the operands; Section 3.1, Listing 1,
 * for the sum that defines every element of C).
 *
 * The three-phase shape of the interface is the paper's inspector / executor
 * split (Section 3.1, Listing 2; Section 3.4 "Data transformer"): the weight
 * matrix is analysed and re-stored once, the product is then executed many
 * times against changing activations.
 *
 * No HIP or C++ type appears here.  Pointers are tagged HOST or DEVICE.
 * No call aborts or throws; every failure is a status code.
 */
#ifndef SPMM_CDNA4_H
#define SPMM_CDNA4_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmm_plan spmm_plan_t; /* opaque */

typedef enum {
    SPMM_OK = 0,
    SPMM_ERR_INVALID_ARG = 1, /* null pointer, negative or oversized dimension, N < 1,
                                 misaligned device pointer, host-only plan executed */
    SPMM_ERR_INVALID_CSR = 2, /* row_ptr[0] != 0, decreasing row_ptr, column outside [0, K) */
    SPMM_ERR_ALLOC = 3,       /* host or device allocation failed */
    SPMM_ERR_HIP = 4,         /* any other HIP runtime failure (sticky error cleared) */
    SPMM_ERR_UNSUPPORTED = 5  /* size outside the index range of the kernels */
} spmm_status_t;

/* Schedule constants and sizes of a plan (all read-only facts). */
typedef struct {
    int64_t M, K, nnz;
    int32_t ufi;           /* rows per panel: height of the register tile (the paper's UFi): 8, 4, 2 or 1 */
    int32_t ufk;           /* enumerated columns per chunk, the unit a wave requests and multiplies at
                              a time (the paper's UFk): 8, or 16 / 32 / 64 in plans made for B of at
                              most 32 / 16 / 8 columns */
    int32_t group_nnz;     /* nonzero budget of one row group (one wave's work item) */
    int32_t group_panels;  /* most panels a row group may hold */
    int64_t n_groups;      /* row groups = wave-level work items, in launch order */
    int64_t n_blocks;      /* workgroups of one launch (8 wave slots each) */
    int64_t n_split;       /* row groups that are pieces of a panel too heavy for one group */
    int64_t n_enum;        /* enumerated columns: B rows a column tile must fetch per execute */
    int64_t n_chunks;      /* chunks: runs of at most ufk enumerated columns of one pattern */
    int64_t stream_words;  /* 32-bit words of the staged stream (headers, column indices, values, padding) */
    int64_t device_bytes;  /* device memory the plan holds (0 for a host-only plan) */
    int64_t sorted_rows;   /* 1: the plan's rows are the matrix's rows sorted by length, longest first
                              (SPMM_ARRAY_ROWMAP gives the order); 0: the plan's rows are the matrix's */
    int64_t n_cross;       /* panels cut into more pieces than one workgroup has waves: their
                              workgroups' sums meet in scratch memory of the plan */
    int64_t scratch_bytes; /* scratch memory of the plan that executes write (part of device_bytes): the
                              sums of panels cut across workgroups and of plans cut along K; 0 when
                              n_cross is 0 and k_slices is 1 */
    int64_t k_slices;      /* 1, or the number of column ranges of A (2, 4 or 8) the plan is cut into:
                              the plan then has k_slices * slice_rows rows, row s * slice_rows + i
                              holding the entries of row i whose columns lie in range s */
    int64_t slice_rows;    /* rows per range of such a plan: M rounded up to a multiple of 8 (M when
                              k_slices is 1) */
    int64_t slice_cols;    /* columns per range: ceil(K / k_slices) */
} spmm_plan_info_t;

/* Optional inspector settings; zero in a field means "let the inspector choose". */
typedef struct {
    int32_t group_nnz;     /* override the nonzero budget per row group (>= 8) */
    int32_t group_panels;  /* override the panel cap per row group (>= 1) */
    int32_t host_only;     /* nonzero: build the plan in host memory only (no device needed;
                              such a plan can be described and exported but not executed) */
    int32_t ufi;           /* force the rows per panel: 1, 2, 4 or 8 (0 = choose) */
    int32_t n_hint;        /* number of B columns the plan will mostly be executed with
                              (0 = unknown, >= 0).  Only the choice of the schedule
                              constants looks at it, as the paper's tuner does per bCols
                              (Section 3.5); the plan stays valid for every N. */
    int32_t sort_rows;     /* > 0: sort the rows by length, longest first, before forming panels
                              (C is still written in the caller's row order); < 0: keep the row
                              order; 0: sort when the rows longer than four times the mean hold
                              a quarter of the entries and the chosen panels are taller than one row */
    int32_t force_wide;    /* nonzero: spmm_execute uses the 64-bit addressing kernels also where B
                              is small enough for 32-bit offsets (lets small inputs exercise them) */
    int32_t threads;       /* host threads of the inspector, 1..64 (0 = one per two million entries,
                              at most 16 and at most the machine's; the plan does not depend on it) */
    int32_t depth;         /* chunks of B rows a wave keeps in flight (the software pipeline's depth,
                              the paper's unroll(k, UFk) axis of Figure 2): 1, 2, 3, 4 or 8;
                              0 = the depth tuned per kernel instance.  A depth the register budget
                              of an instance cannot hold is lowered to the deepest one it can. */
    int32_t cross;         /* whether a panel heavier than eight group budgets and than 1/1024 of all
                              entries is cut across workgroups (their sums meet in scratch memory of
                              the plan and a second, small launch adds them): < 0 never (no scratch,
                              any number of executes of the plan may overlap); > 0 always; 0: when the
                              row lengths are skewed (see sort_rows), A holds 2^20 entries or more and
                              n_hint is 0 or above 32.  Such a plan also halves its group budget. */
    int32_t ufk;           /* force the enumerated columns per chunk: 8, 16, 32 or 64 (0 = choose from
                              n_hint: 8 for more than 32 columns or unknown, else 16 / 32 / 64 for up to
                              32 / 16 / 8 columns; always 8 for more than 2^24 columns of A and with
                              force_wide).  A plan with wider chunks computes every N on column tiles
                              of 32 / 16 / 8 (or 4) columns and cannot address a B beyond 4 GiB
                              (spmm_execute then returns SPMM_ERR_UNSUPPORTED). */
    int32_t probe;         /* nonzero: a measuring plan.  spmm_execute requests and awaits every row
                              of B exactly as the product does but skips the multiply-adds, and C
                              becomes all zeros: the time of such an execute is the on-chip gather
                              ceiling of this plan's own index stream.  Not combinable with
                              force_wide, depth or chunks wider than 16 columns (SPMM_ERR_INVALID_ARG);
                              a B that needs 64-bit addressing is refused (SPMM_ERR_UNSUPPORTED). */
    int32_t kslices;       /* cut the plan along K: 2, 4 or 8 column ranges; 1 = never; 0 = choose.
                              Every workgroup then works on one range and workgroup b of the launch
                              on range b mod kslices, so that each of the GPU's eight L2 caches (one
                              per XCD, workgroups are dealt to the XCDs in turn) holds the rows of B of
                              one range only; the ranges' sums of C meet in scratch memory of the plan
                              (kslices * slice_rows * 128 floats) and a last, small launch adds them
                              in range order.  Chosen (0) when a column tile of B is larger than one
                              L2 (more than 8192 columns of A at more than 64 columns of B or an
                              unknown number, more than 16384 at 33 to 64), A holds 2^20 entries or
                              more and its rows at least 32 entries per range on average, and when
                              the tile is exactly one L2 and the rows hold 1024 entries or more; never for
                              plans with chunks wider than 8 (SPMM_ERR_INVALID_ARG if both are forced).
                              At most one execute of such a plan may be in flight at a time. */
} spmm_options_t;

/*
 * Inspector (paper Section 3.2 "Enumeration", Section 3.3 "Data
 * transformation", Section 3.4 "Data transformer"; here from CSR in O(nnz log)
 * rather than from dense A).  Validates the CSR, orders the columns of every
 * row, picks the panel height `ufi` and the group budget from the shape, the
 * number of nonzeros and the B-column hint, sorts the rows by length when their
 * lengths are very uneven (so that a panel holds rows of like length; C keeps
 * the caller's row order), enumerates nnz-balanced row groups,
 * merges the columns of each panel of `ufi` rows into enumerated columns tagged
 * with their nonzero pattern, re-stores the values in schedule order and
 * uploads the result.
 *
 *   plan     HOST  out; set to NULL on failure
 *   M, K     rows / columns of A; 0 is legal
 *   row_ptr  HOST  int32[M+1], row_ptr[0] == 0, non-decreasing; nnz = row_ptr[M]
 *   col_idx  HOST  int32[nnz], each in [0, K); any order inside a row; duplicates
 *                  are legal and are summed
 *   vals     HOST  float[nnz]; finite values (explicit zeros are ordinary terms)
 *
 * The three arrays are only read during the call; the caller may free them when
 * it returns.  The plan owns its device memory on the device that is current at
 * the time of the call.
 */
spmm_status_t spmm_plan_create(spmm_plan_t **plan, int64_t M, int64_t K,
                               const int32_t *row_ptr, const int32_t *col_idx,
                               const float *vals);

/*
 * Same, with explicit settings (opts may be NULL = all zero).  The settings are
 * the only way to steer the inspector: the library reads no environment
 * variable.
 */
spmm_status_t spmm_plan_create_ex(spmm_plan_t **plan, int64_t M, int64_t K,
                                  const int32_t *row_ptr, const int32_t *col_idx,
                                  const float *vals, const spmm_options_t *opts);

/*
 * Executor (paper Section 3.3 "Sparse Coarsen", Listings 5-7): C <- A x B.
 *
 *   B       DEVICE  const float[K*N], row-major, leading dimension N, finite values
 *   N       columns of B and C, >= 1 (32, 64 and 128 have tuned kernels; every
 *           other N runs through masked column tiles of at most 128 columns; tiles
 *           of one width share a kernel launch, a narrower rest takes a launch of
 *           its own, so N = 256 is one launch and N = 130 costs one of 128 columns
 *           and one of 2; tiles of 64 when 128 columns of B exceed one L2 cache
 *           and 64 fit)
 *   C       DEVICE  float[M*N], row-major, leading dimension N; every element is
 *           overwritten (rows of A without nonzeros become +0.0); must not alias B
 *   stream  hipStream_t passed as void* (NULL = the default stream)
 *
 * The device that was current at plan creation must be current again (else
 * SPMM_ERR_INVALID_ARG), and `stream`, B and C must belong to it.
 * Asynchronous: kernels are enqueued on `stream` and the call returns.  It
 * allocates nothing and does not synchronise.  The plan is read-only during
 * execution (pieces of a split panel meet in on-chip memory, not in the plan),
 * so any number of executes of one plan may be in flight on any streams -- unless the
 * plan holds panels cut across workgroups (info.n_cross > 0): their sums meet in scratch
 * memory of the plan, so at most one execute of such a plan may be in flight at a time;
 * the same holds for a plan cut along K (info.k_slices > 1), whose ranges' sums meet in
 * scratch memory of the plan and are added by a last launch, 128 columns at a time.
 * Results are bit-identical from run to run.  B and C must be 4-byte aligned.
 * Every N runs on the kernels that handle four columns per lane (the last lane of
 * a row stores only the columns that exist; rows that are not 16-byte aligned cost
 * some cache efficiency), except products that need 64-bit addressing of B with N
 * not a multiple of 4, which run on a one-column-per-lane kernel.
 */
spmm_status_t spmm_execute(const spmm_plan_t *plan, const float *B, int32_t N,
                           float *C, void *stream);

/*
 * spmm_execute for callers that cannot tolerate any device allocation behind the
 * product, not even the plan's own: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation calls.  Same arguments, same result bit for bit.
 * The sums of panels cut across workgroups (info.n_cross > 0) go to a scratch array that
 * is part of the library's code object (6 MiB per device, held until the process ends)
 * instead of the plan's scratch memory; plans without such panels run exactly as
 * spmm_execute.  The call allocates and frees nothing; the first call on a device (or
 * the creation of a plan with cut panels on it) asks the runtime for the array's address.
 *
 * One column tile of a launch needs 512 * ufi bytes per workgroup of a cut panel; the
 * call packs as many column tiles into a launch as the array holds and returns
 * SPMM_ERR_UNSUPPORTED, enqueuing nothing, when a single tile does not fit, and for
 * every plan cut along K (info.k_slices > 1: its sums need more than the array holds).
 * All plans and all callers on one device share the array, which keeps the last call's
 * content (every launch overwrites what it reads, nothing needs clearing): calls that
 * overlap in time on one device race, also on different streams and for different plans.
 */
spmm_status_t spmm_execute_static(const spmm_plan_t *plan, const float *B, int32_t N,
                                  float *C, void *stream);

/*
 * The calls below manage and describe a plan.  The paper defines no counterpart for them
 * (its transformed matrix lives as long as the generated program and is never inspected):
 * they exist for ownership (destroy), for the bit-exact re-derivation of the row groups and
 * the format round trip in the tests (describe, get_groups, get_array) and for messages.
 */

/* Frees the plan and its device memory.  NULL is a no-op returning SPMM_OK. */
spmm_status_t spmm_plan_destroy(spmm_plan_t *plan);

/* Read-only introspection: schedule constants and sizes. */
spmm_status_t spmm_plan_describe(const spmm_plan_t *plan, spmm_plan_info_t *out);

/*
 * Row groups in launch order, five int32 each:
 *   row_begin, row_end   rows of the plan the group covers: rows of A (and of C),
 *                        or, when info.sorted_rows is set, positions in the
 *                        length-sorted row order (SPMM_ARRAY_ROWMAP); in a plan cut
 *                        along K, row s * info.slice_rows + i is range s of row
 *                        (or position) i, and rows M .. slice_rows - 1 of a range are empty
 *   nnz_begin, nnz_end   its range in the schedule-ordered value sequence; for a
 *                        group of whole panels this equals the range
 *                        ptr[row_begin] .. ptr[row_end] of the row pointer of the
 *                        plan's row order (row_ptr itself unless rows are sorted)
 *   flags                bit 0: the group is one piece of a split panel; bit 3: of a panel
 *                        cut into more pieces than a workgroup has waves (info.n_cross)
 * Order: pieces of split panels first (heaviest panel first, pieces in order),
 * then groups of whole panels (heaviest first); ties keep row order.  In a plan cut
 * along K both parts list range after range (heaviest first inside a range), and the
 * workgroups (8 groups each, never of two ranges) are then dealt to the ranges in turn.
 *   out  HOST int32[5 * cap];  cap must be >= info.n_groups.
 */
spmm_status_t spmm_plan_get_groups(const spmm_plan_t *plan, int32_t *out, int64_t cap);

/*
 * Raw copies of the plan's schedule-ordered arrays, for format round-trip tests
 * and byte accounting.  Only a host-only plan keeps them (a plan on a device
 * holds them in device memory and drops the host mirror): on any other plan the
 * call returns SPMM_ERR_INVALID_ARG.  Layouts are those the kernels read:
 *   SPMM_ARRAY_HDR     one word per chunk, launch order (host-side copy): bits 0-7
 *                      pattern (panel rows that own a value in some column of the
 *                      chunk), bits 8-14 number of real columns (at most info.ufk),
 *                      bit 15 last chunk of its panel
 *   SPMM_ARRAY_WINS    one word per LDS staging window of a group: bits 0-15 chunks,
 *                      bits 16-31 words (at most 1024; 2048 when info.ufk is 32 or 64)
 *   SPMM_ARRAY_STREAM  the windows back to back, each as: the headers of its chunks
 *                      (zero-padded to a multiple of 8 words); ufk column words per
 *                      chunk (bits 0-23 the column index, unused slots repeat a real
 *                      column; bits 24-31 the slot's own pattern where leftovers of
 *                      several patterns share a chunk and the slot's pattern is
 *                      smaller than the chunk's, else 0); per chunk one block of ufk
 *                      float bit patterns per set pattern row in ascending row order
 *                      (zeros in unused slots and where a slot lacks the row)
 *   SPMM_ARRAY_ITEMS   16 words per wave slot, 8 slots per workgroup, launch order:
 *                      first row, rows, first chunk, chunks, first record word, flags
 *                      (1 piece of a split panel, 2 idle slot, 4 workgroup with split
 *                      panels, 8 workgroup of a panel cut across workgroups), the
 *                      slot's share of the split-panel sums (pieces to add, first
 *                      piece's slot, tile row, row of C), first window, windows, a copy
 *                      of the first window's SPMM_ARRAY_WINS entry, and for a panel cut
 *                      across workgroups the number of its workgroups, the scratch slot
 *                      of its first one and this workgroup's place among them
 *                      (rows are rows of the plan, except the row of C, which is
 *                      always a row of the matrix, plus s * slice_rows in a plan cut along K)
 *   SPMM_ARRAY_ROWMAP  M words when info.sorted_rows is set, else none: the row of
 *                      A and C that each row of the plan stands for (rows by
 *                      decreasing length, equal lengths in ascending row order); in a
 *                      plan cut along K k_slices * slice_rows words: for plan row
 *                      s * slice_rows + i the value s * slice_rows + (row of A and C)
 *   SPMM_ARRAY_CROSS   12 words per panel cut across workgroups (info.n_cross entries, in the
 *                      order their workgroups are launched): first scratch slot, workgroups,
 *                      rows of the panel, one unused word, then the row of C of each of the
 *                      panel's rows (8 words, unused ones 0): the input of the launch that
 *                      adds the workgroups' sums
 *   out   HOST, cap_words 32-bit words of room; *n_words (may be NULL) receives the
 *         array's length.  out == NULL only queries the length.  A too small
 *         cap_words copies nothing and returns SPMM_ERR_INVALID_ARG.
 */
enum { SPMM_ARRAY_HDR = 0, SPMM_ARRAY_STREAM = 1, SPMM_ARRAY_WINS = 2, SPMM_ARRAY_ITEMS = 3, SPMM_ARRAY_ROWMAP = 4,
       SPMM_ARRAY_CROSS = 5 };
spmm_status_t spmm_plan_get_array(const spmm_plan_t *plan, int32_t which,
                                  uint32_t *out, int64_t cap_words, int64_t *n_words);

const char *spmm_status_string(spmm_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* SPMM_CDNA4_H */
