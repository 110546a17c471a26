// C ABI of the library (include/spmm.h): plan life cycle, upload, execute-time
// dispatch of the gfx950 kernels.
#include "../../include/spmm.h"

#include <hip/hip_runtime_api.h>

#include <cstring>
#include <new>
#include <vector>

#include "spmm_format.h"
#include "spmm_kernels.h"
#include "spmm_plan.h"

using namespace spmm_fmt;

struct spmm_plan {
    HostPlan host;
    bool on_device = false;
    int device = -1;
    uint32_t *d_stream = nullptr, *d_wins = nullptr, *d_items = nullptr, *d_rowmap = nullptr;
    // Panels cut across workgroups: one scratch slot of ufi x CROSS_ROW_FLOATS floats per
    // (column tile of a launch, workgroup of such a panel), written by every execute, and the
    // table of those panels.
    float *d_cross_sums = nullptr;
    uint32_t *d_cross_table = nullptr;
    // Plans cut along K: the slices' sums of one batch of up to KSLICE_COLS columns
    // (k_slices x slice_rows rows), written by every execute.
    float *d_slice_sums = nullptr;
    int64_t scratch_bytes = 0;
    int64_t device_bytes = 0;
    int64_t stream_words = 0;  // length of host.stream at creation (a device plan drops its host mirror)
    bool force_wide = false;  // spmm_options_t.force_wide: 64-bit addressing kernels also on small inputs
    int depth = 0;            // spmm_options_t.depth: pipeline depth asked for (0 = per-instance default)
    bool probe = false;       // spmm_options_t.probe: loads-only launches (measurement)
};

namespace {

// Columns a plan cut along K computes per pair of launches (the width of its slices' buffer).
constexpr int32_t KSLICE_COLS = 128;

spmm_status_t hip_fail()
{
    (void)hipGetLastError();  // clear the sticky error
    return SPMM_ERR_HIP;
}

template <typename T>
spmm_status_t upload(T **dst, const void *src, size_t bytes, int64_t &total)
{
    *dst = nullptr;
    if (bytes == 0) return SPMM_OK;
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? SPMM_ERR_ALLOC : SPMM_ERR_HIP;
    }
    *dst = static_cast<T *>(p);
    total += (int64_t)bytes;
    if (src) {
        if (hipMemcpy(p, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return hip_fail();
    } else {
        if (hipMemset(p, 0, bytes) != hipSuccess) return hip_fail();
    }
    return SPMM_OK;
}

void release_device(spmm_plan *p)
{
    if (p->d_stream) (void)hipFree(p->d_stream);
    if (p->d_wins) (void)hipFree(p->d_wins);
    if (p->d_items) (void)hipFree(p->d_items);
    if (p->d_rowmap) (void)hipFree(p->d_rowmap);
    if (p->d_cross_sums) (void)hipFree(p->d_cross_sums);
    if (p->d_cross_table) (void)hipFree(p->d_cross_table);
    if (p->d_slice_sums) (void)hipFree(p->d_slice_sums);
    p->d_stream = p->d_wins = p->d_items = p->d_rowmap = p->d_cross_table = nullptr;
    p->d_cross_sums = p->d_slice_sums = nullptr;
    (void)hipGetLastError();
}

}  // namespace

extern "C" {

spmm_status_t spmm_plan_create_ex(spmm_plan_t **plan, int64_t M, int64_t K, const int32_t *row_ptr,
                                  const int32_t *col_idx, const float *vals, const spmm_options_t *opts)
{
    if (!plan) return SPMM_ERR_INVALID_ARG;
    *plan = nullptr;
    InspectorOptions io;
    bool host_only = false, force_wide = false, probe = false;
    int depth = 0;
    if (opts) {
        if (opts->group_nnz < 0 || opts->group_panels < 0 || opts->n_hint < 0) return SPMM_ERR_INVALID_ARG;
        if (opts->ufi != 0 && opts->ufi != 1 && opts->ufi != 2 && opts->ufi != 4 && opts->ufi != 8)
            return SPMM_ERR_INVALID_ARG;
        if (opts->threads < 0 || opts->threads > 64) return SPMM_ERR_INVALID_ARG;
        if (opts->depth != 0 && opts->depth != 1 && opts->depth != 2 && opts->depth != 3 && opts->depth != 4 &&
            opts->depth != 8)
            return SPMM_ERR_INVALID_ARG;
        io.ufi = opts->ufi;
        io.group_nnz = opts->group_nnz;
        io.group_panels = opts->group_panels;
        host_only = opts->host_only != 0;
        io.n_hint = opts->n_hint;
        io.sort_rows = opts->sort_rows;
        io.threads = opts->threads;
        io.cross = opts->cross;
        if (opts->kslices != 0 && opts->kslices != 1 && opts->kslices != 2 && opts->kslices != 4 && opts->kslices != 8)
            return SPMM_ERR_INVALID_ARG;
        io.kslices = opts->kslices;
        if (opts->ufk != 0 && !valid_ufk(opts->ufk)) return SPMM_ERR_INVALID_ARG;
        io.ufk = opts->ufk;
        force_wide = opts->force_wide != 0;
        if (force_wide) io.ufk = UFK;  // the 64-bit addressing kernels read chunks of 8 columns
        if (io.kslices > 1 && io.ufk != 0 && io.ufk != UFK) return SPMM_ERR_INVALID_ARG;  // only plans with chunks of 8 are cut
        depth = opts->depth;
        probe = opts->probe != 0;
        if (probe && (force_wide || depth != 0 || (io.ufk != 0 && io.ufk > 16))) return SPMM_ERR_INVALID_ARG;
    }
    spmm_plan *p = new (std::nothrow) spmm_plan();
    if (!p) return SPMM_ERR_ALLOC;
    const int rc = spmm_inspect(M, K, row_ptr, col_idx, vals, io, p->host);
    if (rc != 0) {
        delete p;
        return (spmm_status_t)rc;
    }
    p->force_wide = force_wide;
    p->depth = depth;
    p->probe = probe;
    if (!host_only) {
        if (hipGetDevice(&p->device) != hipSuccess) {
            delete p;
            return hip_fail();
        }
        const HostPlan &h = p->host;
        spmm_status_t st = SPMM_OK;
        if (st == SPMM_OK) st = upload(&p->d_stream, h.stream.data(), h.stream.size() * 4, p->device_bytes);
        if (st == SPMM_OK) st = upload(&p->d_wins, h.wins.data(), h.wins.size() * 4, p->device_bytes);
        if (st == SPMM_OK) st = upload(&p->d_items, h.items.data(), h.items.size() * 4, p->device_bytes);
        if (st == SPMM_OK) st = upload(&p->d_rowmap, h.rowmap.data(), h.rowmap.size() * 4, p->device_bytes);
        if (st == SPMM_OK && h.n_cross_slots > 0) {
            const size_t slots = (size_t)h.n_cross_slots * CROSS_MAX_TILES;
            int64_t before = p->device_bytes;
            st = upload(&p->d_cross_sums, nullptr, slots * (size_t)h.ufi * CROSS_ROW_FLOATS * sizeof(float), p->device_bytes);
            p->scratch_bytes = p->device_bytes - before;
            if (st == SPMM_OK) st = upload(&p->d_cross_table, h.cross.data(), h.cross.size() * 4, p->device_bytes);
            // set-up for spmm_execute_static: this device's address of the static scratch is looked up here,
            // once, so that the entry point itself finds it ready (a failure only matters to that entry point)
            float *unused = nullptr;
            size_t unused_bytes = 0;
            if (spmm_static_scratch(&unused, &unused_bytes) != 0) (void)hipGetLastError();
        }
        if (st == SPMM_OK && h.k_slices > 1) {
            int64_t before = p->device_bytes;
            st = upload(&p->d_slice_sums, nullptr, (size_t)h.plan_rows * KSLICE_COLS * sizeof(float), p->device_bytes);
            p->scratch_bytes += p->device_bytes - before;
        }
        if (st != SPMM_OK) {
            release_device(p);
            delete p;
            return st;
        }
        p->on_device = true;
    }
    p->stream_words = (int64_t)p->host.stream.size();
    if (p->on_device) {
        // the arrays live on the device now: keep the descriptors (row groups, sizes), not the mirror
        std::vector<uint32_t>().swap(p->host.stream);
        std::vector<uint32_t>().swap(p->host.hdr);
        std::vector<uint32_t>().swap(p->host.wins);
        std::vector<uint32_t>().swap(p->host.items);
        // the row map stays: one bit of it (sorted or not) is part of the description
    }
    *plan = p;
    return SPMM_OK;
}

spmm_status_t spmm_plan_create(spmm_plan_t **plan, int64_t M, int64_t K, const int32_t *row_ptr,
                               const int32_t *col_idx, const float *vals)
{
    return spmm_plan_create_ex(plan, M, K, row_ptr, col_idx, vals, nullptr);
}

namespace {

// cross_sums: scratch for the sums of panels cut across workgroups, with room for
// cross_tiles column tiles of one launch (unused by plans without such panels)
spmm_status_t execute_with(const spmm_plan_t *plan, const float *B, int32_t N, float *C, void *stream,
                           float *cross_sums, int32_t cross_tiles)
{
    if (!plan || N < 1) return SPMM_ERR_INVALID_ARG;
    if (!plan->on_device) return SPMM_ERR_INVALID_ARG;
    const HostPlan &h = plan->host;
    if (h.M == 0) return SPMM_OK;
    if (!C) return SPMM_ERR_INVALID_ARG;
    if (h.K > 0 && !B) return SPMM_ERR_INVALID_ARG;
    if (((uintptr_t)B & 3u) || ((uintptr_t)C & 3u)) return SPMM_ERR_INVALID_ARG;
    // the plan's arrays live on the device that was current when it was created
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return hip_fail();
    if (dev != plan->device) return SPMM_ERR_INVALID_ARG;

    const uint64_t b_total = (uint64_t)h.K * (uint64_t)N * 4u;
    // Narrow addressing: 32-bit byte offsets into B formed by a 24 x 24-bit multiply.
    const bool narrow_ok = b_total <= 0xFFFFFFFFull && h.K < (1 << 24) && (uint64_t)N * 4u < (1u << 24);
    const bool wide = !narrow_ok || (plan->force_wide && b_total > 0);
    // Four columns per lane: 16-byte loads and stores at 4-byte alignment are legal, and a
    // last lane with fewer than four columns reads past the end of its rows of B, which is
    // safe through the buffer descriptor of the narrow addressing only (range-checked).
    const bool quads = !wide || N % 4 == 0;
    spmm_launch_args a;
    a.stream = plan->d_stream;
    a.wins = plan->d_wins;
    a.items = plan->d_items;
    a.rowmap = plan->d_rowmap;
    a.n_blocks = (int32_t)h.n_blocks;
    a.ldn = N;
    a.ldc = N;
    const bool sliced = h.k_slices > 1;
    a.k_slices = h.k_slices;
    a.slice_rows = h.slice_rows;
    a.M = h.M;
    a.col_mask = h.K <= ((int64_t)1 << spmm_fmt::COL_PATTERN_SHIFT) ? spmm_fmt::COL_INDEX_MASK : 0xFFFFFFFFu;
    a.cross_sums = cross_sums;
    a.cross_table = plan->d_cross_table;
    a.n_cross_slots = (uint32_t)h.n_cross_slots;
    a.n_cross = (int32_t)h.n_cross;
    a.probe = plan->probe;
    if (plan->probe && (wide || h.ufk > 16)) return SPMM_ERR_UNSUPPORTED;
    // the scratch of panels cut across workgroups holds so many column tiles of one launch
    const int32_t max_tiles = sliced ? 1 : h.n_cross_slots > 0 ? cross_tiles : 65535;
    // A 128-column tile of B that exceeds one L2 (4 MiB) while a 64-column tile fits: two
    // narrower tiles read the plan twice but keep their rows of B L2-resident (measured on a
    // 16384-column matrix of 13 M nonzeros: 275 against 295 us).
    // (A plan cut along K binds every slice of B to the L2s of its own XCDs instead and runs full tiles.)
    const bool narrow_tiles = !sliced && (int64_t)h.K * 512 > ((int64_t)4 << 20) && (int64_t)h.K * 256 <= ((int64_t)4 << 20);
    // Such a tile fills the L2: two workgroups per CU instead of three keep the rows of B that
    // concurrently running waves sweep inside it (same matrix: 262 against 275 us).
    a.lds_pad = narrow_tiles ? 24u << 10 : 0u;
    // Column tiles of one width share a launch (its workgroups start tile by tile, so a
    // tile begins while the previous one drains); a narrower rest takes a launch of its own.
    // Plans made for narrow B (chunks wider than 8 columns) run every N on their own narrow tiles.
    if (h.ufk != UFK && wide) return SPMM_ERR_UNSUPPORTED;
    auto tile_for = [&](int32_t left, int &slices) -> int32_t {
        if (h.ufk != UFK) {
            slices = h.ufk == 16 ? 8 : h.ufk == 32 ? 16 : left > 4 ? 32 : 64;
            return 256 / slices;
        }
        if (!quads) {
            slices = 1;
            return 64;
        }
        slices = left > 64 ? (narrow_tiles ? 4 : 2) : left > 32 ? 4 : 8;
        return 256 / slices;
    };
    int32_t j0 = 0;
    while (j0 < N) {
        // a plan cut along K takes the columns in batches its slices' buffer holds
        const int32_t left = sliced && N - j0 > KSLICE_COLS ? KSLICE_COLS : N - j0;
        int slices = 0;
        const int32_t tile = tile_for(left, slices);
        int32_t n_tiles = left / tile, cols = n_tiles * tile;
        int rest_slices = 0;
        if (n_tiles == 0 || (left > cols && tile_for(left - cols, rest_slices) == tile)) {
            n_tiles += 1;  // the narrower last tile runs on the same kernel
            cols = left;
        }
        if (n_tiles > max_tiles) {  // grid limit, or the scratch's; the loop takes the rest
            n_tiles = max_tiles;
            cols = n_tiles * tile;
        }
        a.B = B ? B + j0 : nullptr;
        a.C = C + j0;
        if (sliced) {
            // the launch writes the slices' sums, rows of (cols rounded up to 4) floats; its
            // last step adds them into C
            a.C = plan->d_slice_sums;
            a.ldc = (cols + 3) / 4 * 4;
            a.C_out = C + j0;
            a.ldc_out = N;
        }
        a.width = cols;
        a.tile_cols = tile;
        a.n_tiles = n_tiles;
        const uint64_t skipped = (uint64_t)j0 * 4u;
        a.b_bytes = wide || b_total <= skipped ? 0u : (uint32_t)(b_total - skipped);
        const int e = spmm_launch_chunks(a, h.ufi, h.ufk, slices, wide, plan->depth, stream);
        if (e != 0) return SPMM_ERR_HIP;
        j0 += cols;
    }
    return SPMM_OK;
}

}  // namespace

spmm_status_t spmm_execute(const spmm_plan_t *plan, const float *B, int32_t N, float *C, void *stream)
{
    return execute_with(plan, B, N, C, stream, plan ? plan->d_cross_sums : nullptr, CROSS_MAX_TILES);
}

spmm_status_t spmm_execute_static(const spmm_plan_t *plan, const float *B, int32_t N, float *C, void *stream)
{
    if (!plan) return SPMM_ERR_INVALID_ARG;
    const HostPlan &h = plan->host;
    if (h.k_slices > 1 && plan->on_device) return SPMM_ERR_UNSUPPORTED;  // the slices' buffer is beyond the static array
    if (h.n_cross_slots == 0 || !plan->on_device) return execute_with(plan, B, N, C, stream, nullptr, 0);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return hip_fail();
    if (dev != plan->device) return SPMM_ERR_INVALID_ARG;
    float *sums = nullptr;
    size_t bytes = 0;
    if (spmm_static_scratch(&sums, &bytes) != 0) return hip_fail();
    // one column tile of a launch needs a slot of ufi x CROSS_ROW_FLOATS floats per workgroup of a cut panel
    const size_t per_tile = (size_t)h.n_cross_slots * (size_t)h.ufi * CROSS_ROW_FLOATS * sizeof(float);
    if (per_tile > bytes) return SPMM_ERR_UNSUPPORTED;
    const size_t tiles = bytes / per_tile;
    return execute_with(plan, B, N, C, stream, sums, (int32_t)(tiles < 65535 ? tiles : 65535));
}

spmm_status_t spmm_plan_destroy(spmm_plan_t *plan)
{
    if (!plan) return SPMM_OK;
    if (plan->on_device) release_device(plan);
    delete plan;
    return SPMM_OK;
}

spmm_status_t spmm_plan_describe(const spmm_plan_t *plan, spmm_plan_info_t *out)
{
    if (!plan || !out) return SPMM_ERR_INVALID_ARG;
    const HostPlan &h = plan->host;
    std::memset(out, 0, sizeof(*out));
    out->M = h.M;
    out->K = h.K;
    out->nnz = h.nnz;
    out->ufi = h.ufi;
    out->ufk = h.ufk;
    out->group_nnz = h.group_nnz;
    out->group_panels = h.group_panels;
    out->n_groups = (int64_t)(h.groups.size() / 5);
    out->n_blocks = h.n_blocks;
    out->n_split = h.n_split;
    out->n_enum = h.n_enum;
    out->n_chunks = h.n_chunks;
    out->stream_words = plan->stream_words;
    out->device_bytes = plan->device_bytes;
    out->sorted_rows = h.rowmap.empty() ? 0 : 1;
    out->n_cross = h.n_cross;
    out->scratch_bytes = plan->scratch_bytes;
    out->k_slices = h.k_slices;
    out->slice_rows = h.slice_rows;
    out->slice_cols = h.slice_cols;
    return SPMM_OK;
}

spmm_status_t spmm_plan_get_groups(const spmm_plan_t *plan, int32_t *out, int64_t cap)
{
    if (!plan || !out) return SPMM_ERR_INVALID_ARG;
    const HostPlan &h = plan->host;
    const int64_t n = (int64_t)(h.groups.size() / 5);
    if (cap < n) return SPMM_ERR_INVALID_ARG;
    if (n) std::memcpy(out, h.groups.data(), (size_t)n * 5 * sizeof(int32_t));
    return SPMM_OK;
}

spmm_status_t spmm_plan_get_array(const spmm_plan_t *plan, int32_t which, uint32_t *out, int64_t cap_words,
                                  int64_t *n_words)
{
    if (!plan) return SPMM_ERR_INVALID_ARG;
    if (plan->on_device) return SPMM_ERR_INVALID_ARG;  // only host-only plans keep the mirror
    const HostPlan &h = plan->host;
    if (which == SPMM_ARRAY_ROWMAP) {
        // M entries for a plan with sorted rows (the vector carries padding for the kernel), else none
        const int64_t n = h.rowmap.empty() ? 0 : h.plan_rows;
        if (n_words) *n_words = n;
        if (!out) return SPMM_OK;
        if (cap_words < n) return SPMM_ERR_INVALID_ARG;
        if (n) std::memcpy(out, h.rowmap.data(), (size_t)n * 4);
        return SPMM_OK;
    }
    const std::vector<uint32_t> *v = nullptr;
    switch (which) {
    case SPMM_ARRAY_HDR: v = &h.hdr; break;
    case SPMM_ARRAY_STREAM: v = &h.stream; break;
    case SPMM_ARRAY_WINS: v = &h.wins; break;
    case SPMM_ARRAY_ITEMS: v = &h.items; break;
    case SPMM_ARRAY_CROSS: v = &h.cross; break;
    default: return SPMM_ERR_INVALID_ARG;
    }
    if (n_words) *n_words = (int64_t)v->size();
    if (!out) return SPMM_OK;
    if (cap_words < (int64_t)v->size()) return SPMM_ERR_INVALID_ARG;
    if (!v->empty()) std::memcpy(out, v->data(), v->size() * 4);
    return SPMM_OK;
}

const char *spmm_status_string(spmm_status_t status)
{
    switch (status) {
    case SPMM_OK: return "ok";
    case SPMM_ERR_INVALID_ARG: return "invalid argument";
    case SPMM_ERR_INVALID_CSR: return "invalid CSR structure";
    case SPMM_ERR_ALLOC: return "allocation failed";
    case SPMM_ERR_HIP: return "HIP runtime error";
    case SPMM_ERR_UNSUPPORTED: return "size not supported";
    default: return "unknown status";
    }
}

}  // extern "C"
