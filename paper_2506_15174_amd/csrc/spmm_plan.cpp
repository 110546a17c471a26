// Host inspector: CSR -> nnz-balanced row groups -> per-panel enumeration of
// nonzero patterns -> chunked, schedule-ordered arrays (spmm_format.h).
//
// Paper correspondence: Section 3.2 "Enumeration" (panels of UFI rows, one
// enumerated block per nonzero pattern, columns of equal pattern listed
// together), Section 3.3.3 "Data transformation" and Section 3.4 "Data
// transformer" (values re-stored in the order the schedule consumes them, one
// column index per enumerated column).  The paper scans dense A in O(M K); this
// builds the same structure from CSR in O(nnz) plus a per-row sort only for rows
// whose columns arrive unsorted.  Large inputs are enumerated and laid out by
// several host threads over contiguous ranges of row groups; the result does not
// depend on their number.
#include "spmm_plan.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <system_error>
#include <thread>

#include "spmm_format.h"

using namespace spmm_fmt;

namespace {

enum { ST_OK = 0, ST_INVALID_ARG = 1, ST_INVALID_CSR = 2, ST_ALLOC = 3, ST_UNSUPPORTED = 5 };

struct Group {
    int32_t row_begin, row_end, nnz_begin, nnz_end, flags;
    int32_t seg, nseg;  // piece index / pieces of the panel (split groups only)
    // filled while emitting: the emitter that holds the group's chunks and the group's place in it
    int32_t part = 0;
    int64_t chunk0 = 0, n_chunks = 0, words0 = 0, n_words = 0;
};

// One enumerated column of a panel: a column index with the set of panel rows
// that hold a value there.
struct Entry {
    int32_t col;
    uint32_t pattern;
    float v[MAX_UFI];  // indexed by row inside the panel
};

// ---- schedule selection (all in integers, from M, K, nnz and the caller's hint) ---
//
// The paper tunes the panel height once per architecture and per number of B
// columns by timing candidates (Section 3.5 "Scheduler & Tuner").  The closed rule
// below is the outcome of that exercise on MI355X, fitted to timings of pruned-layer
// shapes (256 .. 8192 rows and columns, 50 .. 98 % pruned) with forced heights.
// `row` is the mean number of entries per row.
//
//   * whatever the width: single rows when the rows of B a column tile touches
//     (K rows of 128 / 256 / 512 bytes for narrow / medium / wide B) exceed the
//     4 MiB of one L2: every wave then sweeps B in ascending row order and waves
//     that run together stay close together in B, which tall panels (pattern by
//     pattern) give up; except that wide B whose 64-column tiles fit one L2
//     (8192 < K <= 16384, run as tiles of 64 columns) takes eight rows from 4096
//     rows on with row >= 1024 (16384 x 16384 at 90 %: 434 against 521 us; at
//     98 %, row 327, single rows win 118 against 159 us);
//   * what a tall panel saves are the columns its rows have in common; two rows of the mean
//     length share about row * row / K of them (`shared` below);
//   * narrow B (hint <= 32 columns): one wave load already covers eight enumerated
//     columns, so tall panels save fewer loads: from 4096 rows on eight rows with
//     row >= 768 and four with row >= 384 in rows at least an eighth full (chunks of 16
//     columns, two per slice: 4096 x 4096 at 50 % 27.7 against 32.3 us with four rows,
//     4096 x 1024 at 50 % 10.2 with four rows against 12.7 us with single rows); four rows
//     under the same condition for 2048 .. 4095 rows (2048 x 8192 at 70 %: 23.9 against
//     27.3 us with two rows); two rows for 1024 .. 2047 rows with row >= 256 in rows at
//     least a third full, for 512 .. 1023 rows with row >= 256; else single rows;
//   * medium B (hint 33 .. 64): eight rows from 4096 rows on with row >= 128 and shared
//     >= 16; four rows for 2048 .. 4095 rows with row >= 256 and shared >= 32; two rows for
//     1024 .. 2047 rows with shared >= 128 and for 512 .. 1023 rows with row >= 64; else
//     single rows;
//   * wide or unknown B: eight rows from 2048 rows on with row >= 128 and shared >= 16
//     (2048 x 8192 at 70 %: 62 against 71 us with four rows); for 1024 .. 2047 rows four
//     rows with row >= 128 and two with row >= 64; two rows for 512 .. 1023 rows with
//     row >= 128; else single rows.
//
// Short rows leave most patterns with one row set, so tall panels share nothing;
// few rows cannot fill the chip with tall panels (a split panel of eight rows owns
// a whole workgroup: 1024 rows give 128 workgroups).
int choose_ufi(int64_t M, int64_t K, int64_t nnz, int32_t n_hint)
{
    const int64_t row = M > 0 ? nnz / M : 0;
    const bool narrow = n_hint > 0 && n_hint <= 32;
    const bool medium = n_hint > 32 && n_hint <= 64;
    const int64_t tile_row_bytes = narrow ? 128 : medium ? 256 : 512;
    const int64_t l2 = (int64_t)4 << 20;
    if (K * tile_row_bytes > l2) {
        // Wide B whose 64-column tiles still fit (the executor then runs tiles of 64 columns):
        // the tile fills the L2, and eight rows pay from much longer rows on than below
        if (!narrow && !medium && K * 256 <= l2 && M >= 4096 && row >= 1024) return 8;
        return 1;
    }
    const int64_t shared = K > 0 ? row * row / K : 0;
    if (n_hint > 0 && n_hint <= 16) {
        // Chunks of 32 or 64 columns, one lane or a few per row of B: a wave load already covers 16
        // to 64 enumerated columns, and what a tall panel saves in loads it pays in multiply slots of
        // absent rows.  Eight rows only where two rows share most of their columns (from 4096 rows
        // on: shared >= 160 for 9 .. 16 columns of B, 320 for 5 .. 8, 640 for up to 4: 4096 x 4096 at
        // 80 %, shared 163, 4 columns: 7.5 us with single rows against 12.3 us with eight); for 9 ..
        // 16 columns also the four and two rows of the rule for 17 .. 32 columns below.
        const int64_t need = n_hint <= 4 ? 640 : n_hint <= 8 ? 320 : 160;
        if (M >= 4096 && shared >= need) return 8;
        if (n_hint > 8) {
            if (M >= 2048) return row >= 384 && 8 * row >= K ? 4 : 1;
            if (M >= 1024) return row >= 256 && 3 * row >= K ? 2 : 1;
        }
        return 1;
    }
    if (narrow) {
        if (M >= 4096) return row >= 768 ? 8 : row >= 384 && 8 * row >= K ? 4 : 1;
        if (M >= 2048) return row >= 384 && 8 * row >= K ? 4 : 1;
        if (M >= 1024) return row >= 256 && 3 * row >= K ? 2 : 1;
        if (M >= 512) return row >= 256 ? 2 : 1;
        return 1;
    }
    if (medium) {
        if (M >= 4096) return row >= 128 && shared >= 16 ? 8 : 1;
        if (M >= 2048) return row >= 256 && shared >= 32 ? 4 : 1;
        if (M >= 1024) return shared >= 128 ? 2 : 1;
        if (M >= 512) return row >= 64 ? 2 : 1;
        return 1;
    }
    if (M >= 2048) return row >= 128 && shared >= 16 ? 8 : 1;
    if (M >= 1024) return row >= 128 ? 4 : row >= 64 ? 2 : 1;
    if (M >= 512) return row >= 128 ? 2 : 1;
    return 1;
}

// Panel height for a matrix whose rows are sorted by length (skewed_rows below).
// The longest rows then sit in the same panels and share most of their columns,
// but a panel is processed by one workgroup, cut into at most eight pieces: a
// panel much heavier than a compute unit's fair share of the matrix (nnz / 256)
// becomes the tail of the launch.  The height is the largest power of two h <= 8
// with h * (longest row) <= 2 * fair share (measured on Zipf-distributed row
// lengths from 1024 to 16384 rows: the best forced height follows this bound
// within 12 %); narrow B halves the gain of a tall panel, so it takes two rows
// where wide B would take four or more, else single rows.  A tile of B beyond one
// L2 keeps single rows as above (for more than 64 columns the executor narrows
// the tile to 64 columns first).  Height 1 means the rows are not sorted at all.
//
// When panels may be cut across workgroups (cross_allowed below) a heavy panel is no
// longer bound to one workgroup and the tail argument falls away: wide B takes eight
// rows and medium B four (measured on the same matrices with every height forced and the
// group budget halved: 13 % and 6 % faster in geometric mean than the bound above;
// narrow B gains nothing from taller panels and keeps the bound).
int choose_ufi_skewed(int64_t K, int64_t nnz, int64_t max_row, int32_t n_hint, bool cross)
{
    const bool narrow = n_hint > 0 && n_hint <= 32;
    const bool medium = n_hint > 32 && n_hint <= 64;
    const int64_t l2 = (int64_t)4 << 20;
    const int64_t tile_row_bytes = narrow ? 128 : medium ? 256 : K * 512 > l2 ? 256 : 512;
    if (K * tile_row_bytes > l2) return 1;
    if (cross && !narrow) return medium ? 4 : 8;
    const int64_t fair = std::max<int64_t>(1, nnz / 256);
    int h = 1;
    while (h < MAX_UFI && 2 * h * max_row <= 2 * fair) h *= 2;
    if (narrow) return h >= 4 ? 2 : 1;
    return h;
}

// Columns per chunk.  A slice of a wave (the lanes that share one row of B, four columns
// per lane) should own two column slots of every chunk: with one slot per slice the fixed
// work per chunk (header, row branches, offsets) outweighs its multiply-adds.  B of up to 32
// columns runs on 8 slices (16 columns per chunk), up to 16 columns on 16 slices (32), up to
// 8 columns on 32 slices (64).  Matrices of more than 2^24 columns keep 8: their column
// words hold no slot pattern and their B needs 64-bit addressing, which only the kernels for
// chunks of 8 have.
int choose_ufk(int64_t K, int32_t n_hint)
{
    if (K > ((int64_t)1 << COL_PATTERN_SHIFT) || n_hint <= 0 || n_hint > 32) return 8;
    return n_hint > 16 ? 16 : n_hint > 8 ? 32 : 64;
}

// Nonzero budget G of a row group and the cap GP on the panels one group packs.
// P panels of mean weight `mean`:
//   * fewer than 4096 panels: a typical panel is cut into ppt = min(8, ceil(8192 / P))
//     pieces so that the launch holds about 8192 waves (4096 waves, from fewer than 2048
//     panels, for B of at most 16 columns; a quarter as many was no better);
//   * 4096 panels or more: panels stay whole, and beyond 8192 panels GP =
//     ceil(P / 8192) of them (at most 16) share a wave.
// G = ceil(5 mean GP / (4 ppt)), rounded up to a multiple of 32 inside [32, 1024];
// the quarter of headroom keeps panels near the mean on the typical piece count.
// Single rows of a matrix of 1024 .. 2047 rows meant for B of at most 64 columns are not cut
// below 128 entries, nor into more than two pieces below 256: such products take 3 to 5 us, and
// waves of 32 entries cost them 10 to 20 % in start-up (every wave first fetches its
// descriptor, its first window and its first rows of B) and in workgroups to dispatch, while
// whole rows of 200 and more entries leave the chip short of waves (1024 x 1024 at 80 %,
// 64 columns: 4.4 us in halves against 5.8 us whole).
// Wider B and matrices of fewer rows need the finer cut to occupy the chip.
void choose_group_budget(int64_t M, int64_t nnz, int ufi, int32_t n_hint, int32_t &G_out, int32_t &GP_out)
{
    const int64_t P = std::max<int64_t>(1, (M + ufi - 1) / ufi);
    const int64_t mean = (nnz + P - 1) / P;
    // B of at most 16 columns: half as many waves of twice the work (a wave's chunk of 32 or 64
    // columns is little arithmetic against its fixed start-up; 2048 x 4096 at 90 %, 4 columns:
    // 5.6 us with rows cut in two against 7.4 us cut in four)
    const int64_t waves = n_hint > 0 && n_hint <= 16 ? 4096 : 8192;
    const int64_t ppt = P < waves / 2 ? std::min<int64_t>(8, (waves + P - 1) / P) : 1;
    const int64_t GP = std::min<int64_t>(16, std::max<int64_t>(1, (P + 8191) / 8192));
    int64_t g = (5 * mean * GP + 4 * ppt - 1) / (4 * ppt);
    if (ufi == 1 && M >= 1024 && M < 2048 && n_hint > 0 && n_hint <= 64)
        g = std::max<int64_t>(g, std::min<int64_t>((5 * mean + 7) / 8, 128));
    g = (g + 31) / 32 * 32;
    if (g < 32) g = 32;
    if (g > 1024) g = 1024;
    G_out = (int32_t)g;
    GP_out = (int32_t)GP;
}

// Panels may be cut across workgroups (their sums then meet in scratch memory and a second,
// small launch adds them) when the caller insists (setting > 0), or, by default, when the
// row lengths are skewed and the matrix holds at least 2^20 entries: on smaller products
// the second launch costs more than the balance gains (2048 x 2048 Zipf rows: + 3 us on
// 9 .. 16 us), and matrices of even row lengths have no panel that outlasts the others.
// Narrow B (hint of 32 columns or fewer) keeps every panel in one workgroup: its products
// are short and the finer cut lost on most of them (8192 x 8192 Zipf rows: 25 -> 29 us).
bool cross_allowed(int32_t setting, bool skewed, int64_t nnz, int32_t n_hint)
{
    if (setting != 0) return setting > 0;
    const bool narrow = n_hint > 0 && n_hint <= 32;
    return skewed && !narrow && nnz >= ((int64_t)1 << 20);
}

// Slices along K.  A column tile of B larger than one L2 (4 MiB per XCD) is re-fetched over
// and over by waves that sweep different parts of it.  The plan is then cut into column
// ranges whose share of the tile takes at most half an L2, every workgroup works on one
// range only, and workgroup b takes range b mod k_slices: workgroups are handed to the
// eight XCDs in turn, so each L2 holds one range of B (for two or four ranges, two or four
// XCDs share a range).  The ranges' partial sums of C meet in a buffer that a second launch
// adds up, which costs 8 k_slices M bCols bytes of traffic and a launch: only for matrices
// of at least 2^20 entries whose rows hold at least 32 entries per range on average
// (1024 per row where the tile is exactly one L2).
// Measured on a 16384 x 16384 matrix of 13 M entries with Zipf row lengths, 128 columns:
// 145 us uncut (two tiles of 64 columns), 106 + 9 us in four ranges bound to XCDs, 153 us in
// four ranges not bound to them; matrices whose tile of B fits the L2 gain nothing.
// Plans made for narrow B (chunks wider than 8) are never cut.
int choose_kslices(int32_t setting, int64_t M, int64_t K, int64_t nnz, int32_t n_hint, int ufk)
{
    if (ufk != UFK || M <= 0 || K < 8) return 1;
    if ((M + MAX_UFI) * 8 > (int64_t)INT32_MAX) return 1;
    if (setting == 2 || setting == 4 || setting == 8) return setting;
    if (setting != 0) return 1;
    const bool medium = n_hint > 32 && n_hint <= 64;
    const int64_t tile_row_bytes = medium ? 256 : 512;
    const int64_t l2 = (int64_t)4 << 20;
    if (K * tile_row_bytes < l2 || nnz < ((int64_t)1 << 20)) return 1;
    int ns = 2;
    while (ns < 8 && (K + ns - 1) / ns * tile_row_bytes > l2 / 2) ns *= 2;
    // a tile that just fills the L2 shares it with the plan's stream: two slices pay from rows of
    // 1024 entries on (8192 x 8192, 128 columns: 5 % faster at 50 to 80 % sparsity, 2 % at 90 %,
    // 3 to 6 % slower from 95 % on)
    const int64_t min_row = K * tile_row_bytes > l2 ? 32 * ns : 1024;
    if (nnz < min_row * M) return 1;
    return ns;
}

// Row lengths so uneven that sorting the rows pays: the rows longer than four
// times the mean hold at least a quarter of the entries.
bool skewed_rows(const int32_t *row_ptr, int64_t M, int64_t nnz)
{
    if (M < 2 || nnz == 0) return false;
    int64_t heavy = 0;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t len = row_ptr[i + 1] - row_ptr[i];
        if (len * M > 4 * nnz) heavy += len;
    }
    return 4 * heavy >= nnz;
}

struct Emitter {
    // creation order: one header per chunk, ufk column slots per chunk, and the
    // chunks' value blocks back to back (ufk words per set pattern row)
    std::vector<uint32_t> hdr, cols, vals;
    int64_t n_enum = 0;
    int ufi = MAX_UFI;
    int UFK = spmm_fmt::UFK;      // columns per chunk of this plan
    bool merge = true;            // leftovers of different patterns may share a chunk
    std::vector<Entry> leftovers; // scratch of panel()

    // Emits one chunk of `count` entries.  Its pattern is the union of the entries'
    // patterns; an entry whose own pattern is smaller keeps it in the top byte of
    // its column word and has zeros in the value blocks of the rows it lacks.
    void chunk(const Entry *e, int count, bool end_panel)
    {
        uint32_t pattern = 0;
        for (int u = 0; u < count; ++u) pattern |= e[u].pattern;
        uint32_t h = pattern | ((uint32_t)count << HDR_COUNT_SHIFT);
        if (end_panel) h |= HDR_END_PANEL;
        hdr.push_back(h);
        for (int u = 0; u < UFK; ++u) {
            uint32_t c = 0;
            if (count > 0) {
                const Entry &s = e[u < count ? u : count - 1];
                c = (uint32_t)s.col;
                if (u < count && s.pattern != pattern) c |= s.pattern << COL_PATTERN_SHIFT;
            }
            cols.push_back(c);
        }
        for (int r = 0; r < ufi; ++r) {
            if (!(pattern & (1u << r))) continue;
            for (int u = 0; u < UFK; ++u) {
                uint32_t bits = 0;
                if (u < count && (e[u].pattern & (1u << r))) std::memcpy(&bits, &e[u].v[r], 4);
                vals.push_back(bits);
            }
        }
        n_enum += count;
    }

    // Emits the chunks of one panel (or one piece of a panel) whose entries are
    // ordered so that equal patterns are adjacent: first the full chunks of every
    // pattern, then the leftovers (fewer than ufk entries per pattern), packed ufk
    // at a time in pattern order.  A leftover chunk costs one step of the kernel
    // whatever it holds, so sharing it between patterns saves both B loads and
    // multiply slots: the paper's compaction of rarely used enumerated blocks
    // (Section 3.2.2), done in the data instead of the code.
    void panel(const std::vector<Entry> &ents)
    {
        if (ents.empty()) {
            chunk(nullptr, 0, true);
            return;
        }
        const size_t n = ents.size();
        leftovers.clear();
        size_t n_full = 0;
        for (size_t i = 0; i < n;) {
            size_t j = i + 1;
            while (j < n && ents[j].pattern == ents[i].pattern) ++j;
            const size_t full = (j - i) / (size_t)UFK;
            n_full += full;
            const size_t rest0 = merge ? i + full * (size_t)UFK : j;
            for (size_t q = rest0; q < j; ++q) leftovers.push_back(ents[q]);
            if (!merge) n_full += (j - i) % (size_t)UFK ? 1 : 0;
            i = j;
        }
        // pass 2: emit
        size_t emitted = 0;
        for (size_t i = 0; i < n;) {
            size_t j = i + 1;
            while (j < n && ents[j].pattern == ents[i].pattern) ++j;
            const size_t stop = merge ? i + (j - i) / (size_t)UFK * (size_t)UFK : j;
            for (size_t q = i; q < stop; q += (size_t)UFK) {
                const int count = (int)std::min<size_t>((size_t)UFK, stop - q);
                emitted += 1;
                chunk(&ents[q], count, emitted == n_full && leftovers.empty());
            }
            i = j;
        }
        for (size_t q = 0; q < leftovers.size(); q += (size_t)UFK) {
            const int count = (int)std::min<size_t>((size_t)UFK, leftovers.size() - q);
            chunk(&leftovers[q], count, q + (size_t)UFK >= leftovers.size());
        }
    }
};

// Row groups in creation order, from row_ptr alone.  Panels (ufi consecutive
// rows) are taken in order.  A panel heavier than the budget G is cut into
// nseg pieces of equal size of its schedule order: want = min(8, ceil(pn / G))
// rounded up to a power of two and raised to the panel height (a workgroup holds
// 8 / ufi split panels, so that the pieces of its panels fill its eight wave slots
// exactly), size = ceil(pn / want),
// nseg = ceil(pn / size); the last piece takes the rest.
// A panel heavier than both eight budgets and 1 / CROSS_SHARE of all entries (and
// `cross` permitting) is cut across blocks instead: parts = ceil(pn / that bound), at
// most MAX_CROSS_PARTS, eight pieces per part, size = ceil(pn / (8 parts)),
// nseg = ceil(pn / size); its pieces fill blocks of eight in order.
// Lighter panels are packed greedily: a group closes when the next panel would
// exceed the budget or the panel cap.
std::vector<Group> make_groups(const int32_t *row_ptr, int64_t M, int ufi, int64_t G, int64_t GP, bool cross)
{
    std::vector<Group> groups;
    const int64_t P = (M + ufi - 1) / ufi;
    const int64_t part_bound = std::max<int64_t>(WAVES_PER_WG * G, (int64_t)row_ptr[M] / CROSS_SHARE);
    bool open = false;
    Group cur{};
    int64_t cur_panels = 0;
    auto flush = [&]() {
        if (open) groups.push_back(cur);
        open = false;
    };
    for (int64_t p = 0; p < P; ++p) {
        const int64_t r0 = p * ufi, r1 = std::min<int64_t>(M, r0 + ufi);
        const int64_t a = row_ptr[r0], b = row_ptr[r1];
        const int64_t pn = b - a;
        if (pn > G) {
            flush();
            int64_t want = std::min<int64_t>(WAVES_PER_WG, (pn + G - 1) / G);
            while (want & (want - 1)) want += 1;
            want = std::max<int64_t>(want, ufi);  // a block holds 8 / ufi split panels: fewer pieces would leave its waves idle
            const bool across = cross && pn > part_bound;
            if (across) want = WAVES_PER_WG * std::min<int64_t>(MAX_CROSS_PARTS, (pn + part_bound - 1) / part_bound);
            const int64_t size = (pn + want - 1) / want;
            const int64_t nseg = (pn + size - 1) / size;
            for (int64_t s = 0; s < nseg; ++s) {
                Group g{};
                g.row_begin = (int32_t)r0;
                g.row_end = (int32_t)r1;
                g.nnz_begin = (int32_t)(a + s * size);
                g.nnz_end = (int32_t)std::min<int64_t>(b, a + (s + 1) * size);
                g.flags = across ? FLAG_SPLIT | FLAG_CROSS : FLAG_SPLIT;
                g.seg = (int32_t)s;
                g.nseg = (int32_t)nseg;
                groups.push_back(g);
            }
            continue;
        }
        if (open && ((int64_t)cur.nnz_end - cur.nnz_begin + pn > G || cur_panels == GP)) flush();
        if (!open) {
            cur = Group{};
            cur.row_begin = (int32_t)r0;
            cur.nnz_begin = (int32_t)a;
            cur.flags = 0;
            cur_panels = 0;
            open = true;
        }
        cur.row_end = (int32_t)r1;
        cur.nnz_end = (int32_t)b;
        cur_panels += 1;
    }
    flush();
    return groups;
}

// Threads the enumeration may use: one per 2 M entries, at most 16 and at most what
// the machine has, unless the caller names a count.
int worker_count(int64_t nnz, int32_t asked)
{
    if (asked >= 1) return std::min(asked, 64);
    int64_t n = std::min<int64_t>(16, std::max<int64_t>(1, nnz / (2 << 20)));
    const unsigned hw = std::thread::hardware_concurrency();
    if (hw > 0) n = std::min<int64_t>(n, hw);
    return (int)n;
}

// Cuts the groups (creation order) into at most `want` contiguous ranges of about
// equal numbers of entries; a cut never falls between the pieces of one panel.
// Returns the range boundaries, first 0 and last groups.size().
std::vector<int64_t> range_cuts(const std::vector<Group> &groups, int want)
{
    const int64_t n = (int64_t)groups.size();
    std::vector<int64_t> cuts{0};
    if (n > 0 && want > 1) {
        const int64_t total = (int64_t)groups.back().nnz_end - groups.front().nnz_begin + n;  // + n: empty groups weigh too
        int64_t done = 0;
        for (int64_t g = 0; g < n; ++g) {
            const bool boundary = !(groups[(size_t)g].flags & FLAG_SPLIT) || groups[(size_t)g].seg == 0;
            if (boundary && g > cuts.back() && done * want >= total * (int64_t)cuts.size()) cuts.push_back(g);
            done += (int64_t)groups[(size_t)g].nnz_end - groups[(size_t)g].nnz_begin + 1;
        }
    }
    if (cuts.back() != n || n == 0) cuts.push_back(n);
    return cuts;
}

}  // namespace

int spmm_inspect(int64_t M, int64_t K, const int32_t *row_ptr, const int32_t *col_idx,
                 const float *vals, const InspectorOptions &opts, HostPlan &out)
{
    if (M < 0 || K < 0 || M > INT32_MAX || K > INT32_MAX) return ST_INVALID_ARG;
    if (!row_ptr) return ST_INVALID_ARG;
    if (row_ptr[0] != 0) return ST_INVALID_CSR;
    for (int64_t i = 0; i < M; ++i)
        if (row_ptr[i + 1] < row_ptr[i]) return ST_INVALID_CSR;
    const int64_t nnz = row_ptr[M];
    if (nnz > 0 && (!col_idx || !vals)) return ST_INVALID_ARG;
    for (int64_t p = 0; p < nnz; ++p)
        if (col_idx[p] < 0 || (int64_t)col_idx[p] >= K) return ST_INVALID_CSR;

    try {
        out = HostPlan();
        out.M = M;
        out.K = K;
        out.nnz = nnz;
        // ---- 0. row order ------------------------------------------------------
        // Rows of very different lengths: the plan's rows are the matrix's rows
        // sorted by length, longest first (stable), so that a panel holds rows of
        // like length (long rows share most of their columns, which is what a
        // tall panel turns into fewer loads of B) and C is written through a map.
        int64_t max_row = 0;
        for (int64_t i = 0; i < M; ++i) max_row = std::max<int64_t>(max_row, row_ptr[i + 1] - row_ptr[i]);
        int ufi = opts.ufi;
        const bool forced_ufi = ufi == 1 || ufi == 2 || ufi == 4 || ufi == 8;
        const bool skewed = skewed_rows(row_ptr, M, nnz);
        bool cross = cross_allowed(opts.cross, skewed, nnz, opts.n_hint);
        out.ufk = valid_ufk(opts.ufk) && K <= ((int64_t)1 << COL_PATTERN_SHIFT) ? opts.ufk : choose_ufk(K, opts.n_hint);
        // slices along K: the heights below then see the columns of one slice
        const int NS = choose_kslices(opts.kslices, M, K, nnz, opts.n_hint, out.ufk);
        const int64_t KS = NS > 1 ? (K + NS - 1) / NS : K;                              // columns per slice
        const int64_t MS = NS > 1 ? (M + MAX_UFI - 1) / MAX_UFI * MAX_UFI : M;          // plan rows per slice
        const int64_t MP = NS > 1 ? NS * MS : M;                                        // plan rows
        out.k_slices = NS;
        out.slice_rows = MS;
        out.slice_cols = KS;
        out.plan_rows = MP;
        if (NS > 1) {
            // the longest row of a slice
            max_row = 0;
            int64_t in_slice[8];
            for (int64_t i = 0; i < M; ++i) {
                std::fill(in_slice, in_slice + NS, (int64_t)0);
                for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) in_slice[(int64_t)col_idx[q] / KS] += 1;
                max_row = std::max(max_row, *std::max_element(in_slice, in_slice + NS));
            }
            // A slice's panels are lighter by the number of slices: where the tallest panel of
            // its longest rows is no longer the tail of the launch, no panel needs to be cut
            // across workgroups (the 16384 x 16384 matrix above, four slices, eight rows:
            // 112 us with every panel in one workgroup, 119 us with the heavy ones cut)
            if (opts.cross == 0 && cross) {
                const bool medium = opts.n_hint > 32 && opts.n_hint <= 64;
                if (choose_ufi_skewed(KS, nnz, max_row, opts.n_hint, false) >= (medium ? 4 : 8)) cross = false;
            }
        }
        if (!forced_ufi) {
            // a forced sort asks for the height a sorted matrix would get
            const bool as_sorted = opts.sort_rows > 0 || (opts.sort_rows == 0 && skewed);
            ufi = as_sorted ? choose_ufi_skewed(KS, nnz, max_row, opts.n_hint, cross) : choose_ufi(M, KS, nnz, opts.n_hint);
        }
        // single rows share nothing: sorting them would only scatter the rows of C
        const bool sorted = opts.sort_rows > 0 || (opts.sort_rows == 0 && skewed && ufi > 1);
        // row_order[i]: the matrix row that row i of a slice stands for (sorted plans only)
        std::vector<uint32_t> row_order;
        std::vector<int32_t> own_ptr;
        if (sorted) {
            row_order.resize((size_t)M);
            std::iota(row_order.begin(), row_order.end(), 0u);
            std::stable_sort(row_order.begin(), row_order.end(), [&](uint32_t x, uint32_t y) {
                return row_ptr[x + 1] - row_ptr[x] > row_ptr[y + 1] - row_ptr[y];
            });
        }
        // Row i of the plan is slice i / MS of matrix row mrow(i % MS) (none for the rows that
        // pad a slice); out_row(i) is the row of the output buffer it is written to: a row of
        // C, or of the slices' buffer.  plan_ptr is the row pointer of the plan's own rows.
        auto mrow = [&](int64_t i) -> int64_t {
            const int64_t w = NS > 1 ? i % MS : i;
            return w >= M ? -1 : sorted ? (int64_t)row_order[(size_t)w] : w;
        };
        auto src = [&](int64_t i) -> int64_t {  // out_row
            if (NS == 1) return sorted ? (int64_t)row_order[(size_t)i] : i;
            const int64_t w = i % MS;
            return i - w + (w < M && sorted ? (int64_t)row_order[(size_t)w] : w);
        };
        if (sorted || NS > 1) {
            own_ptr.assign((size_t)MP + 1, 0);
            for (int64_t i = 0; i < MS; ++i) {
                const int64_t m = mrow(i);
                if (m < 0) continue;
                if (NS == 1) {
                    own_ptr[(size_t)i + 1] = row_ptr[m + 1] - row_ptr[m];
                } else {
                    for (int64_t q = row_ptr[m]; q < row_ptr[m + 1]; ++q)
                        own_ptr[(size_t)((int64_t)col_idx[q] / KS * MS + i) + 1] += 1;
                }
            }
            for (int64_t i = 0; i < MP; ++i) own_ptr[(size_t)i + 1] += own_ptr[(size_t)i];
            if (sorted) {
                out.rowmap.resize((size_t)MP);
                for (int64_t i = 0; i < MP; ++i) out.rowmap[(size_t)i] = (uint32_t)src(i);
            }
        }
        const int32_t *plan_ptr = sorted || NS > 1 ? own_ptr.data() : row_ptr;
        // ---- 1. group budget and row groups, from the row pointer alone ----------
        int32_t auto_g = 0, auto_gp = 0;
        choose_group_budget(MP, nnz, ufi, opts.n_hint, auto_g, auto_gp);
        // heavy panels cut as finely as needed: half the budget, so that the launch is made of
        // lighter pieces throughout (measured with the heights above: stress matrix 162 -> 154 us,
        // 8192 x 8192 lognormal rows of sigma 1.5 94 -> 81 us at 128 columns, 60 -> 53 us at 64)
        if (cross) auto_g = std::max<int32_t>(32, auto_g / 2 / 32 * 32);
        // skewed rows in a plan cut along K whose panels all stay inside a workgroup: a quarter, so
        // that more of the medium panels are cut into eight pieces (the 16384 x 16384 matrix above,
        // four slices: 106 us against 109 us with half and 117 us with the whole budget)
        else if (NS > 1 && skewed) auto_g = std::max<int32_t>(32, auto_g / 4 / 32 * 32);
        out.group_nnz = opts.group_nnz > 0 ? std::max(8, opts.group_nnz) : auto_g;
        out.group_panels = opts.group_panels > 0 ? opts.group_panels : auto_gp;
        const int64_t G = out.group_nnz;
        const int64_t GP = out.group_panels;
        std::vector<Group> groups = make_groups(plan_ptr, MP, ufi, G, GP, cross);
        out.ufi = ufi;
        const int UFI = ufi;  // panel height of this plan
        const int UFK = out.ufk;  // columns per chunk of this plan (shadows the default)
        const int WINW = win_words(UFK), LOOK = lookahead(UFK);
        const int N_PATTERNS = (1 << UFI) - 1;
        const int SPLIT_PANELS_PER_WG = WAVES_PER_WG / UFI;
        const int64_t n_groups = (int64_t)groups.size();

        // ---- 2. enumeration and emission, panel by panel ----------------------
        // The groups are cut into contiguous ranges of about equal weight (never
        // between the pieces of one panel); every range is enumerated by a thread of
        // its own into an emitter of its own, and the emitters are joined in order.
        const bool merge_leftovers = K <= ((int64_t)1 << COL_PATTERN_SHIFT);  // the top byte of a column word must be free
        auto emit_range = [&](int64_t g_begin, int64_t g_end, Emitter &em) {
            std::vector<int32_t> order;                  // canonical order of one row
            std::vector<int32_t> ccol[MAX_UFI];          // canonical columns per panel row
            std::vector<float> cval[MAX_UFI];
            std::vector<Entry> merged, by_pattern, piece;
            struct Flat { int32_t entry; int32_t row; };
            std::vector<Flat> flat;
            int64_t gi = g_begin;
            while (gi < g_end) {
                Group &g0 = groups[gi];
                const bool split = (g0.flags & FLAG_SPLIT) != 0;
                const int64_t g_last = split ? gi + g0.nseg - 1 : gi;  // pieces of a panel are adjacent
                if (!split) {
                    g0.chunk0 = (int64_t)em.hdr.size();
                    g0.words0 = (int64_t)em.vals.size();
                }
                const int64_t first_panel = g0.row_begin / UFI;
                const int64_t last_panel = (g0.row_end + UFI - 1) / UFI;  // exclusive
                for (int64_t p = first_panel; p < last_panel; ++p) {
                    const int64_t r0 = p * UFI, r1 = std::min<int64_t>(MP, r0 + UFI);
                    const int rows = (int)(r1 - r0);
                    // canonical rows: stable order by column (duplicates keep stored order)
                    for (int r = 0; r < rows; ++r) {
                        const int64_t m = mrow(r0 + r);
                        const int64_t a = m < 0 ? 0 : row_ptr[m], b = m < 0 ? 0 : row_ptr[m + 1];
                        const int64_t len = b - a;
                        ccol[r].resize((size_t)len);
                        cval[r].resize((size_t)len);
                        bool sorted = true;
                        for (int64_t q = a + 1; q < b; ++q)
                            if (col_idx[q] < col_idx[q - 1]) { sorted = false; break; }
                        if (sorted) {
                            std::copy(col_idx + a, col_idx + b, ccol[r].begin());
                            std::copy(vals + a, vals + b, cval[r].begin());
                        } else {
                            order.resize((size_t)len);
                            std::iota(order.begin(), order.end(), 0);
                            std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
                                return col_idx[a + x] < col_idx[a + y];
                            });
                            for (int64_t q = 0; q < len; ++q) {
                                ccol[r][(size_t)q] = col_idx[a + order[(size_t)q]];
                                cval[r][(size_t)q] = vals[a + order[(size_t)q]];
                            }
                        }
                        if (NS > 1) {
                            // this slice's columns: a contiguous range of the canonical row
                            const int64_t sl = (r0 + r) / MS;
                            const auto lo = std::lower_bound(ccol[r].begin(), ccol[r].end(), (int32_t)std::min<int64_t>(sl * KS, INT32_MAX));
                            const auto hi = std::lower_bound(ccol[r].begin(), ccol[r].end(), (int32_t)std::min<int64_t>((sl + 1) * KS, INT32_MAX));
                            const size_t i0 = (size_t)(lo - ccol[r].begin()), i1 = (size_t)(hi - ccol[r].begin());
                            ccol[r].erase(ccol[r].begin() + (ptrdiff_t)i1, ccol[r].end());
                            ccol[r].erase(ccol[r].begin(), ccol[r].begin() + (ptrdiff_t)i0);
                            cval[r].erase(cval[r].begin() + (ptrdiff_t)i1, cval[r].end());
                            cval[r].erase(cval[r].begin(), cval[r].begin() + (ptrdiff_t)i0);
                        }
                    }
                    // merge the rows' column lists.  The t-th occurrence of a column in
                    // a row meets the t-th occurrences in the other rows, so a column
                    // stored twice in one row yields two enumerated columns.
                    merged.clear();
                    size_t head[MAX_UFI] = {};
                    uint32_t layer[MAX_UFI] = {};
                    for (;;) {
                        int32_t best_col = INT32_MAX;
                        uint32_t best_layer = UINT32_MAX;
                        bool any = false;
                        for (int r = 0; r < rows; ++r) {
                            if (head[r] >= ccol[r].size()) continue;
                            const int32_t c = ccol[r][head[r]];
                            if (!any || c < best_col || (c == best_col && layer[r] < best_layer)) {
                                best_col = c;
                                best_layer = layer[r];
                                any = true;
                            }
                        }
                        if (!any) break;
                        Entry e{};
                        e.col = best_col;
                        e.pattern = 0;
                        for (int r = 0; r < rows; ++r) {
                            if (head[r] >= ccol[r].size()) continue;
                            if (ccol[r][head[r]] == best_col && layer[r] == best_layer) {
                                e.pattern |= 1u << r;
                                e.v[r] = cval[r][head[r]];
                                const size_t nx = head[r] + 1;
                                layer[r] = (nx < ccol[r].size() && ccol[r][nx] == best_col) ? layer[r] + 1 : 0;
                                head[r] = nx;
                            }
                        }
                        merged.push_back(e);
                    }
                    // list columns of equal pattern together (stable: ascending column inside a pattern)
                    by_pattern.resize(merged.size());
                    {
                        size_t count[(1 << MAX_UFI) + 1] = {0};
                        for (const Entry &e : merged) count[e.pattern + 1]++;
                        for (int q = 1; q <= N_PATTERNS + 1; ++q) count[q] += count[q - 1];
                        for (const Entry &e : merged) by_pattern[count[e.pattern]++] = e;
                    }
                    if (!split) {
                        em.panel(by_pattern);
                        continue;
                    }
                    // split panel: cut the schedule order (pattern by pattern, column by
                    // column, row by row) at multiples of the budget; an enumerated
                    // column that straddles a cut is divided between the two pieces.
                    flat.clear();
                    for (size_t e = 0; e < by_pattern.size(); ++e)
                        for (int r = 0; r < UFI; ++r)
                            if (by_pattern[e].pattern & (1u << r)) flat.push_back(Flat{(int32_t)e, r});
                    const int64_t base = g0.nnz_begin;
                    for (int64_t s = gi; s <= g_last; ++s) {
                        Group &gs = groups[s];
                        gs.chunk0 = (int64_t)em.hdr.size();
                        gs.words0 = (int64_t)em.vals.size();
                        piece.clear();
                        for (int64_t q = gs.nnz_begin - base; q < gs.nnz_end - base; ++q) {
                            const Flat &f = flat[(size_t)q];
                            if (piece.empty() || q == gs.nnz_begin - base || flat[(size_t)q - 1].entry != f.entry) {
                                Entry e{};
                                e.col = by_pattern[(size_t)f.entry].col;
                                e.pattern = 0;
                                piece.push_back(e);
                            }
                            piece.back().pattern |= 1u << f.row;
                            piece.back().v[f.row] = by_pattern[(size_t)f.entry].v[f.row];
                        }
                        em.panel(piece);
                        gs.n_chunks = (int64_t)em.hdr.size() - gs.chunk0;
                        gs.n_words = (int64_t)em.vals.size() - gs.words0;
                    }
                }
                if (!split) {
                    g0.n_chunks = (int64_t)em.hdr.size() - g0.chunk0;
                    g0.n_words = (int64_t)em.vals.size() - g0.words0;
                }

                gi = g_last + 1;
            }
        };
        std::vector<int64_t> cuts = range_cuts(groups, worker_count(nnz, opts.threads));
        const size_t n_ranges = cuts.size() - 1;
        std::vector<Emitter> parts(n_ranges);
        for (size_t t = 0; t < n_ranges; ++t) {
            parts[t].ufi = UFI;
            parts[t].UFK = UFK;
            parts[t].merge = merge_leftovers;
            const int64_t share = cuts[t + 1] > cuts[t] ? (int64_t)groups[(size_t)cuts[t + 1] - 1].nnz_end -
                                                              groups[(size_t)cuts[t]].nnz_begin
                                                        : 0;
            parts[t].hdr.reserve((size_t)(share / 4 + (cuts[t + 1] - cuts[t]) + 16));
            parts[t].cols.reserve((size_t)(share / 4 + (cuts[t + 1] - cuts[t]) + 16) * UFK);
            parts[t].vals.reserve((size_t)(share + share / 2 + 64));
        }
        if (n_ranges == 1) {
            emit_range(cuts[0], cuts[1], parts[0]);
        } else {
            std::vector<std::thread> workers;
            std::vector<int> failed(n_ranges, 0);
            auto job = [&](size_t t) {
                try {
                    emit_range(cuts[t], cuts[t + 1], parts[t]);
                } catch (...) {
                    failed[t] = 1;  // no exception may leave a thread: reported as an allocation failure below
                }
            };
            for (size_t t = 0; t < n_ranges; ++t) {
                try {
                    workers.emplace_back(job, t);
                } catch (const std::system_error &) {
                    job(t);  // no thread to be had: this one does the range itself
                }
            }
            for (std::thread &w : workers) w.join();
            for (int f : failed)
                if (f) throw std::bad_alloc();
        }
        int64_t total_chunks = 0, total_value_words = 0, total_enum = 0;
        for (size_t t = 0; t < n_ranges; ++t) {
            for (int64_t g = cuts[t]; g < cuts[t + 1]; ++g) groups[(size_t)g].part = (int32_t)t;
            total_chunks += (int64_t)parts[t].hdr.size();
            total_value_words += (int64_t)parts[t].vals.size();
            total_enum += parts[t].n_enum;
        }

        // ---- 3. launch order and blocks ---------------------------------------
        // Split panels first, heaviest panel first (stable), each with its pieces
        // in order; then the groups of whole panels, heaviest first (stable).
        // Blocks of WAVES_PER_WG wave slots are filled in that order.  The pieces
        // of a panel never straddle a block and a block holds at most
        // SPLIT_PANELS_PER_WG split panels; slots left over stay idle.
        std::vector<int64_t> split_heads, whole;
        for (int64_t i = 0; i < n_groups; ++i) {
            const Group &g = groups[(size_t)i];
            if (!(g.flags & FLAG_SPLIT)) whole.push_back(i);
            else if (g.seg == 0) split_heads.push_back(i);
        }
        auto panel_nnz = [&](int64_t head) {
            const Group &g0 = groups[(size_t)head];
            return (int64_t)groups[(size_t)(head + g0.nseg - 1)].nnz_end - g0.nnz_begin;
        };
        std::stable_sort(split_heads.begin(), split_heads.end(),
                         [&](int64_t x, int64_t y) { return panel_nnz(x) > panel_nnz(y); });
        std::stable_sort(whole.begin(), whole.end(), [&](int64_t x, int64_t y) {
            return (groups[(size_t)x].nnz_end - groups[(size_t)x].nnz_begin) >
                   (groups[(size_t)y].nnz_end - groups[(size_t)y].nnz_begin);
        });
        // Plans cut along K: every block works on one slice (slice by slice here, heaviest
        // first inside a slice); the blocks are dealt out to the slices in turn at the end.
        auto slice_of = [&](int64_t gi) { return NS > 1 ? (int64_t)groups[(size_t)gi].row_begin / MS : (int64_t)0; };
        if (NS > 1) {
            std::stable_sort(split_heads.begin(), split_heads.end(), [&](int64_t x, int64_t y) { return slice_of(x) < slice_of(y); });
            std::stable_sort(whole.begin(), whole.end(), [&](int64_t x, int64_t y) { return slice_of(x) < slice_of(y); });
        }

        // upper bound of the stream: headers (padded per window), columns, values
        const int64_t bound_words = total_chunks * (1 + UFK) + total_value_words + 8 * total_chunks / 4 + 64;
        if (total_chunks + CHUNK_TAIL_PAD >= ((int64_t)1 << 31) - 8 || bound_words >= ((int64_t)1 << 32) ||
            n_groups >= ((int64_t)1 << 31) - WAVES_PER_WG)
            return ST_UNSUPPORTED;

        out.hdr.resize((size_t)(total_chunks + CHUNK_TAIL_PAD), 0u);
        out.groups.reserve((size_t)n_groups * 5);
        int64_t c_at = 0;
        uint64_t stream_at = 0;

        // One group's place in the launch-ordered arrays.  `place` cuts the group's
        // chunks into staging windows and fills its descriptor; the windows' words
        // are written afterwards (fill_group), many groups at a time.
        struct Placed { int64_t group; uint64_t stream0; uint32_t win0; int64_t chunk_at; };
        std::vector<Placed> placed;
        placed.reserve((size_t)n_groups);
        auto place = [&](int64_t gi, uint32_t *it) {
            const Group &g = groups[(size_t)gi];
            const Emitter &em = parts[(size_t)g.part];
            out.groups.push_back(g.row_begin);
            out.groups.push_back(g.row_end);
            out.groups.push_back(g.nnz_begin);
            out.groups.push_back(g.nnz_end);
            out.groups.push_back(g.flags);
            const uint32_t win0 = (uint32_t)out.wins.size();
            const uint64_t stream0 = stream_at;
            int64_t c = 0;
            while (c < g.n_chunks) {
                // widest run of chunks whose window still fits
                int64_t wc = 0, vw = 0;
                while (c + wc < g.n_chunks) {
                    const uint32_t pattern = em.hdr[(size_t)(g.chunk0 + c + wc)] & HDR_PATTERN_MASK;
                    const int64_t add = (int64_t)UFK * __builtin_popcount(pattern);
                    const int64_t hdr_w = ((wc + 1 + 7) / 8) * 8;
                    const int64_t words = hdr_w + (wc + 1) * UFK + vw + add;
                    // the kernels read column slots up to LOOKAHEAD chunks past the last
                    // one (values never used): those reads must stay inside the window
                    if (words > WINW || hdr_w + (wc + 1 + LOOK) * UFK > WINW) break;
                    wc += 1;
                    vw += add;
                }
                const int64_t ww = ((wc + 7) / 8) * 8 + wc * UFK + vw;
                out.wins.push_back((uint32_t)wc | ((uint32_t)ww << 16));
                stream_at += (uint64_t)ww;
                c += wc;
            }
            placed.push_back(Placed{gi, stream0, win0, c_at});
            it[IT_ROW0] = (uint32_t)g.row_begin;
            it[IT_NROWS] = (uint32_t)(g.row_end - g.row_begin);
            it[IT_CHUNK0] = (uint32_t)c_at;
            it[IT_NCHUNKS] = (uint32_t)g.n_chunks;
            it[IT_STREAM0] = (uint32_t)stream0;
            it[IT_FLAGS] = (uint32_t)g.flags;
            it[IT_WIN0] = win0;
            it[IT_NWINS] = (uint32_t)out.wins.size() - win0;
            it[IT_WIN_FIRST] = out.wins.size() > win0 ? out.wins[win0] : 0u;
            c_at += g.n_chunks;
        };
        // writes one placed group: its headers into the header list and every window as
        // [headers (padded to 8 words) | column slots | value blocks] into the stream
        auto fill_group = [&](const Placed &pl) {
            const Group &g = groups[(size_t)pl.group];
            const Emitter &em = parts[(size_t)g.part];
            std::copy(em.hdr.begin() + g.chunk0, em.hdr.begin() + g.chunk0 + g.n_chunks, out.hdr.begin() + pl.chunk_at);
            uint32_t *dst = out.stream.data() + pl.stream0;
            int64_t c = 0, v_at = g.words0;
            for (uint32_t w = pl.win0; c < g.n_chunks; ++w) {
                const int64_t wc = out.wins[w] & 0xFFFFu, ww = out.wins[w] >> 16;
                const int64_t hdr_words = ((wc + 7) / 8) * 8;
                const int64_t vw = ww - hdr_words - wc * UFK;
                std::copy(em.hdr.begin() + g.chunk0 + c, em.hdr.begin() + g.chunk0 + c + wc, dst);
                std::fill(dst + wc, dst + hdr_words, 0u);
                std::copy(em.cols.begin() + (g.chunk0 + c) * UFK, em.cols.begin() + (g.chunk0 + c + wc) * UFK, dst + hdr_words);
                std::copy(em.vals.begin() + v_at, em.vals.begin() + v_at + vw, dst + hdr_words + wc * UFK);
                dst += ww;
                c += wc;
                v_at += vw;
            }
        };
        auto new_block = [&](uint32_t flags) {
            const size_t at = out.items.size();
            out.items.resize(at + (size_t)WAVES_PER_WG * ITEM_WORDS, 0u);
            for (int w = 0; w < WAVES_PER_WG; ++w) out.items[at + (size_t)w * ITEM_WORDS + IT_FLAGS] = FLAG_IDLE | flags;
            out.n_blocks += 1;
            return at;
        };

        // blocks of split panels
        {
            size_t at = 0;
            int used = WAVES_PER_WG, panels = SPLIT_PANELS_PER_WG;  // forces a new block
            int64_t slice_now = -1;
            for (int64_t head : split_heads) {
                const Group &g0 = groups[(size_t)head];
                const int nseg = g0.nseg;
                if (slice_of(head) != slice_now) {  // a block never mixes slices
                    slice_now = slice_of(head);
                    used = WAVES_PER_WG;
                }
                if (g0.flags & FLAG_CROSS) {
                    // a panel cut across blocks: its pieces fill blocks of their own, eight at a
                    // time; after its barrier wave r of every block adds row r of the block's
                    // pieces into the block's scratch slot, and a second launch adds the slots in order
                    const int nparts = (nseg + WAVES_PER_WG - 1) / WAVES_PER_WG;
                    const uint32_t slot0 = (uint32_t)out.n_cross_slots;
                    for (int part = 0; part < nparts; ++part) {
                        at = new_block(FLAG_SYNC | FLAG_CROSS);
                        const int first = part * WAVES_PER_WG, here = std::min(WAVES_PER_WG, nseg - first);
                        for (int sidx = 0; sidx < here; ++sidx) {
                            uint32_t *it = &out.items[at + (size_t)sidx * ITEM_WORDS];
                            place(head + first + sidx, it);
                            it[IT_FLAGS] |= FLAG_SYNC;
                            out.n_split += 1;
                        }
                        for (int w = 0; w < WAVES_PER_WG; ++w) {
                            uint32_t *it = &out.items[at + (size_t)w * ITEM_WORDS];
                            it[IT_X_NPARTS] = (uint32_t)nparts;
                            it[IT_X_SLOT0] = slot0;
                            it[IT_X_PART] = (uint32_t)part;
                            if (w < g0.row_end - g0.row_begin) {
                                it[IT_RED_NSEG] = (uint32_t)here;
                                it[IT_RED_SLOT0] = 0u;
                                it[IT_RED_R] = (uint32_t)w;
                                it[IT_RED_ROW] = (uint32_t)src(g0.row_begin + w);
                            }
                        }
                    }
                    const size_t e = out.cross.size();
                    out.cross.resize(e + CROSS_ENTRY_WORDS, 0u);
                    out.cross[e + CE_SLOT0] = slot0;
                    out.cross[e + CE_NPARTS] = (uint32_t)nparts;
                    out.cross[e + CE_NROWS] = (uint32_t)(g0.row_end - g0.row_begin);
                    for (int r = 0; r < g0.row_end - g0.row_begin; ++r)
                        out.cross[e + CE_ROW0 + (size_t)r] = (uint32_t)src(g0.row_begin + r);
                    out.n_cross += 1;
                    out.n_cross_slots += nparts;
                    used = WAVES_PER_WG;  // the next split panel starts a block of its own
                    panels = SPLIT_PANELS_PER_WG;
                    continue;
                }
                if (used + nseg > WAVES_PER_WG || panels == SPLIT_PANELS_PER_WG) {
                    at = new_block(FLAG_SYNC);
                    used = 0;
                    panels = 0;
                }
                for (int sidx = 0; sidx < nseg; ++sidx) {
                    uint32_t *it = &out.items[at + (size_t)(used + sidx) * ITEM_WORDS];
                    place(head + sidx, it);
                    it[IT_FLAGS] |= FLAG_SYNC;
                    out.n_split += 1;
                }
                // after the barrier wave UFI * panels + r adds row r of this panel
                for (int r = 0; r < g0.row_end - g0.row_begin; ++r) {
                    uint32_t *it = &out.items[at + (size_t)(UFI * panels + r) * ITEM_WORDS];
                    it[IT_RED_NSEG] = (uint32_t)nseg;
                    it[IT_RED_SLOT0] = (uint32_t)used;
                    it[IT_RED_R] = (uint32_t)r;
                    it[IT_RED_ROW] = (uint32_t)src(g0.row_begin + r);
                }
                used += nseg;
                panels += 1;
            }
        }
        // blocks of whole-panel groups
        {
            size_t at = 0;
            int used = WAVES_PER_WG;
            int64_t slice_now = -1;
            for (int64_t gi2 : whole) {
                if (slice_of(gi2) != slice_now) {
                    slice_now = slice_of(gi2);
                    used = WAVES_PER_WG;
                }
                if (used == WAVES_PER_WG) {
                    at = new_block(0);
                    used = 0;
                }
                place(gi2, &out.items[at + (size_t)used * ITEM_WORDS]);
                used += 1;
            }
        }
        if (NS > 1) {
            // Block b of the launch works on slice b mod NS: workgroups go to the XCDs in
            // turn, so an XCD's L2 sees the rows of B of one slice (of 8 / NS slices' worth of
            // XCDs).  A slice with fewer blocks than the longest gets idle blocks.
            const size_t BW = (size_t)WAVES_PER_WG * ITEM_WORDS;
            std::vector<std::vector<size_t>> of_slice((size_t)NS);
            for (size_t b = 0; b < (size_t)out.n_blocks; ++b) {
                int64_t sl = 0;
                for (int w = 0; w < WAVES_PER_WG; ++w) {
                    const uint32_t *it = &out.items[b * BW + (size_t)w * ITEM_WORDS];
                    if (!(it[IT_FLAGS] & FLAG_IDLE)) {
                        sl = (int64_t)it[IT_ROW0] / MS;
                        break;
                    }
                }
                of_slice[(size_t)sl].push_back(b);
            }
            size_t longest = 0;
            for (const std::vector<size_t> &v : of_slice) longest = std::max(longest, v.size());
            std::vector<uint32_t> dealt(longest * (size_t)NS * BW, 0u);
            for (size_t i = 0; i < longest; ++i)
                for (size_t sl = 0; sl < (size_t)NS; ++sl) {
                    uint32_t *dst = dealt.data() + (i * (size_t)NS + sl) * BW;
                    if (i < of_slice[sl].size())
                        std::copy(out.items.begin() + (ptrdiff_t)(of_slice[sl][i] * BW),
                                  out.items.begin() + (ptrdiff_t)((of_slice[sl][i] + 1) * BW), dst);
                    else
                        for (int w = 0; w < WAVES_PER_WG; ++w) dst[(size_t)w * ITEM_WORDS + IT_FLAGS] = FLAG_IDLE;
                }
            out.items.swap(dealt);
            out.n_blocks = (int64_t)(longest * (size_t)NS);
        }
        out.wins.push_back(0u);  // look-ahead slot
        // the windows' words, contiguous runs of placed groups per thread
        out.stream.resize((size_t)stream_at + STREAM_TAIL_PAD, 0u);
        {
            const int want = worker_count(nnz, opts.threads);
            const size_t n_placed = placed.size();
            std::vector<size_t> from{0};
            for (int t = 1; t < want; ++t) {
                // first placed group at or past the t-th share of the stream
                const uint64_t target = stream_at / (uint64_t)want * (uint64_t)t;
                size_t lo = from.back(), hi = n_placed;
                while (lo < hi) {
                    const size_t mid = (lo + hi) / 2;
                    if (placed[mid].stream0 < target) lo = mid + 1; else hi = mid;
                }
                from.push_back(lo);
            }
            from.push_back(n_placed);
            auto fill_range = [&](size_t a, size_t b) noexcept {
                for (size_t i = a; i < b; ++i) fill_group(placed[i]);  // copies into sized arrays: nothing throws
            };
            if (want == 1) {
                fill_range(0, n_placed);
            } else {
                std::vector<std::thread> workers;
                for (int t = 0; t < want; ++t) {
                    try {
                        workers.emplace_back(fill_range, from[(size_t)t], from[(size_t)t + 1]);
                    } catch (const std::system_error &) {
                        fill_range(from[(size_t)t], from[(size_t)t + 1]);
                    }
                }
                for (std::thread &w : workers) w.join();
            }
        }
        out.n_chunks = total_chunks;
        out.n_enum = total_enum;
        // the kernel may fetch the map entries of a whole panel at once
        if (sorted) out.rowmap.resize((size_t)MP + MAX_UFI, 0u);
    } catch (const std::bad_alloc &) {
        out = HostPlan();
        return ST_ALLOC;
    } catch (...) {
        out = HostPlan();  // length errors of the containers and the like: the input is too large to lay out
        return ST_UNSUPPORTED;
    }
    return ST_OK;
}
