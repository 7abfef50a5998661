// C ABI of the sparse MLP training step: argument checking, layer / MLP handles, the
// one-off mirror build, and the kernel sequence of a training step.
#include "../../include/nerva_sparse.h"
#include "../../include/nerva_sparse_bench.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <algorithm>
#include <climits>
#include <atomic>
#include <functional>
#include <mutex>
#include <vector>

#include "kernels.h"

using namespace nerva;

// Workspace of mlp_train_step_static: one array per GPU, part of the library's code object, held
// from the moment the library is loaded on a device until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress; the device address it yields (one per device) is
// what kernels, copies and fills are given.
constexpr size_t kStaticScratchBytes = NERVA_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once resolved
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (resolved once per device, with that device current).
hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

thread_local std::string g_last_error;
std::atomic<int> g_partition_mode{0};  // see nerva_set_partition_mode

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(NERVA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(expr)                                        \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);    \
    } while (0)

inline hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }
inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace

// What a bound pattern owns on the device besides scratch: the mirror and the partition tables.  A
// layer keeps two sets: sparse_linear_rebind builds the new pattern's structures in the spare set while
// the current one stays valid, and swaps on success; buffers are reused when large enough, so
// repeated topology updates do not allocate.
struct PatternBuffers {
    int32_t *indptr_t = nullptr;    // [cols + 1]
    int32_t *mirror_mem = nullptr;  // indices_t | perm | pos_t | values_t, round_up(nnz, 64) elements each
    size_t mirror_ints = 0;
    int32_t *plan_mem = nullptr, *plan_t_mem = nullptr;
    size_t plan_ints = 0, plan_t_ints = 0;
};

struct nerva_layer {
    int32_t rows = 0, cols = 0, nnz = 0, activation = 0, max_batch = 0;
    // caller-owned
    const int32_t *indptr = nullptr;
    const int32_t *indices = nullptr;
    float *values = nullptr;
    float *bias = nullptr;
    // owned: CSR of W^T and the position maps (views into cur.mirror_mem / cur.indptr_t)
    PatternBuffers cur, spare;
    int32_t *indptr_t = nullptr;   // [cols+1]
    int32_t *indices_t = nullptr;  // [nnz] row index of each mirror entry
    float *values_t = nullptr;     // [nnz]
    int32_t *perm = nullptr;       // [nnz] mirror position -> CSR position
    int32_t *pos_t = nullptr;      // [nnz] CSR position -> mirror position
    // static work partitions of W (by rows) and of the mirror (by W's columns): views into cur.plan_mem / cur.plan_t_mem
    RowBlocks plan{}, plan_t{};
    // owned scratch of the set-up kernels: counters of the mirror build, then 4 status ints
    int32_t *build_work = nullptr;
    size_t build_work_ints = 0;
    int32_t *status = nullptr;     // [4] result of the device-side CSR check
    // owned: partial rows of huge-row work-groups, shared by the forward and the transposed product
    float *scratch = nullptr;
    size_t scratch_floats = 0;
    int64_t scratch_ld = 0;
    // owned: per-tile partial products of the column-tiled SDDMM (only for layers whose input
    // at max_batch columns does not fit an L2)
    float *partial = nullptr;
    size_t partial_floats = 0;
    int64_t partial_stride = 0, partial_db_at = 0;
    int32_t partial_tiles = 0;
    // owned, only on the dense route (sparse_linear_enable_dense, or chosen when the pattern was bound): a
    // zero-filled dense copy of W (rows x dense_ld, dense_ld = cols rounded up to kDenseLdAlign) and a dense
    // gradient of the same shape
    bool dense_on = false;
    float *dense = nullptr, *dense_g = nullptr;
    int64_t dense_ld = 0;
    // owned, only for a matrix that stores every entry and has at most kFullMaxRows rows
    bool full = false;               // the bound pattern is such a matrix
    float *full_scratch = nullptr;   // slice partials of the streaming product, (slices * rows, full_scratch_ld); kept once allocated
    int64_t full_scratch_ld = 0;
    // values_t lags behind values[]: a training step updated this layer as the first layer of an MLP,
    // whose mirror no product reads, and left the mirror's values alone.  Whoever reads values_t next
    // (a step that has the layer further up, sparse_linear_backward, sparse_linear_sync_values)
    // refreshes it first.
    bool mirror_stale = false;
};

// Optional per-kernel timing of mlp_train_step: one HIP event before every launch and one after
// the last launch of each of the first `max_steps` steps after mlp_profile_enable.  A launch's
// time is the span to the next event: kernels of a step run back to back on one stream, so the
// spans add up to the step and each carries the cost of one event, not two.
struct StepProfiler {
    bool on = false;
    int32_t max_steps = 0, step = 0, slot = 0;
    std::vector<std::string> names;    // one per launch of a step, in launch order
    std::vector<hipEvent_t> events;    // [step][slot 0 .. n, end of step], grown while recording
    void release()
    {
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        events.clear();
        names.clear();
        on = false;
        step = slot = 0;
    }
};

struct nerva_mlp {
    std::vector<nerva_layer *> layers;
    std::vector<float *> vel;
    std::vector<float *> bias_vel;
    int32_t max_batch = 0;
    int32_t flags = 0;
    // fused head of a small output layer: per-column losses [max_batch]
    bool head = false;
    float *head_scratch = nullptr;
    StepProfiler prof;
};

namespace {

struct Layout {
    int64_t ld = 0;
    std::vector<int64_t> A, dZ, g, db;
    int64_t bytes = 0;
};

Layout make_layout(const nerva_mlp *m, int32_t batch)
{
    Layout L;
    L.ld = round_up(batch, 32);  // rows start on 128-byte boundaries
    int64_t off = 0;
    auto take = [&](int64_t floats) {
        int64_t o = off;
        off += round_up(floats * 4, 256);
        return o;
    };
    for (const nerva_layer *l : m->layers) {
        L.A.push_back(take(static_cast<int64_t>(l->rows) * L.ld));
        L.dZ.push_back(take(static_cast<int64_t>(l->rows) * L.ld));
        L.g.push_back(take(l->nnz));
        L.db.push_back(take(l->rows));
    }
    L.bytes = off;
    return L;
}

// Rows by stored entries descending, ties by row id: one counting sort, O(rows + longest row), that
// every partition of a pattern is then read off from.
struct RowsByLength {
    std::vector<int32_t> order;
    int32_t longest = 0;
};

RowsByLength rows_by_length(int32_t rows, const int32_t *indptr)
{
    RowsByLength R;
    for (int32_t i = 0; i < rows; ++i) R.longest = std::max(R.longest, indptr[i + 1] - indptr[i]);
    std::vector<int32_t> start(static_cast<size_t>(R.longest) + 2, 0);
    for (int32_t i = 0; i < rows; ++i) ++start[R.longest - (indptr[i + 1] - indptr[i]) + 1];
    for (size_t k = 1; k < start.size(); ++k) start[k] += start[k - 1];
    R.order.resize(rows);
    for (int32_t i = 0; i < rows; ++i) R.order[start[R.longest - (indptr[i + 1] - indptr[i])]++] = i;
    return R;
}

// Rows are grouped by the number of waves that share one row: 2^lg, the smallest power of two
// that leaves each wave at most `target` stored entries, target = nnz / 4096 kept within 8..64
// (measured: with every gather of a pass in flight, fewer and longer shares beat more waves).  A
// row of more than 4 * kWavesPerBlock * huge_target entries is huge: it is cut into work-groups
// of at most 2 * kWavesPerBlock * huge_target entries each, huge_target = nnz / 16384 within
// 8..64 -- finer than `target`, because the few huge rows decide the run time and need many
// work-groups (a dense 10 x 8192 layer: 320 work-groups instead of 130).
struct RowPlan {
    std::vector<int32_t> row_order;  // ordinary rows
    std::vector<int32_t> blocks;     // 4 ints per work-group, huge ones first
    std::vector<int32_t> huge_rows;  // 4 ints per huge row
    std::vector<int32_t> waves;      // 4 ints per wave, kWavesPerBlock waves per work-group
    int32_t n_huge_blocks = 0;
    int32_t n_blocks() const { return static_cast<int32_t>(blocks.size() / 4); }
    int32_t n_huge_rows() const { return static_cast<int32_t>(huge_rows.size() / 4); }
};

// skip_upto >= 0: rows with at most that many entries are left out (they go to the packed path);
// only_upto: rows with more entries than that are left out (they go to the staged kernels).
RowPlan plan_rows(int32_t rows, const int32_t *indptr, const RowsByLength &by_len, int32_t skip_upto = -1, int32_t only_upto = INT32_MAX)
{
    RowPlan P;
    const int64_t nnz = indptr[rows];
    // entries per wave aimed at: ordinary rows, and (finer, for more work-groups on the few rows
    // that decide the run time) the shares of huge rows
    int64_t target = nnz / 4096;
    if (target < 8) target = 8;
    if (target > 64) target = 64;
    int64_t huge_target = nnz / 16384;
    if (huge_target < 8) huge_target = 8;
    if (huge_target > 64) huge_target = 64;
    const int64_t block_cap = huge_target * kWavesPerBlock;
    int max_lg = 0;
    while ((1 << max_lg) < kWavesPerBlock) ++max_lg;
    std::vector<int8_t> ordinary(rows);
    std::vector<int32_t> count(max_lg + 1, 0);
    const bool row_split_only = g_partition_mode.load() == NERVA_PARTITION_ROW_SPLIT;
    int32_t n_ordinary = 0;
    for (int32_t i = 0; i < rows; ++i) {   // huge rows keep row order: their work-groups are also their scratch slots
        const int64_t n = indptr[i + 1] - indptr[i];
        ordinary[i] = 0;
        if (n <= skip_upto || n > only_upto) continue;
        if (!row_split_only && n > 4 * block_cap) {
            const int32_t parts = static_cast<int32_t>((n + 2 * block_cap - 1) / (2 * block_cap));
            const int64_t share = (n + parts - 1) / parts;
            const int32_t first = P.n_blocks();
            for (int32_t q = 0; q < parts; ++q) {
                const int64_t b = indptr[i] + q * share;
                const int64_t e = b + share < indptr[i + 1] ? b + share : indptr[i + 1];
                P.blocks.insert(P.blocks.end(), {kHugeFlag | q, i, static_cast<int32_t>(b), static_cast<int32_t>(e)});
            }
            P.huge_rows.insert(P.huge_rows.end(), {i, first, parts, 0});
            continue;
        }
        int lg = 0;
        if (!row_split_only)   // (plain row splitting: one wave per row whatever its length)
            while (lg < max_lg && (n + (1 << lg) - 1) / (1 << lg) > target) ++lg;
        ordinary[i] = 1;
        ++count[lg];
        ++n_ordinary;
    }
    P.n_huge_blocks = P.n_blocks();
    // A class whose rows do not fill its last work-group hands that work-group's rows (its longest)
    // to the next class, twice the waves per row, if that class's own last work-group has room for
    // them: one work-group fewer to schedule.  (The 1024 x 3072
    // layer of the paper's MLP at 90 % sparsity has 1023 rows of one class and 1 of the next: 513
    // work-groups on a chip that holds 512 at a time.)  The class is monotone in the row's length, so
    // in the order "longest first" every class is one run of rows and the rows handed up are the
    // first of their class's run: only the counts move.
    if (!row_split_only && skip_upto < 0 && only_upto == INT32_MAX) {
        for (int lg = 0; lg < max_lg; ++lg) {
            const int32_t left_over = count[lg] % (kWavesPerBlock >> lg), above = kWavesPerBlock >> (lg + 1);
            // ... where the next class has room for them in a work-group it needs anyway
            if (!left_over || (count[lg + 1] + left_over + above - 1) / above != (count[lg + 1] + above - 1) / above) continue;
            count[lg] -= left_over;
            count[lg + 1] += left_over;
        }
    }
    // ordinary rows longest first, ties in row order: the classes follow each other, heaviest first, and
    // inside a class the rows of a work-group are alike and the work-groups that take longest start first
    P.row_order.reserve(n_ordinary);
    for (int32_t r : by_len.order)
        if (ordinary[r]) P.row_order.push_back(r);
    {
        int32_t f = 0;
        for (int lg = max_lg; lg >= 0; --lg) {
            const int32_t end = f + count[lg], per_block = kWavesPerBlock >> lg;
            for (; f < end; f += per_block) {
                const int32_t n_rows = end - f < per_block ? end - f : per_block;
                P.blocks.insert(P.blocks.end(), {lg | (n_rows << 8), f, 0, 0});
            }
            f = end;
        }
    }
    // The same partition per wave: each of the 2^lg waves of a row takes a contiguous share of
    // its entries, a multiple of 4 entries long (the kernels work on 1, 2 or 4 entries at a time).
    P.waves.resize(P.blocks.size() * kWavesPerBlock);
    int32_t *out = P.waves.data();
    for (int32_t b = 0; b < P.n_blocks(); ++b) {
        const int32_t info = P.blocks[4 * b], y = P.blocks[4 * b + 1];
        const bool huge = (info & kHugeFlag) != 0;
        const int lg = huge ? max_lg : (info & 0xff);
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const int part = w & ((1 << lg) - 1);
            int32_t row = -1;
            int64_t p0 = 0, p1 = 0;
            bool lead = false;
            if (huge) {
                row = y; p0 = P.blocks[4 * b + 2]; p1 = P.blocks[4 * b + 3];
                lead = w == 0 && (info & ~kHugeFlag) == 0;
            } else if ((w >> lg) < (info >> 8)) {
                row = P.row_order[y + (w >> lg)];
                p0 = indptr[row]; p1 = indptr[row + 1];
                lead = part == 0;
            }
            int64_t per = ((p1 - p0) + (1 << lg) - 1) >> lg;
            per = (per + 3) / 4 * 4;
            const int64_t s0 = p0 + part * per < p1 ? p0 + part * per : p1;
            const int64_t s1 = s0 + per < p1 ? s0 + per : p1;
            *out++ = row;
            *out++ = static_cast<int32_t>(s0);
            *out++ = static_cast<int32_t>(s1);
            *out++ = part | (lg << 4) | (lead ? 256 : 0) | (huge ? 512 : 0);
        }
    }
    return P;
}

// Rows of at most kPackMaxLen entries, longest first (ties in row order), 4 ints per row
// {row, first entry, entries, 0}, padded with {-1, 0, 0, 0} to a multiple of 64 rows.  Empty when
// there are fewer than kPackMinRows of them: the packed path pays off on large matrices only.
std::vector<int32_t> short_row_table(int32_t rows, const int32_t *indptr, const RowsByLength &by_len, int32_t *n_short)
{
    int32_t n = 0;
    for (int32_t i = 0; i < rows; ++i) n += indptr[i + 1] - indptr[i] <= kPackMaxLen;
    *n_short = 0;
    std::vector<int32_t> t;
    if (n < kPackMinRows || indptr[rows] == 0 || g_partition_mode.load() == NERVA_PARTITION_ROW_SPLIT) return t;
    t.assign(static_cast<size_t>(round_up(n, 64)) * 4, 0);
    for (int64_t k = n; k < round_up(n, 64); ++k) t[4 * k] = -1;
    int32_t k = 0;
    for (int32_t i : by_len.order) {
        const int32_t len = indptr[i + 1] - indptr[i];
        if (len > kPackMaxLen) continue;
        t[4 * k] = i; t[4 * k + 1] = indptr[i]; t[4 * k + 2] = len;
        ++k;
    }
    *n_short = n;
    return t;
}

// Share of the stored entries that gather one of the kHotRows most referenced operand rows;
// `other` is the transposed orientation (its row lengths are the reference counts).
float hot_row_share(int32_t other_rows, const int32_t *other_indptr, const RowsByLength &other_by_len)
{
    const int64_t nnz = other_indptr[other_rows];
    if (nnz == 0) return 0.f;
    if (other_rows <= kHotRows) return 1.f;
    int64_t top = 0;
    for (int32_t k = 0; k < kHotRows; ++k) {
        const int32_t r = other_by_len.order[k];
        top += other_indptr[r + 1] - other_indptr[r];
    }
    return static_cast<float>(static_cast<double>(top) / static_cast<double>(nnz));
}

// Row ranges and slot order of the staged product (RowBlocks::staged_*) for a matrix whose products
// run at up to max_batch columns; empty when that product would never be chosen.  The segment
// bounds (`ends`) depend on the column indices: the host API fills them here, a layer on the device.
struct StagedPlan {
    std::vector<int32_t> rows;    // [ranges * kStageRangeRows]
    std::vector<int32_t> ends;    // [ranges * (cblocks + 1) * kStageRangeRows] (host API only)
    std::vector<int32_t> groups;  // [ranges]
    int32_t ranges = 0, cblocks = 0;
    int32_t longest_share = 0;    // most entries any one slot serves
    int32_t n_rows = 0;           // rows the plan covers
    int64_t nnz = 0;              // and their stored entries
    size_t ends_ints() const { return static_cast<size_t>(ranges) * (cblocks + 1) * kStageRangeRows; }
};

StagedPlan plan_staged(int32_t all_rows, int32_t cols, const int32_t *indptr, const RowsByLength &by_len, int32_t max_batch,
                       int32_t min_len = 0)
{
    StagedPlan H;
    // the rows the plan covers: all of them, or those of at least min_len stored entries
    std::vector<int32_t> covered;
    int64_t nnz = 0;
    for (int32_t r = 0; r < all_rows; ++r)
        if (indptr[r + 1] - indptr[r] >= min_len) {
            covered.push_back(r);
            nnz += indptr[r + 1] - indptr[r];
        }
    const int32_t rows = static_cast<int32_t>(covered.size());  // from here on: rows of the plan, covered[k] their ids
    const bool preferred = g_partition_mode.load() == NERVA_PARTITION_PREFER_STAGED;
    if (g_partition_mode.load() == NERVA_PARTITION_ROW_SPLIT || max_batch < kStageMinBatch || nnz == 0) return H;
    const int32_t n_tiles = (max_batch + kStageCols - 1) / kStageCols;
    int32_t want = kStageTargetGroups / n_tiles;
    if (want > rows / 64) want = rows / 64;
    // (ranges cut by cost are not equally long: leave an eighth of the slots as slack)
    const int32_t at_least = (rows + kStageRangeRows * 7 / 8 - 1) / (kStageRangeRows * 7 / 8);
    if (want < at_least) want = at_least;
    // one work-group fits a compute unit at a time: fill the last round of the grid as well
    if (static_cast<int64_t>(want) * n_tiles > kStageTargetGroups) {
        const int64_t rounds = (static_cast<int64_t>(want) * n_tiles + kStageTargetGroups - 1) / kStageTargetGroups;
        want = static_cast<int32_t>(rounds * kStageTargetGroups / n_tiles);
    }
    if (!preferred && static_cast<double>(nnz) < static_cast<double>(kStageMinReuse) * want * cols) return H;
    const int32_t cblocks = (cols + kStageRows - 1) / kStageRows;
    if ((static_cast<int64_t>(want) + at_least) * (cblocks + 1) * kStageRangeRows > (1ll << 28)) return H;  // tables beyond 1 GiB
    // ranges of about equal cost: a stored entry costs one gather, a segment about two more
    auto cost = [&](int32_t r) {
        const int64_t len = indptr[r + 1] - indptr[r];
        return len + 2 * (len < cblocks ? len : cblocks) + 1;
    };
    int64_t total = 0;
    for (int32_t k = 0; k < rows; ++k) total += cost(covered[k]);
    // A row of 16 lanes serves a row alone.  A row much longer than a wave's fair share of its range
    // would make that wave the range's critical path: it gets the four lane rows of a wave instead, each a
    // quarter of every segment ("quad": four slots, group-aligned).
    const int64_t quad_len = std::max<int64_t>(256, total / want / 32);
    auto slots_of = [&](int32_t r) { return indptr[r + 1] - indptr[r] >= quad_len ? 4 : 1; };
    std::vector<int32_t> range_of(all_rows, -1);
    int32_t ranges = 0;
    {
        int32_t range = 0, in_range = 0;
        int64_t done = 0;
        for (int32_t k = 0; k < rows; ++k) {
            const int32_t r = covered[k];
            const bool next = range + 1 < want && done * want >= total * (range + 1);
            if ((next || in_range + slots_of(r) > kStageRangeRows) && in_range > 0) {
                ++ranges;
                in_range = 0;
            }
            if (next) ++range;
            done += cost(r);
            in_range += slots_of(r);
            range_of[r] = ranges;
        }
        ++ranges;
    }
    H.ranges = ranges;
    H.cblocks = cblocks;
    H.n_rows = rows;
    H.nnz = nnz;
    H.rows.assign(static_cast<size_t>(ranges) * kStageRangeRows, -1);
    H.groups.assign(ranges, 0);
    // inside a range: longest first, ties in row order -- the global order, read range by range;
    // quads come first (the longest rows), so they start at multiples of 4
    std::vector<int32_t> slot(ranges, 0);
    for (int32_t r : by_len.order) {
        const int32_t q = range_of[r];
        if (q < 0) continue;
        const int32_t copies = slots_of(r), len = indptr[r + 1] - indptr[r];
        const int32_t share = copies == 4 ? (len + 3) / 4 : len;
        if (share > H.longest_share) H.longest_share = share;
        for (int32_t c = 0; c < copies; ++c)
            H.rows[static_cast<size_t>(q) * kStageRangeRows + slot[q] + c] = copies == 4 ? (r | kStageQuad) : r;
        slot[q] += copies;
    }
    for (int32_t q = 0; q < ranges; ++q) H.groups[q] = (slot[q] + 63) / 64;
    return H;
}

// the segment bounds of a plan from host copies of the pattern (what staged_ends_kernel computes for a layer)
void fill_staged_ends_host(StagedPlan &H, const int32_t *indptr, const int32_t *indices)
{
    H.ends.assign(H.ends_ints(), 0);
    for (int32_t q = 0; q < H.ranges; ++q) {
        int32_t *e = H.ends.data() + static_cast<size_t>(q) * (H.cblocks + 1) * kStageRangeRows;
        for (int32_t slot = 0; slot < kStageRangeRows; ++slot) {
            int32_t r = H.rows[static_cast<size_t>(q) * kStageRangeRows + slot];
            if (r < 0) continue;
            r &= ~kStageQuad;
            const int32_t *lo = indices + indptr[r], *hi = indices + indptr[r + 1];
            for (int32_t b = 0; b <= H.cblocks; ++b) {
                if (b > 0) lo = std::lower_bound(lo, hi, b * kStageRows);
                e[static_cast<size_t>(b) * kStageRangeRows + slot] = static_cast<int32_t>(lo - indices);
            }
        }
    }
}

// All partitions of one orientation of a pattern, planned on the host from its row pointers, laid
// out as they go to the device: `staging` is copied to the start of the plan's device memory, the
// segment bounds of the staged plan (ends_ints ints, computed on the device) follow it.
struct HostPlan {
    std::vector<int32_t> staging;
    size_t blocks_at = 0, huge_at = 0, waves_at = 0, staged_at = 0, long_at = 0, rest_at = 0, short_at = 0, order_at = 0, groups_at = 0;
    size_t ends_ints = 0;
    RowBlocks view{};   // counts and flags filled in; pointers are set once the device address is known
    size_t total_ints() const { return staging.size() + ends_ints; }
};

HostPlan make_plan(int32_t rows, const int32_t *indptr_host, const RowsByLength &by_len, int32_t max_batch, int32_t other_rows,
                   float hot_share)
{
    HostPlan hp;
    const RowPlan P = plan_rows(rows, indptr_host, by_len);
    int32_t n_short = 0;
    const std::vector<int32_t> short_rows = short_row_table(rows, indptr_host, by_len, &n_short);
    const int32_t longest_row = by_len.longest;
    // The staged product serves all rows, or, where the rows differ widely in length and the short
    // ones have the packed path to go to, the rows beyond that path's length limit only.
    StagedPlan H;
    bool staged_partial = false;
    if (n_short > 0 && n_short < rows && g_partition_mode.load() == NERVA_PARTITION_BALANCED &&
        static_cast<int64_t>(longest_row) * rows > 4 * static_cast<int64_t>(indptr_host[rows])) {
        H = plan_staged(rows, other_rows, indptr_host, by_len, max_batch, kPackMaxLen + 1);
        staged_partial = H.ranges > 0;
    }
    if (!staged_partial) H = plan_staged(rows, other_rows, indptr_host, by_len, max_batch);
    RowPlan Q, Z;
    if (n_short > 0) Q = plan_rows(rows, indptr_host, by_len, kPackMaxLen);
    // the short rows' partition: for the SDDMM beside a partial staged plan, and for the launches that serve the
    // long rows inside column tiles and the short ones outside (operands beyond the L2s)
    if (n_short > 0 && n_short < rows) Z = plan_rows(rows, indptr_host, by_len, -1, kPackMaxLen);
    int64_t long_nnz = 0;
    for (int32_t r = 0; r < rows; ++r)
        if (indptr_host[r + 1] - indptr_host[r] > kPackMaxLen) long_nnz += indptr_host[r + 1] - indptr_host[r];
    // 16-byte records first so that they stay 16-byte aligned
    std::vector<int32_t> &st = hp.staging;
    st.reserve(P.blocks.size() + P.huge_rows.size() + P.waves.size() + H.rows.size() + Q.waves.size() + Z.waves.size() +
               short_rows.size() + P.row_order.size() + H.groups.size() + 1);
    hp.blocks_at = st.size(); st.insert(st.end(), P.blocks.begin(), P.blocks.end());
    hp.huge_at = st.size(); st.insert(st.end(), P.huge_rows.begin(), P.huge_rows.end());
    hp.waves_at = st.size(); st.insert(st.end(), P.waves.begin(), P.waves.end());
    hp.staged_at = st.size(); st.insert(st.end(), H.rows.begin(), H.rows.end());  // (multiples of kStageRangeRows: what follows stays 16-byte aligned)
    hp.long_at = st.size(); st.insert(st.end(), Q.waves.begin(), Q.waves.end());
    hp.rest_at = st.size(); st.insert(st.end(), Z.waves.begin(), Z.waves.end());
    hp.short_at = st.size(); st.insert(st.end(), short_rows.begin(), short_rows.end());
    hp.order_at = st.size(); st.insert(st.end(), P.row_order.begin(), P.row_order.end());
    hp.groups_at = st.size(); st.insert(st.end(), H.groups.begin(), H.groups.end());
    if (st.empty()) st.push_back(0);
    hp.ends_ints = H.ends_ints();
    RowBlocks &v = hp.view;
    v.n_short = n_short;
    v.hot_share = hot_share;
    v.n_long_blocks = Q.n_blocks();
    v.n_blocks = P.n_blocks();
    v.n_huge_rows = P.n_huge_rows();
    v.n_huge_blocks = P.n_huge_blocks;
    v.staged_ranges = H.ranges;
    v.staged_cblocks = H.cblocks;
    v.staged_preferred = g_partition_mode.load() == NERVA_PARTITION_PREFER_STAGED;
    v.staged_longest_share = H.longest_share;
    v.staged_longest_row = longest_row;
    v.staged_partial = staged_partial;
    v.n_rest_blocks = Z.n_blocks();
    v.long_nnz = static_cast<int32_t>(long_nnz);
    v.staged_row_count = H.n_rows;
    v.staged_nnz = static_cast<int32_t>(H.nnz);
    return hp;
}

// the plan's tables at their device address
RowBlocks plan_view(const HostPlan &hp, const int32_t *mem)
{
    RowBlocks v = hp.view;
    v.blocks = reinterpret_cast<const int4 *>(mem + hp.blocks_at);
    v.huge_rows = reinterpret_cast<const int4 *>(mem + hp.huge_at);
    v.waves = reinterpret_cast<const int4 *>(mem + hp.waves_at);
    v.row_order = mem + hp.order_at;
    v.long_waves = reinterpret_cast<const int4 *>(mem + hp.long_at);
    v.rest_waves = reinterpret_cast<const int4 *>(mem + hp.rest_at);
    v.short_rows = reinterpret_cast<const int4 *>(mem + hp.short_at);
    v.staged_rows = v.staged_ranges ? mem + hp.staged_at : nullptr;
    v.staged_ends = v.staged_ranges ? mem + hp.staging.size() : nullptr;
    v.staged_groups = v.staged_ranges ? mem + hp.groups_at : nullptr;
    return v;
}

void free_pattern_buffers(PatternBuffers &b)
{
    (void)hipFree(b.indptr_t);
    (void)hipFree(b.mirror_mem);
    (void)hipFree(b.plan_mem);
    (void)hipFree(b.plan_t_mem);
    b = PatternBuffers{};
}

void free_layer_buffers(nerva_layer *l)
{
    free_pattern_buffers(l->cur);
    free_pattern_buffers(l->spare);
    (void)hipFree(l->build_work);
    (void)hipFree(l->status);
    (void)hipFree(l->scratch);
    (void)hipFree(l->partial);
    (void)hipFree(l->dense);
    (void)hipFree(l->dense_g);
    (void)hipFree(l->full_scratch);
}

// Room for `need` elements of 4 bytes in *ptr, whose capacity is *have: kept if large enough, else
// replaced by a larger allocation (the old contents are not kept).  On failure nothing changes.
template <typename T>
hipError_t reserve(T **ptr, size_t *have, size_t need)
{
    if (need <= *have && *ptr) return hipSuccess;
    if (need == 0) need = 1;
    const size_t want = need + need / 8;
    void *fresh = nullptr;
    const hipError_t e = hipMalloc(&fresh, want * 4);
    if (e != hipSuccess) return e;
    (void)hipFree(*ptr);
    *ptr = static_cast<T *>(fresh);
    *have = want;
    return hipSuccess;
}

// Marks the start of one launch with an event while profiling is on; costs one branch otherwise.
struct Timed {
    StepProfiler &P;
    hipStream_t s;
    bool live;
    Timed(StepProfiler &p, hipStream_t st, const char *kind, int layer) : P(p), s(st), live(p.on && p.step < p.max_steps)
    {
        if (!live) return;
        if (P.step == 0) {
            char buf[64];
            snprintf(buf, sizeof buf, "%s[%d]", kind, layer);
            P.names.push_back(buf);
        }
        hipEvent_t b = nullptr;
        if (hipEventCreate(&b) != hipSuccess) { live = false; return; }
        P.events.push_back(b);
        (void)hipEventRecord(b, s);
    }
};

int check_batch(int32_t batch, int32_t ld, const char *name)
{
    if (batch <= 0) return fail(NERVA_ERR_ARGUMENT, "batch must be positive (got %d)", batch);
    if (ld < batch) return fail(NERVA_ERR_SHAPE, "%s = %d is smaller than batch = %d", name, ld, batch);
    if (ld >= (1 << 30)) return fail(NERVA_ERR_SHAPE, "%s = %d: rows of 4 GiB or more are not supported", name, ld);
    return NERVA_OK;
}

}  // namespace

extern "C" {

const char *nerva_last_error(void) { return g_last_error.c_str(); }

const char *nerva_build_info(void) { return "nerva_sparse 0.1 gfx950 fp32/int32"; }

int nerva_validate_csr_host(int32_t rows, int32_t cols, int64_t nnz, const int32_t *indptr,
                            const int32_t *indices)
{
    if (rows < 0 || cols < 0 || nnz < 0) return fail(NERVA_ERR_ARGUMENT, "negative size");
    if (!indptr || (nnz > 0 && !indices)) return fail(NERVA_ERR_ARGUMENT, "null pattern array");
    if (nnz > INT32_MAX) return fail(NERVA_ERR_ARGUMENT, "nnz does not fit int32 indices");
    if (indptr[0] != 0) return fail(NERVA_ERR_CSR, "indptr[0] = %d, expected 0", indptr[0]);
    for (int32_t i = 0; i < rows; ++i) {
        const int64_t b = indptr[i], e = indptr[i + 1];
        if (e < b) return fail(NERVA_ERR_CSR, "indptr decreases at row %d", i);
        if (e > nnz) return fail(NERVA_ERR_CSR, "indptr[%d] = %lld exceeds nnz = %lld", i + 1, (long long)e, (long long)nnz);
        for (int64_t p = b; p < e; ++p) {
            const int32_t j = indices[p];
            if (j < 0 || j >= cols) return fail(NERVA_ERR_CSR, "column index %d out of range at position %lld", j, (long long)p);
            if (p > b && indices[p - 1] >= j)
                return fail(NERVA_ERR_CSR, "column indices not strictly ascending in row %d", i);
        }
    }
    if (indptr[rows] != nnz) return fail(NERVA_ERR_CSR, "indptr[rows] = %d, expected nnz = %lld", indptr[rows], (long long)nnz);
    return NERVA_OK;
}

int nerva_set_partition_mode(int32_t mode)
{
    if (mode != NERVA_PARTITION_BALANCED && mode != NERVA_PARTITION_ROW_SPLIT && mode != NERVA_PARTITION_PREFER_STAGED) return fail(NERVA_ERR_ARGUMENT, "unknown partition mode %d", mode);
    g_partition_mode.store(mode);
    return NERVA_OK;
}

int nerva_plan_rows_host(int32_t rows, const int32_t *indptr_host, int32_t *row_order_host,
                         int32_t *blocks_host, int32_t *huge_rows_host, int32_t *waves_host, int32_t *counts_host)
{
    if (rows <= 0 || !indptr_host || !counts_host) return fail(NERVA_ERR_ARGUMENT, "bad argument");
    const RowPlan P = plan_rows(rows, indptr_host, rows_by_length(rows, indptr_host));
    counts_host[0] = static_cast<int32_t>(P.row_order.size());
    counts_host[1] = P.n_blocks();
    counts_host[2] = P.n_huge_rows();
    counts_host[3] = P.n_huge_blocks;
    if (row_order_host && !P.row_order.empty()) memcpy(row_order_host, P.row_order.data(), P.row_order.size() * 4);
    if (blocks_host && !P.blocks.empty()) memcpy(blocks_host, P.blocks.data(), P.blocks.size() * 4);
    if (huge_rows_host && !P.huge_rows.empty()) memcpy(huge_rows_host, P.huge_rows.data(), P.huge_rows.size() * 4);
    if (waves_host && !P.waves.empty()) memcpy(waves_host, P.waves.data(), P.waves.size() * 4);
    return NERVA_OK;
}

int nerva_plan_short_rows_host(int32_t rows, const int32_t *indptr_host, int32_t *short_rows_host,
                               int32_t *long_waves_host, int32_t *counts_host)
{
    if (rows <= 0 || !indptr_host || !counts_host) return fail(NERVA_ERR_ARGUMENT, "bad argument");
    int32_t n_short = 0;
    const RowsByLength by_len = rows_by_length(rows, indptr_host);
    const std::vector<int32_t> t = short_row_table(rows, indptr_host, by_len, &n_short);
    RowPlan Q;
    if (n_short > 0) Q = plan_rows(rows, indptr_host, by_len, kPackMaxLen);
    counts_host[0] = n_short;
    counts_host[1] = Q.n_blocks();
    counts_host[2] = Q.n_huge_blocks;
    if (short_rows_host && !t.empty()) memcpy(short_rows_host, t.data(), t.size() * 4);
    if (long_waves_host && !Q.waves.empty()) memcpy(long_waves_host, Q.waves.data(), Q.waves.size() * 4);
    return NERVA_OK;
}

int nerva_plan_staged_host(int32_t rows, int32_t cols, const int32_t *indptr_host, const int32_t *indices_host,
                           int32_t max_batch, int32_t min_entries, int32_t *slot_rows_host, int32_t *ends_host,
                           int32_t *counts_host)
{
    if (rows <= 0 || cols <= 0 || min_entries < 0 || !indptr_host || !counts_host || (indptr_host[rows] > 0 && !indices_host))
        return fail(NERVA_ERR_ARGUMENT, "bad argument");
    static_assert(NERVA_STAGE_ROWS == kStageRows && NERVA_STAGE_COLS == kStageCols && NERVA_STAGE_MIN_BATCH == kStageMinBatch &&
                  NERVA_STAGE_RANGE_ROWS == kStageRangeRows && NERVA_STAGE_QUAD == kStageQuad, "header and kernels disagree");
    StagedPlan H = plan_staged(rows, cols, indptr_host, rows_by_length(rows, indptr_host), max_batch, min_entries);
    if (ends_host && H.ranges) fill_staged_ends_host(H, indptr_host, indices_host);
    counts_host[0] = H.ranges;
    counts_host[1] = H.cblocks;
    if (slot_rows_host && !H.rows.empty()) memcpy(slot_rows_host, H.rows.data(), H.rows.size() * 4);
    if (ends_host && !H.ends.empty()) memcpy(ends_host, H.ends.data(), H.ends.size() * 4);
    return NERVA_OK;
}

// Density from which a layer bound by sparse_linear_create / sparse_linear_rebind takes the dense route by
// itself (process-wide; nerva_set_dense_threshold).  The default is the measured cut-over on the paper's MLP.
std::atomic<float> g_dense_threshold{kDenseFromDensity};

static bool dense_shape_ok(int32_t rows, int32_t cols)
{
    // (a thin full matrix has its own streaming kernels; the copy and the dense gradient stay below 2 GiB each)
    return rows >= 64 && cols >= 64 && static_cast<int64_t>(rows) * round_up(cols, kDenseLdAlign) < (1ll << 29);
}

// The dense copy for the dense route: allocated zero, then filled from the stored entries; and the dense gradient.
static hipError_t build_dense_copies(nerva_layer *l, hipStream_t s)
{
    l->dense_ld = round_up(l->cols, kDenseLdAlign);
    const size_t bytes = static_cast<size_t>(l->rows) * l->dense_ld * 4;
    hipError_t e = hipMalloc(&l->dense, bytes);
    if (e == hipSuccess) e = hipMalloc(&l->dense_g, bytes);
    if (e == hipSuccess) e = hipMemsetAsync(l->dense, 0, bytes, s);
    if (e == hipSuccess) e = launch_dense_refresh(l->indptr, l->indices, l->values, l->rows, l->dense, l->dense_ld, s);
    return e;
}

static hipError_t refresh_dense_copies(const nerva_layer *l, hipStream_t s)
{
    return launch_dense_refresh(l->indptr, l->indices, l->values, l->rows, l->dense, l->dense_ld, s);
}

// Y = act(W X + b) through the dense copy
static hipError_t dense_forward(const nerva_layer *l, const float *X, int64_t ldx, float *Y, int64_t ldy, int32_t batch,
                                hipStream_t s)
{
    DenseArgs d{};
    d.W = l->dense; d.ldw = l->dense_ld; d.trans = 0; d.X = X; d.ldx = ldx; d.Y = Y; d.ldy = ldy; d.bias = l->bias;
    d.rows = l->rows; d.cols = l->cols; d.batch = batch; d.relu = l->activation == NERVA_ACT_RELU;
    return launch_dense_product(d, s);
}

// dX = (W^T dZ) * [mask > 0] through the same copy
static hipError_t dense_transposed(const nerva_layer *l, const float *dZ, int64_t lddz, float *dX, int64_t lddx,
                                   const float *mask, int64_t ldmask, int32_t batch, hipStream_t s)
{
    DenseArgs d{};
    d.W = l->dense; d.ldw = l->dense_ld; d.trans = 1; d.X = dZ; d.ldx = lddz; d.Y = dX; d.ldy = lddx;
    d.YM = mask; d.ldym = ldmask; d.rows = l->rows; d.cols = l->cols; d.batch = batch;
    return launch_dense_product(d, s);
}

static int enable_dense(nerva_layer *layer, hipStream_t s);

// the dense route needs a batch wide enough to fill its 16-column tiles
static bool use_dense(const nerva_layer *l, int32_t batch) { return l->dense_on && batch >= 16; }

// Message for the status word of the device-side CSR check (launch_validate_csr).
static int csr_status_error(const int32_t *st)
{
    const int f = st[0];
    if (f & kCsrBadFirst) return fail(NERVA_ERR_CSR, "indptr[0] is not 0");
    if (f & kCsrDecreasing) return fail(NERVA_ERR_CSR, "indptr decreases at row %d", st[1]);
    if (f & kCsrBeyondNnz) return fail(NERVA_ERR_CSR, "indptr[%d] lies outside [0, nnz]", st[1]);
    if (f & kCsrBadLast) return fail(NERVA_ERR_CSR, "indptr[rows] differs from nnz");
    if (f & kCsrColumnRange) return fail(NERVA_ERR_CSR, "column index out of range at position %d", st[2]);
    if (f & kCsrNotAscending) return fail(NERVA_ERR_CSR, "column indices not strictly ascending at position %d", st[2]);
    return fail(NERVA_ERR_CSR, "pattern is not canonical CSR (status 0x%x)", f);
}

// Everything a pattern allows to be precomputed, for a layer `l` that describes the NEW pattern (sizes,
// caller-owned arrays, max_batch) and owns the buffers to build into: l->spare receives the mirror and the
// partition tables (l->cur, if any, is not touched), the scratch buffers grow as needed.  What grows with
// the stored entries runs on the device: the CSR check, the mirror with its position maps (a stable
// counting sort by column) and the staged plans' segment bounds; the row partitions, which depend on the
// row lengths only, are planned on the host from copies of the two row-pointer arrays.  On failure
// (NERVA_ERR_CSR, NERVA_ERR_HIP) nothing that a product reads has been changed.  On success the caller swaps
// l->spare into l->cur and adopts `plan`, `plan_t`.
struct BuiltPattern {
    RowBlocks plan{}, plan_t{};
    int64_t partial_stride = 0, partial_db_at = 0;
    int32_t partial_tiles = 0;
    int64_t scratch_ld = 0, full_scratch_ld = 0;
    bool full = false;
};

static int build_structures(nerva_layer *l, int32_t nnz, const int32_t *indptr, const int32_t *indices, const float *values,
                            BuiltPattern *out, hipStream_t s)
{
    const int32_t rows = l->rows, cols = l->cols, max_batch = l->max_batch;
    PatternBuffers &B = l->spare;
    // 1. the pattern is checked where it lives; the row pointers come to the host for the partitions
    std::vector<int32_t> h_indptr(static_cast<size_t>(rows) + 1), h_indptr_t(static_cast<size_t>(cols) + 1);
    int32_t h_status[4] = {0, 0, 0, 0};
    if (!l->status) HIP_TRY(hipMalloc(&l->status, 4 * sizeof(int32_t)));
    HIP_TRY(launch_validate_csr(rows, cols, nnz, indptr, indices, l->status, s));
    HIP_TRY(hipMemcpyAsync(h_indptr.data(), indptr, h_indptr.size() * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_status, l->status, sizeof h_status, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (h_status[0] != 0) return csr_status_error(h_status);

    // 2. the mirror, on the device, into the spare set
    const size_t n64 = static_cast<size_t>(round_up(nnz > 0 ? nnz : 1, 64));
    const int32_t T = mirror_tiles(rows, cols, nnz);
    size_t indptr_t_have = B.indptr_t ? static_cast<size_t>(cols) + 1 : 0;
    HIP_TRY(reserve(&B.indptr_t, &indptr_t_have, static_cast<size_t>(cols) + 1));
    HIP_TRY(reserve(&B.mirror_mem, &B.mirror_ints, 4 * n64));
    HIP_TRY(reserve(&l->build_work, &l->build_work_ints, mirror_work_ints(cols, T)));
    int32_t *indices_t = B.mirror_mem, *perm = B.mirror_mem + n64, *pos_t = B.mirror_mem + 2 * n64;
    float *values_t = reinterpret_cast<float *>(B.mirror_mem + 3 * n64);
    HIP_TRY(launch_build_mirror(rows, cols, nnz, indptr, indices, B.indptr_t, indices_t, perm, pos_t, l->build_work, T, s));
    HIP_TRY(hipMemcpyAsync(h_indptr_t.data(), B.indptr_t, h_indptr_t.size() * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(launch_gather(values_t, values, perm, nnz, s));
    // ... while the host orders the rows by length
    const RowsByLength by_len = rows_by_length(rows, h_indptr.data());
    HIP_TRY(hipStreamSynchronize(s));
    const RowsByLength by_len_t = rows_by_length(cols, h_indptr_t.data());

    // 3. the partitions of both orientations (integer work on row lengths), then their tables to the device
    const HostPlan hp = make_plan(rows, h_indptr.data(), by_len, max_batch, cols, hot_row_share(cols, h_indptr_t.data(), by_len_t));
    const HostPlan hp_t = make_plan(cols, h_indptr_t.data(), by_len_t, max_batch, rows, hot_row_share(rows, h_indptr.data(), by_len));
    HIP_TRY(reserve(&B.plan_mem, &B.plan_ints, hp.total_ints()));
    HIP_TRY(reserve(&B.plan_t_mem, &B.plan_t_ints, hp_t.total_ints()));
    HIP_TRY(hipMemcpyAsync(B.plan_mem, hp.staging.data(), hp.staging.size() * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(B.plan_t_mem, hp_t.staging.data(), hp_t.staging.size() * 4, hipMemcpyHostToDevice, s));
    out->plan = plan_view(hp, B.plan_mem);
    out->plan_t = plan_view(hp_t, B.plan_t_mem);
    if (out->plan.staged_ranges)
        HIP_TRY(launch_staged_ends(indptr, indices, out->plan.staged_rows, const_cast<int32_t *>(out->plan.staged_ends),
                                   out->plan.staged_ranges, out->plan.staged_cblocks, s));
    if (out->plan_t.staged_ranges)
        HIP_TRY(launch_staged_ends(B.indptr_t, indices_t, out->plan_t.staged_rows, const_cast<int32_t *>(out->plan_t.staged_ends),
                                   out->plan_t.staged_ranges, out->plan_t.staged_cblocks, s));

    // 4. scratch buffers (they hold nothing between calls: grown in place)
    {
        // room for the column-tiled SDDMM at max_batch columns, if that batch would be tiled
        const int w = tile_columns(cols, max_batch, nnz, rows, out->plan.hot_share, false, true);
        int32_t tiles = w > 0 ? (max_batch + w - 1) / w : 0;
        if (out->plan.staged_rows && (max_batch + kStageCols - 1) / kStageCols > tiles) tiles = (max_batch + kStageCols - 1) / kStageCols;
        // ... and for the backward pass on one gather stream (products in mirror order, one slice per tile of the
        // transposed product), which runs where every row of the mirror is short
        if (out->plan_t.n_short == cols && out->plan_t.n_long_blocks == 0) {
            const int wt = tile_columns(rows, max_batch, nnz, cols, out->plan_t.hot_share, false);
            if (wt > 0 && (max_batch + wt - 1) / wt > tiles) tiles = (max_batch + wt - 1) / wt;
        }
        out->partial_tiles = 0;
        if (tiles > 0) {
            out->partial_db_at = round_up(nnz, 64);
            out->partial_stride = out->partial_db_at + round_up(rows, 64);
            const size_t floats = static_cast<size_t>(tiles) * out->partial_stride;
            if (floats * 4 <= (4ull << 30)) {  // (beyond that it is too large to be worth it: the untiled kernel stays)
                HIP_TRY(reserve(&l->partial, &l->partial_floats, floats));
                out->partial_tiles = tiles;
            }
        }
        const int64_t slots = out->plan.n_huge_blocks > out->plan_t.n_huge_blocks ? out->plan.n_huge_blocks : out->plan_t.n_huge_blocks;
        out->scratch_ld = round_up(max_batch, 64);
        if (slots > 0) HIP_TRY(reserve(&l->scratch, &l->scratch_floats, static_cast<size_t>(slots) * out->scratch_ld));
        out->full = rows <= kFullMaxRows && static_cast<int64_t>(nnz) == static_cast<int64_t>(rows) * cols;
        out->full_scratch_ld = round_up(max_batch, 64);
        if (out->full && !l->full_scratch) {
            const int64_t slices = (cols + kFullSlice - 1) / kFullSlice;
            HIP_TRY(hipMalloc(&l->full_scratch, static_cast<size_t>(slices) * rows * out->full_scratch_ld * 4));
        }
    }
    HIP_TRY(hipStreamSynchronize(s));  // the host staging vectors die at return
    return NERVA_OK;
}

// The spare set, just built, becomes the layer's pattern; the set it replaces becomes the spare one.
static void adopt_pattern(nerva_layer *l, int32_t nnz, const int32_t *indptr, const int32_t *indices, float *values, const BuiltPattern &bp)
{
    std::swap(l->cur, l->spare);
    const size_t n64 = static_cast<size_t>(round_up(nnz > 0 ? nnz : 1, 64));
    l->nnz = nnz; l->indptr = indptr; l->indices = indices; l->values = values;
    l->indptr_t = l->cur.indptr_t;
    l->indices_t = l->cur.mirror_mem;
    l->perm = l->cur.mirror_mem + n64;
    l->pos_t = l->cur.mirror_mem + 2 * n64;
    l->values_t = reinterpret_cast<float *>(l->cur.mirror_mem + 3 * n64);
    l->plan = bp.plan; l->plan_t = bp.plan_t;
    l->partial_stride = bp.partial_stride; l->partial_db_at = bp.partial_db_at; l->partial_tiles = bp.partial_tiles;
    l->scratch_ld = bp.scratch_ld;
    l->full_scratch_ld = bp.full_scratch_ld;
    l->full = bp.full;
    l->mirror_stale = false;
}

int sparse_linear_create(nerva_layer **out, int32_t rows, int32_t cols, int32_t nnz, const int32_t *indptr,
                         const int32_t *indices, float *values, float *bias, int32_t activation, int32_t max_batch,
                         void *stream)
{
    if (!out) return fail(NERVA_ERR_ARGUMENT, "out is null");
    *out = nullptr;
    if (rows <= 0 || cols <= 0 || nnz < 0) return fail(NERVA_ERR_ARGUMENT, "bad layer size %d x %d, nnz %d", rows, cols, nnz);
    if (!indptr || (nnz > 0 && (!indices || !values))) return fail(NERVA_ERR_ARGUMENT, "null pattern or values pointer");
    if (activation != NERVA_ACT_NONE && activation != NERVA_ACT_RELU) return fail(NERVA_ERR_ARGUMENT, "unknown activation %d", activation);
    if (max_batch <= 0 || max_batch >= (1 << 30)) return fail(NERVA_ERR_ARGUMENT, "max_batch must be positive (got %d)", max_batch);
    nerva_layer *l = new (std::nothrow) nerva_layer;
    if (!l) return fail(NERVA_ERR_ARGUMENT, "out of host memory");
    l->rows = rows; l->cols = cols; l->activation = activation; l->max_batch = max_batch; l->bias = bias;
    BuiltPattern bp;
    const int rc = build_structures(l, nnz, indptr, indices, values, &bp, as_stream(stream));
    if (rc != NERVA_OK) {
        free_layer_buffers(l);
        delete l;
        return rc;
    }
    adopt_pattern(l, nnz, indptr, indices, values, bp);
    // the density-adaptive choice: dense products where the pattern is dense enough for them to be the faster ones
    if (dense_shape_ok(rows, cols) && static_cast<double>(nnz) >= static_cast<double>(g_dense_threshold.load()) * rows * cols) {
        const int rd = enable_dense(l, as_stream(stream));
        if (rd != NERVA_OK) {
            free_layer_buffers(l);
            delete l;
            return rd;
        }
    }
    *out = l;
    return NERVA_OK;
}

int sparse_linear_rebind(nerva_layer *layer, int32_t nnz, const int32_t *indptr, const int32_t *indices, float *values,
                         void *stream)
{
    if (!layer) return fail(NERVA_ERR_ARGUMENT, "layer is null");
    if (nnz < 0 || !indptr || (nnz > 0 && (!indices || !values))) return fail(NERVA_ERR_ARGUMENT, "null pattern or values pointer");
    hipStream_t s = as_stream(stream);
    HIP_TRY(hipStreamSynchronize(s));  // launches already queued on this stream still use the old structures
    BuiltPattern bp;
    const int rc = build_structures(layer, nnz, indptr, indices, values, &bp, s);
    if (rc != NERVA_OK) return rc;  // the layer keeps its old pattern: only the spare set and scratch buffers were written
    adopt_pattern(layer, nnz, indptr, indices, values, bp);
    if (!layer->dense_on && dense_shape_ok(layer->rows, layer->cols) &&
        static_cast<double>(nnz) >= static_cast<double>(g_dense_threshold.load()) * layer->rows * layer->cols)
        return enable_dense(layer, s);   // (a pattern that has grown dense; a route once taken is kept)
    if (layer->dense_on) {
        // the dense copies hold the old pattern's entries: cleared and filled again
        const size_t bytes = static_cast<size_t>(layer->rows) * layer->dense_ld * 4;
        HIP_TRY(hipMemsetAsync(layer->dense, 0, bytes, s));
        HIP_TRY(refresh_dense_copies(layer, s));
        HIP_TRY(hipStreamSynchronize(s));
    }
    return NERVA_OK;
}

static int enable_dense(nerva_layer *layer, hipStream_t s)
{
    if (layer->dense_on) return NERVA_OK;
    if (static_cast<int64_t>(layer->rows) * round_up(layer->cols, kDenseLdAlign) >= (1ll << 31))
        return fail(NERVA_ERR_SHAPE, "a %d x %d layer is too large for the dense route", layer->rows, layer->cols);
    hipError_t e = build_dense_copies(layer, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        (void)hipFree(layer->dense);
        (void)hipFree(layer->dense_g);
        layer->dense = layer->dense_g = nullptr;
        return hip_fail(e, "sparse_linear_enable_dense");
    }
    layer->dense_on = true;
    return NERVA_OK;
}

int sparse_linear_enable_dense(nerva_layer *layer, void *stream)
{
    if (!layer) return fail(NERVA_ERR_ARGUMENT, "layer is null");
    return enable_dense(layer, as_stream(stream));
}

int nerva_set_dense_threshold(float density)
{
    if (!(density >= 0.f)) return fail(NERVA_ERR_ARGUMENT, "the density threshold must not be negative");
    g_dense_threshold.store(density);
    return NERVA_OK;
}

int sparse_linear_sync_values(nerva_layer *layer, void *stream)
{
    if (!layer) return fail(NERVA_ERR_ARGUMENT, "layer is null");
    hipStream_t s = as_stream(stream);
    HIP_TRY(launch_gather(layer->values_t, layer->values, layer->perm, layer->nnz, s));
    layer->mirror_stale = false;
    if (layer->dense_on) HIP_TRY(refresh_dense_copies(layer, s));
    return NERVA_OK;
}

void sparse_linear_destroy(nerva_layer *layer)
{
    if (!layer) return;
    free_layer_buffers(layer);
    delete layer;
}

int sparse_linear_mirror(const nerva_layer *layer, const int32_t **indptr_t, const int32_t **indices_t,
                         const float **values_t, const int32_t **perm)
{
    if (!layer) return fail(NERVA_ERR_ARGUMENT, "layer is null");
    if (indptr_t) *indptr_t = layer->indptr_t;
    if (indices_t) *indices_t = layer->indices_t;
    if (values_t) *values_t = layer->values_t;
    if (perm) *perm = layer->perm;
    return NERVA_OK;
}

int sparse_linear_forward(const nerva_layer *layer, const float *X, int32_t ldx, float *Y, int32_t ldy,
                          int32_t batch, void *stream)
{
    if (!layer || !X || !Y) return fail(NERVA_ERR_ARGUMENT, "null argument");
    int rc = check_batch(batch, ldx, "ldx");
    if (rc == NERVA_OK) rc = check_batch(batch, ldy, "ldy");
    if (rc == NERVA_OK && batch > layer->max_batch) rc = fail(NERVA_ERR_SHAPE, "batch %d exceeds the layer's max_batch %d", batch, layer->max_batch);
    if (rc != NERVA_OK) return rc;
    if (use_dense(layer, batch)) {
        // a stand-alone call cannot know whether the caller has changed values[] since the last one
        HIP_TRY(refresh_dense_copies(layer, as_stream(stream)));
        HIP_TRY(dense_forward(layer, X, ldx, Y, ldy, batch, as_stream(stream)));
        return NERVA_OK;
    }
    SpmmArgs a{};
    a.blocks = layer->plan; a.nnz = layer->nnz; a.scratch = layer->scratch; a.scratch_ld = layer->scratch_ld;
    a.indptr = layer->indptr; a.indices = layer->indices; a.values = layer->values; a.bias = layer->bias;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy;
    a.rows = layer->rows; a.x_rows = layer->cols; a.batch = batch; a.relu = layer->activation == NERVA_ACT_RELU;
    a.full_scratch = layer->full ? layer->full_scratch : nullptr; a.full_scratch_ld = layer->full_scratch_ld;
    HIP_TRY(launch_spmm(a, as_stream(stream)));
    return NERVA_OK;
}

int sparse_linear_backward(nerva_layer *layer, const float *X, int32_t ldx, const float *Y, int32_t ldy,
                           const float *dY, int32_t lddy, float *dX, int32_t lddx, float *dvalues, float *dbias,
                           int32_t batch, void *stream)
{
    if (!layer || !dY) return fail(NERVA_ERR_ARGUMENT, "null argument");
    const bool relu = layer->activation == NERVA_ACT_RELU;
    if (relu && !Y) return fail(NERVA_ERR_ARGUMENT, "a ReLU layer needs its output Y for the backward pass");
    if (dvalues && !X) return fail(NERVA_ERR_ARGUMENT, "dvalues needs the layer input X");
    int rc = check_batch(batch, lddy, "lddy");
    if (rc == NERVA_OK && relu) rc = check_batch(batch, ldy, "ldy");
    if (rc == NERVA_OK && dvalues) rc = check_batch(batch, ldx, "ldx");
    if (rc == NERVA_OK && dX) rc = check_batch(batch, lddx, "lddx");
    if (rc == NERVA_OK && batch > layer->max_batch) rc = fail(NERVA_ERR_SHAPE, "batch %d exceeds the layer's max_batch %d", batch, layer->max_batch);
    if (rc != NERVA_OK) return rc;
    hipStream_t s = as_stream(stream);
    if (dX && use_dense(layer, batch) && !relu) {
        HIP_TRY(refresh_dense_copies(layer, s));
        HIP_TRY(dense_transposed(layer, dY, lddy, dX, lddx, nullptr, 0, batch, s));
    } else if (dX) {
        HIP_TRY(launch_gather(layer->values_t, layer->values, layer->perm, layer->nnz, s));
        layer->mirror_stale = false;
        SpmmArgs a{};
        a.blocks = layer->plan_t; a.nnz = layer->nnz; a.scratch = layer->scratch; a.scratch_ld = layer->scratch_ld;
        a.indptr = layer->indptr_t; a.indices = layer->indices_t; a.values = layer->values_t;
        a.X = dY; a.ldx = lddy;
        if (relu) { a.XM = Y; a.ldxm = ldy; }
        a.Y = dX; a.ldy = lddx; a.rows = layer->cols; a.x_rows = layer->rows; a.batch = batch;
        HIP_TRY(launch_spmm(a, s));
    }
    if (dvalues || dbias) {
        SddmmArgs a{};
        a.blocks = layer->plan;
        a.indptr = layer->indptr; a.indices = layer->indices;
        a.dZ = dY; a.lddz = lddy;
        if (relu) { a.ZM = Y; a.ldzm = ldy; }
        a.X = X; a.ldx = ldx; a.g = dvalues; a.db = dbias;
        a.rows = layer->rows; a.x_rows = layer->cols; a.batch = batch; a.nnz = layer->nnz;
        a.partial = layer->partial; a.partial_stride = layer->partial_stride;
        a.partial_db_at = layer->partial_db_at; a.partial_tiles = layer->partial_tiles;
        a.skip_products = dvalues ? 0 : 1;  // only the bias gradient is wanted
        HIP_TRY(launch_sddmm(a, s));
    }
    return NERVA_OK;
}

int sgd_update_values(float *values, float *velocity, const float *grad, int64_t n, float lr, float momentum,
                      void *stream)
{
    if (n < 0) return fail(NERVA_ERR_ARGUMENT, "n is negative");
    if (n > 0 && (!values || !velocity || !grad)) return fail(NERVA_ERR_ARGUMENT, "null argument");
    HIP_TRY(launch_momentum(values, velocity, grad, n, lr, momentum, 0, as_stream(stream)));
    return NERVA_OK;
}

int sgd_update_values_nesterov(float *values, float *velocity, const float *grad, int64_t n, float lr, float momentum,
                               void *stream)
{
    if (n < 0) return fail(NERVA_ERR_ARGUMENT, "n is negative");
    if (n > 0 && (!values || !velocity || !grad)) return fail(NERVA_ERR_ARGUMENT, "null argument");
    HIP_TRY(launch_momentum(values, velocity, grad, n, lr, momentum, 1, as_stream(stream)));
    return NERVA_OK;
}

int softmax_cross_entropy(const float *Z, int32_t ldz, const int32_t *labels, int32_t classes, int32_t batch,
                          float *dZ, int32_t lddz, float *loss_out, void *stream)
{
    if (!Z || !labels || !dZ) return fail(NERVA_ERR_ARGUMENT, "null argument");
    if (classes <= 0) return fail(NERVA_ERR_ARGUMENT, "classes must be positive");
    int rc = check_batch(batch, ldz, "ldz");
    if (rc == NERVA_OK) rc = check_batch(batch, lddz, "lddz");
    if (rc != NERVA_OK) return rc;
    HIP_TRY(launch_softmax_ce(Z, ldz, labels, classes, batch, dZ, lddz, loss_out, as_stream(stream)));
    return NERVA_OK;
}

int mlp_create(nerva_mlp **out, int32_t n_layers, nerva_layer *const *layers, float *const *velocities,
               float *const *bias_velocities, int32_t max_batch, int32_t flags)
{
    if (!out) return fail(NERVA_ERR_ARGUMENT, "out is null");
    *out = nullptr;
    if (n_layers <= 0 || !layers || !velocities || !bias_velocities) return fail(NERVA_ERR_ARGUMENT, "null or empty layer list");
    if (max_batch <= 0) return fail(NERVA_ERR_ARGUMENT, "max_batch must be positive");
    if (flags & ~(NERVA_MLP_UNFUSED | NERVA_MLP_NESTEROV | NERVA_MLP_SEPARATE_HEAD)) return fail(NERVA_ERR_ARGUMENT, "unknown flags 0x%x", flags);
    for (int32_t l = 0; l < n_layers; ++l) {
        if (!layers[l]) return fail(NERVA_ERR_ARGUMENT, "layer %d is null", l);
        if (layers[l]->nnz > 0 && !velocities[l]) return fail(NERVA_ERR_ARGUMENT, "velocity of layer %d is null", l);
        if (layers[l]->bias && !bias_velocities[l]) return fail(NERVA_ERR_ARGUMENT, "bias velocity of layer %d is null", l);
        if (layers[l]->max_batch < max_batch)
            return fail(NERVA_ERR_SHAPE, "layer %d was created for batches up to %d, the MLP asks for %d", l, layers[l]->max_batch, max_batch);
        if (l > 0 && layers[l]->cols != layers[l - 1]->rows)
            return fail(NERVA_ERR_SHAPE, "layer %d has %d inputs but layer %d has %d outputs", l, layers[l]->cols, l - 1, layers[l - 1]->rows);
        const int32_t want = l + 1 < n_layers ? NERVA_ACT_RELU : NERVA_ACT_NONE;
        if (layers[l]->activation != want)
            return fail(NERVA_ERR_ARGUMENT, "layer %d: hidden layers must be ReLU and the last layer linear", l);
    }
    nerva_mlp *m = new (std::nothrow) nerva_mlp;
    if (!m) return fail(NERVA_ERR_ARGUMENT, "out of host memory");
    {
        // set-up time: the address of the static workspace on this device, so that
        // mlp_train_step_static has nothing left to look up
        void *ptr = nullptr;
        const hipError_t e = static_scratch(&ptr);
        if (e != hipSuccess) {
            delete m;
            return hip_fail(e, "address of the static workspace");
        }
    }
    m->layers.assign(layers, layers + n_layers);
    m->vel.assign(velocities, velocities + n_layers);
    m->bias_vel.assign(bias_velocities, bias_velocities + n_layers);
    m->max_batch = max_batch;
    m->flags = flags;
    const nerva_layer *last = layers[n_layers - 1];
    m->head = n_layers >= 2 && !(flags & NERVA_MLP_SEPARATE_HEAD) && head_ok(last->rows, last->cols, last->nnz);
    if (m->head || (n_layers >= 2 && last->full && last->rows <= kFullMaxRows)) {   // per-column losses between two launches of a step
        const size_t bytes = static_cast<size_t>(max_batch) * 4;
        hipError_t e = hipMalloc(&m->head_scratch, bytes);
        if (e == hipSuccess) e = hipMemset(m->head_scratch, 0, bytes);
        if (e != hipSuccess) {
            if (m->head_scratch) (void)hipFree(m->head_scratch);
            delete m;
            return fail(NERVA_ERR_HIP, "head work space: %s", hipGetErrorString(e));
        }
    }
    *out = m;
    return NERVA_OK;
}

int mlp_rebind_velocity(nerva_mlp *mlp, int32_t layer_index, float *velocity)
{
    if (!mlp) return fail(NERVA_ERR_ARGUMENT, "mlp is null");
    if (layer_index < 0 || layer_index >= static_cast<int32_t>(mlp->layers.size()))
        return fail(NERVA_ERR_ARGUMENT, "layer index %d out of range", layer_index);
    if (!velocity && mlp->layers[layer_index]->nnz > 0) return fail(NERVA_ERR_ARGUMENT, "velocity is null");
    mlp->vel[layer_index] = velocity;
    return NERVA_OK;
}

void mlp_destroy(nerva_mlp *mlp)
{
    if (!mlp) return;
    mlp->prof.release();
    if (mlp->head_scratch) (void)hipFree(mlp->head_scratch);
    delete mlp;
}

int mlp_profile_enable(nerva_mlp *mlp, int32_t max_steps)
{
    if (!mlp || max_steps < 0) return fail(NERVA_ERR_ARGUMENT, "bad argument");
    mlp->prof.release();
    mlp->prof.on = max_steps > 0;
    mlp->prof.max_steps = max_steps;
    return NERVA_OK;
}

int mlp_profile_read(nerva_mlp *mlp, int32_t max_slots, int32_t *n_slots_host, double *ms_sum_host,
                     int32_t *steps_host)
{
    if (!mlp || !n_slots_host || !ms_sum_host || !steps_host) return fail(NERVA_ERR_ARGUMENT, "null argument");
    StepProfiler &P = mlp->prof;
    const int32_t n = static_cast<int32_t>(P.names.size());
    if (n > max_slots) return fail(NERVA_ERR_ARGUMENT, "%d slots, room for %d", n, max_slots);
    *n_slots_host = n;
    *steps_host = P.step;
    for (int32_t k = 0; k < n; ++k) ms_sum_host[k] = 0.0;
    if (P.events.size() != static_cast<size_t>(P.step) * (n + 1)) return fail(NERVA_ERR_HIP, "event bookkeeping is inconsistent");
    for (int32_t t = 0; t < P.step; ++t)
        for (int32_t k = 0; k < n; ++k) {
            const size_t i = static_cast<size_t>(t) * (n + 1) + k;
            HIP_TRY(hipEventSynchronize(P.events[i + 1]));
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, P.events[i], P.events[i + 1]));
            ms_sum_host[k] += ms;
        }
    return NERVA_OK;
}

const char *mlp_profile_slot_name(const nerva_mlp *mlp, int32_t slot)
{
    if (!mlp || slot < 0 || slot >= static_cast<int32_t>(mlp->prof.names.size())) return "";
    return mlp->prof.names[slot].c_str();
}

size_t mlp_workspace_bytes(const nerva_mlp *mlp, int32_t batch)
{
    if (!mlp || batch <= 0) return 0;
    return static_cast<size_t>(make_layout(mlp, batch).bytes);
}

int mlp_workspace_layout(const nerva_mlp *mlp, int32_t batch, int64_t *layout_host)
{
    if (!mlp || !layout_host) return fail(NERVA_ERR_ARGUMENT, "null argument");
    if (batch <= 0) return fail(NERVA_ERR_ARGUMENT, "batch must be positive");
    const Layout L = make_layout(mlp, batch);
    layout_host[0] = L.ld;
    for (size_t l = 0; l < mlp->layers.size(); ++l) {
        layout_host[1 + 4 * l + 0] = L.A[l];
        layout_host[1 + 4 * l + 1] = L.dZ[l];
        layout_host[1 + 4 * l + 2] = L.g[l];
        layout_host[1 + 4 * l + 3] = L.db[l];
    }
    return NERVA_OK;
}

static int check_step_args(const nerva_mlp *mlp, const float *X, int32_t ldx, int32_t batch, void *workspace,
                           size_t workspace_bytes, Layout &L)
{
    if (!mlp || !X || !workspace) return fail(NERVA_ERR_ARGUMENT, "null argument");
    int rc = check_batch(batch, ldx, "ldx");
    if (rc != NERVA_OK) return rc;
    if (batch > mlp->max_batch) return fail(NERVA_ERR_SHAPE, "batch %d exceeds max_batch %d", batch, mlp->max_batch);
    L = make_layout(mlp, batch);
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(NERVA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (workspace_bytes < static_cast<size_t>(L.bytes))
        return fail(NERVA_ERR_WORKSPACE, "workspace has %zu bytes, %lld needed", workspace_bytes, (long long)L.bytes);
    return NERVA_OK;
}

// Y = act(W X + b) of one layer of a step
static SpmmArgs forward_args(const nerva_layer *ly, const float *in, int64_t ldin, float *out, int64_t ldout, int32_t batch)
{
    SpmmArgs a{};
    a.blocks = ly->plan; a.nnz = ly->nnz; a.scratch = ly->scratch; a.scratch_ld = ly->scratch_ld;
    a.indptr = ly->indptr; a.indices = ly->indices; a.values = ly->values; a.bias = ly->bias;
    a.X = in; a.ldx = ldin; a.Y = out; a.ldy = ldout;
    a.rows = ly->rows; a.x_rows = ly->cols; a.batch = batch; a.relu = ly->activation == NERVA_ACT_RELU;
    a.full_scratch = ly->full ? ly->full_scratch : nullptr; a.full_scratch_ld = ly->full_scratch_ld;
    return a;
}

static int forward_chain(nerva_mlp *mlp, const float *X, int32_t ldx, int32_t batch, char *ws, const Layout &L,
                         hipStream_t s, size_t n_layers)
{
    const float *in = X;
    int64_t ldin = ldx;
    for (size_t l = 0; l < n_layers; ++l) {
        const nerva_layer *ly = mlp->layers[l];
        float *A = reinterpret_cast<float *>(ws + L.A[l]);
        const SpmmArgs a = forward_args(ly, in, ldin, A, L.ld, batch);
        if (use_dense(ly, batch)) {
            Timed tm(mlp->prof, s, "dense_forward", static_cast<int>(l));
            HIP_TRY(dense_forward(ly, in, ldin, A, L.ld, batch, s));
        } else {
            Timed tm(mlp->prof, s, "spmm_forward", static_cast<int>(l));
            HIP_TRY(launch_spmm(a, s));
        }
        in = A;
        ldin = L.ld;
    }
    return NERVA_OK;
}

int mlp_forward(nerva_mlp *mlp, const float *X, int32_t ldx, int32_t batch, void *workspace, size_t workspace_bytes,
                void *stream)
{
    Layout L;
    int rc = check_step_args(mlp, X, ldx, batch, workspace, workspace_bytes, L);
    if (rc != NERVA_OK) return rc;
    return forward_chain(mlp, X, ldx, batch, static_cast<char *>(workspace), L, as_stream(stream), mlp->layers.size());
}

static int train_step(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels, int32_t batch, float lr,
                      float momentum, void *workspace, const Layout &L, float *loss_out, void *stream);

int mlp_train_step(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels, int32_t batch, float lr,
                   float momentum, void *workspace, size_t workspace_bytes, float *loss_out, void *stream)
{
    Layout L;
    int rc = check_step_args(mlp, X, ldx, batch, workspace, workspace_bytes, L);
    if (rc != NERVA_OK) return rc;
    if (!labels) return fail(NERVA_ERR_ARGUMENT, "labels is null");
    return train_step(mlp, X, ldx, labels, batch, lr, momentum, workspace, L, loss_out, stream);
}

int mlp_train_step_static(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels, int32_t batch, float lr,
                          float momentum, float *loss_out, void *stream)
{
    if (!mlp || !X || !labels) return fail(NERVA_ERR_ARGUMENT, "null argument");
    if (mlp->prof.on) return fail(NERVA_ERR_ARGUMENT, "per-launch timing creates events: not available in mlp_train_step_static");
    int rc = check_batch(batch, ldx, "ldx");
    if (rc != NERVA_OK) return rc;
    if (batch > mlp->max_batch) return fail(NERVA_ERR_SHAPE, "batch %d exceeds max_batch %d", batch, mlp->max_batch);
    const Layout L = make_layout(mlp, batch);
    if (static_cast<size_t>(L.bytes) > kStaticScratchBytes)
        return fail(NERVA_ERR_WORKSPACE, "this MLP at batch %d needs a workspace of %lld bytes, the static one has %zu: use mlp_train_step with a workspace of your own",
                    batch, (long long)L.bytes, kStaticScratchBytes);
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);  // a table look-up once mlp_create has run on this device
    if (e != hipSuccess) return hip_fail(e, "address of the static workspace");
    // nothing in the workspace has to start at zero: every stage writes what the next one reads
    return train_step(mlp, X, ldx, labels, batch, lr, momentum, ws, L, loss_out, stream);
}

static int train_step(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels, int32_t batch, float lr,
                      float momentum, void *workspace, const Layout &L, float *loss_out, void *stream)
{
    int rc = NERVA_OK;
    hipStream_t s = as_stream(stream);
    char *ws = static_cast<char *>(workspace);
    const int n = static_cast<int>(mlp->layers.size());
    const bool fused = !(mlp->flags & NERVA_MLP_UNFUSED);
    const int nesterov = (mlp->flags & NERVA_MLP_NESTEROV) ? 1 : 0;
    auto A = [&](int l) { return reinterpret_cast<float *>(ws + L.A[l]); };
    auto dZ = [&](int l) { return reinterpret_cast<float *>(ws + L.dZ[l]); };

    // a layer that was last trained as the first layer of another MLP: its mirror's values are behind
    for (int l = 1; l < n; ++l) {
        nerva_layer *ly = mlp->layers[l];
        if (!ly->mirror_stale) continue;
        HIP_TRY(launch_gather(ly->values_t, ly->values, ly->perm, ly->nnz, s));
        ly->mirror_stale = false;
    }
    if (mlp->layers[0]->nnz > 0) mlp->layers[0]->mirror_stale = true;  // neither pipeline below writes layer 0's mirror

    // feedforward, then the loss gradient / batch size
    const nerva_layer *last = mlp->layers[n - 1];
    const bool head = mlp->head && head_ok(last->rows, last->cols, last->nnz);  // (a rebind may have grown the layer)
    bool ce_fused = false;  // softmax cross-entropy in the finish pass of the output layer's forward product
    int bias_done = -1;     // a layer whose biases the launch that formed its dZ has already updated
    // backpropagate and optimize, last layer first.  Layer l's transposed product T_l runs before
    // anything updates layer l's weights, so every gradient sees the weights of the step's start.
    auto make_T = [&](int l) {
        // dZ_{l-1} = (W_l^T dZ_l) * [A_{l-1} > 0]: the ReLU derivative of the layer below is
        // applied as the transposed product is stored
        nerva_layer *ly = mlp->layers[l];
        SpmmArgs t{};
        t.blocks = ly->plan_t; t.nnz = ly->nnz; t.scratch = ly->scratch; t.scratch_ld = ly->scratch_ld;
        t.indptr = ly->indptr_t; t.indices = ly->indices_t; t.values = ly->values_t;
        t.X = dZ(l); t.ldx = L.ld; t.Y = dZ(l - 1); t.ldy = L.ld;
        t.YM = A(l - 1); t.ldym = L.ld;
        t.rows = ly->cols; t.x_rows = ly->rows; t.batch = batch;
        return t;
    };
    auto make_S = [&](int l) {
        nerva_layer *ly = mlp->layers[l];
        SddmmArgs g{};
        g.blocks = ly->plan;
        g.indptr = ly->indptr; g.indices = ly->indices;
        g.dZ = dZ(l); g.lddz = L.ld;
        g.X = l > 0 ? A(l - 1) : X; g.ldx = l > 0 ? L.ld : ldx;
        g.rows = ly->rows; g.x_rows = ly->cols; g.batch = batch; g.nnz = ly->nnz;
        g.partial = ly->partial; g.partial_stride = ly->partial_stride;
        g.partial_db_at = ly->partial_db_at; g.partial_tiles = ly->partial_tiles;
        if ((head || ce_fused) && l == n - 1 && loss_out) { g.loss_cols = mlp->head_scratch; g.loss_out = loss_out; g.loss_n = batch; }
        if (fused) {
            g.fused = 1; g.nesterov = nesterov; g.lr = lr; g.momentum = momentum;
            g.values = ly->values; g.velocity = mlp->vel[l];
            if (l > 0) { g.values_t = ly->values_t; g.pos_t = ly->pos_t; g.perm = ly->perm; }  // the first layer's mirror is never read
            if (ly->dense_on) { g.dense = ly->dense; g.dense_ld = ly->dense_ld; }
            if (l != bias_done) { g.bias = ly->bias; g.bias_velocity = mlp->bias_vel[l]; }
        } else {
            g.g = reinterpret_cast<float *>(ws + L.g[l]);
            g.db = reinterpret_cast<float *>(ws + L.db[l]);
        }
        return g;
    };

    // A saturated output layer too large for the head: its forward product streams the operand, and the finish pass of
    // that product can form the loss gradient as it stores the logits, when the layer's backward pass (one streaming
    // launch as well) is there to take the mean of the per-column losses.
    SpmmArgs last_F{};
    if (!head && fused && n >= 2 && mlp->head_scratch && !use_dense(last, batch)) {
        last_F = forward_args(last, A(n - 2), L.ld, A(n - 1), L.ld, batch);
        last_F.ce_labels = labels; last_F.ce_dZ = dZ(n - 1); last_F.ce_lddz = L.ld; last_F.ce_loss_cols = mlp->head_scratch;
        ce_fused = true;  // (make_S then asks for the mean of the losses)
        ce_fused = spmm_softmax_epilogue_ok(last_F) && full_backward_ok(make_T(n - 1), make_S(n - 1));
    }
    rc = forward_chain(mlp, X, ldx, batch, ws, L, s, head || ce_fused ? n - 1 : n);
    if (rc != NERVA_OK) return rc;
    if (ce_fused) {
        Timed tm(mlp->prof, s, "spmm_forward+softmax_ce", n - 1);
        HIP_TRY(launch_spmm(last_F, s));
    } else if (head) {
        // output layer, loss and the gradient handed to layer n-2 in one launch
        HeadArgs h{};
        h.indptr = last->indptr; h.indices = last->indices; h.values = last->values; h.bias = last->bias;
        h.indptr_t = last->indptr_t; h.indices_t = last->indices_t; h.values_t = last->values_t;
        h.rows = last->rows; h.cols = last->cols; h.batch = batch;
        h.X = A(n - 2); h.ldx = L.ld; h.Z = A(n - 1); h.ldz = L.ld; h.labels = labels;
        h.dZ = dZ(n - 1); h.lddz = L.ld; h.dX = dZ(n - 2); h.lddx = L.ld;
        h.loss_cols = mlp->head_scratch;  // their mean is taken by the launch that runs S_{n-1}
        Timed tm(mlp->prof, s, "spmm_forward+softmax_ce+spmm_transposed", n - 1);
        HIP_TRY(launch_head(h, s));
    } else {
        Timed tm(mlp->prof, s, "softmax_ce", n - 1);
        HIP_TRY(launch_softmax_ce(A(n - 1), L.ld, labels, last->rows, batch, dZ(n - 1), L.ld, loss_out, s));
    }

    if (fused) {
        // Launch order T_{n-1} | T_{n-2} + S_{n-1} | ... | T_1 + S_2 | S_1 + S_0: the fused
        // SDDMM+update S_l of a layer shares a grid with the transposed product of the layer
        // below, which no longer depends on it (S_l only needs dZ_l and must follow T_l).
        // dZ_{l-1} through the dense copy of layer l's weights
        auto dense_T = [&](int l) {
            return dense_transposed(mlp->layers[l], dZ(l), L.ld, dZ(l - 1), L.ld, A(l - 1), L.ld, batch, s);
        };
        // `pending`: a layer whose transposed product has run and whose S has not.  Where a layer's T and S
        // can share their gathers (backward_fused_ok) they run as one launch and nothing stays pending.
        int pending = -1;
        // S_l through the dense gradient: for a layer on the dense route whose operands allow 16-byte accesses
        auto dense_S_ok = [&](int l) {
            const nerva_layer *ly = mlp->layers[l];
            const float *in = l > 0 ? A(l - 1) : X;
            const int64_t ldin = l > 0 ? L.ld : ldx;
            return use_dense(ly, batch) && ly->nnz > 0 && ldin % 4 == 0 && (reinterpret_cast<uintptr_t>(in) & 15u) == 0 &&
                   !(head && l == n - 1 && loss_out);
        };
        auto run_S_alone = [&](int l) -> int {
            if (dense_S_ok(l)) {
                nerva_layer *ly = mlp->layers[l];
                DenseUpdateArgs u{};
                u.indptr = ly->indptr; u.indices = ly->indices; u.dZ = dZ(l); u.lddz = L.ld;
                u.G = ly->dense_g; u.ldg = ly->dense_ld; u.D = ly->dense; u.ldw = ly->dense_ld;
                u.values = ly->values; u.velocity = mlp->vel[l];
                if (l > 0) { u.values_t = ly->values_t; u.pos_t = ly->pos_t; }
                if (l != bias_done) { u.bias = ly->bias; u.bias_velocity = mlp->bias_vel[l]; }
                u.rows = ly->rows; u.cols = ly->cols; u.batch = batch; u.nesterov = nesterov; u.lr = lr; u.momentum = momentum;
                Timed tm(mlp->prof, s, "dense_sddmm_update", l);
                HIP_TRY(launch_dense_sddmm_update(u, l > 0 ? A(l - 1) : X, l > 0 ? L.ld : ldx, s));
                return NERVA_OK;
            }
            Timed tm(mlp->prof, s, "sddmm_update", l);
            HIP_TRY(launch_sddmm(make_S(l), s));
            return NERVA_OK;
        };
        if (head) pending = n - 1;  // the head launch has run T_{n-1}
        for (int l = head ? n - 2 : n - 1; l >= 1; --l) {
            // dZ_l is ready: T_l (which hands dZ_{l-1} down) and S_l
            const SpmmArgs t = make_T(l);
            if (use_dense(mlp->layers[l], batch)) {
                if (pending >= 0 && (rc = run_S_alone(pending)) != NERVA_OK) return rc;
                { Timed tm(mlp->prof, s, "dense_transposed", l); HIP_TRY(dense_T(l)); }
                pending = l;
                continue;
            }
            const SddmmArgs g_same = make_S(l);
            if (full_backward_ok(t, g_same)) {
                if (pending >= 0 && (rc = run_S_alone(pending)) != NERVA_OK) return rc;
                pending = -1;
                SddmmArgs g_full = g_same;
                if (bias_done < 0 && mlp->layers[l - 1]->bias) {
                    // dZ_{l-1} is formed a whole row per wave: the bias gradient of layer l-1 is that row's sum
                    g_full.below_bias = mlp->layers[l - 1]->bias; g_full.below_bias_velocity = mlp->bias_vel[l - 1];
                    bias_done = l - 1;
                }
                Timed tm(mlp->prof, s, "backward_full", l);
                HIP_TRY(launch_full_backward(t, g_full, s));
                continue;
            }
            if (backward_fused_ok(t, g_same)) {
                if (pending >= 0 && (rc = run_S_alone(pending)) != NERVA_OK) return rc;
                pending = -1;
                Timed tm(mlp->prof, s, "backward_fused", l);
                HIP_TRY(launch_backward_fused(t, g_same, s));
                continue;
            }
            if (pending >= 0) {
                const SddmmArgs g = make_S(pending);
                if (!dense_S_ok(pending) && can_pair(t, g)) {
                    Timed tm(mlp->prof, s, "spmm_transposed+sddmm_update", l);
                    HIP_TRY(launch_pair(t, g, s));
                } else {
                    { Timed tm(mlp->prof, s, "spmm_transposed", l); HIP_TRY(launch_spmm(t, s)); }
                    if ((rc = run_S_alone(pending)) != NERVA_OK) return rc;
                }
            } else {
                Timed tm(mlp->prof, s, "spmm_transposed", l);
                HIP_TRY(launch_spmm(t, s));
            }
            pending = l;
        }
        // the first layer has no transposed product: its S, with the one still pending if any
        if (pending >= 0) {
            const SddmmArgs gp = make_S(pending), g0 = make_S(0);
            if (pending == 1 && !dense_S_ok(0) && !dense_S_ok(1) && can_pair(g0, gp)) {
                Timed tm(mlp->prof, s, "sddmm_update+sddmm_update", 0);
                HIP_TRY(launch_pair(g0, gp, s));  // the larger layer's work-groups start first
            } else {
                if ((rc = run_S_alone(pending)) != NERVA_OK) return rc;
                if (pending != 0 && (rc = run_S_alone(0)) != NERVA_OK) return rc;
            }
        } else if ((rc = run_S_alone(0)) != NERVA_OK) {
            return rc;
        }
    } else {
        for (int l = n - 1; l >= 0; --l) {
            nerva_layer *ly = mlp->layers[l];
            if (l > 0 && !(head && l == n - 1)) {
                if (use_dense(ly, batch)) {
                    Timed tm(mlp->prof, s, "dense_transposed", l);
                    HIP_TRY(dense_transposed(ly, dZ(l), L.ld, dZ(l - 1), L.ld, A(l - 1), L.ld, batch, s));
                } else {
                    Timed tm(mlp->prof, s, "spmm_transposed", l);
                    HIP_TRY(launch_spmm(make_T(l), s));
                }
            }
            const SddmmArgs g = make_S(l);
            {
                Timed tm(mlp->prof, s, "sddmm", l);
                HIP_TRY(launch_sddmm(g, s));
            }
            {
                Timed tm(mlp->prof, s, "momentum_values", l);
                HIP_TRY(launch_momentum(ly->values, mlp->vel[l], g.g, ly->nnz, lr, momentum, nesterov, s));
            }
            if (ly->bias) {
                Timed tm(mlp->prof, s, "momentum_bias", l);
                HIP_TRY(launch_momentum(ly->bias, mlp->bias_vel[l], g.db, ly->rows, lr, momentum, nesterov, s));
            }
            if (l > 0) {
                Timed tm(mlp->prof, s, "mirror_refresh", l);
                HIP_TRY(launch_gather(ly->values_t, ly->values, ly->perm, ly->nnz, s));
            }
            if (ly->dense_on) {
                Timed tm(mlp->prof, s, "dense_refresh", l);
                HIP_TRY(refresh_dense_copies(ly, s));
            }
        }
    }
    if (mlp->prof.on && mlp->prof.step < mlp->prof.max_steps) {
        hipEvent_t e = nullptr;  // closes the last launch of the step
        HIP_TRY(hipEventCreate(&e));
        mlp->prof.events.push_back(e);
        HIP_TRY(hipEventRecord(e, s));
        ++mlp->prof.step;
    }
    return NERVA_OK;
}

int nerva_copy_f32(float *dst, const float *src, int64_t n, void *stream)
{
    if (n < 0 || (n > 0 && (!dst || !src))) return fail(NERVA_ERR_ARGUMENT, "bad argument");
    HIP_TRY(launch_copy(dst, src, n, as_stream(stream)));
    return NERVA_OK;
}

}  // extern "C"
