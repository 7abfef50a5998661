// Internal launch interface between the C ABI (api.hip) and the gfx950 kernels (kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nerva {

constexpr int kWavesPerBlock = 16;   // 1024 threads

// Static partition of the rows of a CSR matrix over work-groups, built once per pattern.
// A work-group has kWavesPerBlock waves.  Ordinary rows: the work-group serves
// (kWavesPerBlock >> lg) rows, 2^lg waves per row, each wave taking a contiguous share of the
// row's stored entries.  Huge rows (more entries than a whole work-group should take) are cut
// into several work-groups; each produces a partial result that a second, small kernel adds
// up in share order.  Huge work-groups come first, so blockIdx.x is also their scratch slot.
struct RowBlocks {
    const int32_t *row_order;  // [rows - n_huge_rows] ordinary row ids, grouped by lg (descending)
    const int4 *blocks;        // [n_blocks] ordinary: {lg | rows served << 8, first slot of row_order, 0, 0}
                               //            huge:     {kHugeFlag | share index, row, first entry, end entry}
    const int4 *huge_rows;     // [n_huge_rows] {row, first work-group, number of work-groups, 0}
    const int4 *waves;         // [n_blocks * kWavesPerBlock] the same partition spelled out per wave:
                               // {row or -1, first entry, end entry, part | lg << 4 | lead << 8 | huge << 9}
    int32_t n_blocks;
    int32_t n_huge_rows;
    int32_t n_huge_blocks;
    // Optional second partition, built for matrices with many short rows (n_short > 0): rows of
    // at most kPackMaxLen entries are listed longest first and served one row per lane group,
    // 64/GS rows per wave (spmm_packed_kernel); the remaining rows keep a partition of their
    // own, huge work-groups first exactly as in `waves` (same scratch slots, same huge_rows).
    const int4 *short_rows;    // [n_short rounded up to a multiple of 64] {row or -1, first entry, entries, 0}
    const int4 *long_waves;    // [n_long_blocks * kWavesPerBlock], records as in `waves`
    int32_t n_short;
    int32_t n_long_blocks;
    // Share of the stored entries whose gathered operand row is one of the kHotRows most
    // referenced ones: when it is large the gathers hit in cache without any column tiling.
    float hot_share;
    // Optional third form, for the staged product (spmm_staged_kernel; staged_rows != nullptr).
    // The rows are cut into staged_ranges ranges of at most kStageRangeRows rows and about equal
    // work; inside a range the rows are listed longest first (slot 0, 1, ...; unused slots hold
    // -1).  A row much longer than its range's mean takes four slots, a multiple of 4 onwards, marked
    // kStageQuad: the four lane rows of one wave then serve a quarter of each of its segments each
    // and their results are added at the end.  Every row is cut into segments at the multiples of kStageRows in its column indices:
    // staged_ends[(range * (staged_cblocks + 1) + b) * kStageRangeRows + slot] is the position of
    // the slot's first stored entry with column >= b * kStageRows (b = 0: the row's first entry,
    // b = staged_cblocks: one past its last; unused slots: 0 throughout).
    const int32_t *staged_rows;    // [staged_ranges * kStageRangeRows]
    const int32_t *staged_ends;
    const int32_t *staged_groups;  // [staged_ranges] rows of the range / 64, rounded up
    int32_t staged_ranges;
    int32_t staged_cblocks;
    int32_t staged_longest_share;  // most stored entries any one lane row serves
    int32_t staged_longest_row;    // stored entries of the longest row
    int32_t staged_partial;        // the plan covers the rows of more than kPackMaxLen entries only: the others are
                                   // short_rows and take the packed kernel
    int32_t staged_row_count;      // rows the plan covers
    const int4 *rest_waves;        // where there are both short and longer rows: partition of the rows of at most kPackMaxLen
    int32_t n_rest_blocks;         //   entries alone, records as in `waves` (no huge rows among them)
    int32_t long_nnz;              // stored entries of the rows beyond kPackMaxLen (those of long_waves)
    int32_t staged_nnz;            // and their stored entries
    int32_t staged_preferred;      // measurement aid: take the staged kernels wherever they can run
};
constexpr int32_t kStageRows = 512;      // operand rows held in LDS at a time
constexpr int32_t kStageCols = 64;       // columns of the operand (examples) per work-group
constexpr int32_t kStageJ = 8;           // rows per row of 16 lanes
constexpr int32_t kStageQuad = 1 << 30;  // flag in staged_rows: the slot is one of the four of a split row
constexpr int32_t kStageRangeRows = 512; // rows per work-group: 16 waves x 4 lane rows x kStageJ
constexpr int32_t kStageMinBatch = 128;  // narrower batches never take the staged product
constexpr int32_t kStageTargetGroups = 256;  // work-groups wanted at max_batch (one per compute unit)
constexpr float kStageMinReuse = 2.f;    // stored entries per staged operand row and work-group, at least
constexpr int32_t kStageLongSegment = 10;       // mean entries per segment from which staging pays whatever the operand's size: products
constexpr int32_t kStageLongSegmentSddmm = 20;  // ... and the SDDMM (measured on 8192 x 8192 uniform at batch 1024, 1 / 2 / 3 / 5 % density:
                                                // products 142 / 301 / 407 / - us against 235 / 278 / 349 / 442 staged, SDDMM 162 / 289 / 407 / - against 317 / 369 / 460 / 584)
constexpr int64_t kStageBigOperand = 48ll << 20;  // operand bytes no set of L2s holds: staging pays for shorter segments,
constexpr int32_t kStageSegmentBigOperand = 7;    // ... from this many entries per segment on
constexpr int32_t kHotRows = 1024;
constexpr int32_t kHugeFlag = 0x40000000;
constexpr int32_t kPackMaxLen = 128;     // longest row served by the packed path
constexpr int32_t kPackMinRows = 2048;   // fewer short rows than this: no packed path
constexpr int32_t kPackSets = 1;         // row sets (64/GS rows each) per wave; measured on the wide MLP: 1 / 2 / 4 / 8 sets give 500 / 504 / 527 / 548 us per step

// Y = epilogue( W * gather(X) ) for a CSR matrix W (rows x cols); also used on the CSC
// mirror, where "rows" are W's columns.
struct SpmmArgs {
    RowBlocks blocks;
    const int32_t *indptr;   // [rows+1]
    const int32_t *indices;  // [nnz]
    const float *values;     // [nnz]
    const float *bias;       // [rows] or nullptr
    const float *X;          // gathered operand, (cols, ldx)
    int64_t ldx;
    const float *XM;         // optional (cols, ldxm): operand row j is X[j,c] * [XM[j,c] > 0]
    int64_t ldxm;
    float *Y;                // (rows, ldy)
    int64_t ldy;
    const float *YM;         // optional (rows, ldym): result is multiplied by [YM[i,c] > 0]
    int64_t ldym;
    int32_t rows;
    int32_t x_rows;          // rows of the gathered operand (columns of the sparse matrix)
    int32_t batch;
    int32_t relu;            // clamp the result at zero
    int32_t nnz;             // length of indices/values
    float *scratch;          // partial rows of huge-row work-groups, (n_huge_blocks, scratch_ld)
    int64_t scratch_ld;
    // Only for a matrix that stores every entry and has at most kFullMaxRows rows (a saturated
    // output layer): values[] is then the row-major dense matrix, and the product streams the
    // operand once for all rows instead of gathering it once per row.  Partial results of the
    // kFullSlice-column slices of W: full_scratch[(slice * rows + row) * full_scratch_ld + column].
    float *full_scratch;     // or nullptr: the matrix is not full, or has too many rows
    int64_t full_scratch_ld;
    // Optional epilogue for an output layer served that way (spmm_softmax_epilogue_ok): the softmax
    // cross-entropy of the logits Y against ce_labels -- ce_dZ = (softmax(Y) - onehot) / batch, one
    // loss per column into ce_loss_cols (their mean is taken by a later launch, SddmmArgs::loss_cols).
    const int32_t *ce_labels;  // [batch] or nullptr: no epilogue
    float *ce_dZ;              // (rows, ce_lddz)
    int64_t ce_lddz;
    float *ce_loss_cols;       // [batch]
};
bool spmm_softmax_epilogue_ok(const SpmmArgs &a);
constexpr int32_t kFullMaxRows = 16;
constexpr int32_t kFullSlice = 128;   // columns of W (rows of the operand) per work-group
hipError_t launch_spmm(const SpmmArgs &a, hipStream_t s);

// g[p] = <dZ[row(p),:], X[indices[p],:]>, db[i] = sum_c dZ[i,c]; optionally followed, inside
// the same kernel, by the momentum step on values/velocity (and bias/bias_velocity).
struct SddmmArgs {
    RowBlocks blocks;
    const int32_t *indptr;
    const int32_t *indices;
    const float *dZ;         // (rows, lddz)
    int64_t lddz;
    const float *ZM;         // optional (rows, ldzm): dZ is multiplied by [ZM > 0]
    int64_t ldzm;
    const float *X;          // (cols, ldx)
    int64_t ldx;
    float *g;                // [nnz] or nullptr
    float *db;               // [rows] or nullptr
    int32_t rows;
    int32_t x_rows;          // rows of X (columns of the sparse matrix)
    int32_t batch;
    int32_t skip_products;   // only db is wanted: do not touch indptr/indices/X
    // fused momentum step (fused != 0): g/db are not stored unless non-null
    int32_t fused;
    int32_t nesterov;
    float lr, momentum;
    float *values;           // [nnz]
    float *velocity;         // [nnz]
    float *values_t;         // mirror values or nullptr
    const int32_t *pos_t;    // CSR position -> mirror position (needed iff values_t)
    const int32_t *perm;     // mirror position -> CSR position (only the fused backward pass needs it)
    float *bias;             // [rows] or nullptr
    float *bias_velocity;    // [rows] or nullptr
    // by-product, unrelated to the layer: *loss_out = mean(loss_cols[0..loss_n)), summed in one fixed
    // order by the first wave of the launch.  The head kernel leaves one loss per batch column; a
    // grid-wide sum inside it would need device-scope fences, which write back and invalidate the L2s.
    // launch_full_backward only: the biases of the layer BELOW and their momentum buffer, or nullptr.  That layer's
    // bias gradient is the row sum of the dX this launch forms, a wave per row, so its update can ride along
    // (the caller then leaves the biases out of that layer's own update).
    float *below_bias;
    float *below_bias_velocity;
    const float *loss_cols;  // or nullptr
    float *loss_out;
    int32_t loss_n;
    // column-tiled route for operands X that no L2 holds: per-tile partial products
    // [tile][partial_stride] (values first, then the per-row sums of dZ at partial_db_at), added in
    // tile order by a second kernel that also applies the update.  nullptr: route not available.
    float *partial;
    int64_t partial_stride;   // floats per tile, >= partial_db_at + rows
    int64_t partial_db_at;    // >= nnz
    int32_t partial_tiles;    // tiles the buffer has room for
    int32_t nnz;
    // dense copy of a layer on the dense route (or nullptr): the fused update stores every new
    // weight there too, dense[row * dense_ld + col]
    float *dense;
    int64_t dense_ld;
};
// Column-tile width (in columns) the products use when their gathered operand has x_rows rows and
// does not fit an L2; 0: no tiling.  Shared by the kernels' dispatch and by the sizing of the
// SDDMM partial buffer when a layer is created.
int tile_columns(int32_t x_rows, int32_t batch, int64_t nnz, int32_t rows, float hot_share, bool masked, bool for_sddmm = false);
hipError_t launch_sddmm(const SddmmArgs &a, hipStream_t s);

// Transposed product and SDDMM of one layer on one gather stream (backward_fused_kernel).
struct BackwardArgs {
    RowBlocks blocks;            // the mirror's partition (its table of short rows)
    const int32_t *indices;      // mirror: row of W of each entry
    const float *values;         // mirror values
    const float *dZ;             // (rows of W, lddz): gathered
    int64_t lddz;
    const float *X;              // (cols of W, ldx): the layer's input; second operand of the products and mask of dX
    int64_t ldx;
    float *dX;                   // (cols of W, lddx)
    int64_t lddx;
    int32_t mask;                // multiply dX by [X > 0]
    int32_t rows, x_rows, batch, nnz;   // rows = mirror rows = columns of W; x_rows = rows of W
    float *partial;              // [tile][partial_stride]: products in mirror order
    int64_t partial_stride;
    const int32_t *perm;         // mirror position -> CSR position
    // what the second pass does with the sums: store them (g, db: CSR order) and / or the momentum step
    float *g, *db;
    int32_t fused, nesterov;
    float lr, momentum;
    float *w, *velocity, *w_t;   // values[], velocity[] (CSR order), mirror values
    float *bias, *bias_velocity;
};
bool backward_fused_ok(const SpmmArgs &t, const SddmmArgs &g);
hipError_t launch_backward_fused(const SpmmArgs &t, const SddmmArgs &g, hipStream_t s);
bool full_backward_ok(const SpmmArgs &t, const SddmmArgs &g);
hipError_t launch_full_backward(const SpmmArgs &t, const SddmmArgs &g, hipStream_t s);

// Two independent launches in one grid (both on the 16-byte path, batch <= 1024, one column tile).
bool can_pair(const SpmmArgs &a, const SddmmArgs &b);
bool can_pair(const SddmmArgs &a, const SddmmArgs &b);
hipError_t launch_pair(const SpmmArgs &a, const SddmmArgs &b, hipStream_t s);
hipError_t launch_pair(const SddmmArgs &a, const SddmmArgs &b, hipStream_t s);

hipError_t launch_momentum(float *w, float *v, const float *g, int64_t n, float lr, float mu, int nesterov,
                           hipStream_t s);
// values_t[q] = values[perm[q]]
hipError_t launch_gather(float *values_t, const float *values, const int32_t *perm, int64_t n,
                         hipStream_t s);
hipError_t launch_softmax_ce(const float *Z, int64_t ldz, const int32_t *labels, int32_t classes,
                             int32_t batch, float *dZ, int64_t lddz, float *loss, hipStream_t s);
hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t s);

// Dense route of a layer whose density is high (the density-adaptive layer the paper plans in
// "Discussion and Conclusion" and Appendix C.3).  One zero-filled dense copy of the weights, row-major
// W[i * ldw + j] with ldw = cols rounded up to kDenseLdAlign (zero off the pattern and in the padding), serves
// the forward product, the transposed product (the same copy read down its columns) and, through a dense
// gradient G = dZ X^T of the same shape, the update of the stored entries.
constexpr int32_t kDenseLdAlign = 64;
constexpr float kDenseFromDensity = 0.4f;   // layers at least this dense take the dense route by themselves (measured cut-over)
struct DenseArgs {
    const float *W;      // the dense copy, (rows, ldw)
    int64_t ldw;
    int32_t trans;       // 0: Y (rows x batch) = act(W X + b);  1: Y (cols x batch) = (W^T X) * [YM > 0]
    const float *X;      // (cols, ldx) or, transposed, (rows, ldx)
    int64_t ldx;
    float *Y;
    int64_t ldy;
    const float *bias;   // [rows] or nullptr (forward only)
    const float *YM;     // optional: result is multiplied by [YM > 0]
    int64_t ldym;
    int32_t rows, cols, batch;
    int32_t relu;
};
hipError_t launch_dense_product(const DenseArgs &a, hipStream_t s);
// G = dZ X^T (rows x cols, dense), then per stored entry the momentum step with its element of G, the new weight
// written to values[], the mirror and the dense copy; bias gradient = row sums of dZ.  Needs 16-byte aligned
// operands with leading dimensions that are multiples of 4.
struct DenseUpdateArgs {
    const int32_t *indptr, *indices;
    const float *dZ;     // (rows, lddz)
    int64_t lddz;
    float *G;            // (rows, ldg) scratch
    int64_t ldg;
    float *D;            // the dense copy
    int64_t ldw;
    float *values, *velocity, *values_t;   // values_t may be nullptr
    const int32_t *pos_t;
    float *bias, *bias_velocity;           // may be nullptr
    int32_t rows, cols, batch, nesterov;
    float lr, momentum;
};
hipError_t launch_dense_sddmm_update(const DenseUpdateArgs &a, const float *X, int64_t ldx, hipStream_t s);
// D[i * ld + j] = values[p] for every stored entry p = (i, j); the rest of D is not touched (zero since allocation)
hipError_t launch_dense_refresh(const int32_t *indptr, const int32_t *indices, const float *values, int32_t rows, float *D, int64_t ld,
                                hipStream_t s);

// ---- binding a pattern: the work that grows with the number of stored entries, on the device ----
// Check that device arrays hold a canonical CSR pattern.  status (device, 4 ints) receives
// {OR of the kCsr* flags found, first row with wrong row pointers, first entry with a wrong column
// index, 0}; rows whose pointers are wrong are not walked, so nothing outside the arrays is read.
enum : int32_t { kCsrBadFirst = 1, kCsrDecreasing = 2, kCsrBeyondNnz = 4, kCsrBadLast = 8, kCsrColumnRange = 16, kCsrNotAscending = 32 };
hipError_t launch_validate_csr(int32_t rows, int32_t cols, int32_t nnz, const int32_t *indptr, const int32_t *indices,
                               int32_t *status, hipStream_t s);
// CSC mirror of a canonical CSR pattern (stable counting sort by column): indptr_t[cols + 1],
// indices_t[nnz] (row of each mirror entry), perm[nnz] (mirror position -> CSR position), pos_t[nnz]
// (the inverse).  work: mirror_work_ints(cols, T) ints of scratch, T = mirror_tiles(rows, cols, nnz).
int32_t mirror_tiles(int32_t rows, int32_t cols, int32_t nnz);
size_t mirror_work_ints(int32_t cols, int32_t T);
hipError_t launch_build_mirror(int32_t rows, int32_t cols, int32_t nnz, const int32_t *indptr, const int32_t *indices,
                               int32_t *indptr_t, int32_t *indices_t, int32_t *perm, int32_t *pos_t, int32_t *work, int32_t T,
                               hipStream_t s);
// RowBlocks::staged_ends from RowBlocks::staged_rows and the pattern
hipError_t launch_staged_ends(const int32_t *indptr, const int32_t *indices, const int32_t *slot_rows, int32_t *ends, int32_t ranges,
                              int32_t n_cb, hipStream_t s);

// The end of the forward pass and the start of the backward pass for a small output layer, in
// one launch: logits Z = W X + b, softmax cross-entropy (loss and dZ = (softmax - onehot) / batch),
// and the gradient handed to the layer below, dX = (W^T dZ) * [X > 0] (X is that layer's ReLU
// output).  Every step is local to a column of the batch, so a work-group owns 4 columns.
constexpr int kHeadMaxRows = 32;
struct HeadArgs {
    const int32_t *indptr, *indices;      // W in CSR (rows x cols)
    const float *values, *bias;           // bias may be null
    const int32_t *indptr_t, *indices_t;  // its mirror: CSR of W^T
    const float *values_t;
    int32_t rows, cols, batch;
    const float *X;                       // (cols, ldx)
    int64_t ldx;
    float *Z;                             // (rows, ldz)
    int64_t ldz;
    const int32_t *labels;                // [batch]
    float *dZ;                            // (rows, lddz)
    int64_t lddz;
    float *dX;                            // (cols, lddx)
    int64_t lddx;
    float *loss_cols;                     // [batch]: per-column losses; a later launch takes their mean (SddmmArgs)
};
bool head_ok(int32_t rows, int32_t cols, int32_t nnz);
hipError_t launch_head(const HeadArgs &a, hipStream_t s);

}  // namespace nerva
