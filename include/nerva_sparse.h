/* nerva_sparse.h -- C ABI of the truly sparse MLP training step on MI355X (gfx950).
 *
 * The library implements the four sparse operations that Section 4 of the paper
 * ("Nerva: a Truly Sparse Implementation of Neural Networks") names as essential,
 *
 *     A = S B        feedforward              (sparse_linear_forward)
 *     A = S^T B      backpropagation          (sparse_linear_backward, dX)
 *     S = A B^T      on the pattern of S      (sparse_linear_backward, dvalues)
 *     S = aS + bT    momentum, same pattern   (sgd_update_values)
 *
 * and one iteration of the training loop of the Appendix B listing
 * (feedforward -> loss gradient / batch size -> backpropagate -> optimize) as
 * mlp_train_step, for an MLP with ReLU hidden layers and a softmax cross-entropy
 * loss (Section 5.1).
 *
 * Conventions shared by every call
 * --------------------------------
 * - S (the weight matrix W of a layer) is CSR, rows = n_out, cols = n_in, zero-based
 *   int32 row pointers `indptr[rows+1]` and column indices `indices[nnz]`, fp32
 *   `values[nnz]`.  Column indices are strictly ascending inside a row.  Empty rows are
 *   legal.  The pattern is static: no call ever writes indptr or indices.
 * - Dense matrices hold one example per column (Appendix B listing: Xtrain[:, batch]).
 *   They are fp32, row-major (features, ld): element (i, c) is at base[i*ld + c], with
 *   ld >= batch.  Columns batch..ld-1 are padding: never written, and their contents
 *   never influence a result.  Calls are fastest when every ld is a multiple of 4 and
 *   every base pointer is 16-byte aligned; other values take a slower kernel.
 * - Biases are dense fp32 vectors of length rows (Section 3: biases are not sparsified).
 * - Every pointer is a DEVICE pointer owned by the caller unless the comment says
 *   "host".  The library owns only what *_create builds and frees it in *_destroy.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Except for
 *   the *_create calls, every call only enqueues kernels on that stream: it allocates
 *   nothing, never synchronises, and may be captured in a HIP graph.  Calls on one
 *   handle from several streams at once are not ordered by the library.
 * - Return value: 0 on success, a negative nerva_status otherwise; nothing has been
 *   enqueued when an argument error is returned.  nerva_last_error() gives a
 *   thread-local message for the last failing call.
 */
#ifndef NERVA_SPARSE_H
#define NERVA_SPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nerva_status {
    NERVA_OK = 0,
    NERVA_ERR_ARGUMENT = -1,   /* null pointer, negative size, unknown flag          */
    NERVA_ERR_SHAPE = -2,      /* leading dimension < batch, layer sizes do not chain */
    NERVA_ERR_CSR = -3,        /* pattern is not canonical CSR                        */
    NERVA_ERR_WORKSPACE = -4,  /* workspace too small or misaligned                   */
    NERVA_ERR_HIP = -5         /* a HIP runtime call failed                           */
} nerva_status;

typedef struct nerva_layer nerva_layer; /* one sparse linear layer: pattern, mirror, tables */
typedef struct nerva_mlp nerva_mlp;     /* a chain of layers + optimiser state pointers     */

enum { NERVA_ACT_NONE = 0, NERVA_ACT_RELU = 1 };

/* Message of the last failing call on this thread ("" if none). Host pointer, valid
 * until the next failing call on the thread. */
const char *nerva_last_error(void);

/* Library version and the GPU architecture the kernels were compiled for ("gfx950"). */
const char *nerva_build_info(void);

/* Check that HOST arrays describe a canonical CSR pattern: indptr[0] = 0, non-decreasing,
 * indptr[rows] = nnz, every column index in [0, cols), strictly ascending per row.
 * Returns NERVA_OK or NERVA_ERR_CSR / NERVA_ERR_ARGUMENT.  Needs no GPU. */
int nerva_validate_csr_host(int32_t rows, int32_t cols, int64_t nnz,
                            const int32_t *indptr_host, const int32_t *indices_host);

/* The static work partition the kernels use, computed on HOST arrays (needs no GPU; exposed so
 * that it can be checked).  A work-group has NERVA_WAVES_PER_BLOCK waves.  Ordinary rows are
 * grouped by lg = log2(waves that share one row), the smallest lg that keeps a wave's share at or
 * below the target; a work-group serves NERVA_WAVES_PER_BLOCK >> lg of them, and a class whose
 * rows do not fill its last work-group hands that work-group's rows, its longest, to class lg + 1
 * where that class's own last work-group has room for them (one work-group fewer).  A row with more stored entries than one work-group should
 * take is "huge": it is cut into several work-groups whose partial results a second kernel adds
 * in order.  Outputs (any array may be NULL to get only the counts):
 *   counts_host[4]            {ordinary rows, work-groups, huge rows, huge work-groups}
 *   row_order_host[rows]      ordinary row ids in serving order: by lg descending, inside one lg by
 *                             stored entries descending, ties by row id
 *   blocks_host[4*nb]         per work-group, huge ones first:
 *                               ordinary {lg | rows served << 8, first position of row_order, 0, 0}
 *                               huge     {NERVA_HUGE_FLAG | share index, row, first entry, end entry}
 *   huge_rows_host[4*nh]      per huge row {row, first work-group, number of work-groups, 0}
 *   waves_host[4*16*nb]       the same partition per wave, 16 waves per work-group:
 *                               {row or -1 (idle), first entry, end entry,
 *                                share index in the work-group | lg << 4 | owner-of-row flag << 8 | huge << 9}
 *                             shares of one row are contiguous, in order, multiples of 4 entries
 * nb <= rows + nnz / 128 and nh <= rows bound the sizes. */
enum { NERVA_WAVES_PER_BLOCK = 16, NERVA_HUGE_FLAG = 0x40000000 };
int nerva_plan_rows_host(int32_t rows, const int32_t *indptr_host, int32_t *row_order_host,
                         int32_t *blocks_host, int32_t *huge_rows_host, int32_t *waves_host,
                         int32_t *counts_host);

/* The second partition, which the products Y = S X and Y = S^T X use on matrices with many short
 * rows (HOST arrays, needs no GPU).  Rows of at most NERVA_PACK_MAX_LEN stored entries are listed
 * longest first (ties in row order) and are served one row per group of lanes, several rows per
 * wave; the remaining rows get a partition of their own with the records of waves_host above.
 * With fewer than NERVA_PACK_MIN_ROWS short rows (or no stored entry) there is no second
 * partition and every count is 0.  Outputs (arrays may be NULL to get only the counts):
 *   counts_host[3]            {short rows, work-groups of the remaining rows, huge ones among them}
 *   short_rows_host[4*ns64]   ns64 = short rows rounded up to a multiple of 64:
 *                               {row, first entry, entries, 0}, padding {-1, 0, 0, 0}
 *   long_waves_host[4*16*nl]  per wave of the nl work-groups of the remaining rows */
enum { NERVA_PACK_MAX_LEN = 128, NERVA_PACK_MIN_ROWS = 2048 };
int nerva_plan_short_rows_host(int32_t rows, const int32_t *indptr_host, int32_t *short_rows_host,
                               int32_t *long_waves_host, int32_t *counts_host);

/* The static part of the staged product (HOST arrays, needs no GPU).  For batches of at least
 * NERVA_STAGE_MIN_BATCH columns and matrices with several stored entries per column and row
 * range, Y = S X (and Y = S^T X on the mirror) copies NERVA_STAGE_ROWS rows of X at a time into a
 * compute unit's local memory and serves from there every stored entry whose column falls into
 * that block of rows, while the results of the work-group's rows wait in registers.  The rows
 * are cut into ranges of consecutive rows, at most NERVA_STAGE_RANGE_ROWS each and of about equal
 * work, one work-group per (range, tile of NERVA_STAGE_COLS batch columns); inside a range the
 * rows are listed by stored entries descending (ties in row order), four consecutive list slots
 * being served side by side; every row is cut into segments at the multiples of
 * NERVA_STAGE_ROWS in its column indices.  A row with at least max(256, total work / ranges / 32)
 * stored entries takes four slots, from a multiple of 4 on, each marked NERVA_STAGE_QUAD: the four
 * serve a quarter of each of its segments each, so that no single row outlasts its range.
 * Rows with fewer than min_entries stored entries are left out of the plan (0: every row is in).
 * A layer whose rows differ widely in length (longest row > 4 x the mean) and which has the second
 * partition above is bound with min_entries = NERVA_PACK_MAX_LEN + 1: its long rows are staged, its
 * short rows take the packed path (the other kernels on a partition of their own where the
 * operand is not column-tiled; likewise the SDDMM) in a second launch.  With min_entries > 0 the
 * ranges are runs of consecutive covered rows.  The SDDMM S = A B^T uses the same plan of S.
 * Outputs (arrays may be NULL to get only the counts):
 *   counts_host[2]      {ranges, column blocks nb}; both 0 when no product of this matrix at up
 *                       to max_batch columns would be staged
 *   slot_rows_host[ranges * NERVA_STAGE_RANGE_ROWS]
 *                       row in each slot of each range (| NERVA_STAGE_QUAD in the four slots of a
 *                       split row), -1 in unused slots
 *   ends_host[ranges * (nb + 1) * NERVA_STAGE_RANGE_ROWS]
 *                       [(range * (nb + 1) + b) * NERVA_STAGE_RANGE_ROWS + slot] = position of the
 *                       slot's first stored entry with column >= b * NERVA_STAGE_ROWS (b = nb: one
 *                       past the row's last entry); 0 throughout for unused slots */
enum { NERVA_STAGE_ROWS = 512, NERVA_STAGE_COLS = 64, NERVA_STAGE_MIN_BATCH = 128, NERVA_STAGE_RANGE_ROWS = 512,
       NERVA_STAGE_QUAD = 1 << 30 };
int nerva_plan_staged_host(int32_t rows, int32_t cols, const int32_t *indptr_host, const int32_t *indices_host,
                           int32_t max_batch, int32_t min_entries, int32_t *slot_rows_host, int32_t *ends_host,
                           int32_t *counts_host);

/* ---- layer -------------------------------------------------------------------------
 * sparse_linear_create binds a layer to the caller's pattern, values and bias arrays
 * (which must outlive the layer) and builds, once, what a static pattern allows to be
 * precomputed: the CSC mirror of W (CSR of W^T: indptr_t[cols+1], indices_t[nnz] = row
 * indices ascending per column, values_t[nnz]) and the maps between CSR and mirror
 * positions.  The paper leaves A = S^T B to the vendor library (Section 4); the mirror
 * exists because the topology is static (Section 6).  The call checks the pattern on the
 * device (NERVA_ERR_CSR if not canonical; one status word comes back), builds the mirror there
 * (a stable counting sort by column: the same bits on every run), plans the row partitions on
 * the host from a copy of the row pointers (4 * (rows + cols) bytes), allocates device memory
 * and synchronises `stream`.  activation: NERVA_ACT_RELU for hidden layers, NERVA_ACT_NONE
 * for the output layer (Section 5.1). `bias` may be NULL (no bias).  max_batch bounds the
 * batch of later calls on this layer (a later call with a larger batch returns
 * NERVA_ERR_SHAPE) and is the batch the static tables are laid out for: the scratch rows of
 * huge-row work-groups, the row ranges of the staged products (nerva_plan_staged_host; a much
 * smaller batch falls back to the other kernels), and, where the SDDMM would run in column
 * tiles at that batch, a buffer of per-tile partial products: tiles x (nnz + rows) floats, at
 * most 4 GiB (beyond that the SDDMM stays untiled).  Device memory owned by the layer besides
 * that buffer: 16 bytes per stored entry (mirror and position maps) and the partition tables (a
 * 16-byte record per wave of each partition; with a staged plan 4 bytes per row and block of 512
 * columns, for the matrix and for its mirror) -- twice that once the layer has been rebound (see
 * sparse_linear_rebind) -- and the counters of the mirror build (4 bytes per column and row tile,
 * at most 128 MiB).  */
int sparse_linear_create(nerva_layer **out, int32_t rows, int32_t cols, int32_t nnz,
                         const int32_t *indptr, const int32_t *indices,
                         float *values, float *bias, int32_t activation, int32_t max_batch,
                         void *stream);
void sparse_linear_destroy(nerva_layer *layer);

/* Topology-update hook for dynamic sparse training (Section 2, "Sparse Training"; announced as
 * the next step in "Discussion and Conclusion"): the caller has written a new pattern for the
 * same rows x cols matrix -- entries pruned, others grown, nnz free to change -- as a canonical
 * CSR in device arrays indptr[rows+1], indices[nnz], values[nnz] (caller-owned; they replace the
 * arrays given at creation, which the layer no longer touches; bias, activation and max_batch
 * stay).  The call waits for the stream, checks the pattern as sparse_linear_create does, builds
 * the mirror, the position maps and the partitions in a second set of buffers that the layer keeps
 * for this purpose, then switches over: repeated updates of about the same size allocate nothing.
 * On any error (bad CSR: NERVA_ERR_CSR, allocation: NERVA_ERR_HIP) the layer keeps its old pattern
 * and stays usable.  Momentum buffers are the caller's: after a rebind of a layer
 * that belongs to an MLP, hand the MLP a velocity array of the new length, mapped to the new
 * entries as the method prescribes (zero for grown ones), with mlp_rebind_velocity, and ask
 * mlp_workspace_bytes / mlp_workspace_layout again: the workspace holds one float per stored
 * entry of every layer, so its size and offsets move with nnz.  Everything proportional
 * to nnz runs on the device; the host plans the partitions from the row lengths (measured on an
 * MI355X: 0.3 ms for a 1024 x 3072 layer with 315 k entries, 1.6 ms for a 16384 x 16384 matrix with
 * 2.7 M) -- cheap enough for a topology update every few hundred steps, not meant for every step. */
int sparse_linear_rebind(nerva_layer *layer, int32_t nnz, const int32_t *indptr,
                         const int32_t *indices, float *values, void *stream);

/* Density-adaptive layer ("Discussion and Conclusion" and Appendix C.3: dense computation where a layer is
 * not sparse enough for the sparse kernels to win; Section 5.3 shows masks winning at 50 % sparsity and the
 * sparse kernels from about 80 % on).  A layer on the dense route keeps one zero-filled dense copy of its
 * weights (rows x cols floats, columns padded to a multiple of 64; owned by the layer) and a dense gradient of
 * the same shape.  On batches of at least 16 columns its products Y = S X and Y = S^T X run as fp32 MFMA
 * products on that copy, and inside mlp_train_step S = A B^T is formed as a dense product of which only the
 * entries on the pattern are used.  values[] stays the layer's state, in CSR, and the momentum update touches
 * the stored entries only: the pattern is as immutable as on the sparse route, and every update the library
 * applies is written to the copy as well.  Results agree with the sparse route to rounding (other summation
 * order); entries off the pattern contribute 0 * x, so an operand that holds Inf/NaN spreads differently.
 * sparse_linear_create and sparse_linear_rebind take the route by themselves for a pattern of at least 40 %
 * density with at least 64 rows and 64 columns (the cut-over measured on the 3072-1024-512-10 network at batch
 * 100: the dense route's step takes 81 - 91 us whatever the density, the sparse route's 106 us at 50 % and
 * 57 us at 80 % sparsity); this call switches any layer over by hand.  A route once taken is kept across sparse_linear_rebind.
 * Errors: NERVA_ERR_SHAPE (rows x cols beyond 2^31), NERVA_ERR_HIP. */
int sparse_linear_enable_dense(nerva_layer *layer, void *stream);

/* The library keeps derived copies of values[] (the mirror's values, the dense copies above) and
 * updates them whenever it updates values[], with one exception: mlp_train_step leaves the mirror's
 * values of the MLP's FIRST layer alone, because no product of the step reads them (the first layer's
 * input gradient is not computed).  The layer remembers that: the next call that reads them -- a
 * training step of an MLP that has the layer at a later position, sparse_linear_backward, this call --
 * refreshes them first.  After the CALLER has written values[] (loaded weights, a prune-and-grow
 * step without rebind), this call brings all copies up to date; mlp_train_step and mlp_forward rely
 * on them.  sparse_linear_forward / sparse_linear_backward refresh what they read on every call and
 * do not need it. */
int sparse_linear_sync_values(nerva_layer *layer, void *stream);

/* Device pointers of the mirror, for inspection: indptr_t[cols+1], indices_t[nnz],
 * values_t[nnz], perm[nnz] (mirror position -> CSR position). Any output may be NULL.
 * values_t of a layer that mlp_train_step has trained as an MLP's first layer may be behind
 * values[] (see sparse_linear_sync_values, which brings it up to date). */
int sparse_linear_mirror(const nerva_layer *layer, const int32_t **indptr_t,
                         const int32_t **indices_t, const float **values_t,
                         const int32_t **perm);

/* Feedforward, A = S B (Section 4) with the dense bias and the layer's activation:
 *     Y[i,c] = act( bias[i] + sum_{p in row i} values[p] * X[indices[p], c] )
 * X is (cols, ldx), Y is (rows, ldy), 0 < batch <= ldx, ldy.  X and Y must not overlap. */
int sparse_linear_forward(const nerva_layer *layer, const float *X, int32_t ldx,
                          float *Y, int32_t ldy, int32_t batch, void *stream);

/* Backpropagation through one layer (Section 4, A = S^T B and S = A B^T on S's pattern).
 * With dZ = dY * [Y > 0] for a ReLU layer (the mask comes from the layer OUTPUT Y, as
 * backpropagate(Y, dY) in the Appendix B listing; derivative 0 at 0) and dZ = dY otherwise:
 *     dX[j,c]    = sum_{p : indices[p] = j} values[p] * dZ[row(p), c]     (skipped if dX == NULL)
 *     dvalues[p] = sum_c dZ[row(p), c] * X[indices[p], c]                 (skipped if NULL)
 *     dbias[i]   = sum_c dZ[i, c]                                         (skipped if NULL)
 * X (cols, ldx) is the layer input of the forward pass, Y (rows, ldy) its output (may be
 * NULL for NERVA_ACT_NONE), dY (rows, lddy), dX (cols, lddx).  All gradients use the
 * current contents of values[]; dX first refreshes the mirror's values from values[], so
 * the caller may have changed values[] by any means since the last call. */
int sparse_linear_backward(nerva_layer *layer, const float *X, int32_t ldx,
                           const float *Y, int32_t ldy, const float *dY, int32_t lddy,
                           float *dX, int32_t lddx, float *dvalues, float *dbias,
                           int32_t batch, void *stream);

/* Momentum step on raw arrays that share one pattern (Section 4: S = aS + bT applied
 * directly to the value arrays), used for values[] and for biases alike:
 *     velocity[k] <- momentum * velocity[k] - lr * grad[k]
 *     values[k]   <- values[k] + velocity[k]            for k in [0, n)
 * No dampening, no weight decay.  The index arrays of the pattern are not arguments:
 * the update cannot touch them. */
int sgd_update_values(float *values, float *velocity, const float *grad, int64_t n,
                      float lr, float momentum, void *stream);

/* The same step with Nesterov momentum, the optimiser of the paper's experiments (Section 5.1:
 * momentum 0.9, Nesterov, no weight decay): the weight moves by the look-ahead of the velocity,
 *     velocity[k] <- momentum * velocity[k] - lr * grad[k]
 *     values[k]   <- values[k] + momentum * velocity[k] - lr * grad[k]
 * For a constant lr this is the usual formulation buf <- momentum*buf + grad,
 * values <- values - lr*(grad + momentum*buf) with velocity = -lr*buf. */
int sgd_update_values_nesterov(float *values, float *velocity, const float *grad, int64_t n,
                               float lr, float momentum, void *stream);

/* Softmax cross-entropy on logits Z (classes, ldz), mean over the batch, and its gradient
 * divided by the batch size (Appendix B listing: loss.gradient(Y, T) / batch_size):
 *     lse_c = log sum_i exp Z[i,c]      (computed with the column maximum subtracted)
 *     *loss_out = (1/batch) sum_c ( lse_c - Z[labels[c], c] )
 *     dZ[i,c]   = ( exp(Z[i,c] - lse_c) - [i == labels[c]] ) / batch
 * labels: int32[batch] in [0, classes) (not checked on the device).  dZ may alias Z.
 * loss_out: one device float (may be NULL). */
int softmax_cross_entropy(const float *Z, int32_t ldz, const int32_t *labels,
                          int32_t classes, int32_t batch, float *dZ, int32_t lddz,
                          float *loss_out, void *stream);

/* ---- MLP training step ---------------------------------------------------------------
 * mlp_create chains n_layers layers (layer l's cols = layer l-1's rows; hidden layers
 * ReLU, last layer NERVA_ACT_NONE) and binds the momentum buffers: velocities[l] is
 * float[nnz_l], bias_velocities[l] is float[rows_l] (device, caller-owned, normally zero
 * at the start; bias_velocities[l] may be NULL iff the layer has no bias).  The handle
 * keeps the layer pointers: destroy the MLP before its layers.  max_batch bounds `batch`
 * of later calls and must not exceed any layer's max_batch.  flags: bitwise OR of the NERVA_MLP_* values below. */
enum {
    NERVA_MLP_DEFAULT = 0,
    /* Run S = A B^T, the momentum update and the mirror refresh as separate kernels that
     * store the gradient arrays in the workspace (the composition of the calls above),
     * instead of one fused kernel per layer that never stores dvalues. */
    NERVA_MLP_UNFUSED = 1,
    /* Nesterov momentum (see sgd_update_values_nesterov) for weights and biases. */
    NERVA_MLP_NESTEROV = 2,
    /* A small output layer (at most 32 rows and 8192 stored entries, as the 10-class layers
     * of Section 5.1) normally runs its forward product, the softmax cross-entropy and its
     * transposed product in one launch, each work-group owning four columns of the batch.
     * This flag keeps them in separate launches, as the output layers beyond those limits always
     * run (where a saturated one has the loss gradient formed by the finish pass of its forward
     * product and its whole backward pass in one streaming launch). */
    NERVA_MLP_SEPARATE_HEAD = 4
};
int mlp_create(nerva_mlp **out, int32_t n_layers, nerva_layer *const *layers,
               float *const *velocities, float *const *bias_velocities,
               int32_t max_batch, int32_t flags);
void mlp_destroy(nerva_mlp *mlp);

/* After sparse_linear_rebind on layer `layer_index` of the MLP: the momentum buffer float[new nnz]
 * (device, caller-owned) that later training steps use for that layer's weights. */
int mlp_rebind_velocity(nerva_mlp *mlp, int32_t layer_index, float *velocity);

/* Bytes of scratch mlp_train_step needs for `batch` columns (256-byte aligned base). */
size_t mlp_workspace_bytes(const nerva_mlp *mlp, int32_t batch);

/* Where mlp_train_step keeps its intermediates inside the workspace, so that a caller can
 * read them after a step.  layout_host (HOST, int64[1 + 4*n_layers]) receives
 *   [0]        ld, the leading dimension (in floats) of every matrix in the workspace
 *   [1+4l+0]   byte offset of A_l   (rows_l, ld): output of layer l (last layer: logits)
 *   [1+4l+1]   byte offset of dZ_l  (rows_l, ld): gradient w.r.t. the pre-activation
 *   [1+4l+2]   byte offset of g_l   float[nnz_l]  (written only with NERVA_MLP_UNFUSED)
 *   [1+4l+3]   byte offset of db_l  float[rows_l] (written only with NERVA_MLP_UNFUSED) */
int mlp_workspace_layout(const nerva_mlp *mlp, int32_t batch, int64_t *layout_host);

/* One iteration of the training loop (Appendix B listing) on one mini-batch:
 *   feedforward:    A_l = act(W_l A_{l-1} + b_l), A_0 = X (cols_1, ldx)
 *   loss gradient:  dZ_L = softmax-CE gradient / batch, *loss_out = mean cross-entropy
 *   backpropagate:  dZ_{l-1} = (W_l^T dZ_l) * [A_{l-1} > 0]   (not for the first layer),
 *                   g_l = (dZ_l A_{l-1}^T) on W_l's pattern, db_l = row sums of dZ_l;
 *                   every gradient uses the weights as they were when the call started
 *   optimize:       momentum step (see sgd_update_values) on values_l and bias_l.
 * labels: int32[batch].  workspace: device scratch of at least mlp_workspace_bytes().
 * loss_out: one device float (may be NULL). */
int mlp_train_step(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels,
                   int32_t batch, float lr, float momentum, void *workspace,
                   size_t workspace_bytes, float *loss_out, void *stream);

/* mlp_train_step for callers that cannot allocate device memory or keep a workspace of their own --
 * code under HIP graph capture, tight training loops, harnesses that forbid hipMalloc.  The same
 * step with the same kernels and the same results, but the intermediates (what mlp_workspace_layout
 * describes) live in a workspace that is part of the library itself: a static device array of
 * NERVA_STATIC_WORKSPACE_BYTES that every GPU on which the library runs holds until the process
 * ends.  The call allocates nothing and frees nothing (no hipMalloc, no events, no host buffers
 * that outlive it); per-launch timing (nerva_sparse_bench.h) is therefore refused while it is on.
 * The caller still passes the batch, the labels and loss_out, and owns the weights and momentum
 * buffers as before; the intermediates cannot be read back.  An MLP / batch whose workspace
 * (mlp_workspace_bytes) exceeds the static one is rejected with NERVA_ERR_WORKSPACE and a message
 * that names both sizes; nothing has been enqueued then.  The array is shared by every call on
 * that GPU and keeps the previous call's contents (nothing in it has to start at zero): calls on
 * different streams, or on different MLPs, that overlap in time on one GPU race -- order them on one
 * stream or with events.  The array's device address is looked up when the first MLP is created on
 * a device (mlp_create), so a captured call does no look-up. */
#define NERVA_STATIC_WORKSPACE_BYTES (32u << 20)
int mlp_train_step_static(nerva_mlp *mlp, const float *X, int32_t ldx, const int32_t *labels,
                          int32_t batch, float lr, float momentum, float *loss_out, void *stream);

/* Forward pass only (inference on a batch): logits (rows_L, ld) are left in the
 * workspace at the A_L offset. */
int mlp_forward(nerva_mlp *mlp, const float *X, int32_t ldx, int32_t batch,
                void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NERVA_SPARSE_H */
