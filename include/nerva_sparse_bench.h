/* nerva_sparse_bench.h -- measurement aids of the library, kept apart from the product's C ABI
 * (nerva_sparse.h): a partition mode for A/B timings, per-launch event timing of a training
 * step, and a plain copy kernel of known size that memory-traffic counters are scaled by.
 * Benchmarks and tests use them; a training program needs none of them.
 */
#ifndef NERVA_SPARSE_BENCH_H
#define NERVA_SPARSE_BENCH_H

#include "nerva_sparse.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid: which partition later sparse_linear_create / sparse_linear_rebind /
 * nerva_plan_*_host calls build (process-wide; layers already bound keep theirs).
 * NERVA_PARTITION_BALANCED (default): the partition nerva_plan_rows_host describes.  NERVA_PARTITION_ROW_SPLIT:
 * plain row splitting -- one wave per row whatever its length, no huge rows, no packed short
 * rows, no staged products -- so that the balanced partition can be timed against it on the same
 * matrix.  NERVA_PARTITION_PREFER_STAGED: the balanced partition, but the staged products and the
 * staged SDDMM (see nerva_plan_staged_host) run wherever they can (batch of at least
 * NERVA_STAGE_MIN_BATCH columns, a multiple of 4), also where the library's own rule expects them
 * to be slower. */
enum { NERVA_PARTITION_BALANCED = 0, NERVA_PARTITION_ROW_SPLIT = 1, NERVA_PARTITION_PREFER_STAGED = 2 };
int nerva_set_partition_mode(int32_t mode);

/* Measurement aid: the density from which sparse_linear_create / sparse_linear_rebind put a layer on the
 * dense route by themselves (process-wide; layers already bound keep their route).  Default 0.4; a value above
 * 1 keeps every later layer on the sparse route, 0 sends every layer of at least 64 x 64 down the dense one. */
int nerva_set_dense_threshold(float density);

/* Per-kernel timing of mlp_train_step with HIP events, for benchmarks.  After
 * mlp_profile_enable(mlp, max_steps > 0) the next max_steps training steps record an event
 * before every kernel launch and one after the last, on the step's stream (events are created
 * on the fly: a profiled step allocates, must not be captured in a graph, and runs slower than
 * a plain one).  mlp_profile_read waits for the recorded events and returns, per launch slot of
 * a step (in launch order), the elapsed milliseconds from its event to the next one, summed over
 * the recorded steps (the launches of a step run back to back, so the slots add up to the step); the slots keep their
 * meaning until the next mlp_profile_enable.  mlp_profile_enable(mlp, 0) switches timing off
 * and frees the events.  Slot names look like "spmm_forward[0]", "sddmm_update[2]".
 *   n_slots_host, steps_host: HOST int32; ms_sum_host: HOST double[max_slots]. */
int mlp_profile_enable(nerva_mlp *mlp, int32_t max_steps);
int mlp_profile_read(nerva_mlp *mlp, int32_t max_slots, int32_t *n_slots_host,
                     double *ms_sum_host, int32_t *steps_host);
const char *mlp_profile_slot_name(const nerva_mlp *mlp, int32_t slot);

/* Plain device copy dst[k] = src[k], k in [0, n): the known-size kernel that memory
 * traffic counters are calibrated against.  Not part of the training path. */
int nerva_copy_f32(float *dst, const float *src, int64_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* NERVA_SPARSE_BENCH_H */
