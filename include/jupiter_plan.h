/*
 * jupiter_plan.h -- the parallelism planner of the Jupiter paper (Sec. IV-B) as host-only C entry points of
 * libjupiter_stage.so: where to cut the model into stages, and how to cut a prompt into sub-sequences,
 * from profiled latencies.  Nothing here touches a GPU; all pointers are HOST pointers, arrays are
 * borrowed for the duration of the call only.  Status codes and jup_last_error() as in jupiter_stage.h.
 *
 * The latency function q(x, y) -- one sub-sequence of x tokens through a stage whose cache already holds
 * y tokens -- is what `python -m paper_2504_08242_amd.profile_qxy` measures on this GPU.
 */
#ifndef JUPITER_PLAN_H
#define JUPITER_PLAN_H

#include "jupiter_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optimal model partition (Sec. IV-B.1, Eq. 1): cuts n_layers layers into n_devices contiguous stages,
 * stage n on device n (the devices keep their order), every device at least one layer, so that the slowest
 * stage is as fast as possible:  A(1..y, D_n) = min_l max{ A(1..l, D_{n-1}), T(l+1..y, d_n) }.
 *   layer_time    [n_devices][n_layers] row-major: profiled time of layer l on device n (any unit, >= 0)
 *   layer_mem     [n_layers]: memory the layer needs (parameters and KVCache; any unit, >= 0)
 *   mem_budget    [n_devices]: T(i..j, n) is infinite when the layers' memory exceeds mem_budget[n]
 *   last_layer    out [n_devices]: 1-based index of the last layer of every stage (last_layer[n_devices-1]
 *                 = n_layers); among equally good cuts the one with the earliest cut points, last stage first
 *   slowest       out: A(1..n_layers, D), the time of the slowest stage
 * Errors: JUP_EINVAL (NULL, sizes < 1, negative or NaN entries), JUP_ECAP when no partition fits the memory
 * budgets or there are fewer layers than devices (outputs untouched), JUP_ENOMEM.
 */
JUP_API jup_status_t jup_plan_layers(int32_t n_layers, int32_t n_devices, const double *layer_time,
                             const double *layer_mem, const double *mem_budget, int32_t *last_layer,
                             double *slowest);

typedef struct jup_seq_plan jup_seq_plan_t; /* opaque: the solved tables for every length up to s_max */

/*
 * Optimal sequence partition (Sec. IV-B.2, Eq. 2 and 3) for every prompt length y = 1..s_max and every number
 * of sub-sequences k = 1..4*n_devices at once:
 *     W(1..y, k) = min_l max{ W(1..l, k-1), T*(y-l, l) },   T*(x, l) = q(x, l) if x >= b, else infinite,
 * the latency of the slowest sub-sequence of the most balanced partition of y tokens into k sub-sequences of
 * at least b tokens (b: the shortest sub-sequence that still keeps the accelerator busy).
 *   xs, ys   strictly increasing grids of profiled sub-sequence lengths (xs[0] >= 1) and cached lengths (ys[0] >= 0)
 *   q        [nx][ny] row-major: profiled latency at (xs[i], ys[j]), > 0
 * Between profiled points q is interpolated (the paper approximates unprofiled points by interpolation):
 * bilinear inside the grid; above xs[nx-1] and above ys[ny-1] the outermost segment is continued linearly; below
 * xs[0] the latency of xs[0] is used (a shorter sub-sequence is not faster once the device is under-used) and
 * below ys[0] that of ys[0]; a continued value never falls below the smallest profiled latency, so q stays
 * positive everywhere.
 * Cost: 2*n_devices*s_max^2 evaluations of q; s_max <= 16384, n_devices <= 64.
 * Errors: JUP_EINVAL, JUP_ENOMEM.
 */
JUP_API jup_status_t jup_seq_plan_create(const int32_t *xs, int32_t nx, const int32_t *ys, int32_t ny, const double *q,
                                 int32_t b, int32_t n_devices, int32_t s_max, jup_seq_plan_t **out);
/*
 * The same tables with the cut points l of Eq. 2 restricted to multiples of `granule` tokens (1..16384): every
 * sub-sequence but the last is then a whole number of granules.  The paper's recurrence is granule = 1; on this GPU
 * the stage's kernels work on tiles of 256 token rows, q(x, y) is a staircase in x (a chunk of 513 tokens costs as much
 * as one of 768) that a coarse profiling grid does not show, and a plan is only as good as its q: granule = 256 keeps
 * the planner on the points where the interpolated q is true.
 */
JUP_API jup_status_t jup_seq_plan_create_aligned(const int32_t *xs, int32_t nx, const int32_t *ys, int32_t ny,
                                         const double *q, int32_t b, int32_t granule, int32_t n_devices,
                                         int32_t s_max, jup_seq_plan_t **out);
JUP_API void jup_seq_plan_destroy(jup_seq_plan_t *plan);

/* q(x, y) as the planner sees it (the interpolation rule above); NaN for a NULL plan, x < 1 or y < 0. */
JUP_API double jup_seq_plan_q(const jup_seq_plan_t *plan, int32_t x, int32_t y);

/*
 * The most balanced partition of a prompt of y tokens into exactly k sub-sequences.
 *   lengths   out [k]: the sub-sequence lengths in order (may be NULL)
 *   slowest   out: W(1..y, k) (may be NULL)
 *   total     out: the sum of the sub-sequences' latencies h_i = q(|s_i|, tokens before s_i) (may be NULL)
 * Among equally balanced partitions the one whose last sub-sequence is longest is reported (the smallest l of
 * Eq. 2), and so on towards the front.
 * Errors: JUP_EINVAL (NULL plan, y outside 1..s_max, k outside 1..4*n_devices), JUP_ECAP when y tokens cannot
 * be cut into k sub-sequences of at least b tokens (outputs untouched).
 */
JUP_API jup_status_t jup_seq_plan_partition(const jup_seq_plan_t *plan, int32_t y, int32_t k, int32_t *lengths,
                                    double *slowest, double *total);

/*
 * The number of sub-sequences for a prompt of y tokens (Sec. IV-B.2, Eq. 4): the k in 1..4*n_devices whose
 * partition minimises   Latency = sum_i h_i + (n_devices - 1) * W(1..y, k)   (the smallest such k).
 *   k_out     out: that k
 *   lengths   out [4*n_devices]: the first k entries are the sub-sequence lengths (may be NULL)
 *   latency   out: the estimate of Eq. 4 (may be NULL)
 * Errors: JUP_EINVAL; JUP_ECAP when y < b (no admissible partition at all).
 */
JUP_API jup_status_t jup_seq_plan_best(const jup_seq_plan_t *plan, int32_t y, int32_t *k_out, int32_t *lengths,
                               double *latency);

#ifdef __cplusplus
}
#endif
#endif /* JUPITER_PLAN_H */
