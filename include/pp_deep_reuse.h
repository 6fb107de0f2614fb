/* pp_deep_reuse.h -- C ABI of deep reuse (LSH clustering of neuron vectors) for AMD MI355X (gfx950).
 *
 * The operation.  Deep reuse (paper, section 2.3.2 "Deep Reuse", figure "basicReuse") approximates
 * y = act(x W + bias) -- x holds one row per output position: the unfolded input of a CONV layer or the
 * tokens of a fully-connected one; W is K x M -- by cutting every row of x into neuron vectors of L
 * consecutive values, clustering the neuron vectors of each column segment with locality-sensitive
 * hashing, and computing the dot products of a cluster once, on one of its vectors, for all its
 * members.  The section leaves the hash family, the vector that stands for a cluster and the reuse scope
 * to the papers it cites; this library takes:
 *
 *   segment s       columns sL .. sL+L-1 of x (K a multiple of L)
 *   signature       bit h of sig(i, s) is 1 iff  sum_l x[i][sL+l] * hyperplanes[s][h][l] > 0, the sum
 *                   taken in binary32 as a chain of fused multiply-adds in ascending l, starting from 0
 *   cluster         the rows of one call with equal signature in segment s; its representative rep(s, g)
 *                   is the member with the lowest row index
 *   P[s][g][m]    = sum_l x[rep(s,g)][sL+l] * W[sL+l][m]                      (once per cluster)
 *   y[i][m]       = act( bias[m] + sum_s P[s][sig(i,s)][m] )
 *
 * The hyperplanes are an input (random numbers are the caller's), so a result is a pure function of the
 * arguments.  Storage and arithmetic are binary32.  Pointers named *_dev are device pointers; every other
 * pointer is host memory.  Status codes and flags are those of pp_conv.h.  No call throws.
 */
#ifndef PP_DEEP_REUSE_H
#define PP_DEEP_REUSE_H

#include <stdint.h>

#include "pp_conv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pp_reuse_plan pp_reuse_plan_t; /* opaque; owned by the library */

/* Arrays are host memory, borrowed for the duration of pp_reuse_plan only. */
typedef struct {
    int32_t k, m;             /* reduction length and number of outputs, >= 1 */
    int32_t seg_len;          /* L: length of a neuron vector, 1..32, divides k */
    int32_t hash_bits;        /* H: hyperplanes per segment, 1..12 (at most 2^H clusters per segment) */
    int32_t n_max;            /* the most rows one pp_reuse_run may be given (sizes the plan's workspace) */
    const float *weights;     /* [k][m] row-major */
    const float *bias;        /* [m], or NULL */
    const float *hyperplanes; /* [k/L][H][L] */
    uint32_t flags;           /* PP_FLAG_RELU, PP_FLAG_HOST_ONLY */
} pp_reuse_desc_t;

/* Validates (before any device call; *out_plan is NULL on error), uploads weights, bias and hyperplanes and
 * allocates the workspace: signatures [n_max][k/L] (16 bit), representatives [k/L][2^H] (32 bit) and the
 * cluster products [k/L][2^H][m] (binary32).  PP_ERR_SHAPE: a size out of range, k not a multiple of
 * seg_len, or n_max * max(k, m) beyond 2^31 - 1.  PP_ERR_UNSUPPORTED: an unknown flag, or hyperplanes that do not fit
 * 64 KB of LDS ((k/L) * (H*L + 1) * 4 bytes). */
pp_status_t pp_reuse_plan(const pp_reuse_desc_t *desc, pp_reuse_plan_t **out_plan);

/* Enqueue one pass over n rows (1 <= n <= n_max): four kernels on hip_stream (clear the representatives,
 * hash + elect representatives, cluster products, gather-sum + bias + activation); never synchronises.
 *   x_dev : [n][k] row-major binary32, 16-byte aligned;  y_dev : [n][m] row-major binary32, 16-byte aligned,
 *   must not overlap x_dev (PP_ERR_ALIGN otherwise).
 * Runs of one plan share its workspace and must not overlap in time. */
pp_status_t pp_reuse_run(const pp_reuse_plan_t *plan, const void *x_dev, void *y_dev, int32_t n, void *hip_stream);

/* What the last run on n rows left in the workspace, copied to the host after a device synchronisation:
 * sig_out [n][k/L] signatures (may be NULL), rep_out [k/L][2^H] representative row per cluster, -1 where the
 * cluster is empty (may be NULL).  For tests and for reporting the reuse ratio. */
pp_status_t pp_reuse_read_clusters(const pp_reuse_plan_t *plan, int32_t n, uint16_t *sig_out, int32_t *rep_out);

/* Free the plan.  NULL is a no-op returning PP_OK.  No run of the plan may still be executing. */
pp_status_t pp_reuse_destroy(pp_reuse_plan_t *plan);

#ifdef __cplusplus
}
#endif

#endif /* PP_DEEP_REUSE_H */
