/* pp_block_gemm.h -- C ABI of the block-pruned matrix product for AMD MI355X (gfx950).
 *
 * The operation.  Block-based pruning (paper, section 2.1.2 "Block-Based Pruning", figure
 * "block_pruning") partitions the weight matrix of a fully-connected layer -- or of a CONV layer
 * written as a matrix product, as that section notes -- into blocks and prunes, independently in
 * every block, whole rows and whole columns of the block.  With W the M x K weight matrix cut into
 * blocks of block_m x block_k (the last block row / column is smaller when the sizes do not divide):
 *
 *   Wd[m][k] = W[m][k]  if row (m mod block_m) and column (k mod block_k) are both kept in the block
 *                       that holds (m, k);   0 otherwise
 *   y[m][j]  = act( bias[m] + sum_k Wd[m][k] * x[k][j] ),   x is K x N, y is M x N, both row-major
 *   act = max(., 0) with PP_FLAG_RELU, identity otherwise (a one-to-one operator folded into its
 *   producer, section 2.2).
 *
 * pp_block_gemm_plan is the compile-time half (section 2.3.1's split): for every tile of rows it
 * gathers the columns that any of the tile's blocks keeps into one compact list, packs the weights at
 * those columns (zeros where a block pruned the row) into matrix-core operand order and uploads
 * them.  pp_block_gemm_run multiplies: rows of x named by the compact list are copied
 * memory-to-LDS, so pruned columns cost neither traffic nor arithmetic; pruned rows inside a kept
 * column are zero operands of the matrix cores.
 *
 * Pointers named *_dev are device (HBM) pointers; every other pointer is host memory.  Status codes,
 * dtypes and flags are those of pp_conv.h.  No call throws.
 */
#ifndef PP_BLOCK_GEMM_H
#define PP_BLOCK_GEMM_H

#include <stdint.h>

#include "pp_conv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pp_block_gemm_plan pp_block_gemm_plan_t; /* opaque; owned by the library */

/* Layer description (section 2.1.2).  Arrays are host memory, borrowed for the duration of
 * pp_block_gemm_plan only.  With blocks_m = ceil(m / block_m), blocks_k = ceil(k / block_k), block
 * (bi, bj) has index bi * blocks_k + bj. */
typedef struct {
    int32_t m, k;              /* rows (outputs) and columns (inputs) of the weight matrix, >= 1 */
    int32_t block_m, block_k;  /* block size, >= 1 each */
    const uint8_t *row_keep;   /* [blocks_m*blocks_k*block_m] non-zero = that row of that block is kept; NULL = all kept */
    const uint8_t *col_keep;   /* [blocks_m*blocks_k*block_k] non-zero = that column of that block is kept; NULL = all kept */
    const float *weights;      /* [m*k] row-major; read only where kept */
    const float *bias;         /* [m], or NULL */
    uint32_t flags;            /* PP_FLAG_RELU, PP_FLAG_HOST_ONLY */
    int32_t dtype;             /* pp_dtype_t: storage of x, y and the packed weights; products accumulate in fp32 */
    int32_t variant;           /* 0 auto; 1 generic kernel (any dtype, any n); 2 matrix-core kernel (PP_F16) */
} pp_block_gemm_desc_t;

/* Build a plan.  Validation comes before any device call; on error *out_plan is NULL.  Unless
 * PP_FLAG_HOST_ONLY is set the packed operands are uploaded to the current HIP device with
 * synchronous copies.  PP_ERR_SHAPE: a size < 1, or m * k beyond 2^31 - 1.  PP_ERR_UNSUPPORTED: an
 * unknown dtype, flag or variant, or variant 2 with PP_F32. */
pp_status_t pp_block_gemm_plan(const pp_block_gemm_desc_t *desc, pp_block_gemm_plan_t **out_plan);

/* Enqueue y = act(Wd x + bias) for n columns.
 *   x_dev : [k][n] row-major, plan dtype, 16-byte aligned, caller-owned
 *   y_dev : [m][n] row-major, plan dtype, 16-byte aligned, caller-owned, must not overlap x_dev
 * Asynchronous on hip_stream (a hipStream_t, NULL = default stream).  The matrix-core kernel needs n
 * to be a multiple of 8 (rows of x and y then start on 16-byte boundaries); an automatic plan runs
 * the generic kernel for any other n, a plan with variant 2 forced returns PP_ERR_UNSUPPORTED.
 * n < 1, or k * n or m * n beyond 2^31 - 1 elements: PP_ERR_SHAPE.  Misaligned or overlapping
 * buffers: PP_ERR_ALIGN. */
pp_status_t pp_block_gemm_run(const pp_block_gemm_plan_t *plan, const void *x_dev, void *y_dev, int32_t n, void *hip_stream);

/* Free the plan.  NULL is a no-op returning PP_OK.  No run of the plan may still be executing. */
pp_status_t pp_block_gemm_destroy(pp_block_gemm_plan_t *plan);

/* What the plan built.  Row tile t covers rows t * row_tile .. ; its compact column list is
 * tile_cols[tile_off[t] .. tile_off[t+1]) (ascending, padded to a multiple of 16 by repeating the last
 * column, with zero weights there; an empty list stays empty).  Pointers stay valid until destroy. */
typedef struct {
    int32_t m, k, block_m, block_k;
    int32_t variant;            /* the kernel an n that is a multiple of 8 runs with: 1 or 2 */
    int32_t row_tile;           /* rows per tile (64) */
    int32_t row_tiles;          /* ceil(m / row_tile) */
    int64_t kept_weights;       /* number of (m, k) with Wd structurally kept */
    int64_t executed_weights;   /* row_tile * sum over tiles of the padded list length: what the matrix cores multiply */
    const int32_t *tile_off;    /* [row_tiles + 1] */
    const int32_t *tile_cols;   /* [tile_off[row_tiles]] */
    const int32_t *tile_len;    /* [row_tiles] list length before padding */
} pp_block_gemm_info_t;
pp_status_t pp_block_gemm_query(const pp_block_gemm_plan_t *plan, pp_block_gemm_info_t *out);

/* The packed weights of row tile t decoded back to a dense row_tile x k matrix (fp32; binary16-rounded
 * values for a PP_F16 plan), zeros elsewhere: a round-trip check of the packing.  w_out [row_tile*k]. */
pp_status_t pp_block_gemm_unpack(const pp_block_gemm_plan_t *plan, int32_t tile, float *w_out);

#ifdef __cplusplus
}
#endif

#endif /* PP_BLOCK_GEMM_H */
