/* pp_conv.h -- C ABI of the pattern-pruned 3x3 convolution library for AMD MI355X (gfx950).
 *
 * The operation.  A CONV layer with 3x3 kernels, stride 1, zero padding 1, whose weights
 * have been pruned in the two ways the paper describes in section 2.1.1 ("Pattern-Based
 * Pruning"): every surviving kernel -- the 3x3 slice of one output filter that reads one
 * input channel -- keeps exactly four non-zero weights, at the positions of one pattern out
 * of a small predefined set ("4-entry pattern pruning"); and connectivity pruning removes
 * whole kernels, cutting the link between an input and an output channel (same section, and
 * panel (b) of the figure on pattern / connectivity pruning).  Bias add and ReLU are fused
 * into the layer (one-to-one operators folded into their producer, section 2.2 "DNNFusion").
 *
 *   y[n][co][oy][ox] = act( bias[co] + sum over kept kernels (co,ci), over the four taps t of
 *                           the kernel's pattern:  w(co,ci,t) * X(n, ci, oy + t/3 - 1, ox + t%3 - 1) )
 *   X = x inside the image and 0 outside;  act = max(.,0) with PP_FLAG_RELU, identity otherwise.
 *
 * A tap is numbered t = 3*r + c for row r and column c of the 3x3 window (t = 4 is the
 * centre); a pattern is a 9-bit mask of its four taps.
 *
 * The calls follow the paper's split between compile time and run time (section 2.3.1,
 * "Pattern-Conscious Code Generation"): pp_conv_plan is the per-layer preparation -- it builds
 * the layer-wise representation (pattern types, pattern order in each filter, kernel/channel
 * connections, tile parameters), performs the filter kernel reorder, and packs the weights
 * into a compact filter-kernel-weight stream on the device; pp_conv_run executes the layer
 * with pattern-specialised device code over LDS-staged input tiles (the "load redundancy
 * elimination" of the same section).
 *
 * Pointers named *_dev are device (HBM) pointers; every other pointer is host memory.
 * Nothing in this interface is a C++ or PyTorch type.  No call throws.
 */
#ifndef PP_CONV_H
#define PP_CONV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pp_conv_plan pp_conv_plan_t; /* opaque; created by pp_conv_plan, owned by the library */

typedef enum {
    PP_OK = 0,
    PP_ERR_NULL = 1,        /* a required pointer is NULL */
    PP_ERR_SHAPE = 2,       /* a dimension is < 1 or a size overflows 31-bit element indexing */
    PP_ERR_PATTERN = 3,     /* a mask has bits above bit 8 or not exactly four bits, or a kept kernel's id is out of range */
    PP_ERR_UNSUPPORTED = 4, /* unknown dtype / flag / tuning request, or a host-only plan passed to pp_conv_run */
    PP_ERR_ALLOC = 5,       /* host allocation failed */
    PP_ERR_DEVICE = 6,      /* a HIP call failed (no device, out of device memory, launch error) */
    PP_ERR_ALIGN = 7,       /* a device buffer is not 16-byte aligned, or input and output overlap */
    PP_ERR_SCRATCH = 8      /* pp_conv_run_static: the call needs more scratch memory than the library's static buffer */
} pp_status_t;

/* Storage type of x, y and the packed weights.  Products are accumulated in fp32 in both cases;
 * with PP_F16 the weights are rounded to binary16 (nearest even) when packed and y is rounded
 * to binary16 (nearest even) when stored.  bias stays fp32. */
typedef enum { PP_F32 = 0, PP_F16 = 1 } pp_dtype_t;

enum {
    PP_FLAG_RELU = 1u,      /* y = max(pre, 0) */
    PP_FLAG_DENSE = 2u,     /* unpruned layer: kernel_size^2 weights per kernel, pattern ids and masks not read */
    PP_FLAG_HOST_ONLY = 4u, /* build the plan's host metadata only; touches no device (pp_conv_run then fails) */
    PP_FLAG_POOL2 = 8u      /* a 2x2 max-pool with stride 2 follows the activation and is folded into the layer (the
                               one-to-one / shuffle consumer folded into its producer, section 2.2): y is
                               [n][c_out][ho/2][wo/2]; the convolution's own output size ho x wo must be even */
};

/* Execution parameters (the part of the layer-wise representation that the paper leaves to tuning,
 * section 2.3.1).  A zero field means "let the library choose". */
typedef struct {
    int32_t variant;        /* 0 auto; 1 generic kernel (any layer); 2 tiled pattern-specialised kernel (3x3, stride 1, no
                               fused pool; masks outside its sixteen run as covers of those with zero weights); 3 matrix-core kernel (binary16 storage only: the pruned
                               weights zero-filled to a dense matrix and multiplied on the MFMA units -- the measured
                               alternative to pattern-specialised vector code; any pattern table, kernel size, stride) */
    int32_t filters_per_wave; /* F: output filters whose accumulators one wavefront holds (4, 8 or 16) */
    int32_t rows_per_lane;  /* R: output rows per lane (1, 2, or 4 with F = 4); a lane owns R x 4 adjacent output pixels */
    int32_t lanes_x;        /* LW: lanes across the width of a tile (2, 4, 7, 8, 14 or 16) */
    int32_t waves_f;        /* WF: wavefronts per workgroup that share one input tile, each on its own F filters */
    int32_t split_c;        /* KS: wavefronts per workgroup that split the input channels of a chunk */
    int32_t chunk_c;        /* CC: input channels staged in LDS at a time (multiple of split_c) */
    int32_t staging;        /* how input tiles reach LDS: 1 through registers, one buffer; 2..8 direct global-to-LDS
                               loads into a ring of that many buffers of chunk_c channels (needs rows that start on
                               4-byte boundaries: any fp32 width, even fp16 widths) */
    int32_t split_wg;       /* SW: workgroups that share one output tile, each on its own contiguous range of channel
                               chunks (1..64, at most the number of chunks); the last to finish adds the partial
                               sums up in range order, so results do not depend on who that is */
    int32_t balance;        /* 1: filters and channels take wavefront slots and chunk places in reordered / natural
                               order; 2: they are dealt so that the wavefronts of a workgroup do about equal work
                               between two barriers (the default whenever a workgroup has several wavefronts) */
    /* matrix-core kernel (variant 3) */
    int32_t tile_rows;      /* TR: rows of convolution outputs per workgroup tile (rows of the batch laid out as one tall image) */
    int32_t tile_cols;      /* TC: columns per workgroup tile; TR * TC <= 32 * tiles_per_wave * wg_waves */
    int32_t tiles_per_wave; /* NTW: 32-pixel MFMA column tiles per wavefront (2 or 4) */
    int32_t wg_waves;       /* wavefronts per workgroup (4 or 8), all on the same 64 filters; 8 only with NTW = 4 */
    int32_t autotune;       /* 1: pp_conv_plan times candidate variants and parameters on the device (the rules' own
                               choice, the other kernels that take the layer, other workgroup sizes and tile shapes;
                               fields set in this struct are kept), on scratch buffers of n_hint images and a stream
                               that it creates and frees, and keeps the fastest: the "tuning-decided parameters" of
                               section 2.3.1 decided by measurement.  Takes some milliseconds per candidate and
                               synchronises with its own stream only.  Ignored with PP_FLAG_HOST_ONLY.  The plan
                               reports chosen.autotune = 1 */
    int32_t mfma_kind;      /* which matrix-core kernel: 0 auto; 3 the product kernel of pp_block_gemm.h for 1x1 layers
                               (stride 1, no pool, h * w a multiple of 8: one matrix product per image, connectivity
                               pruning as its column pruning); 1 the general one (tiles transposed in registers on
                               their way into LDS; any kernel size, stride, channel count, fused pool); 2 the
                               direct-load one (3x3, stride 1; a fused pool needs even image sizes; when c_in is not a multiple of 16 the input is
                               first copied into a plan-owned buffer with zero channels appended, n_hint images at a
                               time, so runs of such a plan must not overlap: tiles copied
                               memory-to-LDS as they are and transposed by the LDS read; tile_cols is then a multiple
                               of 30 or of 14: segments of 30 or 14 outputs, of which a workgroup of wg_waves
                               wavefronts holds 2 * wg_waves or 4 * wg_waves; tile_rows = that count divided by
                               the segments per row, tile_cols / 30 or tile_cols / 14) */
    int32_t split_k;        /* direct-load matrix-core kernel only: workgroups that share one output tile, each on its
                               own run of channel chunks (0 auto, 1 none, 2, 4 or 8; must divide the number of
                               16-channel chunks and leave each share at least 2).  Layers with few tiles fill the
                               chip this way.  The shares' partial sums go to a plan-owned binary32 workspace sized
                               for n_hint images and a second small kernel adds them in share order (no atomics:
                               results do not depend on timing), so runs of such a plan must not overlap; a run on
                               more than n_hint images, and pp_conv_run_static, run without the split */
} pp_conv_tuning_t;

/* Layer description (section 2.1.1 for the sparsity, section 2.3.1 for what the layer-wise
 * representation records).  All arrays are host memory, borrowed only for the duration of
 * pp_conv_plan: the plan copies what it needs and the caller may free them afterwards. */
typedef struct {
    int32_t c_in, c_out, h, w;      /* >= 1 each; input is c_in x h x w per image */
    int32_t n_hint;                 /* batch size the plan should be tuned for; <= 0 means 1 */
    int32_t num_patterns;           /* P, 1..255 (ignored with PP_FLAG_DENSE) */
    const uint16_t *pattern_masks;  /* [P] tap masks for kernel_size <= 3 (bit t = K*r + c), exactly taps_per_kernel bits each */
    const int32_t *pattern_id;      /* [c_out*c_in] row-major (co, ci); read only where conn_mask != 0 */
    const uint8_t *conn_mask;       /* [c_out*c_in] non-zero = kernel kept; NULL = all kept */
    const float *weights;           /* [c_out*c_in*taps_per_kernel] the weights of each kernel in ascending tap order,
                                       read only where kept; with PP_FLAG_DENSE [c_out*c_in*K*K], all taps */
    const float *bias;              /* [c_out], or NULL for no bias */
    uint32_t flags;                 /* PP_FLAG_* */
    int32_t dtype;                  /* pp_dtype_t */
    const pp_conv_tuning_t *tuning; /* NULL = all automatic */
    /* Other kernel sizes and strides (the closing paragraph of section 2.1.1 names 3x3, 5x5 and 7x7 kernels; a
     * 1x1 layer has one tap, so only connectivity pruning applies to it).  Zero fields mean the 3x3, stride 1,
     * four-tap layer.  Padding is (K-1)/2 zeros on every side; the convolution's output is
     * ho x wo = (floor((h-1)/stride)+1) x (floor((w-1)/stride)+1). */
    int32_t kernel_size;            /* K: 0 (= 3), 1, 3, 5 or 7 */
    int32_t stride;                 /* 0 (= 1), 1 or 2 */
    int32_t taps_per_kernel;        /* weights kept per kernel: 0 = 4 for K >= 3 and 1 for K = 1; 1..K*K otherwise */
    const uint64_t *pattern_masks64; /* [P] tap masks for kernel_size > 3 (bit t = K*r + c, t < K*K); pattern_masks is
                                        then not read */
} pp_conv_desc_t;

/* Build a plan.  Validation happens before any device call, so invalid descriptions are
 * reported (and *out_plan set to NULL) on a machine without a GPU as well.  Unless
 * PP_FLAG_HOST_ONLY is set, the packed weights and index arrays are uploaded to the current
 * HIP device with synchronous copies; the plan is immutable afterwards. */
pp_status_t pp_conv_plan(const pp_conv_desc_t *desc, pp_conv_plan_t **out_plan);

/* Enqueue one forward pass on n images.
 *   x_dev : [n][c_in][h][w]  contiguous, plan dtype, 16-byte aligned, caller-owned
 *   y_dev : [n][c_out][out_h][out_w] contiguous, plan dtype, 16-byte aligned, caller-owned, must not overlap x_dev
 *           (out_h x out_w as reported by pp_conv_plan_query: h x w for a stride-1 layer without pooling)
 *   hip_stream : a hipStream_t (NULL = the default stream)
 * Returns after the launch without synchronising; launch-configuration errors are returned,
 * asynchronous faults are not.  Misaligned or overlapping x_dev / y_dev are PP_ERR_ALIGN (checked
 * on the host, before anything is launched).  Concurrent runs of one plan on different streams with different
 * y_dev are allowed unless the plan splits channels across workgroups (chosen.split_wg > 1 in
 * pp_conv_plan_query): such a plan owns one partial-sum workspace, sized for n_hint images, and its
 * runs must not overlap; more than n_hint images are processed n_hint at a time.  n <= 0 is
 * PP_ERR_SHAPE. */
pp_status_t pp_conv_run(const pp_conv_plan_t *plan, const void *x_dev, void *y_dev, int32_t n, void *hip_stream);

/* pp_conv_run for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.  It calls no
 * allocator and no allocating library routine; what pp_conv_run takes from a plan-owned workspace
 * (the partial sums and arrival counters of a plan with chosen.split_wg > 1) lives in one static
 * device array of 32 MiB instead -- 64 KiB of counters, the rest partial sums -- which every GPU
 * the library runs on holds until the process ends.  The whole batch goes in one launch, so
 * split_wg * n * c_out * h * w * 4 bytes must fit: otherwise PP_ERR_SCRATCH (likewise beyond 16384
 * output tiles) and nothing is launched.  Plans that need no scratch run exactly as in pp_conv_run.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU race, whatever
 * their plans and streams.  The counters are cleared on the stream by a small kernel before the
 * launch (no memset node), so the call may be recorded into a HIP graph. */
pp_status_t pp_conv_run_static(const pp_conv_plan_t *plan, const void *x_dev, void *y_dev, int32_t n, void *hip_stream);

/* Free the plan's host and device memory.  NULL is a no-op returning PP_OK.  The caller must
 * make sure no pp_conv_run of this plan is still executing. */
pp_status_t pp_conv_destroy(pp_conv_plan_t *plan);

/* The plan's layer-wise representation after the filter kernel reorder (section 2.3.1), in a
 * canonical form that does not depend on tuning.  Filters are listed by position in the new
 * order: kept-kernel count descending, then per-pattern histogram (entry by entry, larger
 * first), then original index ascending.  Inside a filter kernels are ordered by ascending
 * (pattern id, input channel), so kernels of one pattern are consecutive.
 * Pointers stay valid until pp_conv_destroy. */
typedef struct {
    int32_t c_out, c_in, num_patterns, taps; /* taps = weights per kept kernel (4; 9 for a dense 3x3 plan; ...) */
    int32_t out_h, out_w;                    /* size of y per image and filter (after stride and pooling) */
    int64_t k_kept;                          /* number of kept kernels */
    const int32_t *perm;     /* [c_out] perm[pos] = original filter index */
    const int32_t *kcount;   /* [c_out] kept kernels of the filter at pos */
    const int32_t *pat_off;  /* [c_out*(P+1)] prefix sums of that filter's per-pattern counts */
    const int32_t *kidx;     /* [k_kept] input channel of each kernel, filters concatenated in the new order */
    const uint8_t *kpat;     /* [k_kept] pattern id of each kernel */
    const float *wpacked;    /* [k_kept*taps] weights in the same order (fp32, before any binary16 rounding) */
    pp_conv_tuning_t chosen; /* the parameters the plan will run with */
} pp_plan_info_t;
pp_status_t pp_conv_plan_query(const pp_conv_plan_t *plan, pp_plan_info_t *out);

/* Decode the device-format weight stream of a tiled plan back into the canonical order
 * (a round-trip check of the packing).  kidx_out/kpat_out [k_kept], w_out [k_kept*4] (fp32; for
 * a PP_F16 plan the binary16-rounded values).  PP_ERR_UNSUPPORTED if the plan has no stream. */
pp_status_t pp_conv_plan_unpack(const pp_conv_plan_t *plan, int32_t *kidx_out, uint8_t *kpat_out, float *w_out);

/* 2x2 max-pool, stride 2, on [n][c][h][w] (h, w even) -> [n][c][h/2][w/2]; dtype as pp_dtype_t.
 * Not part of the convolution path: provided so that a stack of layers can be chained on the
 * device.  Asynchronous on hip_stream. */
pp_status_t pp_maxpool2x2_run(const void *x_dev, void *y_dev, int32_t n, int32_t c, int32_t h, int32_t w,
                              int32_t dtype, void *hip_stream);

/* Human-readable name of a status code (static storage). */
const char *pp_status_string(pp_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* PP_CONV_H */
