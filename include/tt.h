/*
 * libtt - fused DNN operator kernels executed under transferable schedule
 * records, and the transfer-tuning sweep, for AMD Instinct MI355X (gfx950).
 *
 * The vocabulary follows "Transfer-Tuning: Reusing Auto-Schedules for
 * Efficient Tensor Program Code Generation" (Gibson & Cano, PACT 2022):
 *
 *   kernel        a fused operator group handed to the tuner as one loop nest
 *                 (Section 4.2), e.g. conv2d + bias + ReLU (Algorithm 2);
 *   kernel class  all kernels with the same operator sequence, any sizes
 *                 (Section 4.2); schedules are reused only inside a class;
 *   schedule      the list of loop transformations a kernel is compiled with
 *                 (Section 4.1: Split, Reorder, Fuse, Parallel, Unroll,
 *                 Vectorize, ComputeAt, cache buffer).  Here: one fixed-size
 *                 record of the GPU-native knobs those primitives map to;
 *   transfer      re-applying a schedule tuned for one kernel to another kernel
 *                 of the class: inner factors are kept, outer extents are
 *                 derived from the new shape, and a record that cannot fit is
 *                 invalid (Sections 4.1, 4.2);
 *   sweep         trying every same-class donor schedule on every target
 *                 kernel, standalone, and keeping the fastest, with the default
 *                 schedule as fallback (Section 4.3).
 *
 * Conventions of every entry point
 *   - plain C ABI; every function returns a tt_status (0 = TT_OK, negative = error);
 *   - pointers named x, w, bias, residual, y, a, b, c, ws and `out_dev` are DEVICE
 *     pointers, 16-byte aligned, owned by the caller; all other pointers are HOST
 *     pointers.  The library never allocates or frees device memory;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The
 *     operator entry points only enqueue work on it and return; the caller
 *     synchronises.  tt_transfer_sweep synchronises the stream itself;
 *   - tensors are dense, row-major in the order written (channels-last: NHWC
 *     activations, KRSC filters); element type is tt_dtype of the shape; bias is always the same
 *     type as the activations; accumulation is always float32;
 *   - an operator entry point given a schedule that is invalid for the shape
 *     returns the error and writes nothing: falling back to the default schedule
 *     is the sweep's decision (Section 4.3), not the operator's.  A NULL schedule
 *     means "the default schedule of this kernel";
 *   - split-K partial sums live in the caller's workspace `ws`; its size for a
 *     given (schedule, shape) is tt_plan.workspace_bytes.  Too small a workspace
 *     is TT_ERR_WORKSPACE.
 */
#ifndef TT_H
#define TT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel classes (Section 4.2).  Letters are the paper's labels for ResNet18 (Table 1). */
typedef enum tt_class {
    TT_CONV2D_ADD = 0,           /* A: conv2d + per-output-channel vector, no activation        */
    TT_CONV2D_BIAS_RELU = 1,     /* E: pad, conv2d, + bias, ReLU (Algorithm 2)                  */
    TT_CONV2D_BIAS_ADD_RELU = 2, /* F: conv2d, + bias, + residual tensor, ReLU                  */
    TT_CONV2D_BIAS_RELU6 = 3,    /* conv2d, + bias, clamp to [0,6] (MobileNetV2-shaped nets)    */
    TT_DENSE_ADD = 4,            /* D: dense + vector                                           */
    TT_DENSE_BIAS_RELU = 5,
    TT_DENSE_BIAS_GELU = 6,      /* exact GELU: x/2 * (1 + erf(x / sqrt 2))                      */
    TT_BATCH_MATMUL = 7,
    TT_DWCONV_BIAS_RELU6 = 8,    /* depthwise 3x3 conv, + bias, clamp to [0,6]                  */
    TT_NUM_CLASSES = 9
} tt_class;

typedef enum tt_dtype { TT_F32 = 0, TT_BF16 = 1 } tt_dtype;

typedef enum tt_status {
    TT_OK = 0,
    TT_ERR_INVALID_SCHEDULE = -1, /* the record cannot be applied to this shape (Section 4.2: a split
                                     factor larger than the loop; Section 4.3 reports such pairs as -1) */
    TT_ERR_CLASS_MISMATCH = -2,   /* record of another kernel class (Section 4.2: always invalid)      */
    TT_ERR_BAD_ARG = -3,          /* NULL / misaligned pointer, ill-formed shape or record             */
    TT_ERR_WORKSPACE = -4,        /* workspace smaller than tt_plan.workspace_bytes                    */
    TT_ERR_UNSUPPORTED = -5,      /* valid plan, but no compiled kernel variant implements it          */
    TT_ERR_HIP = -6               /* a HIP runtime call failed                                         */
} tt_status;

/* Why a record is invalid for a shape (tt_plan.reason when status == TT_ERR_INVALID_SCHEDULE). */
typedef enum tt_reason {
    TT_R_NONE = 0,
    TT_R_FACTOR_GT_M = 1,  /* tile_m larger than the M loop (Section 4.2)                */
    TT_R_FACTOR_GT_N = 2,
    TT_R_FACTOR_GT_K = 3,
    TT_R_NOT_DIVISIBLE = 4,/* only with TT_STRICT_DIVISIBLE (Section 4.1: {N : f | N})   */
    TT_R_SPLIT_K = 5,      /* more reduction splits than K tiles                         */
    TT_R_LDS = 6,          /* staged tiles exceed the 160 KiB of LDS a workgroup can use */
    TT_R_K_GRANULE = 7,    /* tile_k is not a multiple of what one matrix-core step of
                              this data type consumes                                    */
    TT_R_GRID = 8,         /* more than 2^31 - 1 workgroups                              */
    TT_R_SKETCH_CLASS = 9  /* the record's sketch has no meaning for this class          */
} tt_reason;

/* The loop-nest skeleton ("sketch") a record's factors refer to. */
typedef enum tt_sketch {
    TT_SK_MFMA = 0,   /* contraction: workgroup tile -> wave tile -> matrix-core block; LDS-staged K loop */
    TT_SK_GEMV = 1,   /* dense classes: a wave per few outputs, lanes split K, wave reduction            */
    TT_SK_DWCONV = 2, /* depthwise: (planes, rows, cols) tile per workgroup, micro-tile per thread       */
    TT_SK_DIRECT = 3  /* any class: one thread per output, the unscheduled loop nest                     */
} tt_sketch;

/* A convolution's sizes.  Memory is channels-last: activations [n,h,w,c], filters [k,r,s,c]
 * ([r,s,c] for depthwise, with k == c), outputs [n,Ho,Wo,k].  The operator is Algorithm 2's:
 * cross-correlation, zero padding, dilation 1, groups 1; only the storage order differs from the
 * paper's NCHW listing, so that the reduction axis is contiguous for the matrix cores. */
typedef struct tt_conv_shape {
    int32_t n, c, h, w, k, r, s, stride_h, stride_w, pad_h, pad_w;
    int32_t dtype; /* tt_dtype */
} tt_conv_shape;

/* C[b,m,n] = sum_k A[b,m,k] * B(b,k,n).  A is [batch,m,k]; B is [batch,n,k] when trans_b = 1
 * and [batch,k,n] when trans_b = 0.  Dense kernels: batch = 1, trans_b = 1, B = weights [out,in]. */
typedef struct tt_gemm_shape {
    int32_t batch, m, n, k, trans_b;
    int32_t dtype; /* tt_dtype */
} tt_gemm_shape;

/*
 * A schedule record.  Every field is an INNER factor or a mode; nothing in it
 * depends on the size of the kernel it was tuned for, so it can be re-applied
 * to any kernel of its class (Section 4.1's Split(N, N/8, 8) form).
 *
 * Meaning per sketch (GEMM view: conv M = n*Ho*Wo, N = k, K = c*r*s; dense and
 * batch matmul M, N, K per batch; depthwise M = Ho, N = Wo, "K" = n*c planes):
 *   TT_SK_MFMA   tile_m x tile_n x tile_k workgroup tile (Split level 1, powers of two 16..256,
 *                tile_k in 16/32/64/128); wave_m x wave_n wave tile (Split level 2); mfma = edge
 *                of the matrix-core block, 16 or 32 (innermost Split); split_k = parallel split of
 *                the reduction (Parallel on a reduction axis); order = workgroup raster (Reorder +
 *                Fuse of the two parallel axes, see tt_plan_tile); vec = elements per global access
 *                (Vectorize); unroll = depth to which the per-tile K-step loop is unrolled (Unroll);
 *                stages = LDS buffers (cache buffer + ComputeAt): 1 or 2 with register-staged loads,
 *                3 or 4 = ring filled by asynchronous global-to-LDS loads (reformulated to 2 where
 *                the ring does not apply: partial 16-byte items, [K][N] operands, odd tile/thread ratios);
 *                5 or 6 = 3x3 convolutions only: the padding stage of Algorithm 2 computed at the
 *                workgroup tile, i.e. the tile's padded input patch cached in LDS for tile_k channels at
 *                a time, plus a ring of 3 or 4 filter buffers (reformulated to 3 or 4 where it does
 *                not apply: other filters or data types, a patch larger than the kernel's buffer, a
 *                channel count tile_k does not divide, a split off the channel-slice boundaries);
 *                7 = dense family with a short reduction (dense layers, unit-stride 1x1 convolutions,
 *                A.B^T products of one batch): cache buffer + ComputeAt one level further out, the whole
 *                [tile_n][K] panel of the second operand cached in LDS once per workgroup, which then
 *                walks down M with the first operand's rows double-buffered a tile ahead
 *                (reformulated to 4 where it does not apply: K not a whole number of tile_k slices or
 *                too long for the LDS, a split reduction, several batches, partial 16-byte items).
 *   TT_SK_GEMV   tile_m (= wave_m) rows and tile_n outputs per workgroup, wave_n outputs per wave,
 *                tile_k = K elements a wave consumes per step (64 lanes x 1/2/4/8), mfma = 0.
 *   TT_SK_DWCONV tile_m x tile_n output rows x cols and tile_k lanes along the plane axis per workgroup,
 *                wave_m x wave_n outputs per thread; vec = channel-contiguous planes per lane (reformulated
 *                to what divides the channel count; the workgroup then covers tile_k * vec planes);
 *                stages = 2 stages the input patch through LDS (kernel with one plane per lane only: a
 *                plan with more has variant_id = -1), mfma = 0.
 *   TT_SK_DIRECT all tile and wave fields 1, mfma = 0.
 */
typedef struct tt_schedule {
    int32_t cls;    /* tt_class the record was tuned for */
    int32_t sketch; /* tt_sketch */
    int32_t tile_m, tile_n, tile_k;
    int32_t wave_m, wave_n;
    int32_t mfma;
    int32_t split_k;
    int32_t order;  /* 0 M-tiles fastest, 1 N-tiles fastest, 2 bands of 8 M-tiles; +3 = XCD-contiguous */
    int32_t vec;    /* 1, 2, 4 or 8 */
    int32_t unroll; /* >= 1 */
    int32_t stages; /* 1..7 (matrix-core sketch), 1 or 2 (others) */
    /* provenance (ignored by tt_schedule_apply): */
    int32_t id;              /* caller's identifier of the record                     */
    int32_t donor_shape[12]; /* the shape the record was tuned on (struct as int32[]) */
    float donor_us;          /* its time on that shape                                */
} tt_schedule;

/*
 * The integer plan tt_schedule_apply derives, a pure function of (record, class, shape, flags).
 * Two kinds of fields:
 *   method   what Sections 4.1 / 4.2 define, independent of how a kernel is written: status and
 *            reason (class mismatch, a factor larger than its loop, strict divisibility, split of
 *            the reduction, grid), the GEMM view M, N, K, the kept inner factors, the derived outer
 *            extents and tails, eff_split_k, k_iters, slabs, order, grid, block, workspace_bytes;
 *   library  how this library's kernels fetch and stage the tiles: eff_vec_*, eff_unroll, stages
 *            (after reformulation), lds_bytes, variant_id, and the reasons TT_R_LDS and
 *            TT_R_K_GRANULE, which are checked after every method rule.  lds_bytes is stages times
 *            the per-stage size the compiled kernel variant reports (tt_variant_info; the kernels of
 *            stages 5..7 report their own layouts); it is 0 when
 *            no variant implements the plan (variant_id = -1: the operator entry points then return
 *            TT_ERR_UNSUPPORTED).
 */
typedef struct tt_plan {
    int32_t status, reason;
    int32_t sketch, batch, M, N, K;
    int32_t tile_m, tile_n, tile_k, wave_m, wave_n, mfma;
    int32_t tiles_m, tiles_n, k_tiles;   /* derived outer extents = ceil(extent / factor) */
    int32_t tail_m, tail_n, tail_k;      /* size of the last tile on each axis            */
    int32_t eff_split_k, k_iters;        /* non-empty reduction splits; K tiles per split */
    int32_t slabs;                       /* batch * eff_split_k (depthwise: plane tiles)  */
    int32_t eff_vec_a, eff_vec_b, eff_vec_c; /* vector widths after reformulation         */
    int32_t eff_unroll;
    int32_t stages, order;
    int32_t grid, block;                 /* workgroups, threads per workgroup             */
    int32_t lds_bytes;
    int64_t workspace_bytes;
    int32_t variant_id;                  /* compiled kernel variant (matrix-core sketch) or 0;
                                            -1 if no kernel implements the plan             */
    int32_t reserved;
} tt_plan;

enum { TT_STRICT_DIVISIBLE = 1 }; /* flags of tt_schedule_apply: factors must divide their loops (Section 4.1) */

/* Library version and a human-readable name for a status code (static storage). */
int tt_version(void);
const char *tt_status_name(int status);
/* Text of the last failed HIP call on this thread (what, HIP's message, HIP's code), or of the last
 * refusal of tt_conv2d_bias_relu_noalloc for lack of static workspace; "" if none. */
const char *tt_last_error(void);

/*
 * The default ("untuned") schedule of a kernel (Section 4.3): valid for every
 * well-formed shape of the class.  `shape` is a tt_conv_shape for the conv and
 * depthwise classes and a tt_gemm_shape otherwise (host pointers).
 */
int tt_schedule_default(int cls, const void *shape, tt_schedule *out);

/*
 * Re-apply a schedule record to a target kernel (Sections 4.1, 4.2): keep the
 * inner factors, derive the outer extents from `shape`, decide validity.
 * Host-only integer work.  Returns plan->status: TT_OK, TT_ERR_INVALID_SCHEDULE
 * (plan->reason says why), TT_ERR_CLASS_MISMATCH or TT_ERR_BAD_ARG.
 */
int tt_schedule_apply(const tt_schedule *sched, int cls, const void *shape, int flags, tt_plan *plan);

/*
 * Host mirror of the device index map: workgroup id -> out[8] =
 * {batch, k-split, m0, m_extent, n0, n_extent, k0, k_extent} (depthwise:
 * {plane tile, 0, row0, rows, col0, cols, plane0, planes}).  Not defined for
 * TT_SK_DIRECT (TT_ERR_BAD_ARG).
 */
int tt_plan_tile(const tt_plan *plan, int64_t wg, int32_t out[8]);

/*
 * Run the device's own index decode for every workgroup of the plan and write
 * 8 int32 per workgroup to out_dev (device, 8 * plan->grid int32).  Used to
 * check that host and device agree bit for bit.
 */
int tt_debug_tile_map(const tt_plan *plan, int32_t *out_dev, void *stream);

/*
 * Debug: the quotient n / d as the kernels compute it (one widening multiply by a precomputed
 * reciprocal, used to turn an output-pixel index into image, row and column), evaluated on the
 * host.  Defined for 0 <= n < 2^31 and 1 <= d < 2^31; returns -1 outside that range.
 */
int64_t tt_debug_fast_div(uint32_t n, uint32_t d);

/*
 * Debug: hardware-rate probes.  Each runs a plain hand-written kernel `reps` times back to back on
 * `stream` (after one untimed run), times the run with events on that stream, synchronises, and writes one
 * figure to *result.  They measure the machine, not the method: a kernel's roofline fraction can be put
 * next to the rate the simplest kernel of its kind reaches on the same GPU.
 *   TT_PROBE_LAUNCH_GAP_US     microseconds per launch of an empty kernel (src, dst, bytes unused)
 *   TT_PROBE_MFMA_BF16_TFLOPS  32x32x16 bf16 matrix products issued back to back by four waves per SIMD;
 *                              dst: at least 1 KB of device memory (never written), bytes its size
 *   TT_PROBE_COPY_LINEAR_GBPS  copy of `bytes` (a multiple of 32 KiB) from src to dst, 16 bytes per lane,
 *                              consecutive lanes on consecutive addresses; result = 2 * bytes / time
 *   TT_PROBE_COPY_TILED_GBPS   the same bytes as a matrix of 512-byte rows copied in tiles of 64 rows x 128
 *                              bytes per workgroup (the order in which a contraction's epilogue writes)
 *   TT_PROBE_L2_READ_GBPS      1024 workgroups read 4 MiB each out of a source of 1..2 MiB (`bytes`) that
 *                              stays in the L2; dst: at least 1 KB of device memory (never written)
 * src and dst are device pointers, 16-byte aligned, owned by the caller; a cold copy figure needs buffers
 * larger than the caches.  TT_ERR_BAD_ARG for sizes or pointers outside these rules.
 */
enum {
    TT_PROBE_LAUNCH_GAP_US = 0,
    TT_PROBE_MFMA_BF16_TFLOPS = 1,
    TT_PROBE_COPY_LINEAR_GBPS = 2,
    TT_PROBE_COPY_TILED_GBPS = 3,
    TT_PROBE_L2_READ_GBPS = 4
};
int tt_debug_probe(int which, const void *src, void *dst, size_t bytes, int reps, void *stream, double *result);

/*
 * conv2d (+bias) (+residual) (+activation) as an implicit GEMM (Algorithm 2; Table 1
 * classes A, E, F).  cls selects the epilogue: TT_CONV2D_ADD (bias, none),
 * TT_CONV2D_BIAS_RELU, TT_CONV2D_BIAS_ADD_RELU (residual required, same layout
 * and type as y), TT_CONV2D_BIAS_RELU6.  x [n,h,w,c], w [k,r,s,c], bias [k],
 * y [n,Ho,Wo,k], Ho = (h + 2 pad_h - r) / stride_h + 1.
 */
int tt_conv2d_bias_relu(const void *x, const void *w, const void *bias, const void *residual, void *y,
                        const tt_conv_shape *shape, int cls, const tt_schedule *sched, void *ws,
                        size_t ws_bytes, void *stream);

/*
 * The same operator for callers that cannot allocate device memory and hold no workspace of their own:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Split-K
 * partial sums go to an array of TT_STATIC_WORKSPACE_BYTES that is part of the library's device code
 * (one copy per GPU, held until the process ends); the call allocates and frees nothing.  A (schedule,
 * shape) whose tt_plan.workspace_bytes exceeds that size is refused with TT_ERR_WORKSPACE (tt_last_error
 * says so) and nothing is launched.  Results are those of tt_conv2d_bias_relu, bit for bit.  Every call
 * on a GPU uses that GPU's one array: calls that may overlap on one GPU (different streams, different
 * host threads) race on it and must be serialised by the caller; calls on one stream are ordered.
 * Nothing in the array has to be cleared between calls: every partial sum a call reads it has written.
 */
#define TT_STATIC_WORKSPACE_BYTES (16 * 1024 * 1024)
int tt_conv2d_bias_relu_noalloc(const void *x, const void *w, const void *bias, const void *residual, void *y,
                                const tt_conv_shape *shape, int cls, const tt_schedule *sched, void *stream);

/*
 * dense (+bias) (+activation): y[m,o] = act(bias[o] + sum_i x[m,i] w[o,i]) (Table 1 class D;
 * Section 4.4.1's dense-only class).  cls: TT_DENSE_ADD, TT_DENSE_BIAS_RELU,
 * TT_DENSE_BIAS_GELU.  shape: batch = 1, trans_b = 1, m rows, n outputs, k inputs.
 */
int tt_dense_bias_relu(const void *x, const void *w, const void *bias, void *y, const tt_gemm_shape *shape,
                       int cls, const tt_schedule *sched, void *ws, size_t ws_bytes, void *stream);

/* Batch matmul c[b] = a[b] B[b] (the loop nest of Algorithm 1 per batch); class TT_BATCH_MATMUL. */
int tt_batch_matmul(const void *a, const void *b, void *c, const tt_gemm_shape *shape,
                    const tt_schedule *sched, void *ws, size_t ws_bytes, void *stream);

/* Depthwise 3x3 conv + bias + clamp[0,6]; x [n,h,w,c], w [3,3,c], y [n,Ho,Wo,c]; class
 * TT_DWCONV_BIAS_RELU6; float32 only. */
int tt_dwconv(const void *x, const void *w, const void *bias, void *y, const tt_conv_shape *shape,
              const tt_schedule *sched, void *stream);

/* One target kernel of a sweep.  bufs: conv {x, w, bias, residual|NULL, y}; dense {x, w, bias, y, NULL};
 * batch matmul {a, b, c, NULL, NULL}; depthwise {x, w, bias, y, NULL}.
 * alt_bufs (host array of n_alt x 5 device pointers, NULL when n_alt = 0): further tensor sets of the same
 * shapes.  The timing functions (tt_time_pair and every sweep) then walk round bufs and the alternatives
 * launch by launch, so that a launch finds none of its operands in a cache once the sets together exceed the
 * caches: the standalone time of a kernel whose inputs come from memory, as inside a network.  With n_alt = 0
 * every launch of a pair reuses bufs (operands of repeated launches stay in the memory-side cache).
 * tt_run_kernels uses bufs only. */
typedef struct tt_kernel_desc {
    int32_t cls;
    int32_t use_count;  /* how often the network runs this kernel (Table 1's "Use Count") */
    const void *shape;  /* host: tt_conv_shape or tt_gemm_shape                           */
    void *bufs[5];      /* device                                                         */
    void *ws;           /* device workspace for split-K records, may be NULL              */
    size_t ws_bytes;
    void *const *alt_bufs;
    int32_t n_alt;
} tt_kernel_desc;

typedef struct tt_sweep_opts {
    int32_t warmup;               /* untimed launches per pair (default 3)                              */
    int32_t samples;              /* timed samples per pair, the median is kept (default 10)            */
    int32_t min_sample_us;        /* launches per sample are chosen so a sample lasts this long (200)   */
    int32_t max_launches;         /* cap on launches per sample (default 64)                            */
    int32_t flags;                /* TT_STRICT_DIVISIBLE                                                */
    int32_t allow_slower_than_default; /* 1: keep the best donor even if the default is faster         */
    /* Cheaper sweeps over a large pool (Section 5.5: "sampling a subset of schedules"; Section 4.4.2:
     * "prioritize kernel classes by the potential improvement"); see tt_sweep_plan for the rule. */
    int32_t pair_budget;          /* 0: every same-class pair; > 0: at most this many donor evaluations */
    int32_t prioritise;           /* 1: spend the budget on the kernels with the largest share of the
                                     untuned time first; 0: sample the pairs uniformly                  */
    uint64_t seed;                /* seed of the sampling                                               */
} tt_sweep_opts;

typedef struct tt_sweep_row {
    int32_t kernel;
    int32_t chosen;      /* index into the pool, -1 = the default schedule */
    int32_t n_valid, n_invalid, n_other_class;
    int32_t n_not_tried; /* same-class pairs a pair budget left out */
    double best_us, default_us;
} tt_sweep_row;

/*
 * The transfer-tuning sweep (Section 4.3).  For each of the nk target kernels:
 * time the default schedule, then every pool record of the kernel's class;
 * records that do not apply are recorded as -1 and skipped; the fastest wins,
 * the default is the fallback and wins ties, equal donors go to the lowest
 * index.  With opts->pair_budget > 0 every default is timed first and only the pairs
 * tt_sweep_plan selects (weights = default time x use count) are tried.  rows (host, nk).  pair_us
 * (host, nk * np doubles, may be NULL): median microseconds per launch, -1 for an invalid pair, -2 for
 * a record of another class, -3 for a pair the budget left out.  evaluations (host, may be NULL): number of timed pairs,
 * sum_k (1 + same-class records).  wall_seconds (host, may be NULL): wall-clock of
 * the call, the paper's "search time".  Synchronises `stream`.
 */
int tt_transfer_sweep(const tt_kernel_desc *kernels, int nk, const tt_schedule *pool, int np,
                      const tt_sweep_opts *opts, void *stream, tt_sweep_row *rows, double *pair_us,
                      int64_t *evaluations, double *wall_seconds);

/*
 * Which (kernel, donor) pairs a budgeted sweep evaluates; host only, a pure function of its arguments.
 * The paper leaves the sampling open ("randomly or using some other selection heuristic", Section 5.5);
 * this library's rule: every same-class pair (k, p) gets the 64-bit key splitmix64(seed + k * np + p + 1)
 * (Steele, Lea and Flood's SplitMix64 finaliser applied to that counter).
 *   prioritise = 0: the `pair_budget` pairs with the smallest keys are evaluated (ties: lower k * np + p),
 *                   a uniform sample without replacement;
 *   prioritise = 1: kernels are visited by decreasing weight[k] (its untuned time times its use count;
 *                   ties: lower k); each takes all its same-class pairs while the budget lasts, the
 *                   kernel the budget runs out on takes its pairs with the smallest keys.
 * pair_budget <= 0 or not below the number of same-class pairs selects them all.  mask (nk * np bytes):
 * 1 = evaluate.  *selected (may be NULL) receives the count.  weight may be NULL when prioritise = 0.
 */
int tt_sweep_plan(const int32_t *kernel_cls, const double *weight, int nk, const int32_t *pool_cls, int np,
                  int pair_budget, int prioritise, uint64_t seed, uint8_t *mask, int64_t *selected);

/*
 * The neighbourhood of a record for local refinement of a transferred schedule (the paper's outlook,
 * Section 6: "vary parameters from schedules transfer-tuned from another model"): every well-formed
 * record that differs from `base` in exactly one knob by one step: a tile, wave or K factor doubled or
 * halved, the other matrix-core block, the neighbouring entries of the split list {1, 2, 3, 4, 6, 8, 12,
 * 16, 32}, any other workgroup order, one stage more or fewer, unrolling on or off (8 / 1), the vector
 * width doubled or halved.  Writes up to cap records to out (host), returns the count (cap = 0 to size).
 * Only TT_SK_MFMA and TT_SK_DWCONV records have neighbours.
 */
int tt_refine_space(const tt_schedule *base, tt_schedule *out, int cap);

/*
 * Local refinement: time `base` and its neighbourhood on the kernel (standalone protocol of `opts`), move
 * to the fastest, repeat up to `rounds` times or until no neighbour is faster.  best / best_us: the
 * record reached and its time; base_us: the time of `base`; tried: number of timed pairs.  A base that
 * does not apply to the kernel is the apply status and nothing is launched.  Synchronises `stream`.
 */
int tt_refine(const tt_kernel_desc *kernel, const tt_schedule *base, int rounds, const tt_sweep_opts *opts,
              void *stream, tt_schedule *best, double *best_us, double *base_us, int32_t *tried);

/*
 * The exhaustive native sweep of ONE kernel (the stand-in for full auto-scheduling, Sections 3 and
 * 5.2): walk tt_schedule_space(cls, dtype, level) with the `explore` protocol, re-try the `finalists`
 * fastest records under every workgroup order and both unroll settings, then time the `finalists`
 * fastest of those and the default with the `full` protocol.  best: the winner (the default record if
 * nothing beats it); n_valid / n_records: records that applied / size of the space.  NULL option
 * pointers select 1 / 3 / 60 us / 16 for explore and the defaults of tt_sweep_opts for full.
 */
int tt_native_sweep(const tt_kernel_desc *kernel, int level, int finalists, const tt_sweep_opts *explore,
                    const tt_sweep_opts *full, void *stream, tt_schedule *best, double *best_us,
                    double *default_us, int32_t *n_valid, int32_t *n_records);

/*
 * Time ONE (kernel, schedule) pair standalone with the sweep's protocol (warm-up,
 * median of samples of back-to-back launches, HIP events on `stream`).
 * sched NULL = default.  median_us / min_us: host.  Returns the apply status
 * (then nothing was launched) or a launch error.
 */
int tt_time_pair(const tt_kernel_desc *kernel, const tt_schedule *sched, const tt_sweep_opts *opts,
                 void *stream, double *median_us, double *min_us);

/*
 * Enqueue a list of kernels back to back on `stream`: kernel i runs use_count times under
 * scheds[i] (NULL entry or NULL array = default schedule), and the whole list runs `repeat` times
 * (a network-shaped pass under the schedules a sweep chose, Section 4.3).  Does not synchronise.
 * Stops at the first error and returns it.
 */
int tt_run_kernels(const tt_kernel_desc *kernels, const tt_schedule *const *scheds, int nk, int repeat,
                   void *stream);

/*
 * Enumerate the schedule space of a class for a data type: every compiled
 * kernel variant crossed with the run-time knobs (split_k, order, stages, vec,
 * unroll).  Writes up to `cap` records to out (host) and returns the total
 * count (call with cap = 0 to size the buffer).  The exhaustive "native" sweep
 * of a kernel is tt_transfer_sweep over this pool.
 */
int tt_schedule_space(int cls, int dtype, int level, tt_schedule *out, int cap);

/*
 * Template arguments of a compiled matrix-core kernel variant (tt_plan.variant_id), and what the
 * kernel itself reports about its use of the chip: out[12] =
 * {dtype, family (0 conv, 1 GEMM with [N][K] B, 2 GEMM with [K][N] B), tile_m, tile_n, tile_k, wave_m,
 * wave_n, mfma, bytes per gathered load (conv family; 0 otherwise), pipeline (0 register-staged,
 * symbol contract_kernel with the first nine arguments; 1 asynchronous ring, symbol
 * contract_async_kernel with the first eight; 2 the 3x3 convolution kernel with the padded input patch
 * in LDS, symbol conv3x3_patch_kernel), LDS bytes of one pipeline stage (pipeline 2: the pixels one patch
 * buffer holds), reduction elements one matrix-core step consumes (tile_k is a multiple of it)}.
 * TT_ERR_BAD_ARG for an id outside the table.
 */
int tt_variant_info(int variant_id, int32_t out[12]);
/* Number of compiled variants: ids 0 .. tt_num_variants() - 1. */
int tt_num_variants(void);

/*
 * Which pre-tuned model to take the donor schedules from (Section 4.4.2, Eq. 1): for every candidate
 * model T the score is the sum over the target's kernel classes c of P_c^2 * sqrt(|W_Tc|), where P_c is
 * the share of class c in the target's untuned time and |W_Tc| the number of tuned kernels of that class
 * model T offers.  class_cost[num_classes] holds the target's untuned time per class in any unit (it is
 * normalised to shares here; all zero is TT_ERR_BAD_ARG); donor_class_count is [n_donors][num_classes],
 * row-major, entries >= 0.  scores[n_donors] (may be NULL) receives every score; *best the index of the
 * highest one, the lowest index winning ties, or -1 when n_donors is 0.  Host only.
 */
int tt_select_donor(const double *class_cost, int num_classes, const int32_t *donor_class_count, int n_donors,
                    double *scores, int32_t *best);

/* Pure selection step of the sweep on given times (host only; the rule tt_transfer_sweep uses). */
int tt_sweep_select(const int32_t *kernel_cls, int nk, const int32_t *pool_cls, int np, const double *pair_us,
                    const double *default_us, int allow_slower_than_default, tt_sweep_row *rows);

#ifdef __cplusplus
}
#endif
#endif /* TT_H */
