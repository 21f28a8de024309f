/*
 * dmath.h -- C ABI of the MI355X (gfx950) implementation of one worker's share of dMath's
 * block-distributed matrix multiply and of convolution lowered to an implicit GEMM.
 *
 * Objects (paper, section 2.1 "Managing Persistent Data in the GPUs"): a matrix is split into
 * non-overlapping dense blocks; the blocks live in GPU memory for the life of the matrix; all
 * GPU memory comes from a pool so that no driver allocation happens after start-up
 * (section 1, "pooling of unused GPU memory").  Precisions (section 1, feature d): double,
 * float, half; half values are widened to float for arithmetic (section 4.2).
 *
 * Conventions of every call
 *   - returns a dmath_status_t, never throws, never aborts; out-parameters are untouched on
 *     error;
 *   - "device pointer" = address in GPU memory, "host pointer" = ordinary process memory;
 *   - compute calls (dmath_gemm, dmath_conv_*) only enqueue work on the context's HIP stream
 *     and return; argument errors are reported at once, device faults at the next
 *     synchronising call (dmath_synchronize, dmath_matrix_get) as DMATH_ERR_DEVICE;
 *   - a context and its handles belong to one host thread.
 *
 * Block split rule: a dimension of length n cut into g parts gives part p the index range
 * [p*ceil(n/g), min(n,(p+1)*ceil(n/g))); a grid that would leave an empty trailing part is
 * refused (DMATH_ERR_LAYOUT).  Each block is its own pool allocation, dense row-major with
 * leading dimension equal to its own column count.
 */
#ifndef DMATH_H
#define DMATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dmath_ctx_s *dmath_ctx_t;       /* opaque, owned by the library */
typedef struct dmath_matrix_s *dmath_matrix_t; /* opaque, owned by its context */

typedef enum { DMATH_F64 = 0, DMATH_F32 = 1, DMATH_F16 = 2 } dmath_dtype_t;
typedef enum { DMATH_OP_N = 0, DMATH_OP_T = 1 } dmath_op_t;

typedef enum {
    DMATH_OK = 0,
    DMATH_ERR_INVALID_ARG = 1, /* null pointer, bad enum value, non-positive size            */
    DMATH_ERR_SHAPE = 2,       /* operand shapes do not fit the operation                     */
    DMATH_ERR_LAYOUT = 3,      /* block grid not allowed (empty trailing block, conv grids)   */
    DMATH_ERR_DTYPE = 4,       /* precision combination not supported                         */
    DMATH_ERR_ALIAS = 5,       /* output handle is also an input                              */
    DMATH_ERR_OOM = 6,         /* the pool cannot satisfy the request                         */
    DMATH_ERR_UNSUPPORTED = 7, /* valid in principle, not implemented (dilation, groups, ...) */
    DMATH_ERR_DEVICE = 8,      /* a HIP call failed                                           */
    DMATH_ERR_SCRATCH_LIMIT = 9 /* dmath_gemm_noalloc: the plan does not fit the fixed scratch array */
} dmath_status_t;

/*
 * Context.  `slab` is a device pointer to `slab_bytes` of GPU memory owned by the CALLER (for
 * example a torch uint8 tensor); the library sub-allocates every block, descriptor table and
 * workspace from it and never frees or reallocates it (section 1: the pool replaces driver
 * allocations).  `hip_stream` is the caller's hipStream_t (NULL = the default stream); all
 * device work of this context is enqueued on it.  dmath_init itself touches neither the slab
 * nor the device.  The slab must outlive the context.
 */
dmath_status_t dmath_init(dmath_ctx_t *ctx, void *slab, size_t slab_bytes, void *hip_stream);

/* Destroys every matrix and cached plan of the context, then the context. */
dmath_status_t dmath_finalize(dmath_ctx_t ctx);

/*
 * Creates a rows x cols matrix of `dtype` cut into a grid_rows x grid_cols grid of blocks
 * (section 2.1).  Contents are uninitialised.  DMATH_ERR_OOM if the pool is exhausted (nothing
 * is leaked in that case).
 */
dmath_status_t dmath_matrix_create(dmath_ctx_t ctx, int64_t rows, int64_t cols, int32_t grid_rows,
                                   int32_t grid_cols, dmath_dtype_t dtype, dmath_matrix_t *out);

/* Returns the blocks to the pool.  Reuse of that memory is ordered after work already enqueued
 * on the context's stream.  Cached plans that mention the matrix are dropped. */
dmath_status_t dmath_matrix_destroy(dmath_matrix_t m);

/*
 * Copies between a monolithic row-major HOST array (leading dimension ld_elems >= cols, in
 * elements of the matrix's dtype; fp16 as raw IEEE binary16 bits) and the blocks.  Both calls
 * run on the context's stream and return after the copy has completed.  Not part of the timed
 * path: operands are meant to stay resident (section 2.1).
 */
dmath_status_t dmath_matrix_set(dmath_matrix_t m, const void *host, int64_t ld_elems);
dmath_status_t dmath_matrix_get(dmath_matrix_t m, void *host, int64_t ld_elems);

/* Shape and grid of a matrix; any out-pointer may be NULL. */
dmath_status_t dmath_matrix_info(dmath_matrix_t m, int64_t *rows, int64_t *cols,
                                 int32_t *grid_rows, int32_t *grid_cols, dmath_dtype_t *dtype);

/* Device pointer, size and leading dimension (elements) of block (bi, bj).  The memory stays
 * owned by the matrix. */
dmath_status_t dmath_matrix_block(dmath_matrix_t m, int32_t bi, int32_t bj, void **dev_ptr,
                                  int64_t *rows, int64_t *cols, int64_t *ld);

/*
 * dst <- src element by element, for any two block grids and any two precisions (section 3.3:
 * "reshape (including a change of ... layout) ... and/or change precision during reshape").
 * Shapes must be equal (DMATH_ERR_SHAPE); src and dst must differ (DMATH_ERR_ALIAS).  Widening is
 * exact; narrowing rounds to nearest even in ONE step (also double -> half), overflow gives
 * +-Inf, NaN stays NaN.  Runs on the context's stream; asynchronous.
 */
dmath_status_t dmath_matrix_reblock(dmath_ctx_t ctx, dmath_matrix_t src, dmath_matrix_t dst);

/*
 * C <- alpha * op(A) * op(B) + beta * C            (abstract: "matrix multiplication";
 * section 1: the back-propagation variants dW = X^T dY (T,N) and dX = dY W^T (N,T))
 *
 * op(X) = X or X^T; a transposed operand is never physically transposed: block (i,k) of op(A)
 * is the transpose of stored block (k,i).  The three block grids are independent of one
 * another (section 3.2, data distribution independence): where partitions do not line up the
 * scheduler cuts tiles at every block boundary of every operand.
 *
 * Precisions: A and B share a dtype; C has the same dtype, except that F16 inputs may write an
 * F32 or an F16 C.  F16 products are exact and are accumulated in fp32, alpha/beta applied in
 * fp32, one final round-to-nearest-even when C is F16 (section 4.2, mixed mode).  F32 uses fp32
 * FMA, F64 fp64 FMA.  alpha and beta are narrowed to the accumulation type.
 * beta == 0: the old C is not read (NaNs in it do not propagate); alpha == 0: A and B are not
 * read.
 *
 * Errors: DMATH_ERR_SHAPE (inner/outer sizes differ), DMATH_ERR_DTYPE, DMATH_ERR_ALIAS (C is
 * A or B), DMATH_ERR_INVALID_ARG (handles of different contexts, bad op), DMATH_ERR_OOM (no
 * room for the plan tables or a split-K workspace).
 * Results are bitwise reproducible from run to run (split-K partial sums are reduced in a
 * fixed order).
 */
dmath_status_t dmath_gemm(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB, double alpha,
                          dmath_matrix_t A, dmath_matrix_t B, double beta, dmath_matrix_t C);

/* What the scheduler decided for a GEMM: filled by dmath_gemm_plan_info without enqueuing
 * anything (host logic only; usable without a GPU). */
typedef struct {
    int64_t m, n, k;
    int32_t m_segments, n_segments, k_segments; /* after refining against every operand's grid */
    int32_t tile_m, tile_n, tile_k;
    int32_t tiles;    /* C tiles                                                       */
    int32_t split_k;  /* partial sums per C tile (1 = none)                            */
    int32_t kernel;   /* 0 = guarded generic kernel, >0 = a specialised kernel id      */
    int32_t cached;   /* 1 if the plan was already in the cache                        */
    int32_t split_tiles; /* C tiles that take partial sums: 0, all of them, or only those
                            left over after the last full round of workgroups            */
    uint64_t workspace_bytes; /* pool memory beyond the operands: split-K partial sums and the
                                 zero-padded scratch panels of k-segments that are not
                                 multiples of tile_k */
} dmath_plan_info_t;

/*
 * dmath_gemm for callers that cannot allocate: code whose stream is under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same arguments, result, status codes
 * and asynchrony as dmath_gemm, but the call takes nothing from the context's pool and makes no
 * driver allocation: what its kernels need beyond the operands (descriptor tables, partial sums
 * of a split k-loop, zero-padded panels of k-tails) lies in a static device array of
 * DMATH_NOALLOC_SCRATCH_BYTES that every GPU running the library holds from the first such call
 * on it until the process ends.
 *   - The array holds ONE plan, the last call's.  A call with the same handles and ops as the
 *     one before it only launches kernels; any other call rewrites the array first, which copies
 *     tables from host memory and waits for the context's stream -- so make the first call for
 *     a set of operands outside stream capture, and do not replay a captured call after the
 *     array has been rewritten.
 *   - All contexts on one GPU share that GPU's array; calls that overlap on one GPU (different
 *     streams) race.  The device that is current at the call is the one whose array is used.
 *   - As with dmath_gemm and a full pool, memory decides: partial sums that do not fit make
 *     the same kernel run unsplit, k-tail panels that do not fit the generic kernel.
 * Errors: those of dmath_gemm; DMATH_ERR_SCRATCH_LIMIT if even the descriptor tables exceed the
 * array (very fine block grids); DMATH_ERR_UNSUPPORTED between dmath_pipeline_begin and _end.
 */
#define DMATH_NOALLOC_SCRATCH_BYTES (32u << 20)
dmath_status_t dmath_gemm_noalloc(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB, double alpha,
                                  dmath_matrix_t A, dmath_matrix_t B, double beta, dmath_matrix_t C);

/* Builds (or finds in the cache) the plan dmath_gemm would use and describes it.  Same
 * argument checks and errors as dmath_gemm.  Section 3.3: the metadata of an operation is
 * computed once and remembered. */
dmath_status_t dmath_gemm_plan_info(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB,
                                    dmath_matrix_t A, dmath_matrix_t B, dmath_matrix_t C,
                                    dmath_plan_info_t *info);

/*
 * Convolution as an implicit GEMM (abstract: "convolutions"; never materialises the lowered
 * matrix).  Tensors are matrices in the blob view of the Caffe family (section 4): each row is
 * one image or one filter, NCHW inside the row:
 *     X, dX : [n x c*h*w]      F, dF : [k x c*r*s]      Y, dY : [n x k*oh*ow]
 * with oh = (h + 2*pad_h - r)/stride_h + 1, ow likewise.  Cross-correlation, no filter flip:
 *     Y[n,k,oh,ow] = sum_{c,r,s} X[n,c,oh*stride_h+r-pad_h, ow*stride_w+s-pad_w] * F[k,c,r,s]
 * with out-of-range input coordinates contributing zero.
 * Block grids: g x 1 (rows = images or filters split over blocks) for every tensor; a grid
 * with more than one block column is DMATH_ERR_LAYOUT.  Precisions and alpha/beta as in
 * dmath_gemm (F16 tensors may produce F32 or F16 results).
 */
typedef struct {
    int32_t n, c, h, w;     /* batch, input channels, input height and width */
    int32_t k, r, s;        /* output channels, filter height and width      */
    int32_t pad_h, pad_w, stride_h, stride_w;
} dmath_conv_desc_t;

/* Y <- alpha * conv(X, F) + beta * Y */
dmath_status_t dmath_conv_fwd(dmath_ctx_t ctx, const dmath_conv_desc_t *desc, double alpha,
                              dmath_matrix_t X, dmath_matrix_t F, double beta, dmath_matrix_t Y);

/* dF[k,c,r,s] <- alpha * sum_{n,oh,ow} dY[n,k,oh,ow] * X[n,c,oh*sh+r-ph,ow*sw+s-pw] + beta * dF
 * (weight gradient of back-propagation, section 1).  Uses a split-K workspace from the pool
 * with a fixed-order reduction. */
dmath_status_t dmath_conv_bwd_filter(dmath_ctx_t ctx, const dmath_conv_desc_t *desc, double alpha,
                                     dmath_matrix_t X, dmath_matrix_t dY, double beta,
                                     dmath_matrix_t dF);

/* dX[n,c,h,w] <- alpha * sum over (k,r,s,oh,ow) with oh*sh+r-ph == h and ow*sw+s-pw == w of
 * dY[n,k,oh,ow] * F[k,c,r,s] + beta * dX   (data gradient). */
dmath_status_t dmath_conv_bwd_data(dmath_ctx_t ctx, const dmath_conv_desc_t *desc, double alpha,
                                   dmath_matrix_t dY, dmath_matrix_t F, double beta,
                                   dmath_matrix_t dX);

/*
 * Pipeline replay (section 3.3: with fixed pipelines the workers "remember the entire forward
 * and backward computations", and one cached identifier replaces the per-operation metadata).
 *   dmath_pipeline_begin : from now on dmath_gemm / dmath_conv_* calls of this context are
 *                          recorded (HIP stream capture) instead of executed.  The context's
 *                          stream must not be the default (NULL) stream.
 *   dmath_pipeline_end   : stops recording and returns the identifier of the recorded sequence.
 *   dmath_pipeline_replay: enqueues the whole sequence with one launch; same results, same
 *                          order, on the same matrices (their contents are read at replay time).
 * Every operation that is recorded must have been executed once before on the same handles,
 * because building a plan copies tables and synchronises: otherwise the call returns
 * DMATH_ERR_UNSUPPORTED (and recording continues).  dmath_matrix_set/get/reblock/create/destroy
 * are refused while recording (DMATH_ERR_UNSUPPORTED).  Destroying a matrix that a pipeline
 * uses, or changing the kernel policy, destroys the pipeline: its identifier is then unknown
 * (DMATH_ERR_INVALID_ARG from replay and destroy).
 */
dmath_status_t dmath_pipeline_begin(dmath_ctx_t ctx);
dmath_status_t dmath_pipeline_end(dmath_ctx_t ctx, int32_t *pipeline_id);
dmath_status_t dmath_pipeline_replay(dmath_ctx_t ctx, int32_t pipeline_id);
dmath_status_t dmath_pipeline_destroy(dmath_ctx_t ctx, int32_t pipeline_id);

/*
 * Re-layout copies that are kept (section 1: the cache of shared objects, "keep what you've
 * seen", switched off where memory is the limit; section 3.3: data reorganised once for the
 * operations that follow).  The specialised convolution kernels read channels-last copies of
 * their activations and permuted copies of their filters, which live in the pool beside the
 * matrices.  A copy is reused, and its rewrite skipped, while the matrix it was made from has not
 * been written since: every library call that writes a matrix (set, reblock, the result of a
 * gemm or convolution, a replayed pipeline) marks it changed.  The activations copied for the
 * forward pass so serve the weight gradient of the same step, and a constant filter is permuted
 * once.  Results are bit-identical with and without reuse.
 *   dmath_set_relayout_reuse: 1 (default) reuse current copies, 0 rewrite them in every call
 *                             (the memory held is the same: the kernels need the copies).
 *   dmath_relayout_stats    : rewrites skipped / done so far, bytes of pool memory the copies hold.
 *                             Any output pointer may be NULL.
 *   dmath_matrix_touch      : declares that the matrix's elements changed without the library
 *                             seeing it.  A matrix whose block pointers were handed out by
 *                             dmath_matrix_block is treated as changed before every use.
 * Nothing is reused across dmath_pipeline_begin / _end / _replay; inside one recording a copy
 * made by a recorded call serves the recorded calls after it.
 */
dmath_status_t dmath_set_relayout_reuse(dmath_ctx_t ctx, int32_t enable);
dmath_status_t dmath_relayout_stats(dmath_ctx_t ctx, uint64_t *reused, uint64_t *written,
                                    size_t *bytes_held);
dmath_status_t dmath_matrix_touch(dmath_matrix_t m);

/*
 * Memory decides first: when the pool cannot hold what the preferred configuration needs beyond
 * the operands (split-K partial sums, re-layout copies), a gemm or convolution call falls back
 * to the configuration that needs none (same results within tolerance, slower) instead of
 * failing; DMATH_ERR_OOM is returned only if not even the plan's tables fit.
 *
 * Selection from timing samples (section 4.1: at start-up the library picks the convolution
 * algorithm from timing samples within the system's memory constraints).  Without tuning, the
 * kernel family, tile shape and split-K count come from a cost model.  The tuners time every
 * configuration the operation admits on the given handles (3 ms of warm-up launches, 20 ms before the first sample, then
 * `trials` launches between two events; the call blocks; a configuration replaces the cost
 * model's choice only if it is more than 2 % faster), leave out those that need more pool memory
 * beyond the operands than `workspace_limit` bytes (split-K partial sums; for convolutions also
 * the re-layout copies the specialised kernels read) or than the pool can give, and remember the
 * fastest under the operation's layout signature (ops, precisions, shapes, block grids,
 * convolution geometry): every later plan with that signature uses it, whichever matrices it is
 * built for.  The result matrix is overwritten (alpha = 1, beta = 0).  Results stay within the
 * same tolerances whatever is chosen (summation order may differ between configurations).
 *   dmath_conv_tune: mode 0 forward, 1 weight gradient, 2 data gradient; X, F, Y are the
 *     tensors in the shapes of dmath_conv_fwd (X or dX, F or dF, Y or dY).
 *   dmath_tune_reset: forgets every choice and drops all plans.
 * Errors: DMATH_ERR_UNSUPPORTED while recording or under kernel policy 1; DMATH_ERR_OOM if no
 * configuration fits; the argument errors of the operation itself.
 */
typedef struct dmath_tune_result {
    int32_t candidates;       /* configurations timed */
    int32_t skipped;          /* configurations left out for memory */
    int32_t kernel;           /* chosen: kernel family (0 generic; convolutions: 1 gathering
                                 MFMA kernels, 2 a 1x1 convolution run as a block GEMM), */
    int32_t tile_m, tile_n;   /*   tile shape, */
    int32_t split_k;          /*   split-K parts, */
    uint64_t workspace_bytes; /*   pool memory beyond the operands */
    double chosen_us;         /* time per call of the chosen configuration */
    double default_us;        /* time per call of the cost model's choice (0: it did not fit) */
} dmath_tune_result_t;

dmath_status_t dmath_gemm_tune(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB,
                               dmath_matrix_t A, dmath_matrix_t B, dmath_matrix_t C,
                               size_t workspace_limit, int32_t trials, dmath_tune_result_t *result);
dmath_status_t dmath_conv_tune(dmath_ctx_t ctx, int32_t mode, const dmath_conv_desc_t *desc,
                               dmath_matrix_t X, dmath_matrix_t F, dmath_matrix_t Y,
                               size_t workspace_limit, int32_t trials, dmath_tune_result_t *result);
dmath_status_t dmath_tune_reset(dmath_ctx_t ctx);

/* Kernel selection: 0 = automatic (specialised kernels where their preconditions hold),
 * 1 = always the guarded generic kernel (for testing and debugging).  Drops cached plans. */
dmath_status_t dmath_set_kernel_policy(dmath_ctx_t ctx, int32_t policy);

/* Waits for all work enqueued on the context's stream. */
dmath_status_t dmath_synchronize(dmath_ctx_t ctx);

/* Pool accounting in bytes: currently allocated, the maximum ever allocated, slab size; any
 * out-pointer may be NULL.  The number of driver allocations made by the library is zero. */
dmath_status_t dmath_pool_stats(dmath_ctx_t ctx, size_t *in_use, size_t *high_water,
                                size_t *capacity);

/* Static string naming a status code. */
const char *dmath_status_string(dmath_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* DMATH_H */
