/*
 * kfac.h - C ABI of the MI355X (gfx950) K-FAC work-item library.
 *
 * The three work items are the ones PipeFisher (arXiv 2211.14133, section
 * 2.3.1 "Work in K-FAC") assigns to pipeline bubbles, per linear layer:
 *
 *   curvature     A = <a a^T>, B = <e e^T> over the tokens of a micro-batch,
 *                 accumulated over the micro-batches of a mini-batch
 *   inversion     (factor + damping I)^-1 through a Cholesky decomposition
 *   precondition  B^-1 G A^-1 for the layer's weight gradient G
 *
 * Each call is one work item (one factor and micro-batch, one factor, one
 * layer), so a scheduler can place them one at a time (section 3.1); the
 * *_grouped / *_batched forms run many independent items in one go and give
 * item by item the same result.
 *
 * Conventions for every entry point
 *  - All matrix pointers are DEVICE pointers; matrices are row-major float32
 *    (the paper computes everything in fp32) unless a dtype argument says
 *    otherwise.  Leading dimensions (ld*) count elements between rows.
 *  - Ownership: every buffer, the workspace included, belongs to the caller.
 *    The library allocates no device memory and keeps no pointer after a call
 *    returns (the one exception, the host-side plan of the chunked inversion,
 *    is described with it).  On the host, the inversion and precondition calls
 *    use a few KB to a few hundred KB of C++ heap for their bookkeeping while
 *    they run (lists of launches and tasks), freed before they return.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is only enqueued; no call synchronises with the host.
 *  - `workspace` is device scratch of at least the size the matching
 *    *_workspace() query returns (0 is a valid answer: then NULL is accepted).
 *    It must be 256-byte aligned and may be reused by the next call on the same
 *    stream.
 *  - Errors that can be seen on the host (null pointers, non-positive sizes,
 *    ld smaller than the row length, workspace too small, unsupported dtype)
 *    are returned as a status before anything is enqueued.  Numerical failure
 *    of an inversion is reported through the device word `info_dev`.
 *  - Item arrays of the grouped forms are HOST arrays, read during the call.
 */
#ifndef KFAC_H
#define KFAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KFAC_OK = 0,
    KFAC_ERR_ARG = 1,         /* null pointer, bad size or leading dimension */
    KFAC_ERR_UNSUPPORTED = 2, /* dtype / option not implemented */
    KFAC_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small */
    KFAC_ERR_HIP = 4          /* a HIP launch reported an error */
} kfac_status;

typedef enum {
    KFAC_F32 = 0, /* float32 activations / errors */
    KFAC_BF16 = 1, /* bfloat16 activations / errors, fp32 accumulation */
    /* float32 activations / errors, each value taken as the sum of three bfloat16 terms and each product as the
     * six bf16 MFMA products that reach 2^-16 of it (the rest is below the rounding of one float32 operation),
     * fp32 accumulation; curvature only.  Launches too small for this path are computed as KFAC_F32. */
    KFAC_F32_BF16X3 = 2,
    /* float32 activations / errors, each tensor scaled by a power of two so that its largest magnitude lies in
     * [2^14, 2^15), each value then taken as the sum of two float16 terms and each product as the three f16 MFMA
     * products that reach 2^-11 of it, fp32 accumulation; curvature only.  Elements below 2^-28 of the tensor's
     * largest lose relative (not absolute) accuracy.  Launches too small for this path are computed as KFAC_F32. */
    KFAC_F32_F16X2 = 3
} kfac_dtype;

/* ---------------------------------------------------------------- curvature
 * Section 2.3 (definition of A_l, B_l) and 2.3.1 (A = U_A U_A^T with U_A the
 * per-example vectors side by side over sqrt(|B|)):
 *
 *     factor = beta * factor + alpha * x^T x
 *
 * x       [n_tokens, d] row-major, leading dimension ldx >= d; every token row
 *         is one example.  Activations for A, output errors for B.
 * factor  [d, d] float32, leading dimension ldf >= d, read (if beta != 0) and
 *         written in full: both triangles are stored and are bitwise equal.
 * alpha   1 / (tokens in the whole mini-batch); beta = 0 for the first
 *         micro-batch of a refresh, 1 for the following ones.
 * The sum over tokens is accumulated in fp32 in short chunks that are then
 * added up, so the rounding error does not grow with n_tokens (float32 input;
 * the bfloat16 variant keeps one fp32 accumulation level per call).
 * bfloat16 input is first repacked into the workspace (its size is part of
 * what the workspace query returns).  KFAC_F32_BF16X3 takes float32 input,
 * writes its three bfloat16 terms into the workspace (6 bytes per element) and
 * accumulates the six bf16 MFMA products of every product in fp32, the five
 * small ones before the large one, 8192 tokens at a time; KFAC_F32_F16X2
 * likewise with two float16 terms (4 bytes per element and one word per item)
 * and three products.  Non-finite inputs give NaN in both.  Limits: sizes must fit in 31 bits;
 * d <= 2^26 for bfloat16 input (KFAC_ERR_UNSUPPORTED beyond).
 */
kfac_status kfac_curvature(const void *x, kfac_dtype dtype, int64_t n_tokens, int64_t d, int64_t ldx,
                           float alpha, float beta, float *factor, int64_t ldf,
                           void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_curvature_workspace(int64_t n_tokens, int64_t d, kfac_dtype dtype);

typedef struct {
    const void *x;    /* device, [n_tokens, d] */
    int64_t n_tokens;
    int64_t d;
    int64_t ldx;
    float *factor;    /* device, [d, d] */
    int64_t ldf;
} kfac_curvature_item;

/* `count` independent curvature items (e.g. both factors of every layer of a
 * stage for one micro-batch) with a common alpha, beta and dtype. */
kfac_status kfac_curvature_grouped(const kfac_curvature_item *items, int64_t count, kfac_dtype dtype,
                                   float alpha, float beta,
                                   void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_curvature_grouped_workspace(const kfac_curvature_item *items, int64_t count, kfac_dtype dtype);

/* ---------------------------------------------------------------- inversion
 * Section 2.3.1: each Kronecker factor is symmetric, so its inverse is taken
 * through a Cholesky decomposition and the inverse from the Cholesky factor.
 * The damping term is this library's addition (the paper does not spell one
 * out): it is added to the diagonal of the factor before the decomposition.
 *
 *     inv = (factor + damping I)^-1
 *
 * factor    [d, d] float32, ldf >= d; only its upper triangle (j >= i) is read.
 * inv       [d, d] float32, ldi >= d; written in full (both triangles, bitwise
 *           symmetric), and only by the last kernel of the call, so an inverse
 *           from an earlier refresh stays usable until then (section 2.3.1:
 *           precondition runs with stale inverses).  Must not overlap factor.
 * info_dev  device int32, written by the call: 0 success; k > 0 the k-th pivot
 *           of the decomposition was not positive (matrix not positive
 *           definite); -1 the input held a non-finite value.  When it is not 0
 *           `inv` is left untouched.
 * Limit: d <= 32640 (255 panels of 128; KFAC_ERR_UNSUPPORTED beyond).
 */
kfac_status kfac_invert(const float *factor, int64_t d, int64_t ldf, float damping,
                        float *inv, int64_t ldi, int32_t *info_dev,
                        void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_invert_workspace(int64_t d);

typedef struct {
    const float *factor; /* device, [d, d] */
    int64_t d;
    int64_t ldf;
    float *inv;          /* device, [d, d] */
    int64_t ldi;
    int32_t *info_dev;   /* device, one word per item */
} kfac_invert_item;

/* `count` independent inversions (e.g. every factor of a stage) advanced
 * together, one panel step of all matrices per launch. */
kfac_status kfac_invert_batched(const kfac_invert_item *items, int64_t count, float damping,
                                void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_invert_batched_workspace(const kfac_invert_item *items, int64_t count);

/* ------------------------------------------------------ chunked inversion
 * Section 3.1 assigns work to bubbles only if it fits, and section 5 notes
 * that the work for a single matrix has to be divisible to use bubbles well.
 * A plan is the fixed sequence of kernel launches of one kfac_invert_batched
 * call, recorded once; a scheduler runs it a few launches at a time, in
 * order, on any stream, between other work.  Running all steps is exactly
 * kfac_invert_batched.  `inv` buffers are written by the last steps only.
 *
 * The plan lives in host memory obtained from the C++ heap (about 4 KB per
 * step: the launch descriptors; the library never allocates device memory).  It keeps
 * the device pointers of `items` and of `workspace`: those must stay valid,
 * and the workspace must not be used by anything else, until the plan has
 * run to its end.  A plan can be reset and run again (next refresh).
 */
typedef struct kfac_invert_plan kfac_invert_plan;

kfac_status kfac_invert_plan_create(const kfac_invert_item *items, int64_t count, float damping,
                                    void *workspace, size_t workspace_bytes, kfac_invert_plan **plan);
/* number of steps (one step = one kernel launch, at most two) */
int64_t kfac_invert_plan_steps(const kfac_invert_plan *plan);
/* index of the next step to run */
int64_t kfac_invert_plan_position(const kfac_invert_plan *plan);
/* model cost of a step in floating point operations (0 for copies, -1 for a bad index) */
double kfac_invert_plan_step_flops(const kfac_invert_plan *plan, int64_t step);
/* what a step does, as a short static string such as "panel solve" (NULL for a bad index) */
const char *kfac_invert_plan_step_label(const kfac_invert_plan *plan, int64_t step);
/* enqueue the next n_steps steps (fewer if the end is reached) on `stream` */
kfac_status kfac_invert_plan_run(kfac_invert_plan *plan, int64_t n_steps, void *stream);
kfac_status kfac_invert_plan_reset(kfac_invert_plan *plan);
void kfac_invert_plan_destroy(kfac_invert_plan *plan);

/* ---------------------------------------- inversion without a workspace argument
 * For callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same computation and result as kfac_invert (bit for bit: the same
 * kernels), with the working arrays in a 32 MiB array that is part of the
 * library's code object instead of a caller workspace.
 *
 *  - d <= kfac_invert_noalloc_max_d() (2048); larger d returns
 *    KFAC_ERR_UNSUPPORTED and nothing is enqueued.  All other argument rules,
 *    info_dev and the "inv untouched on failure" rule are those of kfac_invert.
 *  - The call allocates and frees nothing on the device (no hipMalloc / hipFree,
 *    no allocating library routine); every GPU that runs the library holds its
 *    own copy of the array from the moment the library is loaded until the
 *    process ends.
 *  - The device that `stream` belongs to must be the current device.  The
 *    array's address on a device is looked up on the first call made there
 *    (KFAC_ERR_HIP if that fails).
 *  - All calls on one GPU share that GPU's array: two calls whose work overlaps
 *    in time (different streams, or one stream per thread) race.  Calls on one
 *    stream are ordered and safe.  The array keeps the last call's contents; the
 *    kernels write every element before they read it, so nothing is cleared.
 */
kfac_status kfac_invert_noalloc(const float *factor, int64_t d, int64_t ldf, float damping,
                                float *inv, int64_t ldi, int32_t *info_dev, void *stream);
int64_t kfac_invert_noalloc_max_d(void);

/* ------------------------------------------------------------- precondition
 * Section 2.3.1: (A (x) B)^-1 vec(G) = vec(B^-1 G A^-1), vec stacking columns.
 *
 *     out = b_inv * grad * a_inv
 *
 * b_inv  [d_out, d_out], ldb >= d_out; a_inv [d_in, d_in], lda >= d_in: the
 *        inverses written by kfac_invert (symmetric; the kernels rely on it).
 * grad   [d_out, d_in], ldg >= d_in: the weight gradient in PyTorch's layout.
 * out    [d_out, d_in], ldo >= d_in.  out may be the same buffer as grad.
 */
kfac_status kfac_precondition(const float *b_inv, int64_t d_out, int64_t ldb,
                              const float *a_inv, int64_t d_in, int64_t lda,
                              const float *grad, int64_t ldg, float *out, int64_t ldo,
                              void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_precondition_workspace(int64_t d_out, int64_t d_in);

typedef struct {
    const float *b_inv;
    int64_t d_out;
    int64_t ldb;
    const float *a_inv;
    int64_t d_in;
    int64_t lda;
    const float *grad;
    int64_t ldg;
    float *out;
    int64_t ldo;
} kfac_precondition_item;

/* `count` independent layers in two launches (all left products, then all
 * right products). */
kfac_status kfac_precondition_grouped(const kfac_precondition_item *items, int64_t count,
                                      void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_precondition_grouped_workspace(const kfac_precondition_item *items, int64_t count);

/* The same on the f16 matrix core (the method's un-hidden step, section 3.1, made shorter): each of the four
 * operands (G, B^-1; then T^T, A^-1) is scaled by a power of two from its largest magnitude and taken as two
 * float16 terms, each product as three f16 MFMA products, fp32 accumulation (see KFAC_F32_F16X2).  Same
 * arguments, results to the same tolerance; the workspace is larger (T^T, and 4 bytes per element of every
 * operand).  out must not alias the inputs.  Non-finite inputs give NaN.  Errors as for
 * kfac_precondition_grouped; KFAC_ERR_UNSUPPORTED for d_out or d_in above 2^26. */
kfac_status kfac_precondition_grouped_f16x2(const kfac_precondition_item *items, int64_t count,
                                            void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_precondition_grouped_f16x2_workspace(const kfac_precondition_item *items, int64_t count);

/* The inverses only change when they are refreshed (every few steps under the schedule of section 3.1), the
 * gradient every step: their float16 planes can be made once per refresh and used by every precondition until
 * the next.  kfac_precondition_f16x2_prepare reads b_inv and a_inv of every item (grad and out are ignored) and
 * fills `prepared` (device memory of the caller, kfac_precondition_f16x2_prepared_bytes, 256-byte aligned);
 * kfac_precondition_grouped_f16x2_prepared then computes what kfac_precondition_grouped_f16x2 computes, bit for
 * bit, from `prepared` (made for the same items in the same order), grad and out; its workspace is smaller
 * (kfac_precondition_grouped_f16x2_prepared_workspace).  `prepared` is only read by it.  KFAC_ERR_WORKSPACE also
 * when `prepared` is null, not 256-byte aligned or smaller than kfac_precondition_f16x2_prepared_bytes says. */
kfac_status kfac_precondition_f16x2_prepare(const kfac_precondition_item *items, int64_t count,
                                            void *prepared, size_t prepared_bytes, void *stream);
size_t kfac_precondition_f16x2_prepared_bytes(const kfac_precondition_item *items, int64_t count);
kfac_status kfac_precondition_grouped_f16x2_prepared(const kfac_precondition_item *items, int64_t count,
                                                     const void *prepared, size_t prepared_bytes,
                                                     void *workspace, size_t workspace_bytes, void *stream);
size_t kfac_precondition_grouped_f16x2_prepared_workspace(const kfac_precondition_item *items, int64_t count);

/* ------------------------------------------- bubble filling (host side only)
 * Section 3.1 "Automatic Work Assignments": K-FAC work is taken from a queue
 * and put into the first pipeline bubble that is long enough and lies after the
 * work it depends on; bubbles of later pipeline steps are used when the
 * current ones are full; the result is a static schedule that is repeated.
 *
 * One pipeline step of one device is described by its bubbles (idle
 * intervals, relative to the start of the step, sorted, not overlapping) and
 * the step period (start-to-start time of consecutive steps, precondition
 * included: rule 3 puts it after the last backward pass, outside the bubbles).
 * Work w consists of chunk_count[w] indivisible chunks (durations in
 * chunk_time, concatenated in work order), becomes available at release[w]
 * (time in step 0, e.g. the end of the forward pass of its micro-batch: rule 1)
 * and after every work listed in dep_ids[dep_begin[w] .. dep_begin[w+1])
 * (rule 2: an inversion after all its curvature work; ids must be smaller
 * than w).  Works are placed in index order, chunk by chunk, first fit along
 * the time line: a chunk goes into the first idle interval that starts no
 * earlier than the chunk may and can hold it.  Idle intervals are the bubbles
 * minus what has been placed, so a hole that a later-released chunk left in
 * front of itself is used by a later chunk of the queue that fits (the paper
 * says nothing about such holes; this reading uses the bubbles best).
 *
 * Outputs, one entry per chunk in the same order as chunk_time: the pipeline
 * step (0, 1, ...) and bubble index it went to and its start time relative to
 * that step's start.  *steps_needed receives the number of pipeline steps the
 * whole queue takes (the refresh interval of section 3.1).
 * Returns KFAC_ERR_ARG for malformed input and KFAC_ERR_UNSUPPORTED if a chunk
 * is longer than every bubble (the work has to be cut finer).
 */
kfac_status kfac_assign_work(int64_t n_bubbles, const double *bubble_start, const double *bubble_length,
                             double step_period,
                             int64_t n_works, const int64_t *chunk_count, const double *chunk_time,
                             const double *release, const int64_t *dep_begin, const int64_t *dep_ids,
                             int64_t *out_step, int64_t *out_bubble, double *out_start,
                             int64_t *steps_needed);

/* One pipeline step of GPipe seen from one stage (section 2.1: every forward pass
 * of the step, then every backward pass; t_f, t_b per micro-batch and stage,
 * stages numbered from 0 in forward direction).  Gives what kfac_assign_work
 * needs: forward_end[m] and backward_end[m] (release times of the curvature
 * work of micro-batch m under rule 1; n_micro entries each), the bubbles of
 * the stage (at most 3: before the first forward pass, between the forward and
 * the backward passes, after the last backward pass; caller provides room for
 * 3 starts and 3 lengths) and the length of the step.  Host arrays.
 * KFAC_ERR_ARG for null pointers, stage outside [0, depth), non-positive
 * sizes or times. */
kfac_status kfac_gpipe_stage(int64_t stage, int64_t depth, int64_t n_micro, double t_f, double t_b,
                             double *forward_end, double *backward_end,
                             double *bubble_start, double *bubble_length, int64_t *n_bubbles, double *t_step);

/* Section 3.3 "Performance Modeling", closed forms for one pipeline step:
 *   t_pipe   = c_f * t_f + c_b * t_b
 *   t_bubble = t_pipe - n_micro * (t_f + t_b)
 *   t_kfac   = n_micro * t_curv + t_inv + t_prec
 *   ratio    = (n_micro * t_curv + t_inv) / t_bubble     (steps per refresh)
 * c_f, c_b: forward / backward passes on the critical path of the schedule.
 * out[0..4] = t_pipe, t_bubble, t_kfac, ratio, step time with bubble filling
 * (t_pipe + t_prec).
 */
kfac_status kfac_perf_model(double c_f, double c_b, double t_f, double t_b, int64_t n_micro,
                            double t_curv, double t_inv, double t_prec, double *out);

/* ------------------------------------------------------------------- misc */
const char *kfac_status_string(kfac_status status);

/* Measurement aid (not a step of the method): enqueues a kernel whose waves do nothing but
 * matrix-core instructions on registers, so that a caller can time what the matrix cores of this
 * chip sustain and report a kernel against that ceiling as well as against the published peak.
 *   dtype     KFAC_F32: MFMA 32x32x2 (4096 flops each); KFAC_BF16: MFMA 32x32x16 (32768 flops each)
 *   iters     loop iterations per wave (> 0); each iteration issues 8 independent MFMAs
 *   sink      device buffer of at least 256 bytes, caller-owned (in practice never written)
 *   flops     host pointer; receives the floating-point operations the launch performs
 * The launch is asynchronous on `stream`.  Errors: KFAC_ERR_ARG for null pointers, iters <= 0 or an
 * unknown dtype; KFAC_ERR_HIP if the launch fails. */
kfac_status kfac_mfma_probe(kfac_dtype dtype, int64_t iters, void *sink, double *flops, void *stream);
/* The same with a choice of operand data.  random_operands = 0: constant operands, as kfac_mfma_probe;
 * otherwise operands with random sign and mantissa bits, four sets in rotation (iters is rounded up to a
 * multiple of 4): what the matrix cores sustain when their inputs toggle as real data does, which on this
 * chip is less, because it lowers its clock under the higher power draw. */
kfac_status kfac_mfma_probe_data(kfac_dtype dtype, int random_operands, int64_t iters, void *sink, double *flops,
                                 void *stream);

/* Library version as major * 10000 + minor * 100 + patch. */
int kfac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H */
