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
 *    The library allocates and frees nothing, keeps no pointer after the call
 *    returns and has no global state.
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
    KFAC_BF16 = 1 /* bfloat16 activations / errors, fp32 accumulation */
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
 * added up, so the rounding error does not grow with n_tokens.
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

/* ------------------------------------------------------------------- misc */
const char *kfac_status_string(kfac_status status);

/* Library version as major * 10000 + minor * 100 + patch. */
int kfac_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H */
