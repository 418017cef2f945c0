/*
 * fira.h - C ABI of the MI355X (gfx950) Fira optimizer-step library.
 *
 * Fira ("Can We Achieve Full-rank Training of LLMs under Low-rank Constraint?", arXiv 2410.01623)
 * updates every weight matrix W (m x n) from its gradient G with Algorithm 1 ("Fira with Adam",
 * Appendix A.1).  With a projector P supplied by the caller the loop body is
 *
 *     R  = P^T G                         (Sec. 3.3; R = G Q when m > n, footnote of Sec. 3.3)
 *     M  = b1 M + (1-b1) R,  V = b2 V + (1-b2) R^2,
 *     N  = sqrt(1-b2^t)/(1-b1^t) * M / (sqrt(V) + eps)                      (Eqs. 2-4 on R)
 *     k_i = ||N[:,i]|| / (||R[:,i]|| + eps)                     (Eq. 11, norm-based scaling)
 *     S  = (G - P R) diag(k)                                                  (Sec. 4.1)
 *     S  = S * gamma / max(||S|| / (||S_prev|| + eps), gamma)   (Eq. 12, norm-growth limiter)
 *     W  = W - lr * alpha * (P N + S)                            (Algorithm 1, last two lines)
 *
 * When m > n the same algorithm runs on the transposed problem: one factor k_i per *row* of G,
 * reductions over the rank axis.  m == n is the m <= n case.
 *
 * Conventions
 *   - All `dev_*` pointers are DEVICE (HBM) pointers on the current HIP device; `host_*` pointers
 *     are host pointers.  The library never takes ownership of caller memory.
 *   - W and G are row-major m x n with leading dimension ld >= n (elements), dtype wg_dtype.
 *   - P is row-major min(m,n) x r (P when m <= n, Q when m > n), contiguous.
 *   - The caller allocates ONE device slab of fira_state_bytes() bytes per context; it holds the
 *     optimizer state (M, V, the library's operand copies of P, ||S_prev||, t) and the step's
 *     scratch.  It must stay alive and untouched until fira_destroy().
 *   - Every call enqueues on the HIP stream given to fira_init_state and, unless stated, returns
 *     without synchronising.  fira_step performs no device allocation.
 *   - Every function returns a fira_status (0 = OK, negative = error); errors detectable on the
 *     host are reported before anything is enqueued and leave the state untouched.
 *     fira_last_error() gives a message for the last failure (ctx may be NULL for failures of
 *     fira_init_state).  Non-finite inputs are not checked; they propagate: a non-finite gradient
 *     entry makes the state and the weights of its factor (its column; its row when m > n)
 *     non-finite for good, the limiter's factor is 1 on a step whose norm is not finite, and the other
 *     factors and the other matrices of the call are what they are without it.
 *   - Not thread-safe per context; two contexts are independent.
 */
#ifndef FIRA_H_
#define FIRA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FIRA_API __attribute__((visibility("default")))

typedef struct fira_ctx fira_ctx;

typedef enum {
  FIRA_OK = 0,
  FIRA_ERR_INVALID_ARG = -1,  /* null pointer, bad index, duplicate index, bad enum            */
  FIRA_ERR_SHAPE = -2,        /* m, n, ld, r out of range (need 1 <= r <= min(m,n), ld >= n)   */
  FIRA_ERR_NO_PROJECTOR = -3, /* fira_step on a matrix whose projector was never set            */
  FIRA_ERR_DTYPE = -4,        /* unsupported dtype combination                                  */
  FIRA_ERR_WORKSPACE = -5,    /* dev_state_bytes too small or slab misaligned (256 B)           */
  FIRA_ERR_HIP = -6           /* a HIP runtime call or kernel launch failed                     */
} fira_status;

typedef enum { FIRA_F32 = 0, FIRA_BF16 = 1 } fira_dtype;

/* Input line of Algorithm 1: eta, beta1, beta2, (Adam's) epsilon, GaLore scale alpha, limiter
 * threshold gamma.  gamma = +inf disables the limiter (the "w.o.-limiter" variant, Sec. 5.3). */
typedef struct {
  double lr, beta1, beta2, eps, alpha, gamma;
} fira_hparams;

/* One weight matrix.  wg_dtype is the storage type of W and G (fira_dtype). */
typedef struct {
  int64_t m, n, ld;
  int32_t r;
  int32_t wg_dtype;
} fira_matrix_desc;

/* Scaling-factor granularity: FIRA_SCALE_COLUMN is the paper's Fira (one factor per column, Eq. 11);
 * FIRA_SCALE_MATRIX uses one factor ||N|| / (||R|| + eps) for the whole matrix (Eqs. 9-10, the
 * "Fira-matrix" variant of Sec. 5.3); FIRA_SCALE_NONE sets every factor to 1 (the "GaLore-add" update
 * of Eq. 8 / "Fira-w.o.-scaling" of Sec. 5.3). */
typedef enum { FIRA_SCALE_COLUMN = 0, FIRA_SCALE_MATRIX = 1, FIRA_SCALE_NONE = 2 } fira_scaling;

/* How ||S_t|| (Eq. 12) is obtained.  FIRA_NORM_RESIDUAL forms G - P R tile by tile with an extra
 * rank-r contraction and a second pass over G (exact for any P).  FIRA_NORM_GRAM, the default, uses
 * ||G_i - P R_i||^2 = ||G_i||^2 - ||R_i||^2, which holds when P^T P = I (G_i^T P = R_i^T always) and
 * needs neither.  With a bf16-rounded orthonormal P the identity holds to about 1e-3 of ||R_i||^2,
 * which is harmless while the part of G outside the subspace is not small against the part inside; the
 * difference cancels when the subspace holds nearly all of G (P the leading singular vectors of a
 * gradient of low effective rank, or r close to min(m,n)).  Two gates per matrix therefore decide,
 * whatever this setting says:
 *   1. fira_set_projector estimates ||P^T P - I||; beyond 0.02 the matrix stays on the residual route;
 *   2. the first step after a projector is installed takes the residual route for that matrix and
 *      also forms the Gram value from the same data; the relative difference of the two ||S_t||^2 is kept,
 *      and the following steps take the Gram route only if it was at most 2e-3 (1e-3 of ||S_t||).
 * The second gate is measured once per installed projector, on that step's gradient; a gradient that
 * moves into the subspace later is not noticed until the next installation (select
 * FIRA_NORM_RESIDUAL for such workloads).  fira_get_gate reads both values; fira_set_gate restores
 * them after fira_set_projector (checkpoint resume without a new measurement). */
typedef enum { FIRA_NORM_RESIDUAL = 0, FIRA_NORM_GRAM = 1 } fira_norm_mode;

/* Number of optimizer-state values the METHOD keeps for one matrix: m r + 2 n r + 1 for m <= n
 * (Table "Comparison of different methods"); the transposed count for m > n. */
FIRA_API int64_t fira_method_state_numel(const fira_matrix_desc* d);

/* Bytes of the device slab for `count` matrices: M and V in fp32, the library's bf16 operand
 * copies of P, the per-matrix scalars, and the step's scratch (low-rank intermediates, factors,
 * partial sums, work tables).  Returns 0 on invalid descriptors. */
FIRA_API size_t fira_state_bytes(const fira_matrix_desc* d, int count);

/* Create a context over `count` matrices.  Zeroes M and V, sets t = 0 and "no previous norm"
 * (Algorithm 1, initialisation line).  dev_state: device slab, 256-byte aligned, at least
 * fira_state_bytes(d, count) bytes.  hip_stream: a hipStream_t (NULL = default stream).
 * Host-side resources of the context are released by fira_destroy. */
FIRA_API fira_status fira_init_state(fira_ctx** out, const fira_matrix_desc* d, int count,
                            const fira_hparams* hp, void* dev_state, size_t dev_state_bytes,
                            void* hip_stream);

/* Install the projector of matrix idx (Eq. 7; built by the caller, e.g. every T steps).
 * dev_P: min(m,n) x r row-major, dtype p_dtype; it is copied/converted into the slab, so the
 * caller may free it after the stream has run the call.  For bf16 matrices an fp32 P is rounded
 * to bf16 (nearest even).  M, V, t and ||S_prev|| are kept (Sec. 4.2, loss-spike analysis). */
FIRA_API fira_status fira_set_projector(fira_ctx* ctx, int idx, const void* dev_P, fira_dtype p_dtype);

/* fira_set_projector for `count` distinct matrices idx[0..count) at once (Eq. 7: a training loop
 * installs every matrix's projector at the same step, every T steps): dev_P[i] is the projector of
 * matrix idx[i], all of dtype p_dtype; idx and dev_P are host arrays of length count.  The same
 * copies, the same estimate behind the Gram route's first gate and the same result as `count` single
 * calls, bit for bit, in one launch per phase for every 16 matrices and one read-back of the gate values
 * instead of four launches and a copy per matrix.  A call may wait on the host for the previous call's
 * table of pointers to have reached the device.  Errors found on the host (a bad index, a matrix
 * listed twice, a null pointer, an unknown dtype) leave every projector as it was; a launch failure
 * (FIRA_ERR_HIP) leaves the listed matrices without a projector (fira_step then reports
 * FIRA_ERR_NO_PROJECTOR for them). */
FIRA_API fira_status fira_set_projectors(fira_ctx* ctx, int count, const int* idx, const void* const* dev_P,
                                         fira_dtype p_dtype);

/* One optimizer step (Algorithm 1's loop body below the SVD branch) for `count` distinct
 * matrices idx[0..count), in one grouped launch sequence.  dev_W[i] is updated in place, dev_G[i]
 * is read only; both are m x n with the descriptor's ld and dtype.  t advances by one for each
 * listed matrix.  idx, dev_W, dev_G are host arrays of length count.
 *
 * Capturing a step in a HIP graph: the step size lr * alpha is read from device memory, which
 * fira_set_hparams rewrites in stream order, so a learning-rate schedule reaches a captured step:
 * call fira_set_hparams on the same stream, then replay.  Everything else is decided on the host when
 * the call is made and travels as kernel arguments: beta1, beta2, eps, gamma, the options, the
 * variant, the fusion switch and the route of every listed matrix; and the work list (which W and G
 * pointers, which tiles) sits in one of four cached slots of the slab.  A captured step therefore
 * replays those as they were in force at capture: later changes of them through fira_set_hparams,
 * fira_set_options, fira_set_variant, fira_set_fusion, and fira_set_projector(s) or
 * fira_refresh_projectors calls (which may change a matrix's route) do not reach it, and it must be
 * captured again after any of them.  Capture only from the second step after a projector was
 * installed on (the first one measures the Gram route's gate and reads it back).  While a captured
 * step may still be replayed, do not step more than three other distinct (idx, W, G) lists on the
 * same context: the fifth distinct list reuses the oldest slot and would rewrite the captured one's
 * work list. */
FIRA_API fira_status fira_step(fira_ctx* ctx, int count, const int* idx, void* const* dev_W,
                      const void* const* dev_G);

/* Replace the hyper-parameters (e.g. the learning rate under a schedule); takes effect at the
 * next fira_step.  Enqueues one small kernel on the context's stream, which stores lr * alpha in the
 * slab for the update kernel to read (see fira_step on HIP graphs). */
FIRA_API fira_status fira_set_hparams(fira_ctx* ctx, const fira_hparams* hp);

/* Variant switches (Sec. 5.3 ablations) and the way ||S_t|| is computed.  Defaults: FIRA_SCALE_COLUMN,
 * FIRA_NORM_GRAM. */
FIRA_API fira_status fira_set_options(fira_ctx* ctx, fira_scaling scaling, fira_norm_mode norm_mode);

/* FIRA_VARIANT_FULL is Algorithm 1.  FIRA_VARIANT_ONLY_SCALING is the appendix's "Fira-only-scaling"
 * (Eq. "only-scaling"): the factors are applied to the full gradient and the Adam term is dropped,
 * W <- W - lr * alpha * c * (G diag(k)); the limiter acts on ||G diag(k)||, which needs only the
 * ||G_i||^2 (no back-projection and no orthonormality condition on P).  M, V and t advance as usual. */
typedef enum { FIRA_VARIANT_FULL = 0, FIRA_VARIANT_ONLY_SCALING = 1 } fira_variant;
FIRA_API fira_status fira_set_variant(fira_ctx* ctx, fira_variant variant);

/* Kernel fusion (on by default).  With column factors (Eq. 11), Algorithm 1 proper and FIRA_NORM_GRAM, the
 * listed matrices that take the Gram route run the projection R = P^T G and Adam (Eqs. 2-4) in one
 * kernel that keeps R in registers, provided each of them is bf16 with r % 4 == 0 and 128 <= r <= 512;
 * the listed matrices on the residual route (e.g. in the first step after their projector was
 * installed) run them as two kernels with R in memory in the same step.  Any other step, and every
 * step with enable == 0, runs two kernels for all.  Both compute the same quantities; sums are taken in
 * a different order, so results agree to rounding, not bit for bit.  fira_last_step_fused: 1 if the
 * last fira_step on ctx took the fused kernel for every listed matrix, 0 if not (or ctx is NULL).  A
 * fused step keeps no copy of R: fira_get_lowrank then returns what an earlier two-kernel step left
 * (zeros if there was none). */
FIRA_API fira_status fira_set_fusion(fira_ctx* ctx, int enable);
FIRA_API int fira_last_step_fused(const fira_ctx* ctx);

/* Precision of the back-projection operand Z = N - c k R of bf16 matrices (Algorithm 1's last two lines are
 * computed as W -= lr alpha (P Z + c k G)).  planes = 1, the default: Z is rounded to bf16 once, which puts
 * about 2^-9 relative error on P Z; harmless for one step, but W is stored in bf16, and an element whose
 * update sits next to half an ulp then moves or stays differently from exact arithmetic, one ulp per step
 * for as long as that lasts.  planes = 2: Z is kept as two bf16 planes, its rounding and the rounding of the
 * remainder (16 mantissa bits), the contraction runs over both, and W follows exact arithmetic over long
 * runs; the back-projection does twice the multiplies and the fused projection/Adam kernel is not used.
 * Applies to bf16 matrices with r % 4 == 0, r <= 1024 and column or no factors; others keep one plane. */
FIRA_API fira_status fira_set_z_planes(fira_ctx* ctx, int planes);

/* Copy the state of matrix idx to host memory.  Synchronises the stream.
 * host_M, host_V: fp32, in the paper's orientation (r x n row-major for m <= n, m x r for m > n);
 * either may be NULL.  *s_prev = ||S_{t-1}|| or -1 when no step has run yet.  *t = steps taken. */
FIRA_API fira_status fira_get_state(fira_ctx* ctx, int idx, float* host_M, float* host_V, double* s_prev,
                           int64_t* t);

/* Inverse of fira_get_state (checkpoint restore).  s_prev < 0 means "no previous norm".
 * Synchronises the stream. */
FIRA_API fira_status fira_set_state(fira_ctx* ctx, int idx, const float* host_M, const float* host_V,
                           double s_prev, int64_t t);

/* Limiter diagnostics of the last step of matrix idx: ||S|| before and after limiting and the
 * factor applied (the "gradient norm" curve of Fig. 3).  Synchronises the stream. */
FIRA_API fira_status fira_get_diag(fira_ctx* ctx, int idx, double* s_norm_pre, double* s_norm_post,
                          double* c);

/* The two gate values of the Gram route for matrix idx (see fira_norm_mode): the estimate of
 * ||P^T P - I|| and the measured relative error of the Gram route's ||S_t||^2 (+inf while not yet
 * measured, or before any projector), and the route the last step took for this matrix (0: residual
 * route; 1: Gram route, two kernels; 2: Gram route, fused projection/Adam kernel, which keeps no R).
 * Any output may be NULL.  Synchronises the stream.  fira_set_gate writes the two values back (after
 * fira_set_projector, which resets them), so that a restored run continues on the same route without
 * measuring again; values must be >= 0. */
FIRA_API fira_status fira_get_gate(fira_ctx* ctx, int idx, float* ortho_err, float* gram_err, int* gram_route);
FIRA_API fira_status fira_set_gate(fira_ctx* ctx, int idx, float ortho_err, float gram_err);

/* Copy the scaling factors k_i of the last step of matrix idx (n values for m <= n, m values for
 * m > n) to host memory.  Synchronises the stream. */
FIRA_API fira_status fira_get_factors(fira_ctx* ctx, int idx, float* host_k);

/* Copy the low-rank gradient R_t of the last step of matrix idx to host memory, fp32, in the
 * paper's orientation (r x n row-major for m <= n, m x r for m > n).  Synchronises the stream. */
FIRA_API fira_status fira_get_lowrank(fira_ctx* ctx, int idx, float* host_R);

/* Copy the projector of matrix idx as the kernels use it (rounded to bf16 for bf16 matrices, to the
 * three-way bf16 split for fp32 ones) to host memory: min(m,n) x r fp32, row-major.  Synchronises
 * the stream.  FIRA_ERR_NO_PROJECTOR if none was installed. */
FIRA_API fira_status fira_get_projector(fira_ctx* ctx, int idx, float* host_P);

/* Projector refresh on the device (Sec. 3.3, Eq. 7; Algorithm 1's "if t mod T = 0" branch): for every
 * listed matrix, replaces P by an orthonormal basis of an approximation to the span of the leading r
 * left singular vectors of its gradient (right singular vectors when m > n) and installs it exactly
 * as fira_set_projector would (M, V, t and the remembered norm are kept).  The basis comes from
 * `iters` >= 1 rounds of subspace iteration, Q <- orth(G G^T Q) (or G^T G for m > n), from a random
 * start that is a function of (seed, matrix index) only; it is a rotation of the singular vectors
 * inside that subspace, not the vectors themselves.  For fp32 matrices the product G^T Q runs on the
 * split planes of G as in a step, the product back on a bf16 rounding of G (kept in the workspace),
 * and the orthonormalisation in fp64 as for every matrix: the installed basis is orthonormal to fp32
 * accuracy, the subspace it spans is found with about 8 bits per product, which a few rounds of
 * subspace iteration do not resolve anyway.
 *   dev_G[e]       gradient of matrix idx[e], same layout as in fira_step; read only
 *   dev_workspace  device scratch of fira_refresh_workspace_bytes(ctx, count, idx) bytes, 256-byte
 *                  aligned, owned by the caller, free to reuse once the stream has passed this call
 * Enqueues on the context's stream and returns; the small work lists are uploaded with blocking
 * copies, so the call is not meant for the step's inner loop.  Uses the listed matrices' step
 * scratch (not their state).  The rounds of the iteration work in the matrices' own operand copies of
 * P: if a launch fails on the way (FIRA_ERR_HIP), the listed matrices are left WITHOUT a projector
 * (fira_step reports FIRA_ERR_NO_PROJECTOR for them until one is installed again); M, V, t and the
 * remembered norm are untouched in every case. */
FIRA_API size_t fira_refresh_workspace_bytes(const fira_ctx* ctx, int count, const int* idx);
FIRA_API fira_status fira_refresh_projectors(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G,
                                             int iters, uint64_t seed, void* dev_workspace, size_t workspace_bytes);

/* fira_refresh_projectors for callers that cannot allocate device memory (code that runs under a HIP
 * graph capture, tight serving or training loops, harnesses that forbid hipMalloc): the same computation
 * with the same kernels and the same result, but the workspace is a static device array of
 * FIRA_STATIC_SCRATCH_BYTES that is part of the library's code object, so the call performs no device
 * allocation and takes no workspace argument.  FIRA_ERR_WORKSPACE (nothing enqueued) when the listed
 * matrices need more than that (fira_refresh_workspace_bytes tells how much: about 16 MB for a
 * 2048 x 5461 matrix at r = 512, so a large model is refreshed a few matrices per call).  Every GPU the
 * library is used on holds its own copy of the array until the process ends; all calls on one GPU share
 * it and it keeps the last call's contents (what must start at zero is cleared by the call itself), so
 * two calls that overlap in time on one GPU, e.g. from contexts on different streams, race: serialise
 * them. */
#define FIRA_STATIC_SCRATCH_BYTES (64u << 20)
FIRA_API fira_status fira_refresh_projectors_static(fira_ctx* ctx, int count, const int* idx, const void* const* dev_G,
                                                    int iters, uint64_t seed);

/* Per-kernel timing of the step's launch sequence with HIP events on the context's stream.
 * fira_profile_begin creates the events for up to max_steps steps (the only allocation; it happens
 * here, not in fira_step); every following fira_step records one event before its first kernel
 * and one after each kernel.  fira_profile_end synchronises, adds up the elapsed time of each of
 * the FIRA_NUM_KERNELS kernels over the recorded steps into ms_sum[0..FIRA_NUM_KERNELS) (host
 * array, milliseconds), stores the number of recorded steps in *steps, and destroys the events.
 * Kernel order: fira_kernel_name(k). */
#define FIRA_NUM_KERNELS 6
FIRA_API fira_status fira_profile_begin(fira_ctx* ctx, int max_steps);
FIRA_API fira_status fira_profile_end(fira_ctx* ctx, double* ms_sum, int* steps);
FIRA_API const char* fira_kernel_name(int k);

FIRA_API const char* fira_last_error(const fira_ctx* ctx);

FIRA_API void fira_destroy(fira_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FIRA_H_ */
