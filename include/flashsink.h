/*
 * flashsink.h -- C ABI of libflashsink: fused log-domain Sinkhorn for entropic
 * optimal transport with squared-Euclidean cost on AMD MI355X (gfx950).
 *
 * Problem (paper Section 2.1): source points x in R^{n x d} with weights a,
 * target points y in R^{m x d} with weights b, cost C_ij = |x_i - y_j|^2,
 * regularisation eps > 0, dual potentials f in R^n, g in R^m.  Every half-step
 * is evaluated as a streaming row-wise LogSumExp of biased dot-product scores
 * (Prop. 1); no n x m matrix is ever stored.
 *
 * Conventions common to all entry points
 *  - Every pointer inside fs_problem and every pointer argument is a DEVICE
 *    pointer owned by the caller, unless the argument is marked "host".
 *    Inputs are never written.  Outputs must not alias inputs.
 *  - x, y are row-major with leading dimensions ldx, ldy (in elements, >= d).
 *  - Potentials that cross this interface are the UNSHIFTED f, g of Eq. 2-3, in
 *    float.  The shift by the squared norms (Prop. 1) is internal.
 *  - a == NULL / b == NULL means uniform weights 1/n, 1/m.  Weights must be
 *    positive; a zero weight removes its point from every sum (log 0 = -inf).
 *  - All work is enqueued on the stream given to fs_create.  The streaming passes
 *    are never waited for, except by the calls that return host values
 *    (fs_marginal_err, fs_ot_value, fs_solve_tol, fs_profile_read).  An entry
 *    point may synchronise the stream briefly in its prologue: for d <= 16 it
 *    reads back a few scalars (largest squared norm, size of the given
 *    potentials) that select the score arithmetic, fs_hvp reads back the scalars
 *    of its conjugate-gradient loop, and a call that has to grow the context's
 *    workspace synchronises once before the old workspace is released.
 *  - Errors are reported by status code only; nothing throws or aborts.
 *    Argument validation happens on the host before any launch.  The message
 *    of the last failure on a context is available from fs_last_error.
 *  - A context is not thread-safe; use one per thread/stream.
 *  - The library allocates device memory only for the context's workspace
 *    (derived copies of x and y, squared norms, bias vectors, partial
 *    reductions); it is grown on demand and released by fs_destroy.
 */
#ifndef FLASHSINK_H
#define FLASHSINK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_ctx fs_ctx;

typedef enum {
    FS_OK = 0,
    FS_ERR_INVALID_ARG = 1, /* null pointer, aliasing, bad enum value                  */
    FS_ERR_BAD_SHAPE = 2,   /* n, m, d, p <= 0, ld < d, sizes beyond the supported max */
    FS_ERR_BAD_EPS = 3,     /* eps <= 0 or not finite, n_stages < 1, iters < 0         */
    FS_ERR_BAD_WEIGHTS = 4, /* fs_check_weights: a weight <= 0 or not finite, sum != 1 */
    FS_ERR_UNSUPPORTED = 5, /* dtype/compute combination not available                 */
    FS_ERR_ALLOC = 6,       /* device allocation failed                                */
    FS_ERR_DEVICE = 7,      /* a HIP call failed (message in fs_last_error)            */
    FS_ERR_NONFINITE = 8    /* fs_check_finite: an entry is NaN or infinite            */
} fs_status;

/* storage type of x and y */
typedef enum { FS_F32 = 0, FS_BF16 = 1 } fs_dtype;

/*
 * Arithmetic of the score tile 2<x_i, y_j>:
 *  FS_COMPUTE_FP32       true fp32 products or better.  d <= 16: coordinates centred at the
 *                        common mean (the cost is translation invariant), products
 *                        summed at fp32 accuracy from bf16-split operands, float64-grade
 *                        scores where fp32 ones cannot hold the tolerance; d > 16: the
 *                        contraction runs on the fp64 matrix cores, because at
 *                        |score| ~ 1e3 fp32 products cannot hold 1e-4 absolute.
 *                        Potentials agree with a float64 reference to 1e-4*eps.
 *  FS_COMPUTE_BF16_MFMA  x, y rounded to bfloat16 (RNE), products on the bf16 matrix
 *                        cores with fp32 accumulation; norms are taken from the
 *                        rounded points.  Needs d >= 16.  Agreement 2e-2*eps.
 *                        Plan application in this mode also rounds the plan entries
 *                        (relative to each row's largest) and V to bfloat16 for the
 *                        second contraction; agreement 2e-2 relative (Frobenius).
 *                        fs_hvp needs FS_COMPUTE_FP32.
 */
typedef enum { FS_COMPUTE_FP32 = 0, FS_COMPUTE_BF16_MFMA = 1 } fs_compute;

typedef struct {
    const void *x;      /* n x d, row-major, dtype below                 */
    const void *y;      /* m x d                                         */
    int32_t dtype;      /* fs_dtype                                      */
    int32_t compute;    /* fs_compute                                    */
    int64_t n, m, d;    /* n, m <= 2^24 points, d <= 8192                */
    int64_t ldx, ldy;   /* leading dimensions in elements (>= d)         */
    const float *a;     /* n weights or NULL (uniform)                   */
    const float *b;     /* m weights or NULL (uniform)                   */
} fs_problem;

/*
 * Create a context bound to HIP device `device` and to `hip_stream` (a hipStream_t
 * passed as void*, NULL = the default stream).  Fails with FS_ERR_DEVICE if the
 * device cannot be used.  The context owns its workspace only.
 * device == -1 creates a host-only context: every entry point still validates its
 * arguments and reports argument errors, and otherwise returns FS_ERR_DEVICE without
 * touching a GPU (used to test the interface on machines without one).
 */
fs_status fs_create(fs_ctx **ctx, int device, void *hip_stream);

/* Synchronises the stream, frees the workspace and the context.  NULL is allowed. */
fs_status fs_destroy(fs_ctx *ctx);

const char *fs_status_str(fs_status s);
const char *fs_last_error(const fs_ctx *ctx); /* "" if none; valid until the next call */

/* Library build info: "flashsink <version> gfx950". */
const char *fs_version(void);

/*
 * Squared row norms alpha_i = |pts_i|^2 (Prop. 1, definition of alpha and beta).
 * pts: rows x d (ld elements per row) of `dtype`; out: rows floats.  Accumulated in
 * float64 and rounded once.
 */
fs_status fs_row_norms(fs_ctx *ctx, const void *pts, int32_t dtype, int64_t rows, int64_t d,
                       int64_t ld, float *out);

/*
 * One half-step, Eq. 2 evaluated in the form of Prop. 1 / Alg. 1:
 *   f_i = alpha_i - eps * LSE_j[(2<x_i,y_j> - beta_j + g_j)/eps + log b_j].
 * g: m floats in; f_out: n floats out.
 */
fs_status fs_update_f(fs_ctx *ctx, const fs_problem *prob, float eps, const float *g,
                      float *f_out);

/*
 * The other half-step, Eq. 3 in the form of Prop. 1 / Alg. 3:
 *   g_j = beta_j - eps * LSE_i[(2<y_j,x_i> - alpha_i + f_i)/eps + log a_i].
 */
fs_status fs_update_g(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f,
                      float *g_out);

/*
 * Alternating Sinkhorn with a fixed iteration count (App. B, Gauss-Seidel form):
 * n_stages * iters_per_stage iterations, each "f from g, then g from the new f".
 * Stage s uses eps_s = eps_start * (eps_end/eps_start)^(s/(n_stages-1)), evaluated
 * in double and rounded to float, endpoints exact; n_stages == 1 uses eps_end.
 * f (n floats) and g (m floats) are read as the starting potentials (f is never
 * read by the first half-step, g is) and overwritten with the result.  Between
 * half-steps the potentials are kept in float64 inside the workspace; they are
 * rounded to float once, at the end.
 */
fs_status fs_solve(fs_ctx *ctx, const fs_problem *prob, float eps_start, float eps_end,
                   int32_t n_stages, int32_t iters_per_stage, float *f, float *g);

/*
 * fs_solve for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same arguments, arithmetic and results as fs_solve, but
 * the workspace (derived copies of x and y, norms, biases, potentials, partial reductions) lives in a
 * static device array of 32 MiB inside the library, of which the partial reductions of a pass take at
 * most 8 MiB (so a pass may be cut into fewer column splits than fs_solve would choose).  The call
 * performs no hipMalloc / hipFree and leaves the context's own workspace untouched.  Problems whose
 * workspace does not fit are refused with FS_ERR_BAD_SHAPE before anything is launched (n = m up to
 * 54272 at d = 3, 15360 at d = 16, 22528 at d = 64, 5120 at d = 1024 in bfloat16 mode).
 * Every GPU holds ONE such array for the whole process: calls of this entry point that overlap in time
 * on one GPU -- from any context or stream -- race on it.  Nothing is assumed about its contents on
 * entry (it keeps what the previous call left).  Synchronises like fs_solve.
 */
fs_status fs_solve_noalloc(fs_ctx *ctx, const fs_problem *prob, float eps_start, float eps_end,
                           int32_t n_stages, int32_t iters_per_stage, float *f /* device, in/out */,
                           float *g /* device, in/out */);

/*
 * Alternating Sinkhorn for the label-augmented cost of the dataset-distance application (Section 3.1's remark on
 * generalised costs; Section 4 and its appendix):
 *     C_ij = lambda1 |x_i - y_j|^2 + lambda2 W[lx_i, ly_j],
 * `iters` iterations at eps, "f from g, then g from the new f", from the given potentials (of THIS cost), which are
 * overwritten with the result.  lx [n], ly [m]: device int32 class labels in [0, V); W: device floats, V x V row-major
 * (row = class of the source point).  lambda1 > 0.
 * The n x m cost is never stored and no kernel does a table lookup: W[lx, ly] = <onehot(lx), W[:, ly]> is a
 * contraction, so the library appends V coordinates to device copies of both clouds and runs the squared-Euclidean
 * kernels on them at eps / lambda1; the per-point constants this adds to the cost are absorbed exactly by the
 * potentials, which are mapped on the device on entry and exit.  In FS_COMPUTE_BF16_MFMA mode the table entries are
 * rounded to bfloat16 like the coordinates.  The augmented copies (float, (n + m)(d + V) values) live in the context's
 * second buffer.  Labels outside [0, V): FS_ERR_INVALID_ARG after the run (the potentials are then undefined).
 * Synchronises the stream.
 */
fs_status fs_solve_labeled(fs_ctx *ctx, const fs_problem *prob, const int32_t *lx /* device */,
                           const int32_t *ly /* device */, const float *W /* device */, int32_t V, float lambda1,
                           float lambda2, float eps, int32_t iters, float *f /* device, in/out */,
                           float *g /* device, in/out */);

/*
 * Symmetric (Jacobi, averaged) schedule with a fixed iteration count (Eq. 4-5):
 * in every iteration both updates read the OLD potentials,
 *     f <- f/2 + (1/2) (-eps LSE_j[(g_j - C_ij)/eps + log b_j]),
 *     g <- g/2 + (1/2) (-eps LSE_i[(f_i - C_ij)/eps + log a_i]),
 * at one eps.  f (n floats) and g (m floats) are both read as the starting
 * potentials and overwritten with the result; between iterations they are kept
 * in float64 inside the workspace and rounded to float once, at the end.
 * Same arguments, validation and error behaviour as fs_solve.
 */
fs_status fs_solve_symmetric(fs_ctx *ctx, const fs_problem *prob, float eps, int32_t iters,
                             float *f /* device, in/out */, float *g /* device, in/out */);

/*
 * Alternating Sinkhorn at one eps with early stopping on the row marginal error
 * (Prop. 3; after a g-update the column marginal is exact, so the row error is the
 * whole error).  After every `check_every` iterations, and after `max_iters`, the L1 row
 * error of the current potentials is measured; the iteration stops when it is <= tol.
 * The error comes out of the f-update that begins the next iteration, so a check that
 * does not stop costs no extra pass (it costs one synchronisation).  f is not read on
 * entry (the first half-step computes it from g).  On return f, g are the potentials
 * after *iters_done iterations and *err_row_l1 their measured row error; both are HOST
 * pointers, and the call synchronises the stream.
 */
fs_status fs_solve_tol(fs_ctx *ctx, const fs_problem *prob, float eps, int32_t max_iters,
                       int32_t check_every, float tol, float *f /* device, in/out */,
                       float *g /* device, in/out */, int32_t *iters_done /* host */,
                       float *err_row_l1 /* host */);

/*
 * L1 violation of the marginals of the plan induced by (f, g) (Prop. 3):
 *   r_i = a_i exp((f_i - f_i^+)/eps),  c_j = b_j exp((g_j - g_j^+)/eps),
 *   *err_row_l1 = sum_i |r_i - a_i|,   *err_col_l1 = sum_j |c_j - b_j|,
 * where f^+, g^+ are one half-step from (f, g).  The two results are HOST floats;
 * either pointer may be NULL to skip that side.  Synchronises the stream.
 */
fs_status fs_marginal_err(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f,
                          const float *g, float *err_row_l1 /* host */,
                          float *err_col_l1 /* host */);

/*
 * Value of the dual objective at the given potentials (App. B, the Lagrangian at its
 * stationary plan):  <a,f> + <b,g> - eps (sum_ij P_ij - sum_ij a_i b_j)  with P the plan that
 * (f, g) induce (text after Eq. 3).  At convergence this is the entropic OT value of Eq. 1.
 * Costs one streaming pass (the total mass of P is the sum of the induced row marginals,
 * Prop. 3), always with the accurate score arithmetic.  *value is a HOST double; the call
 * synchronises the stream.
 */
fs_status fs_ot_value(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f /* device */,
                      const float *g /* device */, double *value /* host */);

/*
 * Optional check of the weights (Section 2 takes a and b in the open simplex; the entry points
 * above do not check this, because it costs a pass over the weights): FS_ERR_BAD_WEIGHTS if a
 * weight is not positive and finite, or if a or b does not sum to 1 within tol; FS_OK otherwise.
 * NULL weights (uniform) pass.  sum_a, sum_b: NULL or HOST doubles that receive the sums.
 * Synchronises the stream when there is something to check.
 */
fs_status fs_check_weights(fs_ctx *ctx, const fs_problem *prob, float tol, double *sum_a /* host, nullable */,
                           double *sum_b /* host, nullable */);

/*
 * Optional check of a result (potentials, a plan application, a gradient): FS_ERR_NONFINITE if one
 * of the cnt floats at v (device) is NaN or infinite, FS_OK otherwise; bad_count: NULL or a HOST
 * int64 that receives how many are.  The entry points do not check their outputs themselves (it
 * costs a pass).  Synchronises the stream.
 */
fs_status fs_check_finite(fs_ctx *ctx, const float *v /* device */, int64_t cnt, int64_t *bad_count /* host, nullable */);

/*
 * Debiased Sinkhorn divergence  S = OT(a,b) - OT(a,a)/2 - OT(b,b)/2  (Section 4.2 uses it as the
 * loss of the downstream tasks): each term is the dual value (fs_ot_value) after `iters`
 * alternating iterations from zero potentials at eps -- three fs_solve + fs_ot_value runs inside
 * the library.  f (n floats), g (m floats), device: receive the potentials of the cross term.
 * value: HOST double; terms: NULL or three HOST doubles receiving OT(a,b), OT(a,a), OT(b,b).
 * Synchronises the stream.  The potentials of the self terms live in a second, grow-only buffer
 * of the context (2 max(n, m) floats).
 */
fs_status fs_divergence(fs_ctx *ctx, const fs_problem *prob, float eps, int32_t iters,
                        float *f /* device */, float *g /* device */, double *value /* host */,
                        double *terms /* host, nullable */);

/*
 * out = P V with P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps) for ANY potentials
 * (Prop. 3, Alg. 2): streaming passes, P never stored.
 * V: m x p (ldv), out: n x p (ldo), r_out: NULL or n floats receiving P 1_m.
 * The gradient of Cor. 4 is 2*(diag(a) x - P y) (or with r_out in place of a, App. G).
 * Cost: a pass recomputes all n m scores and takes a block of value columns, so a call is
 * one pass for p <= 8 and ceil(p / 15) passes beyond at d <= 16,
 * ceil(p / 64) passes at d > 16 (when p > 64: ceil(p / 128) with FS_COMPUTE_FP32, ceil(p / 96) with
 * FS_COMPUTE_BF16_MFMA).
 * Accuracy at d <= 16, FS_COMPUTE_FP32: every plan entry enters the products to 2^-17 relative
 * (1e-6 to 3e-6 of the result's norm in practice), values to 24 bits (p <= 8) or 2^-17 (p > 8).
 */
fs_status fs_apply_plan(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f,
                        const float *g, const float *V, int64_t p, int64_t ldv, float *out,
                        int64_t ldo, float *r_out);

/*
 * out = P^T U (Alg. 4).  U: n x p (ldu), out: m x p (ldo), c_out: NULL or m floats
 * receiving P^T 1_n.
 */
fs_status fs_apply_plan_T(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f,
                          const float *g, const float *U, int64_t p, int64_t ldu, float *out,
                          int64_t ldo, float *c_out);

/*
 * Gradient of the entropic OT value with respect to the points of one cloud, for ANY
 * potentials, assembled inside the library on top of one plan application (Cor. 4; the
 * appendix on gradients for the induced-marginal form):
 *   fs_grad_x:  T = P y (n x d),   mode 0:  2 (diag(a) x - T)
 *                                  mode 1:  2 (diag(r) x - T),  r = P 1 the plan's own row marginal
 *                                  mode 2:  x - diag(a)^-1 T    displacement to the barycentric image
 *   fs_grad_y:  T = P^T x (m x d), the same with b, c = P^T 1 and y.
 * grad: rows x d floats (ldg >= d), device, written; it may not overlap an input.  d <= 4096.
 * With bfloat16 point storage the other cloud is widened to float in the workspace first.
 */
fs_status fs_grad_x(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                    int32_t mode, float *grad, int64_t ldg);
fs_status fs_grad_y(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                    int32_t mode, float *grad, int64_t ldg);

/*
 * Hessian-vector product G = T A of the entropic OT value with respect to the source
 * cloud x (Thm. 5): the matrix-free Schur-complement / conjugate-gradient oracle of
 * App. E, built on streamed applications of the plan that (f, g) induce:
 * (2 K + 3) transport-vector products, three transport-matrix products and one
 * Hadamard-weighted transport (Alg. 5), K the number of CG iterations.  The plan's own
 * marginals are used throughout, so (f, g) need not be converged.
 *   A   [n x d] device floats, row stride lda: the direction
 *   tau >= 0    Tikhonov damping of the Schur system (S + tau I); 0 is allowed
 *   eta, max_cg CG stops at relative residual eta or after max_cg iterations
 *   out [n x d] device floats, row stride ldo
 *   cg_iters    HOST int32 (may be NULL): iterations CG took
 * Available for float32 points and FS_COMPUTE_FP32 (FS_ERR_UNSUPPORTED otherwise).
 * Synchronises the stream (CG's scalars are read by the host).
 */
fs_status fs_hvp(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f /* device */,
                 const float *g /* device */, const float *A /* device */, int64_t lda, float tau,
                 float eta, int32_t max_cg, float *out /* device */, int64_t ldo,
                 int32_t *cg_iters /* host, nullable */);

/*
 * Hadamard-weighted transport (Alg. 5) with the second factor of the weights taken from the target
 * cloud, the form Thm. 5 uses:   out = (P o (A y^T)) V,   out_i = sum_j P_ij <A_i, y_j> V_j,
 * for ANY potentials, in streaming passes (P and the weights are formed tile by tile and never stored).
 *   A   [n x d] device floats, row stride lda >= d
 *   V   [m x p] device floats, row stride ldv;   out [n x p] device floats, row stride ldo, written
 * For d <= 16 the weights are formed against the centred points and the mean's share is added from a
 * plain application of the same plan (two streaming passes per block of value columns).
 * Available for float32 points and FS_COMPUTE_FP32 (FS_ERR_UNSUPPORTED otherwise).  out may not
 * overlap an input.  Does not synchronise.
 */
fs_status fs_apply_plan_hadamard(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f /* device */,
                                 const float *g /* device */, const float *A /* device */, int64_t lda,
                                 const float *V /* device */, int64_t p, int64_t ldv, float *out /* device */,
                                 int64_t ldo);

/*
 * Keeping the derived copies of the clouds across entry calls (the norms alpha, beta of Prop. 1 and the
 * tiled / split / centred copies the kernels stream).  Every entry call above prepares them from x and y
 * anew, because the library cannot see whether the caller has changed the points in between.
 * fs_points_keep declares that the clouds of `prob` (the addresses x and y, n, m, d, ldx, ldy, storage and
 * compute mode; the weights may change freely) will not be written until fs_points_release: the next entry
 * call on these clouds prepares the copies as usual, and later calls on the same clouds reuse them and skip
 * that part of their prologue (coordinate sums, mean, derived copies, norms; biases and potentials are
 * always written anew).  The copies live in the context's workspace: a call on other clouds, or one that
 * needs a larger workspace, overwrites them, and the next call on the kept clouds prepares them again, so
 * results never depend on the declaration as long as it is true.  fs_solve_noalloc prepares its copies
 * on every call (its scratch array is shared by all contexts of a GPU).  Host-only state; nothing is launched.
 * Changing the points while the declaration stands gives results for the OLD points.
 */
fs_status fs_points_keep(fs_ctx *ctx, const fs_problem *prob);
fs_status fs_points_release(fs_ctx *ctx);

/*
 * Test and experiment switches of ONE context (there is no process-wide state; a new context has
 * every switch at 0 = the library decides).  Not needed for normal use.
 *   "lowd_splits"        1..1024: split count of the streamed side of the d <= 16 passes
 *   "lowd_score"         32 / 64: fp32-accurate / float64-grade scores in every d <= 16 half-step and
 *                        application (fs_marginal_err and fs_ot_value always take float64-grade scores)
 *   "lowd_precise_valu"  1: float64-grade scores at d <= 3 on the vector ALU instead of the matrix cores
 *   "lowd_precise_any_bias"  1: those matrix-core records also for biases beyond their digit range
 * Unknown keys and values out of range: FS_ERR_INVALID_ARG.  key: HOST string.
 */
fs_status fs_debug_set(fs_ctx *ctx, const char *key /* host */, int64_t value);

/*
 * Timing hook for benchmarks: average duration in milliseconds of the streaming
 * LSE kernel launches recorded with HIP events on the context's stream since the
 * last call of this function, and their count.  Where a solve mixes two LSE
 * kernels (low-d problems: fp32-accuracy and float64-score half-steps), the
 * figures are those of the kernel with the larger total time (the dominant one).
 * Recording is off until fs_profile_enable(ctx, 1).  Synchronises the stream.
 */
fs_status fs_profile_enable(fs_ctx *ctx, int32_t on);
fs_status fs_profile_read(fs_ctx *ctx, double *avg_ms /* host */, int64_t *launches /* host */,
                          double *pairs_per_launch /* host */);

#ifdef __cplusplus
}
#endif
#endif /* FLASHSINK_H */
