// Streaming Hessian-vector product of the entropic OT value with respect to the source cloud
// (Thm. 5, App. E): G = T A = (1/eps) R^T w + E A with w the solution of the (damped) Schur
// complement system, everything expressed through transport applications P v, P^T u, P Y,
// P (diag(w2) Y) and one Hadamard-weighted transport (Alg. 5).  The plan's own marginals r = P 1,
// c = P^T 1 are used throughout (as the appendix on implementation does), so the formulas stay
// consistent for potentials that are not converged.
//
// This file holds the O(n + m) vector kernels and the host loop (conjugate gradients); the
// O(n m) work is done by the plan-application kernels (low-d or fp64 matrix-core path).
#include "fs_internal.h"

#include <math.h>

namespace fs {
namespace {

__device__ inline double block_sum(double v, double *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

// out_i = <X_i, A_i> (row-wise dot products, App. E notation <X, A>)
__global__ void k_rowdot(const float *X, int64_t ldx, const float *A, int64_t lda, int64_t rows, int d, float *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    double s = 0.0;
    for (int k = 0; k < d; ++k) s += (double)X[i * ldx + k] * (double)A[i * lda + k];
    out[i] = (float)s;
}

// cA_i = <A_i, mean> (the share of the common mean in the Hadamard weights)
__global__ void k_rowdot_mean(const float *A, int64_t lda, const double *mean, int64_t rows, int d, float *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    double s = 0.0;
    if (mean)   // (the fp64 matrix-core path does not centre: no share)
        for (int k = 0; k < d; ++k) s += (double)A[i * lda + k] * mean[k];
    out[i] = (float)s;
}

// r1 = 2 (r u - uP),  t1 = r1 / r      (App. E.2, step 1 and the right-hand side of the Schur system)
__global__ void k_rhs_n(const float *r, const float *u, const float *uP, int64_t n, float *r1, float *t1)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float v = 2.0f * (r[i] * u[i] - uP[i]);
    r1[i] = v;
    t1[i] = v / r[i];
}

// rhs = r2 - P^T (r1 / r),  r2 = 2 (P^T u - <P^T A, Y>);  also x = 0, res = p = rhs (CG start)
__global__ void k_rhs_m(const float *Ptu, const float *rd, const float *Ptt1, int64_t m, float *rhs, float *x, float *res,
                        float *pdir)
{
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    const float v = 2.0f * (Ptu[j] - rd[j]) - Ptt1[j];
    rhs[j] = v;
    x[j] = 0.0f;
    res[j] = v;
    pdir[j] = v;
}

__global__ void k_div(const float *a, const float *b, int64_t cnt, float *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cnt) out[i] = a[i] / b[i];
}

// S_tau p = c p - P^T ((P p) / r) + tau p
__global__ void k_schur(const float *cm, const float *pdir, const float *Ptq, float tau, int64_t m, float *Sp)
{
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < m) Sp[j] = cm[j] * pdir[j] - Ptq[j] + tau * pdir[j];
}

__global__ void k_cg_step(float alpha, const float *pdir, const float *Sp, int64_t m, float *x, float *res)
{
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    x[j] += alpha * pdir[j];
    res[j] -= alpha * Sp[j];
}

__global__ void k_cg_dir(float beta, const float *res, int64_t m, float *pdir)
{
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < m) pdir[j] = res[j] + beta * pdir[j];
}

__global__ __launch_bounds__(256) void k_dot(const float *a, const float *b, int64_t cnt, double *part)
{
    __shared__ double sh[256];
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double v = i < cnt ? (double)a[i] * (double)b[i] : 0.0;
    double t = block_sum(v, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = t;
}

__global__ __launch_bounds__(256) void k_sum(const double *part, int64_t cnt, double *dst)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < cnt; i += 256) acc += part[i];
    double t = block_sum(acc, sh);
    if (threadIdx.x == 0) *dst = t;
}

// w1 = (r1 - P w2) / r
__global__ void k_w1(const float *r1, const float *Pw2, const float *r, int64_t n, float *w1)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w1[i] = (r1[i] - Pw2[i]) / r[i];
}

// V2 = diag(w2) Y
__global__ void k_scale_rows(const float *w, const float *Y, int64_t ldy, int64_t rows, int d, float *out)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * d) return;
    int64_t j = e / d;
    int k = (int)(e - j * d);
    out[e] = w[j] * Y[j * ldy + k];
}

// G = (1/eps) R^T w + E A, entry by entry (App. E.1 and E.2, step 3):
//   R^T w = 2 ((r w1 + P w2) X - w1 PY - P (diag(w2) Y))
//   E A   = 2 r A - (4/eps) (r u X - u PY - uP X + B5),   B5 = B5c + <A, mean> PY
// (B5c: Hadamard-weighted transport with the weights taken against the centred streamed points)
__global__ void k_assemble(const float *X, int64_t ldx, const float *A, int64_t lda, const float *PY, const float *PV2,
                           const float *B5c, const float *r, const float *u, const float *uP, const float *w1,
                           const float *Pw2, const float *cA, double inv_eps, int64_t n, int d, float *out, int64_t ldo)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n * d) return;
    int64_t i = e / d;
    int t = (int)(e - i * d);
    const double x = X[i * ldx + t], av = A[i * lda + t], py = PY[e];
    const double ri = r[i], ui = u[i], upi = uP[i];
    const double rtw = 2.0 * ((ri * w1[i] + Pw2[i]) * x - w1[i] * py - PV2[e]);
    const double b5 = (double)B5c[e] + (double)cA[i] * py;
    const double ea = 2.0 * ri * av - 4.0 * inv_eps * (ri * ui * x - ui * py - upi * x + b5);
    out[i * ldo + t] = (float)(rtw * inv_eps + ea);
}

// out_i += <A_i, mean> PV_i: the share of the common mean in the Hadamard weights <A_i, y_j> when the
// application kernel forms them against the centred streamed points
__global__ void k_add_mean_share(const float *A, int64_t lda, const double *mean, const float *PV, int64_t n, int d, int p,
                                 float *out, int64_t ldo)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n * p) return;
    const int64_t i = e / p;
    const int q = (int)(e - i * p);
    double s = 0.0;
    for (int k = 0; k < d; ++k) s += (double)A[i * lda + k] * mean[k];
    out[i * ldo + q] = (float)((double)out[i * ldo + q] + s * (double)PV[e]);
}

inline dim3 g256(int64_t cnt) { return dim3((unsigned)ceil_div(cnt, 256)); }

}  // namespace

fs_status launch_add_mean_share(Ctx *c, const float *A, int64_t lda, const double *mean, const float *PV, int64_t n, int d,
                                int p, float *out, int64_t ldo)
{
    hipLaunchKernelGGL(k_add_mean_share, g256(n * p), dim3(256), 0, c->stream, A, lda, mean, PV, n, d, p, out, ldo);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

size_t hvp_scratch_bytes(int64_t n, int64_t m, int64_t d)
{
    auto al = [](size_t b) { return (b + 255) & ~size_t(255); };
    return 9 * al((size_t)n * 4) + 10 * al((size_t)m * 4) + 3 * al((size_t)n * d * 4) + 2 * al((size_t)m * d * 4) +
           al((size_t)ceil_div(n > m ? n : m, 256) * 8) + al(64);
}

// Potentials must already be in place (biases of both sides for `eps`).  x, y, A, out: device floats.
fs_status hvp_run(Ctx *c, Prepared *P, const float *x, int64_t ldx, const float *y, int64_t ldy, double eps,
                  const float *A, int64_t lda, double tau, double eta, int max_cg, float *out, int64_t ldo,
                  char *scratch, int *cg_iters)
{
    const int64_t n = P->X.cnt, m = P->Y.cnt;
    const int d = (int)P->d;
    hipStream_t st = c->stream;
    char *cur = scratch;
    auto take = [&](size_t bytes) {
        char *p = cur;
        cur += (bytes + 255) & ~size_t(255);
        return p;
    };
    float *r = (float *)take(n * 4), *u = (float *)take(n * 4), *uP = (float *)take(n * 4), *r1 = (float *)take(n * 4),
          *t1 = (float *)take(n * 4), *q1 = (float *)take(n * 4), *w1 = (float *)take(n * 4), *Pw2 = (float *)take(n * 4),
          *cA = (float *)take(n * 4);
    float *cm = (float *)take(m * 4), *Ptu = (float *)take(m * 4), *rd = (float *)take(m * 4), *Ptt1 = (float *)take(m * 4),
          *rhs = (float *)take(m * 4), *w2 = (float *)take(m * 4), *res = (float *)take(m * 4),
          *pdir = (float *)take(m * 4), *Sp = (float *)take(m * 4), *Ptq = (float *)take(m * 4);
    float *PY = (float *)take((size_t)n * d * 4), *PV2 = (float *)take((size_t)n * d * 4),
          *B5c = (float *)take((size_t)n * d * 4);
    float *PtA = (float *)take((size_t)m * d * 4), *V2 = (float *)take((size_t)m * d * 4);
    double *part = (double *)take((size_t)ceil_div(n > m ? n : m, 256) * 8);
    double *scal = (double *)take(64);

    Side *X = &P->X, *Y = &P->Y;
    fs_status s;
    const bool lowd = P->path == Path::LowD;
    // one streamed application: out = P V (res = X) or P^T V (res = Y); hadA: Hadamard weights (Alg. 5)
    auto apply = [&](const Side *rs, const Side *ss, const float *V, int64_t p, int64_t ldv, float *o, int64_t ldo_,
                     float *mass, const float *hadA = nullptr, int64_t lda_ = 0) -> fs_status {
        return lowd ? lowd_apply(c, P, rs, ss, eps, V, p, ldv, o, ldo_, mass, hadA, lda_)
                    : f64_apply(c, P, rs, ss, eps, V, p, ldv, o, ldo_, mass, hadA, lda_);
    };
    auto dot = [&](const float *a, const float *b, int64_t cnt, double *host) -> fs_status {
        hipLaunchKernelGGL(k_dot, g256(cnt), dim3(256), 0, st, a, b, cnt, part);
        hipLaunchKernelGGL(k_sum, dim3(1), dim3(256), 0, st, part, (int64_t)ceil_div(cnt, 256), scal);
        FS_HIP(c, hipMemcpyAsync(host, scal, 8, hipMemcpyDeviceToHost, st));
        FS_HIP(c, hipStreamSynchronize(st));
        return FS_OK;
    };

    // transport-matrix products P Y (with r = P 1) and P^T A (with c = P^T 1); row-wise dots
    if ((s = apply(X, Y, y, d, ldy, PY, d, r)) != FS_OK) return s;
    if ((s = apply(Y, X, A, d, lda, PtA, d, cm)) != FS_OK) return s;
    hipLaunchKernelGGL(k_rowdot, g256(n), dim3(256), 0, st, x, ldx, A, lda, n, d, u);
    hipLaunchKernelGGL(k_rowdot, g256(n), dim3(256), 0, st, PY, (int64_t)d, A, lda, n, d, uP);
    hipLaunchKernelGGL(k_rowdot, g256(m), dim3(256), 0, st, PtA, (int64_t)d, y, ldy, m, d, rd);
    hipLaunchKernelGGL(k_rowdot_mean, g256(n), dim3(256), 0, st, A, lda, lowd ? P->mean : (const double *)nullptr, n, d, cA);
    // right-hand sides
    hipLaunchKernelGGL(k_rhs_n, g256(n), dim3(256), 0, st, r, u, uP, n, r1, t1);
    if ((s = apply(Y, X, u, 1, 1, Ptu, 1, nullptr)) != FS_OK) return s;
    if ((s = apply(Y, X, t1, 1, 1, Ptt1, 1, nullptr)) != FS_OK) return s;
    hipLaunchKernelGGL(k_rhs_m, g256(m), dim3(256), 0, st, Ptu, rd, Ptt1, m, rhs, w2, res, pdir);
    FS_HIP(c, hipGetLastError());

    // conjugate gradients on S_tau w2 = rhs
    double rr = 0.0;
    if ((s = dot(res, res, m, &rr)) != FS_OK) return s;
    const double rr0 = rr;
    int k = 0;
    for (; k < max_cg; ++k) {
        if (!(rr > 0.0) || sqrt(rr) <= eta * sqrt(rr0)) break;
        if ((s = apply(X, Y, pdir, 1, 1, q1, 1, nullptr)) != FS_OK) return s;
        hipLaunchKernelGGL(k_div, g256(n), dim3(256), 0, st, q1, r, n, q1);
        if ((s = apply(Y, X, q1, 1, 1, Ptq, 1, nullptr)) != FS_OK) return s;
        hipLaunchKernelGGL(k_schur, g256(m), dim3(256), 0, st, cm, pdir, Ptq, (float)tau, m, Sp);
        double pSp = 0.0;
        if ((s = dot(pdir, Sp, m, &pSp)) != FS_OK) return s;
        if (!(pSp > 0.0)) break;   // direction in the null space (tau = 0): nothing more to gain
        const double alpha = rr / pSp;
        hipLaunchKernelGGL(k_cg_step, g256(m), dim3(256), 0, st, (float)alpha, pdir, Sp, m, w2, res);
        double rr_new = 0.0;
        if ((s = dot(res, res, m, &rr_new)) != FS_OK) return s;
        hipLaunchKernelGGL(k_cg_dir, g256(m), dim3(256), 0, st, (float)(rr_new / rr), res, m, pdir);
        rr = rr_new;
    }
    if (cg_iters) *cg_iters = k;

    // back-substitution, R^T w, Hadamard-weighted transport, assembly
    if ((s = apply(X, Y, w2, 1, 1, Pw2, 1, nullptr)) != FS_OK) return s;
    hipLaunchKernelGGL(k_w1, g256(n), dim3(256), 0, st, r1, Pw2, r, n, w1);
    hipLaunchKernelGGL(k_scale_rows, g256(m * d), dim3(256), 0, st, w2, y, ldy, m, d, V2);
    if ((s = apply(X, Y, V2, d, d, PV2, d, nullptr)) != FS_OK) return s;
    if ((s = apply(X, Y, y, d, ldy, B5c, d, nullptr, A, lda)) != FS_OK) return s;
    hipLaunchKernelGGL(k_assemble, g256(n * d), dim3(256), 0, st, x, ldx, A, lda, PY, PV2, B5c, r, u, uP, w1, Pw2, cA,
                       1.0 / eps, n, d, out, ldo);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
