/*
 * fs_oracle.c -- float64 CPU oracle for entropic optimal transport with
 * squared-Euclidean cost, solved by log-domain Sinkhorn iterations.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition written out, slow on
 * purpose, and shares no code, header, table or helper with the GPU library.
 * Only the tests, the smoke check and the bench's cpu_baseline leg call it.
 *
 * Everything is the textbook form of the paper's Section 2.1:
 *   - cost       C_ij = sum_k (x_ik - y_jk)^2, by differences (never by norms
 *                and dot products: that algebra belongs to the method under test)
 *   - Eq. 2      f_i <- -eps * LSE_j[(g_j - C_ij)/eps + log b_j]
 *   - Eq. 3      g_j <- -eps * LSE_i[(f_i - C_ij)/eps + log a_i]
 *   - Eq. 4-5    the symmetric (averaged, Jacobi) variant
 *   - plan       P_ij = a_i b_j exp((f_i + g_j - C_ij)/eps)    (text after Eq. 3)
 *   - Eq. 1      primal objective <C,P> + eps*KL(P | a (x) b), generalised KL
 *   - App. B     Lagrangian / dual value
 * LSE is taken in two passes (max, then sum of exp(. - max), then log), which is
 * deliberately NOT the online recurrence the method uses.
 *
 * All arrays are row-major double; the callers widen the float inputs exactly.
 * Rows of a half-step are independent, so OpenMP splits them; no other blocking,
 * fusion or reordering is applied.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int fso_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* C(p, q) = ||p - q||^2 by coordinate differences (Section 2.1, definition of C). */
static double sqdist(const double *p, const double *q, int64_t d)
{
    double c = 0.0;
    for (int64_t k = 0; k < d; ++k) {
        double t = p[k] - q[k];
        c += t * t;
    }
    return c;
}

/* alpha_i = ||pts_i||^2 (Prop. 1 defines alpha, beta this way). */
void fso_row_norms(const double *pts, int64_t rows, int64_t d, double *out)
{
    for (int64_t i = 0; i < rows; ++i) {
        double s = 0.0;
        for (int64_t k = 0; k < d; ++k) s += pts[i * d + k] * pts[i * d + k];
        out[i] = s;
    }
}

/*
 * One Sinkhorn half-step, for the listed rows only (rows == NULL: all rows).
 *
 *   out_r = -eps * LSE_j[ (pot_j - ||p_i - q_j||^2)/eps + log w_j ],  i = rows[r]
 *
 * With (p,q,w,pot) = (x,y,b,g) this is Eq. 2; with (y,x,a,f) it is Eq. 3.
 * A weight of zero gives log 0 = -inf, i.e. the term drops out of the sum; if
 * every term is -inf the LSE is -inf and the potential +inf.
 */
void fso_half_step_rows(const double *p, const double *q, int64_t np, int64_t nq, int64_t d,
                        const double *w, double eps, const double *pot,
                        const int64_t *rows, int64_t n_rows, double *out)
{
    (void)np;
#pragma omp parallel
    {
        double *z = (double *)malloc((size_t)(nq > 0 ? nq : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < n_rows; ++r) {
            int64_t i = rows ? rows[r] : r;
            double zmax = -INFINITY;
            for (int64_t j = 0; j < nq; ++j) {
                z[j] = (pot[j] - sqdist(p + i * d, q + j * d, d)) / eps + log(w[j]);
                if (z[j] > zmax) zmax = z[j];
            }
            if (zmax == -INFINITY) { out[r] = INFINITY; continue; }
            double s = 0.0;
            for (int64_t j = 0; j < nq; ++j) s += exp(z[j] - zmax);
            out[r] = -eps * (zmax + log(s));
        }
        free(z);
    }
}

/* Eq. 2: f from g. */
void fso_update_f(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                  const double *b, double eps, const double *g, double *f_out)
{
    fso_half_step_rows(x, y, n, m, d, b, eps, g, NULL, n, f_out);
}

/* Eq. 3: g from f. */
void fso_update_g(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                  const double *a, double eps, const double *f, double *g_out)
{
    fso_half_step_rows(y, x, m, n, d, a, eps, f, NULL, m, g_out);
}

/*
 * The eps of stage s of an annealed solve: geometric from eps_start to eps_end,
 * both endpoints included, evaluated in double and rounded once to float (the
 * GPU library takes float eps).  One stage: eps_end.
 */
double fso_stage_eps(double eps_start, double eps_end, int n_stages, int s)
{
    if (n_stages <= 1 || s >= n_stages - 1) return (double)(float)eps_end;
    if (s <= 0) return (double)(float)eps_start;
    double e = eps_start * pow(eps_end / eps_start, (double)s / (double)(n_stages - 1));
    return (double)(float)e;
}

/*
 * Alternating (Gauss-Seidel) schedule, App. B second bullet: in every iteration
 * f is computed from the old g, then g from the NEW f.  n_stages * iters
 * iterations in total, eps fixed within a stage; potentials carry over unchanged.
 */
void fso_solve(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
               const double *a, const double *b,
               double eps_start, double eps_end, int n_stages, int iters,
               double *f, double *g)
{
    double *fn = (double *)malloc((size_t)n * sizeof(double));
    double *gn = (double *)malloc((size_t)m * sizeof(double));
    for (int s = 0; s < n_stages; ++s) {
        double eps = fso_stage_eps(eps_start, eps_end, n_stages, s);
        for (int t = 0; t < iters; ++t) {
            fso_update_f(x, y, n, m, d, b, eps, g, fn);
            for (int64_t i = 0; i < n; ++i) f[i] = fn[i];
            fso_update_g(x, y, n, m, d, a, eps, f, gn);
            for (int64_t j = 0; j < m; ++j) g[j] = gn[j];
        }
    }
    free(fn);
    free(gn);
}

/*
 * Symmetric (Jacobi, averaged) schedule, Eq. 4-5: both half-steps read the OLD
 * potentials, and each new potential is the mean of the old one and the update.
 */
void fso_solve_symmetric(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                         const double *a, const double *b, double eps, int iters,
                         double *f, double *g)
{
    double *fn = (double *)malloc((size_t)n * sizeof(double));
    double *gn = (double *)malloc((size_t)m * sizeof(double));
    for (int t = 0; t < iters; ++t) {
        fso_update_f(x, y, n, m, d, b, eps, g, fn);
        fso_update_g(x, y, n, m, d, a, eps, f, gn);
        for (int64_t i = 0; i < n; ++i) f[i] = 0.5 * f[i] + 0.5 * fn[i];
        for (int64_t j = 0; j < m; ++j) g[j] = 0.5 * g[j] + 0.5 * gn[j];
    }
    free(fn);
    free(gn);
}

/* log P_ij = log a_i + log b_j + (f_i + g_j - C_ij)/eps  (plan formula after Eq. 3). */
static double log_plan(const double *xi, const double *yj, int64_t d, double ai, double bj,
                       double fi, double gj, double eps)
{
    return log(ai) + log(bj) + (fi + gj - sqdist(xi, yj, d)) / eps;
}

/* r = P 1_m and c = P^T 1_n of the plan induced by ANY potentials (Prop. 3). */
void fso_marginals(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                   const double *a, const double *b, double eps,
                   const double *f, const double *g, double *r, double *c)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < m; ++j)
            s += exp(log_plan(x + i * d, y + j * d, d, a[i], b[j], f[i], g[j], eps));
        r[i] = s;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i)
            s += exp(log_plan(x + i * d, y + j * d, d, a[i], b[j], f[i], g[j], eps));
        c[j] = s;
    }
}

/* L1 marginal violations: err_row = sum_i |r_i - a_i|, err_col = sum_j |c_j - b_j|. */
void fso_marginal_err(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                      const double *a, const double *b, double eps,
                      const double *f, const double *g, double *err_row, double *err_col)
{
    double *r = (double *)malloc((size_t)n * sizeof(double));
    double *c = (double *)malloc((size_t)m * sizeof(double));
    fso_marginals(x, y, n, m, d, a, b, eps, f, g, r, c);
    double er = 0.0, ec = 0.0;
    for (int64_t i = 0; i < n; ++i) er += fabs(r[i] - a[i]);
    for (int64_t j = 0; j < m; ++j) ec += fabs(c[j] - b[j]);
    *err_row = er;
    *err_col = ec;
    free(r);
    free(c);
}

/*
 * out_i = sum_j P_ij V_j for the listed rows (rows == NULL: all), V is m x p.
 * r_out (nullable) receives sum_j P_ij for the same rows.
 */
void fso_apply_plan_rows(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                         const double *a, const double *b, double eps,
                         const double *f, const double *g, const double *V, int64_t p,
                         const int64_t *rows, int64_t n_rows, double *out, double *r_out)
{
    (void)n;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double mass = 0.0;
        for (int64_t c = 0; c < p; ++c) out[r * p + c] = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            double P = exp(log_plan(x + i * d, y + j * d, d, a[i], b[j], f[i], g[j], eps));
            mass += P;
            for (int64_t c = 0; c < p; ++c) out[r * p + c] += P * V[j * p + c];
        }
        if (r_out) r_out[r] = mass;
    }
}

/*
 * out_j = sum_i P_ij U_i for the listed columns (cols == NULL: all), U is n x p.
 * c_out (nullable) receives sum_i P_ij for the same columns.
 */
void fso_apply_plan_T_rows(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                           const double *a, const double *b, double eps,
                           const double *f, const double *g, const double *U, int64_t p,
                           const int64_t *cols, int64_t n_cols, double *out, double *c_out)
{
    (void)m;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_cols; ++r) {
        int64_t j = cols ? cols[r] : r;
        double mass = 0.0;
        for (int64_t c = 0; c < p; ++c) out[r * p + c] = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double P = exp(log_plan(x + i * d, y + j * d, d, a[i], b[j], f[i], g[j], eps));
            mass += P;
            for (int64_t c = 0; c < p; ++c) out[r * p + c] += P * U[i * p + c];
        }
        if (c_out) c_out[r] = mass;
    }
}

/*
 * Objective values of the plan induced by (f, g), for the pins only:
 *   primal = <C,P> + eps * sum_ij [P log(P/(a b)) - P + a b]        (Eq. 1)
 *   dual   = <a,f> + <b,g> - eps * (sum_ij P_ij - sum_ij a_i b_j)   (App. B Lagrangian
 *            evaluated at its stationary P)
 * with log(P_ij/(a_i b_j)) = (f_i + g_j - C_ij)/eps taken from the exponent.
 */
void fso_objectives(const double *x, const double *y, int64_t n, int64_t m, int64_t d,
                    const double *a, const double *b, double eps,
                    const double *f, const double *g, double *primal, double *dual)
{
    double cp = 0.0, kl = 0.0, mass = 0.0, ab = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : cp, kl, mass, ab)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < m; ++j) {
            double C = sqdist(x + i * d, y + j * d, d);
            double e = (f[i] + g[j] - C) / eps;
            double P = a[i] * b[j] * exp(e);
            cp += C * P;
            kl += P * e - P + a[i] * b[j];
            mass += P;
            ab += a[i] * b[j];
        }
    }
    double af = 0.0, bg = 0.0;
    for (int64_t i = 0; i < n; ++i) af += a[i] * f[i];
    for (int64_t j = 0; j < m; ++j) bg += b[j] * g[j];
    *primal = cp + eps * kl;
    *dual = af + bg - eps * (mass - ab);
}
