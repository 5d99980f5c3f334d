/*
 * fp64 CPU oracle for Local Linear Attention (arxiv 2510.01450).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is slow on
 * purpose and shares no code, header, table or helper with the HIP path.  Only tests/, the smoke
 * check and the CPU-baseline leg of the benchmark may call it.
 *
 * What it computes (Section 2.3, "Local Linear Attention", objective Eq. (lla_obj)):
 * for one head with queries q_i, keys k_j, values v_j and a query row i, fit
 *
 *      f(x) = b + W (x - q_i)
 *
 * by weighted ridge least squares over the visible keys (j <= i when causal, Section 3.2 matrix
 * form with the tril mask), weights w_ij, ridge only on W; the output is the intercept b.
 * The normal equations of that objective are written out and solved directly:
 *
 *      x_j  = [1 ; k_j - q_i]                       (d+1 vector, the design row)
 *      A    = sum_j w_ij x_j x_j^T + lambda * diag(0, 1, ..., 1)
 *      Bv   = sum_j w_ij x_j v_j^T                  ((d+1) x dv)
 *      A Theta = Bv,   o_i = first row of Theta     (the intercept b)
 *
 * A's blocks are omega_i, mu_i and Sigma_i of Eq. (query_specific).  "+lambda I" follows that
 * equation (not the factor a literal derivative of the printed objective would give).
 *
 * Weights: w_ij = exp(scale * <q_i, k_j> - m_i) with m_i the maximum logit over the visible keys
 * of row i.  This is the weight Algorithm 1 (FlashLLA forward) ends up using once all key blocks
 * have been seen (its running maximum equals the true row maximum), and lambda is added to
 * moments of exactly these max-shifted weights, as in Algorithms 1 and 2.
 *
 * Optional extras of the *_ex entry point: a ridge per query row (Appendix C makes lambda a learnable,
 * position-dependent quantity; row i then uses lambda_i in its own normal equations and nothing else
 * changes), and the two per-row statistics of Eq. (lla) that FlashLLA keeps for its backward pass
 * (end of Section 3.2): rho_i = Sigma_i^{-1} mu_i and delta_i = omega_i - mu_i^T rho_i, computed here
 * from the blocks omega_i, mu_i, Sigma_i of A by a second, separate Cholesky of the d x d block.
 *
 * Nothing here is blocked, fused, recentred or iterated: no tilde moments, no relmm, no CG.
 * Build: gcc -O2 -fopenmp -shared -fPIC -o libllla_oracle.so llla_oracle.c -lm
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* In-place Cholesky A = L L^T of a symmetric positive definite p x p matrix (row-major, lower
 * triangle used and overwritten).  Returns 0 on success, 1 if a pivot is not positive. */
static int chol_factor(double *A, int p)
{
    for (int c = 0; c < p; ++c) {
        double diag = A[c * p + c];
        for (int t = 0; t < c; ++t) diag -= A[c * p + t] * A[c * p + t];
        if (!(diag > 0.0)) return 1;
        diag = sqrt(diag);
        A[c * p + c] = diag;
        for (int r = c + 1; r < p; ++r) {
            double s = A[r * p + c];
            for (int t = 0; t < c; ++t) s -= A[r * p + t] * A[c * p + t];
            A[r * p + c] = s / diag;
        }
    }
    return 0;
}

/* Solve L L^T X = B for X (B is p x m, row-major, overwritten by X). */
static void chol_solve(const double *L, int p, double *B, int m)
{
    for (int r = 0; r < p; ++r) {            /* forward: L Y = B */
        for (int t = 0; t < r; ++t)
            for (int c = 0; c < m; ++c) B[r * m + c] -= L[r * p + t] * B[t * m + c];
        for (int c = 0; c < m; ++c) B[r * m + c] /= L[r * p + r];
    }
    for (int r = p - 1; r >= 0; --r) {       /* backward: L^T X = Y */
        for (int t = r + 1; t < p; ++t)
            for (int c = 0; c < m; ++c) B[r * m + c] -= L[t * p + r] * B[t * m + c];
        for (int c = 0; c < m; ++c) B[r * m + c] /= L[r * p + r];
    }
}

/* One query against nk keys.  q: [d]; K: [nk, d]; V: [nk, dv]; out: [dv].
 * scratch: (d+1)*(d+1) + (d+1)*dv + nk doubles.  Returns 0, or 1 if A is not positive definite. */
static int lla_one_query(const double *q, const double *K, const double *V, int nk, int d, int dv,
                         double lambda, double scale, double *out, double *scratch, double *rho,
                         double *delta)
{
    const int p = d + 1;
    double *A = scratch;
    double *Bv = A + (size_t)p * p;
    double *w = Bv + (size_t)p * dv;
    double *x = (double *)malloc(sizeof(double) * p);
    if (!x) return 2;

    /* logits, their maximum over the visible keys, max-shifted weights (Alg. 1, weight lines) */
    double m = -INFINITY;
    for (int j = 0; j < nk; ++j) {
        double s = 0.0;
        for (int a = 0; a < d; ++a) s += q[a] * K[(size_t)j * d + a];
        w[j] = scale * s;
        if (w[j] > m) m = w[j];
    }
    for (int j = 0; j < nk; ++j) w[j] = exp(w[j] - m);

    /* normal equations of Eq. (lla_obj) */
    memset(A, 0, sizeof(double) * p * p);
    memset(Bv, 0, sizeof(double) * p * dv);
    for (int j = 0; j < nk; ++j) {
        x[0] = 1.0;
        for (int a = 0; a < d; ++a) x[a + 1] = K[(size_t)j * d + a] - q[a];
        for (int r = 0; r < p; ++r) {
            const double wx = w[j] * x[r];
            for (int c = 0; c <= r; ++c) A[r * p + c] += wx * x[c];
            for (int c = 0; c < dv; ++c) Bv[r * dv + c] += wx * V[(size_t)j * dv + c];
        }
    }
    for (int r = 1; r < p; ++r) A[r * p + r] += lambda;   /* ridge on W only, not on b */

    if (rho || delta) {
        /* Eq. (lla): rho = Sigma^{-1} mu, delta = omega - mu^T rho, with omega = A[0][0], mu = A[1:,0] and
         * Sigma (ridge included) = A[1:,1:]; the lower triangle of A is what was accumulated above */
        double *Sg = (double *)malloc(sizeof(double) * (size_t)d * d);
        double *rh = (double *)malloc(sizeof(double) * (size_t)d);
        if (!Sg || !rh) { free(Sg); free(rh); free(x); return 2; }
        for (int r = 0; r < d; ++r) {
            for (int c = 0; c <= r; ++c) Sg[r * d + c] = A[(r + 1) * p + (c + 1)];
            rh[r] = A[(r + 1) * p];
        }
        int sbad = chol_factor(Sg, d);
        if (!sbad) {
            chol_solve(Sg, d, rh, 1);
            double dl = A[0];
            for (int r = 0; r < d; ++r) dl -= A[(r + 1) * p] * rh[r];
            if (rho) for (int r = 0; r < d; ++r) rho[r] = rh[r];
            if (delta) *delta = dl;
        }
        free(Sg);
        free(rh);
        if (sbad) { free(x); return 1; }
    }

    int bad = chol_factor(A, p);
    if (!bad) {
        chol_solve(A, p, Bv, dv);
        for (int c = 0; c < dv; ++c) out[c] = Bv[c];      /* row 0 of Theta = intercept */
    }
    free(x);
    return bad;
}

/*
 * Selected rows of one head.
 *   Q [n, d], K [n, d], V [n, dv] row-major fp64; rows[nrows] are 0-based query indices;
 *   causal != 0: row i sees keys 0..i inclusive; causal == 0: every row sees all n keys.
 *   O [nrows, dv] receives the outputs in the order of rows[].
 *   lambda_rows: NULL, or [n] ridges, row i using lambda_rows[i] instead of lambda.
 *   R [nrows, d] and Delta [nrows]: NULL, or receive rho_i and delta_i of Eq. (lla).
 * Returns the number of rows whose normal matrix was not positive definite (0 when lambda > 0).
 */
int llla_oracle_rows_ex(const double *Q, const double *K, const double *V, int n, int d, int dv,
                        double lambda, const double *lambda_rows, double scale, int causal, const int *rows,
                        int nrows, double *O, double *R, double *Delta)
{
    int failures = 0;
    const size_t per = (size_t)(d + 1) * (d + 1) + (size_t)(d + 1) * dv + (size_t)n;
#pragma omp parallel reduction(+ : failures)
    {
        double *scratch = (double *)malloc(sizeof(double) * per);
#pragma omp for schedule(dynamic, 1)
        for (int t = 0; t < nrows; ++t) {
            const int i = rows[t];
            const int nk = causal ? i + 1 : n;
            if (!scratch || i < 0 || i >= n) { failures += 1; continue; }
            failures += lla_one_query(Q + (size_t)i * d, K, V, nk, d, dv, lambda_rows ? lambda_rows[i] : lambda,
                                      scale, O + (size_t)t * dv, scratch, R ? R + (size_t)t * d : NULL,
                                      Delta ? Delta + t : NULL) ? 1 : 0;
        }
        free(scratch);
    }
    return failures;
}

/* The same with one ridge for all rows and no statistics. */
int llla_oracle_rows(const double *Q, const double *K, const double *V, int n, int d, int dv,
                     double lambda, double scale, int causal, const int *rows, int nrows, double *O)
{
    return llla_oracle_rows_ex(Q, K, V, n, d, dv, lambda, NULL, scale, causal, rows, nrows, O, NULL, NULL);
}

/*
 * Decode: one new query against a cache of L keys/values in which the new token's own (k, v) is
 * already the last entry; by the query-independence of Eq. (query_specific) this is the last
 * row of a causal forward over L positions.  q [d], K [L, d], V [L, dv], o [dv].
 */
int llla_oracle_decode(const double *q, const double *K, const double *V, int L, int d, int dv,
                       double lambda, double scale, double *o)
{
    const size_t per = (size_t)(d + 1) * (d + 1) + (size_t)(d + 1) * dv + (size_t)L;
    double *scratch = (double *)malloc(sizeof(double) * per);
    if (!scratch) return 2;
    int bad = lla_one_query(q, K, V, L, d, dv, lambda, scale, o, scratch, NULL, NULL);
    free(scratch);
    return bad;
}

/*
 * Batched decode, OpenMP over the nh independent (batch, head) pairs.
 *   q [nh, d]; K [nh, Lmax, d]; V [nh, Lmax, dv]; lens[nh] valid cache lengths (1..Lmax); o [nh, dv].
 * Returns the number of heads whose normal matrix was not positive definite.
 */
int llla_oracle_decode_batch(const double *q, const double *K, const double *V, const int *lens,
                             int nh, int Lmax, int d, int dv, double lambda, double scale, double *o)
{
    int failures = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : failures)
    for (int h = 0; h < nh; ++h) {
        int L = lens[h];
        if (L < 1 || L > Lmax) { failures += 1; continue; }
        failures += llla_oracle_decode(q + (size_t)h * d, K + (size_t)h * Lmax * d,
                                       V + (size_t)h * Lmax * dv, L, d, dv, lambda, scale,
                                       o + (size_t)h * dv) ? 1 : 0;
    }
    return failures;
}

/*
 * Approximate mode: the paper's own way of getting rho_i (Section 3.1, "Matrix-free inversion via conjugate
 * gradients", and the CG solver of Appendix C).  Sigma_i rho = mu_i is solved by T steps of the textbook
 * conjugate-gradient recursion started at X = 0 (so the first residual and search direction are mu_i), with the
 * matrix only ever applied to a vector, in the matrix-free form of Section 3.1:
 *     Sigma p = sum_j w_j (k_j . p) k_j - (q . p) mu~ - (mu~ . p) q + omega (q . p) q + lambda p,
 * mu~ = sum_j w_j k_j the un-centred first moment.  (The printed solver's correction line reads Y where the search
 * direction P is meant; the matvec equation of Section 3.1 is followed.)  A system whose residual norm is at or below
 * eps when an iteration starts is frozen (the paper's active mask; "at or" so that eps = 0 still stops a system whose
 * residual has become exactly zero instead of dividing 0 by 0).  Then delta = omega - mu . rho and the output is
 * Eq. (lla) with those rho, delta.  Everything in fp64, no blocking.
 * used[t] receives the number of iterations row rows[t] actually performed (may be NULL).
 */
static void cg_one_query(const double *q, const double *K, const double *V, int nk, int d, int dv, double lambda,
                         double scale, int T, double eps, double *out, double *rho_out, double *delta_out, int *used)
{
    double *w = (double *)malloc(sizeof(double) * nk);
    double *mut = (double *)calloc(d, sizeof(double));      /* mu~ */
    double *mu = (double *)malloc(sizeof(double) * d);
    double *x = (double *)calloc(d, sizeof(double));
    double *r = (double *)malloc(sizeof(double) * d);
    double *p = (double *)malloc(sizeof(double) * d);
    double *sp = (double *)malloc(sizeof(double) * d);
    double m = -INFINITY, omega = 0.0;
    for (int j = 0; j < nk; ++j) {
        double s = 0.0;
        for (int a = 0; a < d; ++a) s += q[a] * K[(size_t)j * d + a];
        w[j] = scale * s;
        if (w[j] > m) m = w[j];
    }
    for (int j = 0; j < nk; ++j) {
        w[j] = exp(w[j] - m);
        omega += w[j];
        for (int a = 0; a < d; ++a) mut[a] += w[j] * K[(size_t)j * d + a];
    }
    for (int a = 0; a < d; ++a) { mu[a] = mut[a] - omega * q[a]; r[a] = mu[a]; p[a] = mu[a]; }
    int it = 0;
    for (; it < T; ++it) {
        double rr = 0.0;
        for (int a = 0; a < d; ++a) rr += r[a] * r[a];
        if (sqrt(rr) <= eps) break;                          /* active mask: this system is done (also at rr == 0) */
        double qp = 0.0, mp = 0.0;
        for (int a = 0; a < d; ++a) { qp += q[a] * p[a]; mp += mut[a] * p[a]; sp[a] = 0.0; }
        for (int j = 0; j < nk; ++j) {
            double kp = 0.0;
            for (int a = 0; a < d; ++a) kp += K[(size_t)j * d + a] * p[a];
            for (int a = 0; a < d; ++a) sp[a] += w[j] * kp * K[(size_t)j * d + a];
        }
        double psp = 0.0;
        for (int a = 0; a < d; ++a) {
            sp[a] += -qp * mut[a] - mp * q[a] + omega * qp * q[a] + lambda * p[a];
            psp += p[a] * sp[a];
        }
        const double alpha = rr / psp;
        double rr2 = 0.0;
        for (int a = 0; a < d; ++a) { x[a] += alpha * p[a]; r[a] -= alpha * sp[a]; rr2 += r[a] * r[a]; }
        const double beta = rr2 / rr;
        for (int a = 0; a < d; ++a) p[a] = r[a] + beta * p[a];
    }
    double delta = omega;
    for (int a = 0; a < d; ++a) delta -= mu[a] * x[a];
    for (int c = 0; c < dv; ++c) out[c] = 0.0;
    for (int j = 0; j < nk; ++j) {                           /* Eq. (lla) with the approximate rho */
        double zr = 0.0;
        for (int a = 0; a < d; ++a) zr += (K[(size_t)j * d + a] - q[a]) * x[a];
        const double sj = w[j] * (1.0 - zr) / delta;
        for (int c = 0; c < dv; ++c) out[c] += sj * V[(size_t)j * dv + c];
    }
    if (rho_out) for (int a = 0; a < d; ++a) rho_out[a] = x[a];
    if (delta_out) *delta_out = delta;
    if (used) *used = it;
    free(w); free(mut); free(mu); free(x); free(r); free(p); free(sp);
}

int llla_oracle_rows_cg(const double *Q, const double *K, const double *V, int n, int d, int dv, double lambda,
                        double scale, int causal, int T, double eps, const int *rows, int nrows, double *O,
                        double *R, double *Delta, int *used)
{
    int failures = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : failures)
    for (int t = 0; t < nrows; ++t) {
        const int i = rows[t];
        if (i < 0 || i >= n) { failures += 1; continue; }
        cg_one_query(Q + (size_t)i * d, K, V, causal ? i + 1 : n, d, dv, lambda, scale, T, eps, O + (size_t)t * dv,
                     R ? R + (size_t)t * d : NULL, Delta ? Delta + t : NULL, used ? used + t : NULL);
    }
    return failures;
}

int llla_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
