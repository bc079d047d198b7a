/*
 * CPU oracle for alternating-least-squares matrix factorisation  R ~ X * Theta^T.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, double-precision
 * definition of what the GPU library must compute.  It shares no code with the
 * GPU path; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * Every function states the passage of the paper it follows.  Notation is the
 * paper's: R is m x n with N_z stored entries, X is m x f, Theta is n x f,
 * x_u / theta_v are rows of X / Theta, Omega_u is the set of stored column
 * ids of row u and n_u its size.
 *
 * Readings of the paper taken here
 *   - Omega_u is the sparsity structure: a stored rating of value 0 is an
 *     observation (it adds theta theta^T and lambda to A_u and 0 to b_u).
 *   - the regulariser is the weighted one of eq. (1): lambda * n_u on the
 *     diagonal of A_u (eq. (2) has lambda*I inside the sum over Omega_u).
 *   - the exact solver is Cholesky (A_u is symmetric positive definite); the
 *     paper's LU gives the same solution up to rounding.
 *   - n_u = 0: x_u = 0.
 *   - Algorithm 1's residual update is r = r - alpha * a_p (the printed
 *     "r - alpha p" does not reduce the residual; with f iterations the text
 *     says CG is exact, which only the standard update satisfies).
 *   - Algorithm 1 guards: rs_old == 0 on entry returns x unchanged; a
 *     non-positive or non-finite p^T a_p stops the iteration.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force regularised least squares
 * by QR, f = 1 closed form, identical-theta (Sherman-Morrison) closed form,
 * orthonormal closed form, normal-equation residual, monotone objective,
 * CG(f) == Cholesky, CG finite termination, CSR/CSC symmetry and invariants;
 * implicit feedback: weighted least squares by QR over all columns, f = 1 closed form,
 * alpha = 0 ridge regression, reduction to the explicit update on a fully observed row,
 * monotone implicit cost.
 * The CG-solver ALS sweep (oracle_update_rows_cg): every row against Algorithm 1 run alone on
 * that row's system and against the Krylov-space minimiser from that row's warm start,
 * f_s = 0 leaves x alone, the exact solution is a fixed point, rows without entries become 0.
 * Parity unpinned: none.
 *
 * Build: gcc -O3 -march=native -fopenmp -shared -fPIC (no -ffast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Step (i) of Section 2, eq. (2): A_u = sum_{v in Omega_u} theta_v theta_v^T + lambda*n_u*I
 * (get_hermitian) and b_u = sum_{v in Omega_u} r_uv theta_v (get_bias).
 * A is f x f row-major, full (both triangles). */
void oracle_normal_eq(int f, int64_t n_u, const int32_t *idx, const float *r, const double *Theta,
                      double lambda, double *A, double *b) {
    for (int i = 0; i < f * f; i++) A[i] = 0.0;
    for (int i = 0; i < f; i++) b[i] = 0.0;
    for (int64_t q = 0; q < n_u; q++) {
        const double *t = Theta + (int64_t)idx[q] * f;
        double ruv = (double)r[q];
        for (int i = 0; i < f; i++) {
            double ti = t[i];
            double *Ai = A + (int64_t)i * f;
            for (int j = 0; j < f; j++) Ai[j] += ti * t[j];
            b[i] += ruv * ti;
        }
    }
    for (int i = 0; i < f; i++) A[(int64_t)i * f + i] += lambda * (double)n_u;
}

/* Step (ii) of Section 2 ("solve"), exact: textbook Cholesky A = L L^T followed by
 * L y = b and L^T x = y.  A is overwritten by L (lower triangle), b by x.
 * Returns 0, or -1 if a pivot is not positive. */
int oracle_cholesky_solve(int f, double *A, double *b) {
    for (int j = 0; j < f; j++) {
        double d = A[(int64_t)j * f + j];
        for (int k = 0; k < j; k++) d -= A[(int64_t)j * f + k] * A[(int64_t)j * f + k];
        if (!(d > 0.0)) return -1;
        d = sqrt(d);
        A[(int64_t)j * f + j] = d;
        for (int i = j + 1; i < f; i++) {
            double s = A[(int64_t)i * f + j];
            for (int k = 0; k < j; k++) s -= A[(int64_t)i * f + k] * A[(int64_t)j * f + k];
            A[(int64_t)i * f + j] = s / d;
        }
    }
    for (int i = 0; i < f; i++) {
        double s = b[i];
        for (int k = 0; k < i; k++) s -= A[(int64_t)i * f + k] * b[k];
        b[i] = s / A[(int64_t)i * f + i];
    }
    for (int i = f - 1; i >= 0; i--) {
        double s = b[i];
        for (int k = i + 1; k < f; k++) s -= A[(int64_t)k * f + i] * b[k];
        b[i] = s / A[(int64_t)i * f + i];
    }
    return 0;
}

/* Algorithm 1 (CGSolve) of Section 4.1 in double precision: at most fs
 * iterations from the x passed in, absolute tolerance eps on sqrt(r^T r).
 * A is f x f row-major.  Returns the number of iterations performed. */
int oracle_cg(int f, const double *A, double *x, const double *b, int fs, double eps) {
    double *r = (double *)malloc(sizeof(double) * 3 * (size_t)f);
    double *p = r + f, *ap = p + f;
    double rs_old = 0.0;
    for (int i = 0; i < f; i++) {
        double s = 0.0;
        for (int j = 0; j < f; j++) s += A[(int64_t)i * f + j] * x[j];
        r[i] = b[i] - s;
        p[i] = r[i];
        rs_old += r[i] * r[i];
    }
    int it = 0;
    if (rs_old == 0.0) { free(r); return 0; }
    for (it = 0; it < fs;) {
        double pap = 0.0;
        for (int i = 0; i < f; i++) {
            double s = 0.0;
            for (int j = 0; j < f; j++) s += A[(int64_t)i * f + j] * p[j];
            ap[i] = s;
            pap += p[i] * s;
        }
        if (!(pap > 0.0) || !isfinite(pap)) break;
        double alpha = rs_old / pap;
        double rs_new = 0.0;
        for (int i = 0; i < f; i++) {
            x[i] += alpha * p[i];
            r[i] -= alpha * ap[i];
            rs_new += r[i] * r[i];
        }
        it++;
        if (sqrt(rs_new) < eps) break;
        double beta = rs_new / rs_old;
        for (int i = 0; i < f; i++) p[i] = r[i] + beta * p[i];
        rs_old = rs_new;
    }
    free(r);
    return it;
}

/* "Update X" of Section 2 (eq. (2)) for every row of a CSR matrix, exact solver.
 * With the CSC of R and X in Theta's place it is "Update Theta" (eq. (3)).
 * X is m x f, written; Theta is n x f.  Returns the number of failed pivots. */
int64_t oracle_update_rows(int64_t m, const int64_t *ptr, const int32_t *idx, const float *val,
                           const double *Theta, int f, double lambda, double *X) {
    int64_t bad = 0;
#pragma omp parallel reduction(+ : bad)
    {
        double *A = (double *)malloc(sizeof(double) * ((size_t)f * f + f));
        double *b = A + (size_t)f * f;
#pragma omp for schedule(dynamic, 16)
        for (int64_t u = 0; u < m; u++) {
            int64_t s = ptr[u], n_u = ptr[u + 1] - ptr[u];
            double *x = X + u * f;
            if (n_u == 0) { for (int i = 0; i < f; i++) x[i] = 0.0; continue; }
            oracle_normal_eq(f, n_u, idx + s, val + s, Theta, lambda, A, b);
            if (oracle_cholesky_solve(f, A, b) != 0) bad++;
            for (int i = 0; i < f; i++) x[i] = b[i];
        }
        free(A);
    }
    return bad;
}

/* The same update for a list of selected rows only: X_sel is nsel x f. */
int64_t oracle_update_selected(int64_t nsel, const int64_t *rows, const int64_t *ptr, const int32_t *idx,
                               const float *val, const double *Theta, int f, double lambda, double *X_sel) {
    int64_t bad = 0;
#pragma omp parallel reduction(+ : bad)
    {
        double *A = (double *)malloc(sizeof(double) * ((size_t)f * f + f));
        double *b = A + (size_t)f * f;
#pragma omp for schedule(dynamic, 4)
        for (int64_t q = 0; q < nsel; q++) {
            int64_t u = rows[q];
            int64_t s = ptr[u], n_u = ptr[u + 1] - ptr[u];
            double *x = X_sel + q * f;
            if (n_u == 0) { for (int i = 0; i < f; i++) x[i] = 0.0; continue; }
            oracle_normal_eq(f, n_u, idx + s, val + s, Theta, lambda, A, b);
            if (oracle_cholesky_solve(f, A, b) != 0) bad++;
            for (int i = 0; i < f; i++) x[i] = b[i];
        }
        free(A);
    }
    return bad;
}

/* "Update X" with the approximate solver of Section 4.1: the normal equations
 * of eq. (2), then Algorithm 1 warm-started from the current x_u (X is in/out). */
void oracle_update_rows_cg(int64_t m, const int64_t *ptr, const int32_t *idx, const float *val,
                           const double *Theta, int f, double lambda, int fs, double eps, double *X) {
#pragma omp parallel
    {
        double *A = (double *)malloc(sizeof(double) * ((size_t)f * f + f));
        double *b = A + (size_t)f * f;
#pragma omp for schedule(dynamic, 16)
        for (int64_t u = 0; u < m; u++) {
            int64_t s = ptr[u], n_u = ptr[u + 1] - ptr[u];
            double *x = X + u * f;
            if (n_u == 0) { for (int i = 0; i < f; i++) x[i] = 0.0; continue; }
            oracle_normal_eq(f, n_u, idx + s, val + s, Theta, lambda, A, b);
            oracle_cg(f, A, x, b, fs, eps);
        }
        free(A);
    }
}

/* Sum of squared errors over the stored entries, sum_{(u,v)} (r_uv - x_u^T theta_v)^2:
 * the data term of eq. (1); the RMSE of Section 5.2 is sqrt(sse / N_z).
 * Rows are summed in order, each row's partial sum first. */
double oracle_sse(int64_t m, const int64_t *ptr, const int32_t *idx, const float *val,
                  const double *X, const double *Theta, int f) {
    double total = 0.0;
    for (int64_t u = 0; u < m; u++) {
        double row = 0.0;
        const double *x = X + u * f;
        for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) {
            const double *t = Theta + (int64_t)idx[q] * f;
            double dot = 0.0;
            for (int i = 0; i < f; i++) dot += x[i] * t[i];
            double e = (double)val[q] - dot;
            row += e * e;
        }
        total += row;
    }
    return total;
}

/* The same sum with the rows spread over threads (per-row partial sums are
 * stored and then added in row order, so the result equals oracle_sse). */
double oracle_sse_parallel(int64_t m, const int64_t *ptr, const int32_t *idx, const float *val,
                           const double *X, const double *Theta, int f) {
    double *rows = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < m; u++) {
        double row = 0.0;
        const double *x = X + u * f;
        for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) {
            const double *t = Theta + (int64_t)idx[q] * f;
            double dot = 0.0;
            for (int i = 0; i < f; i++) dot += x[i] * t[i];
            double e = (double)val[q] - dot;
            row += e * e;
        }
        rows[u] = row;
    }
    double total = 0.0;
    for (int64_t u = 0; u < m; u++) total += rows[u];
    free(rows);
    return total;
}

/* The same sum for single-precision factors (read as they are, all arithmetic in double): lets a
 * caller with tens of gigabytes of factors avoid a double-precision copy. */
double oracle_sse_parallel_f32(int64_t m, const int64_t *ptr, const int32_t *idx, const float *val,
                               const float *X, const float *Theta, int f) {
    double *rows = (double *)malloc(sizeof(double) * (size_t)(m > 0 ? m : 1));
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t u = 0; u < m; u++) {
        double row = 0.0;
        const float *x = X + u * f;
        for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) {
            const float *t = Theta + (int64_t)idx[q] * f;
            double dot = 0.0;
            for (int i = 0; i < f; i++) dot += (double)x[i] * (double)t[i];
            double e = (double)val[q] - dot;
            row += e * e;
        }
        rows[u] = row;
    }
    double total = 0.0;
    for (int64_t u = 0; u < m; u++) total += rows[u];
    free(rows);
    return total;
}

/* Regulariser of eq. (1): lambda * ( sum_u n_{x_u} ||x_u||^2 + sum_v n_{theta_v} ||theta_v||^2 ),
 * n_{x_u} / n_{theta_v} being the numbers of stored entries in row u / column v. */
double oracle_regulariser(int64_t m, int64_t n, const int64_t *ptr, const int32_t *idx,
                          const double *X, const double *Theta, int f, double lambda) {
    int64_t *cnt = (int64_t *)calloc((size_t)(n > 0 ? n : 1), sizeof(int64_t));
    double sx = 0.0, st = 0.0;
    for (int64_t u = 0; u < m; u++) {
        int64_t n_u = ptr[u + 1] - ptr[u];
        for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) cnt[idx[q]]++;
        double nn = 0.0;
        for (int i = 0; i < f; i++) nn += X[u * f + i] * X[u * f + i];
        sx += (double)n_u * nn;
    }
    for (int64_t v = 0; v < n; v++) {
        double nn = 0.0;
        for (int i = 0; i < f; i++) nn += Theta[v * f + i] * Theta[v * f + i];
        st += (double)cnt[v] * nn;
    }
    free(cnt);
    return lambda * (sx + st);
}

/* CSC of R from its CSR (equivalently the CSR of R^T): counting sort by column,
 * rows visited in ascending order so every column lists its rows ascending. */
void oracle_csr_to_csc(int64_t m, int64_t n, const int64_t *ptr, const int32_t *idx, const float *val,
                       int64_t *cptr, int32_t *cidx, float *cval) {
    for (int64_t v = 0; v <= n; v++) cptr[v] = 0;
    for (int64_t q = 0; q < ptr[m]; q++) cptr[idx[q] + 1]++;
    for (int64_t v = 0; v < n; v++) cptr[v + 1] += cptr[v];
    int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t v = 0; v < n; v++) cur[v] = cptr[v];
    for (int64_t u = 0; u < m; u++)
        for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) {
            int64_t dst = cur[idx[q]]++;
            cidx[dst] = (int32_t)u;
            cval[dst] = val[q];
        }
    free(cur);
}

/* Degree class of a row for load balancing (not in the paper, which launches
 * one block per row regardless of length): class 0 for n_u = 0, otherwise
 * 1 + floor(log2(n_u)), capped at nclass-1. */
static int degree_class(int64_t n_u, int nclass) {
    if (n_u <= 0) return 0;
    int c = 1;
    while (n_u > 1) { n_u >>= 1; c++; }
    return c < nclass ? c : nclass - 1;
}

/* Rows grouped by degree class, heaviest class first, original order kept
 * inside a class (a stable counting sort).  perm has m entries;
 * class_start has nclass+1 entries: rows of class c occupy
 * perm[class_start[nclass-1-c] .. class_start[nclass-c]). */
void oracle_bin_rows(int64_t m, const int64_t *ptr, int nclass, int32_t *perm, int64_t *class_start) {
    int64_t *count = (int64_t *)calloc((size_t)nclass + 1, sizeof(int64_t));
    for (int64_t u = 0; u < m; u++) count[nclass - 1 - degree_class(ptr[u + 1] - ptr[u], nclass)]++;
    class_start[0] = 0;
    for (int c = 0; c < nclass; c++) class_start[c + 1] = class_start[c] + count[c];
    for (int c = 0; c < nclass; c++) count[c] = class_start[c];
    for (int64_t u = 0; u < m; u++) {
        int slot = nclass - 1 - degree_class(ptr[u + 1] - ptr[u], nclass);
        perm[count[slot]++] = (int32_t)u;
    }
    free(count);
}

/* ---- implicit feedback (Section 5.6) -------------------------------------------------------
 * Cost: sum over ALL m*n pairs of c_uv (p_uv - x_u^T theta_v)^2 with p_uv = 1 if r_uv > 0 else 0 and
 * confidence c_uv = 1 + alpha*r_uv; pairs that are not stored have r_uv = 0 (p = 0, c = 1).
 * Readings: the printed cost has no regulariser, the method it follows has lambda*(|X|^2 + |Theta|^2),
 * not weighted by n_u: that is what is added here.  A stored r_uv <= 0 counts like a missing pair
 * (c = 1 + alpha*max(r,0)); the paper defines p and c for r >= 0 only.
 *
 * The row update is the ridge regression over all n columns, written out as its definition:
 *   A_u = sum_v c_uv theta_v theta_v^T + lambda*I,   b_u = sum_v c_uv p_uv theta_v
 * (no Theta^T Theta shortcut).  cdense is scratch of n doubles, all zero on entry and on return. */
void oracle_implicit_normal_eq(int f, int64_t n, int64_t n_u, const int32_t *idx, const float *r,
                               const double *Theta, double lambda, double alpha, double *A, double *b,
                               double *cdense) {
    for (int i = 0; i < f * f; i++) A[i] = 0.0;
    for (int i = 0; i < f; i++) b[i] = 0.0;
    for (int64_t q = 0; q < n_u; q++) cdense[idx[q]] = r[q] > 0.f ? (double)r[q] : 0.0;
    for (int64_t v = 0; v < n; v++) {
        const double *t = Theta + v * f;
        double ruv = cdense[v];
        double c = 1.0 + alpha * ruv, p = ruv > 0.0 ? 1.0 : 0.0;
        for (int i = 0; i < f; i++) {
            double cti = c * t[i];
            double *Ai = A + (int64_t)i * f;
            for (int j = 0; j < f; j++) Ai[j] += cti * t[j];
            b[i] += c * p * t[i];
        }
    }
    for (int i = 0; i < f; i++) A[(int64_t)i * f + i] += lambda;
    for (int64_t q = 0; q < n_u; q++) cdense[idx[q]] = 0.0;
}

/* Implicit "Update X" for the listed rows (rows == NULL: rows 0..nsel-1), exact solver.
 * Theta is n x f.  With the CSC of R and X it is the implicit "Update Theta".  Returns failed pivots. */
int64_t oracle_implicit_update_selected(int64_t nsel, const int64_t *rows, const int64_t *ptr, const int32_t *idx,
                                        const float *val, const double *Theta, int64_t n, int f, double lambda,
                                        double alpha, double *X_sel) {
    int64_t bad = 0;
#pragma omp parallel reduction(+ : bad)
    {
        double *A = (double *)malloc(sizeof(double) * ((size_t)f * f + f));
        double *b = A + (size_t)f * f;
        double *cdense = (double *)calloc((size_t)n, sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < nsel; q++) {
            int64_t u = rows ? rows[q] : q;
            int64_t s = ptr[u], n_u = ptr[u + 1] - ptr[u];
            oracle_implicit_normal_eq(f, n, n_u, idx + s, val + s, Theta, lambda, alpha, A, b, cdense);
            if (oracle_cholesky_solve(f, A, b) != 0) bad++;
            for (int i = 0; i < f; i++) X_sel[q * f + i] = b[i];
        }
        free(A);
        free(cdense);
    }
    return bad;
}

/* The implicit cost itself, over all m*n pairs, plus lambda*(|X|_F^2 + |Theta|_F^2).  O(m*n*f). */
double oracle_implicit_objective(int64_t m, int64_t n, const int64_t *ptr, const int32_t *idx, const float *val,
                                 const double *X, const double *Theta, int f, double lambda, double alpha) {
    double total = 0.0;
#pragma omp parallel reduction(+ : total)
    {
        double *rdense = (double *)calloc((size_t)n, sizeof(double));
#pragma omp for schedule(static)
        for (int64_t u = 0; u < m; u++) {
            for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) rdense[idx[q]] = val[q] > 0.f ? (double)val[q] : 0.0;
            const double *x = X + u * f;
            double row = 0.0;
            for (int64_t v = 0; v < n; v++) {
                const double *t = Theta + v * f;
                double d = 0.0;
                for (int i = 0; i < f; i++) d += x[i] * t[i];
                double c = 1.0 + alpha * rdense[v], p = rdense[v] > 0.0 ? 1.0 : 0.0;
                row += c * (p - d) * (p - d);
            }
            for (int64_t q = ptr[u]; q < ptr[u + 1]; q++) rdense[idx[q]] = 0.0;
            total += row;
        }
        free(rdense);
    }
    double reg = 0.0;
    for (int64_t q = 0; q < m * f; q++) reg += X[q] * X[q];
    for (int64_t q = 0; q < n * f; q++) reg += Theta[q] * Theta[q];
    return total + lambda * reg;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
