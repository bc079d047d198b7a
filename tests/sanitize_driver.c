/* Runs the input generator and every function of the CPU oracle on the tiny workload (2,000 x 1,000, 60,000
 * entries, f = 16) in one executable that tests/test_sanitizers.py builds with -fsanitize=address,undefined:
 * out-of-bounds accesses, leaks of the per-thread buffers, signed overflow and misaligned accesses in either file
 * end the run with a non-zero status.  It also checks the invariants that need no second implementation
 * (objective non-increasing over exact half-sweeps, transposing twice gives the matrix back).
 * Test infrastructure: it includes the two sources so that nothing else is linked. */
#include <stdio.h>

#include "../workload/synth.c"
#include "../oracle/als_oracle.c"

#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); \
            return 1;                                                   \
        }                                                               \
    } while (0)

int main(void) {
    const int f = 16;
    const double lam = 0.05;
    synth_config cfg = {2000, 1000, 60000, 1.1, 1, 300, 0.8, 8, 0.6, 0.5, 0, 0};
    synth_handle *h = synth_create(&cfg);
    CHECK(h != NULL);
    const int64_t m = cfg.m, n = cfg.n;
    int64_t *deg = malloc(sizeof(int64_t) * m), *ptr = malloc(sizeof(int64_t) * (m + 1));
    CHECK(synth_degrees(h, deg) == 0);
    ptr[0] = 0;
    for (int64_t u = 0; u < m; u++) ptr[u + 1] = ptr[u] + deg[u];
    const int64_t nnz = ptr[m];
    CHECK(nnz == cfg.nnz);
    int32_t *idx = malloc(sizeof(int32_t) * nnz);
    float *val = malloc(sizeof(float) * nnz);
    CHECK(synth_fill_rows(h, 0, m, ptr, idx, val) == 0);
    for (int64_t u = 0; u < m; u++)
        for (int64_t q = ptr[u]; q + 1 < ptr[u + 1]; q++) CHECK(idx[q] < idx[q + 1] && idx[q] >= 0 && idx[q + 1] < n);

    int64_t *cptr = malloc(sizeof(int64_t) * (n + 1)), *rptr = malloc(sizeof(int64_t) * (m + 1));
    int32_t *cidx = malloc(sizeof(int32_t) * nnz), *ridx = malloc(sizeof(int32_t) * nnz);
    float *cval = malloc(sizeof(float) * nnz), *rval = malloc(sizeof(float) * nnz);
    oracle_csr_to_csc(m, n, ptr, idx, val, cptr, cidx, cval);
    oracle_csr_to_csc(n, m, cptr, cidx, cval, rptr, ridx, rval);
    CHECK(memcmp(rptr, ptr, sizeof(int64_t) * (m + 1)) == 0 && memcmp(ridx, idx, sizeof(int32_t) * nnz) == 0 &&
          memcmp(rval, val, sizeof(float) * nnz) == 0);

    double *X = calloc((size_t)m * f, sizeof(double)), *T = malloc(sizeof(double) * n * f);
    uint64_t s = 12345;
    for (int64_t i = 0; i < n * f; i++) {
        s = s * 6364136223846793005ull + 1442695040888963407ull;
        T[i] = (double)(s >> 11) / 9007199254740992.0 / 4.0;
    }
    double prev = 1e300;
    for (int sweep = 0; sweep < 2; sweep++) {
        CHECK(oracle_update_rows(m, ptr, idx, val, T, f, lam, X) == 0);
        double j1 = oracle_sse(m, ptr, idx, val, X, T, f) + oracle_regulariser(m, n, ptr, idx, X, T, f, lam);
        CHECK(j1 <= prev);
        CHECK(oracle_update_rows(n, cptr, cidx, cval, X, f, lam, T) == 0);
        double j2 = oracle_sse(m, ptr, idx, val, X, T, f) + oracle_regulariser(m, n, ptr, idx, X, T, f, lam);
        CHECK(j2 <= j1);
        prev = j2;
    }
    CHECK(fabs(oracle_sse_parallel(m, ptr, idx, val, X, T, f) - oracle_sse(m, ptr, idx, val, X, T, f)) <= 1e-9 * prev);
    oracle_update_rows_cg(m, ptr, idx, val, T, f, lam, 6, 0.0, X);
    oracle_update_rows_cg(n, cptr, cidx, cval, X, f, lam, 3, 1e-3, T);
    int64_t sel[5] = {0, 1, m / 2, m - 2, m - 1};
    double *Xs = malloc(sizeof(double) * 5 * f);
    CHECK(oracle_update_selected(5, sel, ptr, idx, val, T, f, lam, Xs) == 0);
    CHECK(oracle_implicit_update_selected(5, sel, ptr, idx, val, T, n, f, 0.5, 2.0, Xs) == 0);
    CHECK(oracle_implicit_update_selected(3, NULL, ptr, idx, val, T, n, f, 0.5, 2.0, Xs) == 0);
    double cost = oracle_implicit_objective(m, n, ptr, idx, val, X, T, f, 0.5, 2.0);
    CHECK(cost > 0.0);
    int32_t *perm = malloc(sizeof(int32_t) * m);
    int64_t start[25];
    oracle_bin_rows(m, ptr, 24, perm, start);
    CHECK(start[0] == 0 && start[24] == m);
    float *Xf = malloc(sizeof(float) * m * f), *Tf = malloc(sizeof(float) * n * f);
    for (int64_t i = 0; i < m * f; i++) Xf[i] = (float)X[i];
    for (int64_t i = 0; i < n * f; i++) Tf[i] = (float)T[i];
    CHECK(oracle_sse_parallel_f32(m, ptr, idx, val, Xf, Tf, f) > 0.0);

    synth_destroy(h);
    free(deg); free(ptr); free(idx); free(val); free(cptr); free(rptr); free(cidx); free(ridx); free(cval); free(rval);
    free(X); free(T); free(Xs); free(perm); free(Xf); free(Tf);
    printf("sanitize_driver: ok (%lld entries, objective %.6e, implicit cost %.6e, %d threads)\n", (long long)nnz, prev, cost,
           oracle_num_threads());
    return 0;
}
