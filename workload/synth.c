/*
 * Seeded synthetic rating matrices (input generator only).
 *
 * This file produces the INPUTS that both the CPU oracle and the GPU library
 * are run on: a sparse rating matrix R in CSR form with the shape, density,
 * degree skew and rating range of the workloads the paper factorises
 * (Table 2: Netflix / YahooMusic / Hugewiki shapes).  It contains none of the
 * method's arithmetic (no Gram matrices, no solves, no RMSE).
 *
 * Everything is a pure function of (seed, row): a counter-based hash supplies
 * every random number, so rows can be generated in any order, in parallel, or
 * one at a time, and always come out identical.
 *
 * Recipe
 *   degrees    rank-size Zipf law: the row of popularity rank i (0-based) has
 *              degree clip(rint(C*(i+1)^-s), dmin, dmax); C is found by
 *              bisection so the total is the requested nnz, the last few units
 *              are fixed one row at a time in rank order.  Rank -> row id is a
 *              seeded bijection (Feistel network with cycle walking).
 *   columns    a row draws its d distinct column ids from the popularity law
 *              p(rank j) ~ (j+1)^-s_col, successive sampling without
 *              replacement; rank -> column id is a second seeded bijection.
 *              Ids are emitted in ascending order (canonical CSR).
 *   ratings    z = <x*_u, t*_v> + N(0, noise_std) from hidden rank-k factors
 *              ~ N(0, factor_std);  kind 0: clip(rint(z), 1, 5);
 *              kind 1: 10*clip(rint(5 + 2 z), 0, 10)  (0..100 in steps of 10,
 *              zeros are stored entries).  rint = round-half-to-even.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no -march=native and
 * no contraction, so the output does not depend on the host CPU).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t m, n, nnz;
    double row_s;          /* rank-size exponent of row degrees            */
    int64_t dmin, dmax;    /* degree clip                                   */
    double col_s;          /* popularity exponent of columns                */
    int32_t hidden_rank;   /* k of the hidden model                         */
    double factor_std;     /* std of hidden factors                         */
    double noise_std;      /* std of the additive rating noise              */
    int32_t rating_kind;   /* 0: 1..5   1: 0..100 step 10                   */
    uint64_t seed;
} synth_config;

typedef struct {
    synth_config c;
    double *col_cdf;       /* n entries, cumulative popularity over ranks   */
    double *col_w;         /* n entries, weight of rank j                   */
    int32_t *rank_to_col;  /* n entries                                     */
    double *tstar;         /* n x k hidden column factors (by column id)    */
} synth_handle;

/* ---- counter-based random numbers --------------------------------------- */
static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static inline uint64_t hash3(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b) {
    uint64_t h = mix64(seed ^ (stream * 0xD6E8FEB86659FD93ull));
    h = mix64(h ^ a);
    h = mix64(h ^ b);
    return h;
}
static inline double u01(uint64_t h) { return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
static inline double normal01(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b) {
    double u1 = u01(hash3(seed, stream, a, 2 * b));
    double u2 = u01(hash3(seed, stream, a, 2 * b + 1));
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}
enum { S_ROWPERM = 1, S_COLPERM = 2, S_TSTAR = 3, S_XSTAR = 4, S_NOISE = 5, S_DRAW = 6, S_KEY = 7 };

/* seeded bijection on [0, size): balanced Feistel on 2*hb bits + cycle walking */
static inline uint64_t permute_index(uint64_t x, uint64_t size, uint64_t seed, uint64_t stream) {
    int bits = 1;
    while (((uint64_t)1 << bits) < size) bits++;
    if (bits & 1) bits++;
    int hb = bits / 2;
    uint64_t mask = ((uint64_t)1 << hb) - 1;
    do {
        uint64_t l = x >> hb, r = x & mask;
        for (int round = 0; round < 4; round++) {
            uint64_t f = hash3(seed, stream, (uint64_t)round, r) & mask;
            uint64_t nl = r, nr = l ^ f;
            l = nl; r = nr;
        }
        x = (l << hb) | r;
    } while (x >= size);
    return x;
}

/* ---- handle -------------------------------------------------------------- */
void synth_destroy(synth_handle *h) {
    if (!h) return;
    free(h->col_cdf); free(h->col_w); free(h->rank_to_col); free(h->tstar); free(h);
}

synth_handle *synth_create(const synth_config *cfg) {
    if (!cfg || cfg->m <= 0 || cfg->n <= 0 || cfg->n > 0x7fffffff || cfg->hidden_rank <= 0) return NULL;
    synth_handle *h = (synth_handle *)calloc(1, sizeof(*h));
    if (!h) return NULL;
    h->c = *cfg;
    int64_t n = cfg->n; int k = cfg->hidden_rank;
    h->col_cdf = (double *)malloc(sizeof(double) * n);
    h->col_w = (double *)malloc(sizeof(double) * n);
    h->rank_to_col = (int32_t *)malloc(sizeof(int32_t) * n);
    h->tstar = (double *)malloc(sizeof(double) * n * k);
    if (!h->col_cdf || !h->col_w || !h->rank_to_col || !h->tstar) { synth_destroy(h); return NULL; }
    double acc = 0.0;
    for (int64_t j = 0; j < n; j++) {
        h->col_w[j] = pow((double)(j + 1), -cfg->col_s);
        acc += h->col_w[j];
        h->col_cdf[j] = acc;
    }
    for (int64_t j = 0; j < n; j++) h->col_cdf[j] /= acc;
    h->col_cdf[n - 1] = 1.0;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n; j++) {
        h->rank_to_col[j] = (int32_t)permute_index((uint64_t)j, (uint64_t)n, cfg->seed, S_COLPERM);
        for (int q = 0; q < k; q++)
            h->tstar[j * k + q] = cfg->factor_std * normal01(cfg->seed, S_TSTAR, (uint64_t)j, (uint64_t)q);
    }
    return h;
}

/* ---- degrees -------------------------------------------------------------- */
static inline int64_t clipdeg(double v, int64_t lo, int64_t hi) {
    double r = rint(v);
    if (r < (double)lo) return lo;
    if (r > (double)hi) return hi;
    return (int64_t)r;
}

/* deg_out[u] for every row u; returns 0 on success, -1 if nnz is unreachable. */
int synth_degrees(const synth_handle *h, int64_t *deg_out) {
    const synth_config *c = &h->c;
    int64_t m = c->m;
    int64_t dmax = c->dmax < c->n ? c->dmax : c->n;
    int64_t dmin = c->dmin;
    if (dmin * m > c->nnz || dmax * m < c->nnz) return -1;
    double *w = (double *)malloc(sizeof(double) * m);
    if (!w) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; i++) w[i] = pow((double)(i + 1), -c->row_s);
    double lo = 0.0, hi = 1.0;
    for (;;) {   /* grow hi until the total reaches nnz */
        int64_t tot = 0;
#pragma omp parallel for schedule(static) reduction(+ : tot)
        for (int64_t i = 0; i < m; i++) tot += clipdeg(hi * w[i], dmin, dmax);
        if (tot >= c->nnz) break;
        hi *= 2.0;
    }
    for (int it = 0; it < 200; it++) {
        double mid = 0.5 * (lo + hi);
        if (mid == lo || mid == hi) break;
        int64_t tot = 0;
#pragma omp parallel for schedule(static) reduction(+ : tot)
        for (int64_t i = 0; i < m; i++) tot += clipdeg(mid * w[i], dmin, dmax);
        if (tot >= c->nnz) hi = mid; else lo = mid;
    }
    int64_t *byrank = (int64_t *)malloc(sizeof(int64_t) * m);
    if (!byrank) { free(w); return -1; }
    int64_t tot = 0;
    for (int64_t i = 0; i < m; i++) { byrank[i] = clipdeg(hi * w[i], dmin, dmax); tot += byrank[i]; }
    free(w);
    /* tot >= nnz: take the surplus off one unit at a time, in rank order */
    int64_t surplus = tot - c->nnz;
    while (surplus > 0) {
        int64_t before = surplus;
        for (int64_t i = 0; i < m && surplus > 0; i++)
            if (byrank[i] > dmin) { byrank[i]--; surplus--; }
        if (surplus == before) { free(byrank); return -1; }
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; i++) {
        uint64_t u = permute_index((uint64_t)i, (uint64_t)m, c->seed, S_ROWPERM);
        deg_out[u] = byrank[i];
    }
    free(byrank);
    return 0;
}

/* ---- one row --------------------------------------------------------------- */
static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}
typedef struct { double key; int32_t col; } keyed;
static int cmp_keyed_desc(const void *a, const void *b) {
    const keyed *x = (const keyed *)a, *y = (const keyed *)b;
    if (x->key > y->key) return -1;
    if (x->key < y->key) return 1;
    return (x->col > y->col) - (x->col < y->col);
}

static inline float make_rating(const synth_handle *h, int64_t u, int32_t v, const double *xstar) {
    const synth_config *c = &h->c;
    int k = c->hidden_rank;
    const double *t = h->tstar + (int64_t)v * k;
    double z = 0.0;
    for (int q = 0; q < k; q++) z += xstar[q] * t[q];
    z += c->noise_std * normal01(c->seed, S_NOISE, (uint64_t)u, (uint64_t)v);
    double r;
    if (c->rating_kind == 0) {
        r = rint(z);
        if (r < 1.0) r = 1.0;
        if (r > 5.0) r = 5.0;
    } else {
        r = rint(5.0 + 2.0 * z);
        if (r < 0.0) r = 0.0;
        if (r > 10.0) r = 10.0;
        r *= 10.0;
    }
    return (float)r;
}

/* scratch: bitmap of n bits (all zero on entry and on exit), keyed[n] */
static void fill_one_row(const synth_handle *h, int64_t u, int64_t d, int32_t *cols, float *vals,
                         uint64_t *bitmap, keyed *keys) {
    const synth_config *c = &h->c;
    int64_t n = c->n;
    if (d <= 0) return;
    if (d * 8 > n) {
        /* weighted sampling without replacement through exponential keys:
           the d largest of log(u_j)/w_j over all ranks j                     */
        for (int64_t j = 0; j < n; j++) {
            double uu = u01(hash3(c->seed, S_KEY, (uint64_t)u, (uint64_t)j));
            keys[j].key = log(uu) / h->col_w[j];
            keys[j].col = h->rank_to_col[j];
        }
        qsort(keys, (size_t)n, sizeof(keyed), cmp_keyed_desc);
        for (int64_t q = 0; q < d; q++) cols[q] = keys[q].col;
    } else {
        int64_t got = 0; uint64_t draw = 0;
        while (got < d) {
            double uu = u01(hash3(c->seed, S_DRAW, (uint64_t)u, draw++));
            int64_t lo = 0, hi = n - 1;          /* first rank with cdf >= uu */
            while (lo < hi) {
                int64_t mid = (lo + hi) >> 1;
                if (h->col_cdf[mid] >= uu) hi = mid; else lo = mid + 1;
            }
            int32_t v = h->rank_to_col[lo];
            uint64_t bit = (uint64_t)1 << (v & 63);
            if (bitmap[v >> 6] & bit) continue;
            bitmap[v >> 6] |= bit;
            cols[got++] = v;
        }
        for (int64_t q = 0; q < d; q++) bitmap[cols[q] >> 6] = 0;
    }
    qsort(cols, (size_t)d, sizeof(int32_t), cmp_i32);
    double xstar[64];
    int k = c->hidden_rank;
    for (int q = 0; q < k; q++) xstar[q] = c->factor_std * normal01(c->seed, S_XSTAR, (uint64_t)u, (uint64_t)q);
    for (int64_t q = 0; q < d; q++) vals[q] = make_rating(h, u, cols[q], xstar);
}

/* Rows [u0, u1).  rowptr has u1-u0+1 entries (rowptr[i] is the offset of row
 * u0+i relative to the start of colidx/val).  Returns 0 on success.          */
int synth_fill_rows(const synth_handle *h, int64_t u0, int64_t u1, const int64_t *rowptr,
                    int32_t *colidx, float *val) {
    if (!h || u0 < 0 || u1 > h->c.m || u0 > u1 || h->c.hidden_rank > 64) return -1;
    int64_t n = h->c.n;
    int64_t words = (n + 63) / 64;
    int64_t need_keys = 0;
    for (int64_t u = u0; u < u1; u++) {
        int64_t d = rowptr[u - u0 + 1] - rowptr[u - u0];
        if (d < 0 || d > n) return -1;
        if (d * 8 > n) need_keys = 1;
    }
    int fail = 0;
#pragma omp parallel
    {
        uint64_t *bitmap = (uint64_t *)calloc((size_t)words, sizeof(uint64_t));
        keyed *keys = need_keys ? (keyed *)malloc(sizeof(keyed) * (size_t)n) : NULL;
        if (!bitmap || (need_keys && !keys)) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 64)
            for (int64_t u = u0; u < u1; u++) {
                int64_t s = rowptr[u - u0], e = rowptr[u - u0 + 1];
                fill_one_row(h, u, e - s, colidx + s, val + s, bitmap, keys);
            }
        }
        free(bitmap); free(keys);
    }
    return fail ? -1 : 0;
}

int synth_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
