/*
 * libals_gfx950 -- C ABI of the MI355X alternating-least-squares hot path.
 *
 * The library factorises a sparse rating matrix R (m x n, N_z stored entries)
 * as R ~ X * Theta^T with X (m x f) and Theta (n x f), by the per-row
 * normal-equation build and solve of the paper's Section 2:
 *
 *     A_u = sum_{v in Omega_u} theta_v theta_v^T + lambda * n_u * I      (get_hermitian, eq. (2))
 *     b_u = sum_{v in Omega_u} r_uv theta_v                              (get_bias,      eq. (2))
 *     x_u = A_u^-1 b_u                                                    (solve)
 *
 * for every row u (als_update_rows) and, with the roles of X and Theta
 * swapped and the CSC of R in place of its CSR, for every column v
 * (als_update_cols, eq. (3)).  Omega_u is the set of STORED entries of row u
 * (a stored value 0 is an observation), n_u its size.
 *
 * Conventions that hold for every entry point
 *   - "DEVICE" pointers are HIP device memory on the context's GPU, owned by
 *     the caller, never freed or reallocated by the library.  "HOST" pointers
 *     are ordinary host memory.
 *   - Factor matrices are dense, row-major, f contiguous floats per row, the
 *     base pointer 16-byte aligned.
 *   - Sparse matrices are compressed rows: ptr has nrows+1 entries (int32 or
 *     int64, see ptr_is_64), idx holds 0-based int32 column ids ascending and
 *     duplicate-free inside a row, val the float ratings.
 *   - Work is enqueued on the stream given at als_create and the call returns
 *     without waiting, unless stated otherwise.
 *   - Return value: ALS_OK (0) or a negative ALS_E* code; als_last_error gives
 *     the text.  Nothing is printed, nothing aborts.
 */
#ifndef ALS_GFX950_H
#define ALS_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ALS_OK 0
#define ALS_EINVAL (-1)   /* bad argument: null pointer, unsupported f, negative lambda, inconsistent sizes */
#define ALS_EHIP (-2)     /* a HIP runtime call failed (text in als_last_error)                              */
#define ALS_ENUMERIC (-3) /* a kernel met a non-positive pivot or a non-finite value                         */
#define ALS_ENOMEM (-4)   /* device or host allocation failed                                                */

#define ALS_SOLVER_CHOLESKY 0 /* exact solve (the paper's LU baseline of Section 4.1; A_u is SPD)            */
#define ALS_SOLVER_CG 1       /* Algorithm 1: cg_iters iterations warm-started from the current x_u          */

#define ALS_F32 0
#define ALS_BF16 1
#define ALS_F16 2
#define ALS_F32X3 3 /* factor_dtype only: fp32 factors in memory, multiplied on the 16-bit matrix cores as three
                       bf16 parts each (six products per pair, fp32 accumulate): fp32 accuracy, see als_config */
#define ALS_F32X2 4 /* factor_dtype only: fp32 factors in memory, multiplied on the 16-bit matrix cores as two
                       fp16 parts each (three products per pair, fp32 accumulate), see als_config              */

typedef struct als_ctx als_ctx; /* opaque; one per (device, stream); not thread-safe */
/* Every call makes the context's device current while it runs and restores the caller's current device on return. */

/* A sparse matrix in compressed-row form, all arrays DEVICE memory.
 * For als_update_cols pass the CSC of R as the compressed rows of R^T
 * (nrows = n, ncols = m). */
typedef struct als_sparse {
    int64_t nrows, ncols, nnz;
    const void *ptr;    /* nrows+1 offsets, int32 if ptr_is_64 == 0 else int64          */
    int32_t ptr_is_64;
    const int32_t *idx; /* nnz column ids                                              */
    const float *val;   /* nnz ratings                                                 */
} als_sparse;

/* Zero the whole struct first (memset or = {0}) and then set fields: 0 is the default of every optional field. */
typedef struct als_config {
    int32_t f;            /* number of latent features; supported: 16, 32, 64, 100, 128, 256            */
    int32_t solver;       /* ALS_SOLVER_*                                                                */
    int32_t cg_iters;     /* f_s of Algorithm 1 (used when solver == ALS_SOLVER_CG)                      */
    float cg_eps;         /* epsilon of Algorithm 1: stop when sqrt(r^T r) < cg_eps; 0 = fixed f_s steps */
    int32_t factor_dtype; /* ALS_F32 / ALS_BF16 / ALS_F16: element type of the factor matrix that is GATHERED
                             (Theta in als_update_rows, X in als_update_cols).  16-bit elements are multiplied
                             on the 16-bit matrix cores with fp32 accumulation (exact products, so the sums
                             are those of the widened values); solvers and the written factor stay fp32.
                             The rating rides along as three 16-bit parts: exact to 2^-24 of it with ALS_BF16;
                             with ALS_F16 to 2^-24 of max(|r_uv|, 1), the spacing of the smallest fp16 numbers
                             being 2^-24 (ratings and counts of 1 and more, as in Sections 5.1 and 5.6, lose
                             nothing; a rating of 0.02 carries a relative error of up to 3e-6 into b_u).
                             ALS_F32X3: the gathered matrix is fp32 as with ALS_F32, but get_hermitian and get_bias
                             run on the 16-bit matrix cores: every value is cut into three bf16 parts that add up
                             to it exactly, and a product is the sum of the six part products that matter (what is
                             dropped is below 2^-23 of the product, one fp32 rounding).  Same tolerances as
                             ALS_F32, about 1.25 times its speed (Mid shape); f <= 128, explicit feedback only.
                             ALS_F32X2: likewise fp32 in memory, but two fp16 parts per value, h = fp16(s x) and
                             l = fp16(s x - h), rounded to nearest (|s x - h - l| <= 2^-22 |s x|), and the three
                             products h h' + h l' + l h'.  s is a power of two chosen per call from max |x| of the
                             gathered matrix (a reduction that runs before the kernels), so any finite factor is in
                             range; ratings are not scaled and must stay below 65504 in magnitude.  The error of a
                             product is a few 2^-22 of it, of the size of fp32 accumulation rounding: held to the
                             tolerances of ALS_F32.  f <= 128, explicit feedback only                             */
    int32_t herm_dtype;   /* storage type of A_u where it is materialised, i.e. the partial Gram matrices of
                             rows split over several work items (Section 4.2): ALS_F32, or ALS_BF16 with
                             ALS_SOLVER_CG (fp32 accumulate, bf16 in memory; at f = 256 only together
                             with factor_dtype == ALS_F32)                                               */
    int32_t device;       /* HIP device ordinal                                                          */
    void *stream;         /* hipStream_t to enqueue on (NULL = the default stream)                       */
    int32_t chunk;        /* stored entries per work item, a power of two in [64, 2^20]; longer rows are
                             split (0 = default 4096)                                                    */
    int64_t batch_slots;  /* work items whose partial A_u are held at once (0 = about 4 GB worth;
                             larger values than 4,194,303 are taken as that)                                      */
    int32_t profile;      /* 1: bracket every kernel with HIP events (see als_kernel_time)               */
    /* Caller-owned work memory (optional).  workspace: DEVICE, 256-byte aligned, at least
     * als_workspace_bytes(cfg, workspace_max_rows, workspace_max_nnz) bytes, owned by the caller and left alone by
     * it until als_destroy.  With it the library takes no device memory of its own for the update, RMSE, implicit,
     * Gram, check and synchronize calls: status words, work plans, partial Gram matrices and partial sums are all
     * carved from it, and those calls run no hipMalloc / hipFree.  Matrices with more rows (of the compressed
     * form passed in) or more stored entries than the two maxima are refused with ALS_EINVAL and the size that
     * would be needed.  The helper calls outside the per-sweep path (als_hermitian, als_bin_rows, als_csr_to_csc,
     * als_measure_peak) still take temporary device memory of their own for the duration of the call.
     * NULL (and 0 for the three sizes): the library allocates with hipMalloc on first use, may
     * free and reallocate when a larger matrix or batch shows up, and keeps the memory until als_destroy. */
    void *workspace;
    size_t workspace_bytes;
    int64_t workspace_max_rows;
    int64_t workspace_max_nnz;
    int32_t dense_short_rows; /* 0 (default): with ALS_SOLVER_CG and explicit feedback, rows with fewer than
                                 64 stored entries (128: see als_short_row_limit) run Algorithm 1 on the gathered theta_v themselves,
                                 A_u p = G^T (G p) + lambda n_u p, and never form A_u (2 n_u f instead of f^2
                                 multiply-adds per product, no get_hermitian; the iterates differ from the dense
                                 ones by rounding order only).  1: every row builds A_u, as in the paper         */
} als_config;

/* Bytes of workspace a context with this configuration needs for matrices of at most max_rows rows (the larger
 * of m and n when both the CSR and the CSC of R are used) and max_nnz stored entries: bookkeeping, the plans of
 * two such matrices at once (more if they are smaller; when a new plan does not fit, all cached plans are
 * dropped and rebuilt on demand), one partial sum per work item, and partial Gram matrices for
 * min(batch_slots, 2 * max_nnz / chunk + 1) work items.  The workspace, workspace_bytes and workspace_max_* fields
 * of cfg are ignored.  Returns 0 for a configuration als_create would refuse.  Needs no device. */
size_t als_workspace_bytes(const als_config *cfg, int64_t max_rows, int64_t max_nnz);

/* Creates a context.  Without a workspace: allocates small bookkeeping only; work buffers are allocated with
 * hipMalloc on first use and kept until als_destroy.  With a workspace (see als_config): allocates nothing on
 * the device, now or later; a workspace that is too small or misaligned gives ALS_EINVAL. */
int als_create(als_ctx **out, const als_config *cfg);

/* Frees everything the context allocated (waits for its stream first). NULL is allowed. */
void als_destroy(als_ctx *ctx);

/* Text of the last error recorded on this context ("" if none). Valid until the next call. */
const char *als_last_error(const als_ctx *ctx);

/* "Update X" (eq. (2)): for every row u of csr, builds A_u, b_u from Theta
 * (DEVICE, ncols x f, config's factor_dtype) and writes x_u into X (DEVICE,
 * nrows x f float).  With ALS_SOLVER_CG, X is also an input: row u of X is the
 * warm start of Algorithm 1 (rows with fewer than 64 or 128 entries then run it on
 * their gathered theta_v without forming A_u, unless dense_short_rows is set:
 * see als_config).  Rows with n_u = 0 get x_u = 0.  f must equal the
 * config's f; lambda >= 0 (lambda > 0 or n_u >= f is needed for A_u to be SPD).
 * The first call on a matrix (identified by its ptr, nrows, nnz) builds its work plan and sizes the work
 * buffers: it waits for the stream and, without a caller's workspace, allocates.  Later calls on the same matrix
 * only enqueue kernels on the context's stream (no allocation, no wait, no memset), so they may be captured in a
 * HIP graph; the same holds for als_update_cols and the implicit variants.  Errors found by the kernels (a non-positive pivot, a
 * non-finite solution) are reported by the next als_synchronize.  A row whose A_u, b_u or warm start is not finite (a NaN or
 * an overflow in the gathered factor) gets NaN with ALS_SOLVER_CG and is reported the same way. */
int als_update_rows(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f, float *X);

/* "Update Theta" (eq. (3)): the same computation with csc = compressed columns
 * of R (as compressed rows of R^T), X (DEVICE, m x f) gathered and Theta
 * (DEVICE, n x f float) written (and warm start for CG). */
int als_update_cols(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, int f, float *Theta);

/* Training RMSE over the stored entries, sqrt( sum (r_uv - x_u^T theta_v)^2 / N_z )
 * (the metric of Section 5.2 applied to the set given).  X, Theta: DEVICE float.
 * rmse_out: HOST double.  Blocks until the result is available. */
int als_rmse(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, int f, double *rmse_out);

/* Implicit-feedback "Update X" (Section 5.6): the cost is the sum over ALL pairs (u, v) of
 * c_uv (p_uv - x_u^T theta_v)^2 with p_uv = 1 if r_uv > 0 else 0 and c_uv = 1 + alpha * max(r_uv, 0)
 * (pairs that are not stored have r_uv = 0), plus lambda * (|X|_F^2 + |Theta|_F^2) (not weighted by
 * n_u).  For every row u of csr:
 *     A_u = Theta^T Theta + sum_{v in Omega_u} (c_uv - 1) theta_v theta_v^T + lambda I,
 *     b_u = sum_{v in Omega_u, r_uv > 0} c_uv theta_v,     x_u = A_u^-1 b_u
 * which equals the sum over all n columns.  Theta^T Theta is computed once per call by the same
 * gathered kernel.  Arguments as for als_update_rows; alpha >= 0; fp32 storage of A_u.  The gathered factor is
 * fp32, or for f <= 128 bf16 / fp16 (config's factor_dtype): then the columns of a tile get the 16-bit theta and its
 * rows the fp32 product (c_uv - 1) theta cut into three 16-bit parts that add up to it, on the 16-bit matrix cores,
 * and Theta^T Theta is formed from the same 16-bit values.  Rows with n_u = 0 get x_u = 0. */
int als_update_rows_implicit(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, float alpha,
                             int f, float *X);

/* Implicit-feedback "Update Theta": the same with the compressed columns of R and X gathered. */
int als_update_cols_implicit(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, float alpha,
                             int f, float *Theta);

/* The implicit cost of Section 5.6 over all nrows x ncols pairs, regulariser included, evaluated as
 *     sum_{stored} [c (p - d)^2 - d^2] + <X^T X, Theta^T Theta> + lambda (tr X^T X + tr Theta^T Theta),
 * d = x_u^T theta_v (fp32 dots and Gram matrices, fp64 sums).  loss_out: HOST double.  Blocks. */
int als_implicit_loss(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, float lambda,
                      float alpha, int f, double *loss_out);

/* G^T G for a factor matrix G (DEVICE, n x f float): out (DEVICE, f x f floats, row-major, full
 * symmetric).  The dense term of the implicit update; exported for tests. */
int als_gram(als_ctx *ctx, const float *G, int64_t n, int f, float *out);

/* als_gram for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels and the same result layout, but the partial Gram matrices
 * and their sum live in a file-scope device array of 16 MiB that every GPU the library runs on holds until the
 * process ends, so the call runs no hipMalloc, hipFree or other allocating routine and only enqueues kernels on
 * the context's stream.  At most ALS_GRAM_STATIC_MAX_ROWS rows (ALS_EINVAL beyond).  The array holds room for
 * min(512, 16 MiB / slot size) partial matrices (118 at f = 256), so a tall matrix is split into fewer, longer
 * work items than als_gram uses and the fp32 partial sums may differ from its in the last bits; up to
 * 256 * that many rows the two calls split the rows identically and agree bit for bit.  All calls on one GPU share
 * the array: two calls that overlap on one GPU (different streams or contexts) race; calls on one stream are
 * ordered.  Nothing in it needs clearing between calls: every word a call reads it has written before. */
#define ALS_GRAM_STATIC_MAX_ROWS (1ll << 30)
int als_gram_static(als_ctx *ctx, const float *G, int64_t n, int f, float *out);

/* get_hermitian / get_bias alone (Section 2, step (i)) for rows [row0, row0+nrows):
 * A_out (DEVICE, nrows x f x f floats, full symmetric, lambda*n_u on the diagonal
 * included) and b_out (DEVICE, nrows x f).  Meant for tests and breakdown runs. */
int als_hermitian(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f,
                  int64_t row0, int64_t nrows, float *A_out, float *b_out);

/* Load-balancing permutation (not in the paper, which maps one block per row):
 * rows grouped by degree class, class(n_u) = 0 if n_u = 0 else
 * min(1 + floor(log2 n_u), nclass-1); heaviest class first, original row order
 * kept inside a class.  perm_out: DEVICE int32[nrows]; class_start_out: HOST
 * int64[nclass+1] (rows of class c are perm[class_start[nclass-1-c] ..
 * class_start[nclass-c])).  Blocks until done. */
int als_bin_rows(als_ctx *ctx, const als_sparse *csr, int nclass, int32_t *perm_out, int64_t *class_start_out);

/* Compressed columns of R from its compressed rows (the CSC used by
 * als_update_cols), rows ascending inside every column.  cptr_out: DEVICE,
 * ncols+1 offsets of the same width as csr->ptr; cidx_out / cval_out: DEVICE,
 * nnz entries.  Requires nnz < 2^32 (and 64-bit ptr from 2^31 on); allocates
 * about 16 bytes per entry of temporary device memory (8 when the column ids
 * fit into 11 bits) plus at most 130 MB of counters, and waits for the result. */
int als_csr_to_csc(als_ctx *ctx, const als_sparse *csr, void *cptr_out, int32_t *cidx_out, float *cval_out);

/* Waits for the stream and reports ALS_ENUMERIC if any kernel since the last
 * call flagged a non-positive pivot or a non-finite value, ALS_EINVAL if the row
 * offsets of a matrix no longer matched its cached plan (every call that uses a
 * plan compares a fingerprint of ptr on the device; see als_drop_plans). */
int als_synchronize(als_ctx *ctx);

/* Checks a matrix against what the other calls assume and never check themselves: ptr ascending from 0 to nnz,
 * every column id in [0, ncols), the column ids of every row strictly ascending (no duplicates).  An id out of
 * range would make an update read outside the factor matrix.  Returns ALS_EINVAL with the findings in
 * als_last_error; reads the whole matrix once and waits for the result (about the time of one RMSE). */
int als_check_matrix(als_ctx *ctx, const als_sparse *a);

/* Measurement aid (no part of the method): the rate this device sustains on the simplest kernel that can reach a
 * peak -- back-to-back independent MFMAs (flop/s) or a streaming copy of 1 GiB (bytes read + written per second).
 * The roofline fractions of the benchmark are quoted against the published peaks; these are the reachable ones.
 * Allocates its own buffers (2 GiB for the copy), waits for the result.  rate_out: HOST. */
#define ALS_PEAK_MFMA_F32 0  /* v_mfma_f32_16x16x4_f32   */
#define ALS_PEAK_MFMA_BF16 1 /* v_mfma_f32_16x16x32_bf16 */
#define ALS_PEAK_MFMA_F16 2  /* v_mfma_f32_16x16x32_f16  */
#define ALS_PEAK_COPY 3
int als_measure_peak(als_ctx *ctx, int what, double *rate_out);

/* Rows (of als_update_rows / als_update_cols, explicit feedback) with fewer stored entries than the value returned run
 * Algorithm 1 on their gathered theta_v and never form A_u (see dense_short_rows in als_config): 64, or 128 with
 * ALS_F32 factors at f = 100 and f = 128; 0 when no row does (exact solver, dense_short_rows = 1, NULL).  For
 * callers that account for get_hermitian work. */
int als_short_row_limit(const als_ctx *ctx);

/* Forgets the cached work plans (waits for the stream first).  A plan is keyed on a matrix's ptr address, nrows
 * and nnz and holds its degree classes and work items, so the arrays of a matrix must stay unchanged between
 * calls; call this after changing them in place, or when a different matrix with the same nrows and nnz may have
 * been allocated at the address of an earlier one (the kernels stay inside the arrays with a stale plan, but
 * the results are wrong; als_synchronize reports it).  The next call on any matrix rebuilds its plan. */
int als_drop_plans(als_ctx *ctx);

/* Kernel ids for als_kernel_time */
#define ALS_K_HERMITIAN 0
#define ALS_K_SOLVE 1
#define ALS_K_RMSE 2
#define ALS_K_PLAN 3
#define ALS_K_FUSED 4 /* get_hermitian and Algorithm 1 in one kernel (rows shorter than chunk, CG solver) */
#define ALS_K_GRAM 5  /* Theta^T Theta of the implicit update (Section 5.6)                                   */
#define ALS_K_SHORT 6 /* Algorithm 1 on the gathered rows, without A_u (rows with fewer than 64 entries)          */
#define ALS_K_COUNT 7

/* With config.profile = 1: total milliseconds and number of launches of one
 * kernel class since the last als_profile_reset, measured with HIP events on
 * the context's stream.  Blocks until the recorded events have completed.
 * ms_out / launches_out: HOST. */
int als_kernel_time(als_ctx *ctx, int kernel_id, double *ms_out, int64_t *launches_out);
int als_profile_reset(als_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* ALS_GFX950_H */
