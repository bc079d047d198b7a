// Step (ii) of Section 2 ("solve"), exact: x_u = A_u^-1 b_u for a batch of rows whose A_u, b_u were
// accumulated into work-item slots by the get_hermitian kernel.  One workgroup per system: LDL^T
// factorisation of the bordered matrix [A b; b^T .] in LDS (the paper's exact baseline is a batched
// LU, Section 4.1; A_u is symmetric positive definite, so the symmetric factorisation gives the same
// solution with half the work).  Algorithm 1, the approximate solver, lives with the get_hermitian
// kernels because it runs on their accumulator tiles.
#include "tiles.h"

namespace als {

// tile index -> (tile row R, tile column C), R >= C
__device__ __forceinline__ void tile_rc(int tile, int &R, int &C) {
    int r = 0;
    while ((r + 1) * (r + 2) / 2 <= tile) ++r;
    R = r;
    C = tile - r * (r + 1) / 2;
}

// packed lower triangle: element (i, k), k <= i, at i(i+1)/2 + k
__device__ __forceinline__ int tri(int i, int k) { return i * (i + 1) / 2 + k; }

// Sums the slots of one row into a packed lower triangle As[tri(row, col)] (col <= row < F, feature
// coordinates) and bs[0..F).  Adds reg to the diagonal.  Every thread of the block takes part.
template <int F>
__device__ __forceinline__ void load_system(const float *__restrict__ slots, int nslots, float reg, float *As,
                                            float *bs) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = slot_floats(F);
    for (int o = threadIdx.x; o < NTILES * 256; o += blockDim.x) {
        const int tile = o >> 8, r = (o >> 6) & 3, l = o & 63;
        int R, C;
        tile_rc(tile, R, C);
        const int lr = 4 * (l >> 4) + r, lc = l & 15;          // position inside the tile
        const int fr = feature_of(F, R, lr), fc = feature_of(F, C, lc);
        if (fr >= 0 && fc >= 0 && (R > C || lc <= lr)) {        // each unordered pair once
            float v = 0.f;
            for (int s = 0; s < nslots; ++s) v += slots[(int64_t)s * SLOT + o];
            if (fr == fc) v += reg;
            const int hi = fr > fc ? fr : fc, lo = fr > fc ? fc : fr;
            As[tri(hi, lo)] = v;
        }
    }
    for (int o = threadIdx.x; o < NT * 16; o += blockDim.x) {
        const int ft = feature_of(F, o >> 4, o & 15);
        if (ft >= 0) {
            float v = 0.f;
            for (int s = 0; s < nslots; ++s) v += slots[(int64_t)s * SLOT + NTILES * 256 + o];
            bs[ft] = v;
        }
    }
}

// ---- exact solve -------------------------------------------------------------------------------
// Right-looking LDL^T on the bordered matrix: row F of As holds b.  After eliminating column j,
// As[i][j] (i > j) holds L[i][j]*d_j and As[F][j] holds z_j with L z = b; then x solves
// L^T x = D^-1 z.  One barrier per column.
// threads per workgroup: a system of f = 256 fills the LDS of a CU (one workgroup per CU), so the only way
// to have several wavefronts per SIMD hide each other's LDS latency is a larger workgroup
constexpr int ldlt_threads(int F) { return F > 128 ? 1024 : 256; }

template <int F, typename PtrT>
__global__ __launch_bounds__(ldlt_threads(F)) void k_solve_ldlt(const int32_t *__restrict__ perm,
                                                    const int32_t *__restrict__ task_off, int64_t pos0,
                                                    int64_t task0, const PtrT *__restrict__ ptr,
                                                    const float *__restrict__ slots, float lambda,
                                                    float *__restrict__ Xout, int *__restrict__ status) {
    constexpr int SLOT = slot_floats(F);
    __shared__ float As[(F + 1) * (F + 2) / 2];   // packed lower triangle of the bordered matrix, row F = b
    const int64_t pos = pos0 + blockIdx.x;
    const int row = perm[pos];
    const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
    float *x = Xout + (int64_t)row * F;
    if (n_u == 0) {
        for (int q = threadIdx.x; q < F; q += blockDim.x) x[q] = 0.f;
        return;
    }
    const int first = task_off[pos] - (int)task0;
    // the slots of a split row have been summed into its first slot by k_reduce_slots
    load_system<F>(slots + (int64_t)first * SLOT, 1, lambda * (float)n_u, As, As + tri(F, 0));

    constexpr int TX = F > 128 ? 32 : 16, TY = ldlt_threads(F) / TX;   // thread grid over (column k, row i)
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    bool bad = false;
    for (int j = 0; j < F; ++j) {
        __syncthreads();
        float d = As[tri(j, j)];
        if (!(d > 0.f)) { bad = true; d = 1.f; }
        const float invd = 1.f / d;
        // rows i in (j, F] (row F is b), columns k in (j, min(i, F-1)]
        for (int i = j + 1 + ty; i <= F; i += TY) {
            const int ri = tri(i, 0);
            const float lij = As[ri + j] * invd;
            const int kmax = i < F ? i : F - 1;
            for (int k = j + 1 + tx; k <= kmax; k += TX) As[ri + k] -= lij * As[tri(k, j)];
        }
    }
    __syncthreads();
    if (bad && threadIdx.x == 0) atomicOr(status, kStatusBadPivot);
    if (threadIdx.x >= 64) return;
    // back substitution by one wavefront: lane l owns z_l, z_{l+64}, ...
    constexpr int NZ = (F + 63) / 64;
    const int l = threadIdx.x;
    float z[NZ], xs[NZ];
#pragma unroll
    for (int q = 0; q < NZ; ++q) {
        z[q] = (l + 64 * q < F) ? As[tri(F, l + 64 * q)] : 0.f;
        xs[q] = 0.f;
    }
    for (int k = F - 1; k >= 0; --k) {
        float zsel = z[0];
#pragma unroll
        for (int q = 1; q < NZ; ++q) zsel = (k >> 6) == q ? z[q] : zsel;
        const float zk = __shfl(zsel, k & 63);
        float dk = As[tri(k, k)];
        if (!(dk > 0.f)) dk = 1.f;
        const float xk = zk / dk;
        // z_i -= (L[k][i] d_i) x_k for i < k
        const int rk = tri(k, 0);
#pragma unroll
        for (int q = 0; q < NZ; ++q) {
            if (l + 64 * q == k) xs[q] = xk;
            if (l + 64 * q < k) z[q] -= As[rk + l + 64 * q] * xk;
        }
    }
#pragma unroll
    for (int q = 0; q < NZ; ++q)
        if (l + 64 * q < F) {
            x[l + 64 * q] = xs[q];
            if (!isfinite(xs[q])) atomicOr(status, kStatusNonFinite);
        }
}

// ---- dense export (tests, breakdown runs) -----------------------------------------------------
template <int F, typename PtrT>
__global__ __launch_bounds__(256) void k_export_dense(const int32_t *__restrict__ perm,
                                                      const int32_t *__restrict__ task_off, int64_t pos0,
                                                      int64_t task0, const PtrT *__restrict__ ptr,
                                                      const float *__restrict__ slots, float lambda, int64_t row0,
                                                      float *__restrict__ A_out, float *__restrict__ b_out) {
    constexpr int SLOT = slot_floats(F);
    __shared__ float As[F * (F + 1) / 2];
    __shared__ float bs[F];
    const int64_t pos = pos0 + blockIdx.x;
    const int row = perm[pos];
    const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
    const int first = task_off[pos] - (int)task0, nslots = task_off[pos + 1] - task_off[pos];
    load_system<F>(slots + (int64_t)first * SLOT, nslots, lambda * (float)n_u, As, bs);
    __syncthreads();
    float *A = A_out + (row - row0) * (int64_t)F * F;
    for (int o = threadIdx.x; o < F * F; o += blockDim.x) {
        const int r = o / F, c = o % F;
        A[o] = (c <= r) ? As[tri(r, c)] : As[tri(c, r)];
    }
    for (int o = threadIdx.x; o < F; o += blockDim.x) b_out[(row - row0) * (int64_t)F + o] = bs[o];
}

template <int F, typename PtrT>
static hipError_t solve_f(int solver, int cg_iters, float cg_eps, hipStream_t st, const int32_t *perm,
                          const int32_t *task_off, int64_t pos0, int64_t npos, int64_t task0, const void *ptr,
                          const float *slots, float lambda, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    dim3 grid((unsigned)npos);
    (void)cg_iters; (void)cg_eps;
    if (solver != ALS_SOLVER_CHOLESKY) return hipErrorInvalidValue;
    if constexpr (F > 128) {   // wider systems are solved on the register tiles of a workgroup (wide_ldlt.hip)
        return hipErrorInvalidValue;
    } else {
        hipLaunchKernelGGL((k_solve_ldlt<F, PtrT>), grid, dim3(ldlt_threads(F)), 0, st, perm, task_off, pos0, task0,
                           (const PtrT *)ptr, slots, lambda, Xout, status);
        return hipGetLastError();
    }
}

#define ALS_DISPATCH_F(CALL)                       \
    switch (f) {                                   \
        case 16: return CALL(16);                  \
        case 32: return CALL(32);                  \
        case 64: return CALL(64);                  \
        case 100: return CALL(100);                \
        case 128: return CALL(128);                \
        case 256: return CALL(256);                \
        default: return hipErrorInvalidValue;      \
    }

hipError_t launch_solve(int f, int solver, int cg_iters, float cg_eps, bool ptr64, hipStream_t st,
                        const int32_t *perm, const int32_t *task_off, int64_t pos0, int64_t npos, int64_t task0,
                        const void *ptr, const float *slots, float lambda, float *Xout, int *status) {
#define CALL(FF)                                                                                                  \
    (ptr64 ? solve_f<FF, int64_t>(solver, cg_iters, cg_eps, st, perm, task_off, pos0, npos, task0, ptr, slots,    \
                                  lambda, Xout, status)                                                           \
           : solve_f<FF, int32_t>(solver, cg_iters, cg_eps, st, perm, task_off, pos0, npos, task0, ptr, slots,    \
                                  lambda, Xout, status))
    ALS_DISPATCH_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t export_f(hipStream_t st, const int32_t *perm, const int32_t *task_off, int64_t pos0, int64_t npos,
                           int64_t task0, const void *ptr, const float *slots, float lambda, int64_t row0,
                           float *A_out, float *b_out) {
    if (npos <= 0) return hipSuccess;
    hipLaunchKernelGGL((k_export_dense<F, PtrT>), dim3((unsigned)npos), dim3(256), 0, st, perm, task_off, pos0,
                       task0, (const PtrT *)ptr, slots, lambda, row0, A_out, b_out);
    return hipGetLastError();
}

hipError_t launch_export_dense(int f, bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                               int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                               float lambda, int64_t row0, float *A_out, float *b_out) {
#define CALL(FF)                                                                                                   \
    (ptr64 ? export_f<FF, int64_t>(st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, row0, A_out, b_out) \
           : export_f<FF, int32_t>(st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, row0, A_out, b_out))
    ALS_DISPATCH_F(CALL)
#undef CALL
}

}  // namespace als
