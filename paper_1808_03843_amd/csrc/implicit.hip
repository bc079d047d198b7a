// Implicit-feedback ALS (Section 5.6): the cost runs over all m*n pairs, c_uv (p_uv - x_u^T theta_v)^2 with
// p_uv = [r_uv > 0] and c_uv = 1 + alpha r_uv.  The normal equations of a row split into a dense part that
// is the same for every row and a part over the stored entries only,
//     A_u = Theta^T Theta + sum_{v in Omega_u} alpha r_uv theta_v theta_v^T + lambda I,
//     b_u = sum_{v in Omega_u, r_uv > 0} (1 + alpha r_uv) theta_v,
// so the update reuses the gathered get_hermitian kernels with weighted operands (kImplicit) and adds
//   k_gram            Theta^T Theta: the same accumulation loop over the rows of Theta themselves (a true
//                     SYRK with K = n), split over work items whose partial tiles go to slots,
//   k_sum_slots       the sum of those slots, in slot order (deterministic), accumulated in fp64,
//   k_tiles_to_dense  tile layout -> f x f row-major (tests), k_gram_dot: <G_X, G_Theta> and the traces
//                     for the cost function.
#include "hermitian_kernels.h"

namespace als {

// ET: element type of G (16-bit rows are widened in registers; the MFMAs are the fp32 ones)
template <int F, bool WIDE, int ET>
__global__ __launch_bounds__(64) void k_gram(const void *__restrict__ G, int64_t n, int per,
                                             float *__restrict__ slots) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = slot_floats(F);
    const int lane = threadIdx.x;
    const int64_t s0 = (int64_t)blockIdx.x * per;
    const int len = (int)((s0 + per < n) ? per : n - s0);   // >= 1 by the choice of the grid
    v4f acc[NTILES];
#pragma unroll
    for (int q = 0; q < NTILES; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    float b[NT];
    accumulate_tiles<F, false, kDepthSlots, WIDE, ET, rows_all(F), false, kGram>(nullptr, nullptr, G, uniform64(s0), len, acc, b);
    float *out = slots + (int64_t)blockIdx.x * SLOT;
#pragma unroll
    for (int q = 0; q < NTILES; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) out[(q * 4 + r) * 64 + lane] = acc[q][r];
}

// out[o] = slots[0][o] + slots[1][o] + ... for the tile part of a slot
template <int F>
__global__ __launch_bounds__(256) void k_sum_slots(const float *__restrict__ slots, int nslots,
                                                   float *__restrict__ out) {
    constexpr int SLOT = slot_floats(F), TILEPART = tiles_tri(F) * 256;
    const int o = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (o >= TILEPART) return;
    // summed in double: the Gram matrix enters every row's system, and its rounding error is amplified by
    // the condition number of A_u
    double x = 0.0, y = 0.0, z = 0.0, w4 = 0.0;
#pragma unroll 8
    for (int s = 0; s < nslots; ++s) {
        const float4 w = *reinterpret_cast<const float4 *>(slots + (int64_t)s * SLOT + o);
        x += w.x; y += w.y; z += w.z; w4 += w.w;
    }
    *reinterpret_cast<float4 *>(out + o) = make_float4((float)x, (float)y, (float)z, (float)w4);
}

// position o of the tile part -> (tile row R, tile column C, row in tile, column in tile)
__device__ __forceinline__ void tile_pos(int o, int &R, int &C, int &lr, int &lc) {
    const int tile = o >> 8, r = (o >> 6) & 3, l = o & 63;
    int rr = 0;
    while ((rr + 1) * (rr + 2) / 2 <= tile) ++rr;
    R = rr;
    C = tile - rr * (rr + 1) / 2;
    lr = 4 * (l >> 4) + r;
    lc = l & 15;
}

template <int F>
__global__ __launch_bounds__(256) void k_tiles_to_dense(const float *__restrict__ tiles, float *__restrict__ out) {
    const int o = blockIdx.x * 256 + threadIdx.x;
    if (o >= tiles_tri(F) * 256) return;
    int R, C, lr, lc;
    tile_pos(o, R, C, lr, lc);
    const int fr = feature_of(F, R, lr), fc = feature_of(F, C, lc);
    if (fr < 0 || fc < 0) return;
    const float v = tiles[o];
    out[fr * F + fc] = v;   // diagonal tiles hold both triangles: each element is written with its own value
    if (R != C) out[fc * F + fr] = v;
}

// out[0] = <A, B> over the full symmetric matrices, out[1] = tr A, out[2] = tr B (fp64 sums, fixed order)
template <int F>
__global__ __launch_bounds__(256) void k_gram_dot(const float *__restrict__ A, const float *__restrict__ B,
                                                  double *__restrict__ out) {
    __shared__ double red[3][256];
    double dot = 0.0, ta = 0.0, tb = 0.0;
    for (int o = threadIdx.x; o < tiles_tri(F) * 256; o += 256) {
        int R, C, lr, lc;
        tile_pos(o, R, C, lr, lc);
        if (feature_of(F, R, lr) < 0 || feature_of(F, C, lc) < 0) continue;
        const double a = A[o], b = B[o];
        dot += (R != C ? 2.0 : 1.0) * a * b;
        if (R == C && lr == lc) { ta += a; tb += b; }
    }
    red[0][threadIdx.x] = dot; red[1][threadIdx.x] = ta; red[2][threadIdx.x] = tb;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
            for (int k = 0; k < 3; ++k) red[k][threadIdx.x] += red[k][threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x < 3) out[threadIdx.x] = red[threadIdx.x][0];
}

#define ALS_FOR_F(CALL)                       \
    switch (f) {                              \
        case 16: return CALL(16);             \
        case 32: return CALL(32);             \
        case 64: return CALL(64);             \
        case 100: return CALL(100);           \
        case 128: return CALL(128);           \
        default: return hipErrorInvalidValue; \
    }

template <int F>
static hipError_t gram_f(bool wide, int et, hipStream_t st, const void *G, int64_t n, int per, int nslots, float *slots,
                         float *out) {
#define LAUNCH(W, E) hipLaunchKernelGGL((k_gram<F, W, E>), dim3(nslots), dim3(64), 0, st, G, n, per, slots)
    if (et == ALS_F32) { if (wide) LAUNCH(true, ALS_F32); else LAUNCH(false, ALS_F32); }
    else if (et == ALS_BF16) { if (wide) LAUNCH(true, ALS_BF16); else LAUNCH(false, ALS_BF16); }
    else { if (wide) LAUNCH(true, ALS_F16); else LAUNCH(false, ALS_F16); }
#undef LAUNCH
    hipLaunchKernelGGL((k_sum_slots<F>), dim3((tiles_tri(F) * 64 + 255) / 256), dim3(256), 0, st, slots, nslots, out);
    return hipGetLastError();
}

hipError_t launch_gram(int f, bool wide, int et, hipStream_t st, const void *G, int64_t n, int per, int nslots,
                       float *slots, float *out) {
    if (f == 256) {   // the wavefronts of a workgroup share the matrix (wide.hip); the sum of the slots is the same
        if (et != ALS_F32) return hipErrorInvalidValue;
        const hipError_t e = launch_gram_wide(wide, st, (const float *)G, n, per, nslots, slots);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_sum_slots<256>), dim3((tiles_tri(256) * 64 + 255) / 256), dim3(256), 0, st, slots, nslots, out);
        return hipGetLastError();
    }
#define CALL(FF) gram_f<FF>(wide, et, st, G, n, per, nslots, slots, out)
    ALS_FOR_F(CALL)
#undef CALL
}

// Scratch of als_gram_static: the partial Gram matrices (slots) followed by the summed tiles, for callers
// that cannot allocate.  Every GPU the library runs on holds its own copy until the process ends.  The name is
// a host-side stand-in: host code uses the address that hipGetSymbolAddress returns on the current device.
static __device__ __align__(256) float g_gram_scratch[kGramStaticFloats];

hipError_t gram_static_scratch(float **ptr) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_gram_scratch));
    if (e != hipSuccess) return e;
    *ptr = static_cast<float *>(p);
    return hipSuccess;
}

template <int F>
static hipError_t dense_f(hipStream_t st, const float *tiles, float *out) {
    hipLaunchKernelGGL((k_tiles_to_dense<F>), dim3(tiles_tri(F)), dim3(256), 0, st, tiles, out);
    return hipGetLastError();
}
hipError_t launch_tiles_to_dense(int f, hipStream_t st, const float *tiles, float *out) {
    if (f == 256) return dense_f<256>(st, tiles, out);
#define CALL(FF) dense_f<FF>(st, tiles, out)
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F>
static hipError_t dot_f(hipStream_t st, const float *A, const float *B, double *out) {
    hipLaunchKernelGGL((k_gram_dot<F>), dim3(1), dim3(256), 0, st, A, B, out);
    return hipGetLastError();
}
hipError_t launch_gram_dot(int f, hipStream_t st, const float *A, const float *B, double *out) {
    if (f == 256) return dot_f<256>(st, A, B, out);
#define CALL(FF) dot_f<FF>(st, A, B, out)
    ALS_FOR_F(CALL)
#undef CALL
}

// ---- the gathered kernels in implicit mode (fp32 factors, fp32 slots) ----------------------------
template <int F, typename PtrT>
static hipError_t herm_imp_f(bool wide, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk, const int32_t *task_order,
                             int64_t task0, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx,
                             const float *val, const void *Theta, float alpha, float *slots) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)ntasks), block(64);
    const PtrT *p = (const PtrT *)ptr;
    if (wide)
        hipLaunchKernelGGL((k_hermitian<F, PtrT, true, ALS_F32, false, kImplicit>), grid, block, 0, st, task_row,
                           task_chunk, task_order, task0, chunk, p, idx, val, Theta, alpha, slots);
    else
        hipLaunchKernelGGL((k_hermitian<F, PtrT, false, ALS_F32, false, kImplicit>), grid, block, 0, st, task_row,
                           task_chunk, task_order, task0, chunk, p, idx, val, Theta, alpha, slots);
    return hipGetLastError();
}

hipError_t launch_hermitian_implicit(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *task_row,
                                     const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk,
                                     const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                     float alpha, float *slots) {
    if (et != ALS_F32)
        return launch_hermitian_implicit16(f, ptr64, wide, et, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr,
                                           idx, val, Theta, alpha, slots);
    if (f == 256)
        return launch_hermitian_wide_implicit(ptr64, wide, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val,
                                              Theta, alpha, slots);
#define CALL(FF)                                                                                                   \
    (ptr64 ? herm_imp_f<FF, int64_t>(wide, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta,   \
                                     alpha, slots)                                                                 \
           : herm_imp_f<FF, int32_t>(wide, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta,   \
                                     alpha, slots))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT, bool WIDE>
static hipError_t fused_imp_w(int solver, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                              const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                              float alpha, const float *gram, int fs, float eps, float *Xout, int *status) {
    const dim3 grid((unsigned)npos), block(64);
    const PtrT *p = (const PtrT *)ptr;
    if (solver == ALS_SOLVER_CG)
        hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, WIDE, ALS_F32, ALS_SOLVER_CG, kImplicit>), grid, block, 0, st, perm,
                           pos0, p, idx, val, Theta, lambda, alpha, gram, fs, eps, Xout, status);
    else
        hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, WIDE, ALS_F32, ALS_SOLVER_CHOLESKY, kImplicit>), grid, block, 0, st,
                           perm, pos0, p, idx, val, Theta, lambda, alpha, gram, fs, eps, Xout, status);
    return hipGetLastError();
}

template <int F, typename PtrT>
static hipError_t fused_imp_f(bool wide, int solver, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                              const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                              float alpha, const float *gram, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    return wide ? fused_imp_w<F, PtrT, true>(solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram,
                                             fs, eps, Xout, status)
                : fused_imp_w<F, PtrT, false>(solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram,
                                              fs, eps, Xout, status);
}

hipError_t launch_hermitian_cg_implicit(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st, const int32_t *perm,
                                        int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx,
                                        const float *val, const void *Theta, float lambda, float alpha,
                                        const float *gram, int fs, float eps, float *Xout, int *status) {
    if (et != ALS_F32)
        return launch_hermitian_cg_implicit16(f, ptr64, wide, et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda,
                                              alpha, gram, fs, eps, Xout, status);
    if (f == 256)
        return solver == ALS_SOLVER_CG
                   ? launch_hermitian_cg_wide_implicit(ptr64, wide, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha,
                                                       gram, fs, eps, Xout, status)
                   : launch_hermitian_ldlt_wide_implicit(ptr64, wide, st, perm, pos0, npos, ptr, idx, val, Theta, lambda,
                                                         alpha, gram, Xout, status);
#define CALL(FF)                                                                                                     \
    (ptr64 ? fused_imp_f<FF, int64_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram, \
                                      fs, eps, Xout, status)                                                         \
           : fused_imp_f<FF, int32_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram, \
                                      fs, eps, Xout, status))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t solve_imp_f(int solver, hipStream_t st, const int32_t *perm, const int32_t *task_off, int64_t pos0,
                              int64_t npos, int64_t task0, const void *ptr, const float *slots, float lambda,
                              const float *gram, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64);
    if (solver == ALS_SOLVER_CG)
        hipLaunchKernelGGL((k_solve_cg_wave<F, PtrT, false, ALS_SOLVER_CG, kImplicit>), grid, block, 0, st, perm,
                           task_off, pos0, task0, (const PtrT *)ptr, slots, lambda, gram, fs, eps, Xout, status);
    else
        hipLaunchKernelGGL((k_solve_cg_wave<F, PtrT, false, ALS_SOLVER_CHOLESKY, kImplicit>), grid, block, 0, st, perm,
                           task_off, pos0, task0, (const PtrT *)ptr, slots, lambda, gram, fs, eps, Xout, status);
    return hipGetLastError();
}

hipError_t launch_solve_wave_implicit(int f, bool ptr64, int solver, hipStream_t st, const int32_t *perm,
                                      const int32_t *task_off, int64_t pos0, int64_t npos, int64_t task0,
                                      const void *ptr, const float *slots, float lambda, const float *gram, int fs,
                                      float eps, float *Xout, int *status) {
    if (f == 256)
        return solver == ALS_SOLVER_CG
                   ? launch_solve_cg_wide_implicit(ptr64, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, gram, fs,
                                                   eps, Xout, status)
                   : launch_solve_ldlt_wide_implicit(ptr64, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, gram,
                                                     Xout, status);
#define CALL(FF)                                                                                                      \
    (ptr64 ? solve_imp_f<FF, int64_t>(solver, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, gram, fs,    \
                                      eps, Xout, status)                                                              \
           : solve_imp_f<FF, int32_t>(solver, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, gram, fs,    \
                                      eps, Xout, status))
    ALS_FOR_F(CALL)
#undef CALL
}

}  // namespace als
