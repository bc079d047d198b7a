// Implicit feedback (Section 5.6) with 16-bit factor inputs, f <= 128: the gathered kernels of hermitian_kernels.h in
// kImplicit mode on the 16-bit matrix cores (tiles16.h: the rows of a tile get w * theta as three 16-bit parts, the
// columns the plain 16-bit theta).  Instantiations and launchers only, in a translation unit of their own.
#include "hermitian_kernels.h"

namespace als {

#define ALS_FOR_F(CALL)                       \
    switch (f) {                              \
        case 16: return CALL(16);             \
        case 32: return CALL(32);             \
        case 64: return CALL(64);             \
        case 100: return CALL(100);           \
        case 128: return CALL(128);           \
        default: return hipErrorInvalidValue; \
    }

template <int F, typename PtrT>
static hipError_t herm_imp16_f(bool wide, int et, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                               const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                               const int32_t *idx, const float *val, const void *Theta, float alpha, float *slots) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)ntasks), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, E)                                                                                                   \
    hipLaunchKernelGGL((k_hermitian<F, PtrT, W, E, false, kImplicit>), grid, block, 0, st, task_row, task_chunk, task_order, \
                       task0, chunk, p, idx, val, Theta, alpha, slots)
    if (et == ALS_BF16) { if (wide) LAUNCH(true, ALS_BF16); else LAUNCH(false, ALS_BF16); }
    else { if (wide) LAUNCH(true, ALS_F16); else LAUNCH(false, ALS_F16); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_implicit16(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *task_row,
                                       const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                                       int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                       float alpha, float *slots) {
#define CALL(FF)                                                                                                       \
    (ptr64 ? herm_imp16_f<FF, int64_t>(wide, et, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val,  \
                                       Theta, alpha, slots)                                                            \
           : herm_imp16_f<FF, int32_t>(wide, et, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val,  \
                                       Theta, alpha, slots))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t fused_imp16_f(bool wide, int et, int solver, hipStream_t st, const int32_t *perm, int64_t pos0,
                                int64_t npos, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                float lambda, float alpha, const float *gram, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, E, S)                                                                                                \
    hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, W, E, S, kImplicit>), grid, block, 0, st, perm, pos0, p, idx, val, Theta,  \
                       lambda, alpha, gram, fs, eps, Xout, status)
#define BY_SOLVER(W, E)                                                                   \
    do {                                                                                  \
        if (solver == ALS_SOLVER_CG) LAUNCH(W, E, ALS_SOLVER_CG);                         \
        else LAUNCH(W, E, ALS_SOLVER_CHOLESKY);                                           \
    } while (0)
    if (et == ALS_BF16) { if (wide) BY_SOLVER(true, ALS_BF16); else BY_SOLVER(false, ALS_BF16); }
    else { if (wide) BY_SOLVER(true, ALS_F16); else BY_SOLVER(false, ALS_F16); }
#undef BY_SOLVER
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_cg_implicit16(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st,
                                          const int32_t *perm, int64_t pos0, int64_t npos, const void *ptr,
                                          const int32_t *idx, const float *val, const void *Theta, float lambda,
                                          float alpha, const float *gram, int fs, float eps, float *Xout, int *status) {
#define CALL(FF)                                                                                                       \
    (ptr64 ? fused_imp16_f<FF, int64_t>(wide, et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram, \
                                        fs, eps, Xout, status)                                                         \
           : fused_imp16_f<FF, int32_t>(wide, et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, alpha, gram, \
                                        fs, eps, Xout, status))
    ALS_FOR_F(CALL)
#undef CALL
}

}  // namespace als
