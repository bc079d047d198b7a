// get_hermitian kernels for factor_dtype = ALS_F32X3 (tiles_x3.h): fp32 factor rows cut into three bf16 parts and
// multiplied on the 16-bit matrix cores.  The kernels are the templates of hermitian_kernels.h (slot work items;
// whole rows fused with Algorithm 1 or with the exact solver); this file only instantiates and launches them, in
// a translation unit of its own to keep the build parallel.
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
static hipError_t herm_x3_f(bool wide, bool s16, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                            const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                            const int32_t *idx, const float *val, const void *Theta, float *slots) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)ntasks), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, S)                                                                                                  \
    hipLaunchKernelGGL((k_hermitian<F, PtrT, W, ALS_F32X3, S, kExplicit>), grid, block, 0, st, task_row, task_chunk, \
                       task_order, task0, chunk, p, idx, val, Theta, 0.f, slots)
    if (wide) { if (s16) LAUNCH(true, true); else LAUNCH(true, false); }
    else { if (s16) LAUNCH(false, true); else LAUNCH(false, false); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_x3(int f, bool ptr64, bool wide, bool s16, hipStream_t st, const int32_t *task_row,
                               const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                               int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                               float *slots) {
#define CALL(FF)                                                                                                      \
    (ptr64 ? herm_x3_f<FF, int64_t>(wide, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, \
                                    Theta, slots)                                                                     \
           : herm_x3_f<FF, int32_t>(wide, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, \
                                    Theta, slots))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t herm_cg_x3_f(bool wide, int solver, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                               const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                               int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, S)                                                                                                  \
    hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, W, ALS_F32X3, S, kExplicit>), grid, block, 0, st, perm, pos0, p, idx, val, \
                       Theta, lambda, 0.f, (const float *)nullptr, fs, eps, Xout, status)
    if (solver == ALS_SOLVER_CG) { if (wide) LAUNCH(true, ALS_SOLVER_CG); else LAUNCH(false, ALS_SOLVER_CG); }
    else { if (wide) LAUNCH(true, ALS_SOLVER_CHOLESKY); else LAUNCH(false, ALS_SOLVER_CHOLESKY); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_cg_x3(int f, bool ptr64, bool wide, int solver, hipStream_t st, const int32_t *perm,
                                  int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                  const void *Theta, float lambda, int fs, float eps, float *Xout, int *status) {
#define CALL(FF)                                                                                                      \
    (ptr64 ? herm_cg_x3_f<FF, int64_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, \
                                       status)                                                                        \
           : herm_cg_x3_f<FF, int32_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, \
                                       status))
    ALS_FOR_F(CALL)
#undef CALL
}

}  // namespace als
