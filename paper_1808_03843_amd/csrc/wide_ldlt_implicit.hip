// Exact solver at f = 256 for implicit feedback (Section 5.6): the fused kernel and the slot solver in kImplicit
// mode (see wide_ldlt.h for the method).  fp32 factors.
#include "wide_ldlt.h"

namespace als {

hipError_t launch_hermitian_ldlt_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                               int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                               const void *Theta, float lambda, float alpha, const float *gram,
                                               float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    constexpr int WF = 256, NW = kLdltWaves;
    const dim3 grid((unsigned)npos), block(64 * NW);
#define LAUNCH(P, W)                                                                                              \
    hipLaunchKernelGGL((k_hermitian_ldlt_wide<WF, NW, P, W, ALS_F32, kImplicit>), grid, block, 0, st, perm, pos0,  \
                       (const P *)ptr, idx, val, Theta, lambda, alpha, gram, Xout, status)
    if (ptr64) { if (wide) LAUNCH(int64_t, true); else LAUNCH(int64_t, false); }
    else       { if (wide) LAUNCH(int32_t, true); else LAUNCH(int32_t, false); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_solve_ldlt_wide_implicit(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                           int64_t pos0, int64_t npos, int64_t task0, const void *ptr,
                                           const float *slots, float lambda, const float *gram, float *Xout,
                                           int *status) {
    if (npos <= 0) return hipSuccess;
    constexpr int WF = 256, NW = kLdltWaves;
    const dim3 grid((unsigned)npos), block(64 * NW);
    if (ptr64)
        hipLaunchKernelGGL((k_solve_ldlt_wide<WF, NW, int64_t, kImplicit>), grid, block, 0, st, perm, task_off, pos0, task0,
                           (const int64_t *)ptr, slots, lambda, gram, Xout, status);
    else
        hipLaunchKernelGGL((k_solve_ldlt_wide<WF, NW, int32_t, kImplicit>), grid, block, 0, st, perm, task_off, pos0, task0,
                           (const int32_t *)ptr, slots, lambda, gram, Xout, status);
    return hipGetLastError();
}

}  // namespace als
