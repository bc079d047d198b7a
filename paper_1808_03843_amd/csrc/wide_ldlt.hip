// Exact solver at f = 256: launchers; fp32 factor inputs and the slot solver are compiled here, the 16-bit
// element types in wide_ldlt_bf16.hip / wide_ldlt_f16.hip (see wide_ldlt.h for the method).
#include "wide_ldlt.h"

namespace als {

hipError_t launch_hermitian_ldlt_wide(bool ptr64, bool wide, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                                      int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                      const void *Theta, float lambda, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
#define ARGS ptr64, wide, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, Xout, status
    if (et == ALS_F32) return launch_hermitian_ldlt_wide_et<ALS_F32>(ARGS);
    if (et == ALS_BF16) return launch_hermitian_ldlt_wide_bf16(ARGS);
    return launch_hermitian_ldlt_wide_f16(ARGS);
#undef ARGS
}

hipError_t launch_solve_ldlt_wide(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                  int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                  float lambda, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    constexpr int WF = 256, NW = kLdltWaves;
    const dim3 grid((unsigned)npos), block(64 * NW);
    if (ptr64)
        hipLaunchKernelGGL((k_solve_ldlt_wide<WF, NW, int64_t>), grid, block, 0, st, perm, task_off, pos0, task0,
                           (const int64_t *)ptr, slots, lambda, (const float *)nullptr, Xout, status);
    else
        hipLaunchKernelGGL((k_solve_ldlt_wide<WF, NW, int32_t>), grid, block, 0, st, perm, task_off, pos0, task0,
                           (const int32_t *)ptr, slots, lambda, (const float *)nullptr, Xout, status);
    return hipGetLastError();
}

}  // namespace als
