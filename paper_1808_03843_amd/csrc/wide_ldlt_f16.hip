// Exact solver at f = 256, fused kernel for f16 factor inputs (see wide_ldlt.h).
#include "wide_ldlt.h"

namespace als {

hipError_t launch_hermitian_ldlt_wide_f16(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                           int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                           const void *Theta, float lambda, float *Xout, int *status) {
    return launch_hermitian_ldlt_wide_et<ALS_F16>(ptr64, wide, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, Xout, status);
}

}  // namespace als
