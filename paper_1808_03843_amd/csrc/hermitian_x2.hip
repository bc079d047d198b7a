// get_hermitian kernels for factor_dtype = ALS_F32X2 (tiles_x3.h, PARTS = 2): fp32 factor rows scaled by a power of
// two, cut into two fp16 parts and multiplied on the 16-bit matrix cores; and the reduction that finds the scale.  The kernels are the templates of hermitian_kernels.h (slot work items;
// whole rows fused with Algorithm 1 or with the exact solver); this file only instantiates and launches them, in
// a translation unit of its own to keep the build parallel.
#include "hermitian_kernels.h"

namespace als {

// max |x| over n floats as the bits of a non-negative float (they order like unsigned integers); *out must be zero
// before the launch.  A NaN anywhere wins the maximum: the kernels then fall back to scale 1 and the NaN shows up in
// their output, where it is reported like any other non-finite result.
__global__ __launch_bounds__(256) void k_absmax(const float *__restrict__ x, int64_t n, uint32_t *__restrict__ out) {
    uint32_t m = 0u;
    const int64_t n4 = n >> 2, stride = (int64_t)gridDim.x * 256;
    const uint4 *x4 = reinterpret_cast<const uint4 *>(x);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        const uint4 v = x4[i];
        const uint32_t a = v.x & 0x7fffffffu, b = v.y & 0x7fffffffu, c = v.z & 0x7fffffffu, d = v.w & 0x7fffffffu;
        const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
        const uint32_t q = ab > cd ? ab : cd;
        m = m > q ? m : q;
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {   // (n is a multiple of 4 for every supported f; kept general)
        const uint32_t a = __builtin_bit_cast(uint32_t, x[(n4 << 2) + threadIdx.x]) & 0x7fffffffu;
        m = m > a ? m : a;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const uint32_t other = (uint32_t)__shfl_xor((int)m, o);
        m = m > other ? m : other;
    }
    if ((threadIdx.x & 63) == 0 && m != 0u) atomicMax(out, m);
}

hipError_t launch_absmax(hipStream_t st, const float *x, int64_t n, uint32_t *absmax) {
    hipError_t e = fill_zero(st, absmax, 1);
    if (e != hipSuccess || n <= 0) return e;
    int64_t blocks = (n / 4 + 256 * 8 - 1) / (256 * 8);   // 8 or more 16-byte loads per thread
    blocks = blocks < 1 ? 1 : (blocks > 2048 ? 2048 : blocks);
    hipLaunchKernelGGL(k_absmax, dim3((unsigned)blocks), dim3(256), 0, st, x, n, absmax);
    return hipGetLastError();
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

template <int F, typename PtrT>
static hipError_t herm_x2_f(bool wide, bool s16, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                            const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                            const int32_t *idx, const float *val, const void *Theta, float *slots, const uint32_t *absmax) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)ntasks), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, S)                                                                                                  \
    hipLaunchKernelGGL((k_hermitian<F, PtrT, W, ALS_F32X2, S, kExplicit>), grid, block, 0, st, task_row, task_chunk, \
                       task_order, task0, chunk, p, idx, val, Theta, 0.f, slots, absmax)
    if (wide) { if (s16) LAUNCH(true, true); else LAUNCH(true, false); }
    else { if (s16) LAUNCH(false, true); else LAUNCH(false, false); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_x2(int f, bool ptr64, bool wide, bool s16, hipStream_t st, const int32_t *task_row,
                               const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                               int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                               float *slots, const uint32_t *absmax) {
#define CALL(FF)                                                                                                      \
    (ptr64 ? herm_x2_f<FF, int64_t>(wide, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, \
                                    Theta, slots, absmax)                                                             \
           : herm_x2_f<FF, int32_t>(wide, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, \
                                    Theta, slots, absmax))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t herm_cg_x2_f(bool wide, int solver, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                               const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                               int fs, float eps, float *Xout, int *status, const uint32_t *absmax) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(W, S)                                                                                                  \
    hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, W, ALS_F32X2, S, kExplicit>), grid, block, 0, st, perm, pos0, p, idx, val, \
                       Theta, lambda, 0.f, (const float *)nullptr, fs, eps, Xout, status, absmax)
    if (solver == ALS_SOLVER_CG) { if (wide) LAUNCH(true, ALS_SOLVER_CG); else LAUNCH(false, ALS_SOLVER_CG); }
    else { if (wide) LAUNCH(true, ALS_SOLVER_CHOLESKY); else LAUNCH(false, ALS_SOLVER_CHOLESKY); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_cg_x2(int f, bool ptr64, bool wide, int solver, hipStream_t st, const int32_t *perm,
                                  int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                  const void *Theta, float lambda, int fs, float eps, float *Xout, int *status, const uint32_t *absmax) {
#define CALL(FF)                                                                                                      \
    (ptr64 ? herm_cg_x2_f<FF, int64_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, \
                                       status, absmax)                                                                \
           : herm_cg_x2_f<FF, int32_t>(wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, \
                                       status, absmax))
    ALS_FOR_F(CALL)
#undef CALL
}

}  // namespace als
