// get_hermitian + get_bias (Section 2, step (i); Section 3): the gathered, batched SYRK
//     A_u = sum_{v in Omega_u} theta_v theta_v^T,   b_u = sum_{v in Omega_u} r_uv theta_v
// on the fp32 matrix cores of gfx950, and its fusion with the approximate solver (Section 4.1).
//
// One wavefront owns one work item (a row, or a chunk of a long row) and keeps the whole lower
// triangle of A_u in MFMA accumulators: the paper keeps A_u in registers because it is the most
// reused operand (Section 3, Solution 1); here "registers" are the 16x16 accumulator tiles of
// v_mfma_f32_16x16x4_f32.  theta rows are gathered straight into the operand registers (no staging
// buffer): every theta element is used by exactly one wavefront, so there is nothing to share
// through LDS, and a register double buffer hides the gather latency.
//
//   k_hermitian        work items of long rows: the partial A_u, b_u go to a slot in memory.
//   k_hermitian_cg     whole short rows: A_u never leaves the registers; the same wavefront runs
//                      Algorithm 1 (or, in exact mode, an LDL^T factorisation and the triangular solves)
//                      on the accumulator tiles and writes x_u (the paper flushes A_u to global memory
//                      and reads it back in the solver, Section 3 and Observation 4).
//   k_reduce_slots     sums the slots of a split row into its first slot, in slot order.
//   k_solve_cg_wave    the same two solvers for rows whose A_u sits in a slot, one wavefront per row.
#include "hermitian_kernels.h"

namespace als {

// slots[first] += slots[first+1] + ... (in slot order) for every row of the batch with several slots
template <int F, bool S16>
__global__ __launch_bounds__(256) void k_reduce_slots(const int32_t *__restrict__ task_off, int64_t pos0,
                                                      int64_t task0, float *__restrict__ slots) {
    constexpr int SLOT = S16 ? slot_words16(F) : slot_floats(F);
    constexpr int PACKED = S16 ? tiles_tri(F) * 128 : 0;   // words holding bf16 pairs (a multiple of 4)
    const int64_t pos = pos0 + blockIdx.x;
    const int first = task_off[pos] - (int)task0, n = task_off[pos + 1] - task_off[pos];
    if (n <= 1) return;
    const int o = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (o >= SLOT) return;
    float4 *dst = reinterpret_cast<float4 *>(slots + (int64_t)first * SLOT + o);
    if (o < PACKED) {   // sums in fp32, stored back as bf16
        uint4 *dst32 = reinterpret_cast<uint4 *>(dst);
        const uint4 w0 = *dst32;
        float a[8] = {bits_to_float(w0.x << 16), bits_to_float(w0.x & 0xffff0000u), bits_to_float(w0.y << 16),
                      bits_to_float(w0.y & 0xffff0000u), bits_to_float(w0.z << 16), bits_to_float(w0.z & 0xffff0000u),
                      bits_to_float(w0.w << 16), bits_to_float(w0.w & 0xffff0000u)};
#pragma unroll 4
        for (int s = 1; s < n; ++s) {
            const uint4 w = *reinterpret_cast<const uint4 *>(slots + (int64_t)(first + s) * SLOT + o);
            a[0] += bits_to_float(w.x << 16); a[1] += bits_to_float(w.x & 0xffff0000u);
            a[2] += bits_to_float(w.y << 16); a[3] += bits_to_float(w.y & 0xffff0000u);
            a[4] += bits_to_float(w.z << 16); a[5] += bits_to_float(w.z & 0xffff0000u);
            a[6] += bits_to_float(w.w << 16); a[7] += bits_to_float(w.w & 0xffff0000u);
        }
        *dst32 = make_uint4(pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(a[4], a[5]), pack_bf16(a[6], a[7]));
        return;
    }
    float4 v = *dst;
#pragma unroll 8
    for (int s = 1; s < n; ++s) {
        const float4 w = *reinterpret_cast<const float4 *>(slots + (int64_t)(first + s) * SLOT + o);
        v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    }
    *dst = v;
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

// dispatch on the run-time switches that are template parameters of the kernels
template <int F, typename PtrT, bool WIDE, bool S16>
static hipError_t herm_e(int et, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk, const int32_t *task_order, int64_t task0,
                         int64_t ntasks, int chunk, const void *ptr, const int32_t *idx, const float *val,
                         const void *Theta, float *slots) {
    const dim3 grid((unsigned)ntasks), block(64);
    const PtrT *p = (const PtrT *)ptr;
    if (et == ALS_F32)
        hipLaunchKernelGGL((k_hermitian<F, PtrT, WIDE, ALS_F32, S16, kExplicit>), grid, block, 0, st, task_row, task_chunk, task_order, task0,
                           chunk, p, idx, val, Theta, 0.f, slots);
    else if (et == ALS_BF16)
        hipLaunchKernelGGL((k_hermitian<F, PtrT, WIDE, ALS_BF16, S16, kExplicit>), grid, block, 0, st, task_row, task_chunk, task_order, task0,
                           chunk, p, idx, val, Theta, 0.f, slots);
    else
        hipLaunchKernelGGL((k_hermitian<F, PtrT, WIDE, ALS_F16, S16, kExplicit>), grid, block, 0, st, task_row, task_chunk, task_order, task0,
                           chunk, p, idx, val, Theta, 0.f, slots);
    return hipGetLastError();
}

template <int F, typename PtrT>
static hipError_t herm_f(bool wide, int et, bool s16, hipStream_t st, const int32_t *task_row,
                         const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                         const int32_t *idx, const float *val, const void *Theta, float *slots) {
    if (ntasks <= 0) return hipSuccess;
#define ARGS et, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta, slots
    if (s16) return wide ? herm_e<F, PtrT, true, true>(ARGS) : herm_e<F, PtrT, false, true>(ARGS);
    return wide ? herm_e<F, PtrT, true, false>(ARGS) : herm_e<F, PtrT, false, false>(ARGS);
#undef ARGS
}

hipError_t launch_hermitian(int f, bool ptr64, bool wide, int et, bool s16, hipStream_t st, const int32_t *task_row,
                            const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                            const int32_t *idx, const float *val, const void *Theta, float *slots) {
    if (et == ALS_F32X3)
        return launch_hermitian_x3(f, ptr64, wide, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val,
                                   Theta, slots);
    if (f == 256)
        return launch_hermitian_wide(ptr64, wide, et, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val,
                                     Theta, slots);
#define CALL(FF)                                                                                                      \
    (ptr64 ? herm_f<FF, int64_t>(wide, et, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta, \
                                 slots)                                                                               \
           : herm_f<FF, int32_t>(wide, et, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta, \
                                 slots))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT, bool WIDE>
static hipError_t herm_cg_e(int et, int solver, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                            const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                            int fs, float eps, float *Xout, int *status) {
    const dim3 grid((unsigned)npos), block(64);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(E, S)                                                                                                 \
    hipLaunchKernelGGL((k_hermitian_cg<F, PtrT, WIDE, E, S, kExplicit>), grid, block, 0, st, perm, pos0, p, idx, val, Theta, \
                       lambda, 0.f, (const float *)nullptr, fs, eps, Xout, status)
    if (solver == ALS_SOLVER_CHOLESKY) {
        if (et == ALS_F32) LAUNCH(ALS_F32, ALS_SOLVER_CHOLESKY);
        else if (et == ALS_BF16) LAUNCH(ALS_BF16, ALS_SOLVER_CHOLESKY);
        else LAUNCH(ALS_F16, ALS_SOLVER_CHOLESKY);
    } else {
        if (et == ALS_F32) LAUNCH(ALS_F32, ALS_SOLVER_CG);
        else if (et == ALS_BF16) LAUNCH(ALS_BF16, ALS_SOLVER_CG);
        else LAUNCH(ALS_F16, ALS_SOLVER_CG);
    }
#undef LAUNCH
    return hipGetLastError();
}

template <int F, typename PtrT>
static hipError_t herm_cg_f(bool wide, int et, int solver, hipStream_t st, const int32_t *perm, int64_t pos0,
                            int64_t npos, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                            float lambda, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    return wide ? herm_cg_e<F, PtrT, true>(et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps,
                                           Xout, status)
                : herm_cg_e<F, PtrT, false>(et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps,
                                            Xout, status);
}

hipError_t launch_hermitian_cg(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st, const int32_t *perm,
                               int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                               const void *Theta, float lambda, int fs, float eps, float *Xout, int *status) {
    if (et == ALS_F32X3)
        return launch_hermitian_cg_x3(f, ptr64, wide, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout,
                                      status);
    if (f == 256 && solver != ALS_SOLVER_CG)
        return launch_hermitian_ldlt_wide(ptr64, wide, et, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, Xout, status);
    if (f == 256)
        return launch_hermitian_cg_wide(f, ptr64, wide, et, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps,
                                        Xout, status);
#define CALL(FF)                                                                                                     \
    (ptr64 ? herm_cg_f<FF, int64_t>(wide, et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps,   \
                                    Xout, status)                                                                    \
           : herm_cg_f<FF, int32_t>(wide, et, solver, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps,   \
                                    Xout, status))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F, typename PtrT>
static hipError_t solve_wave_f(bool s16, int solver, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                               int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                               float lambda, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    if (solver == ALS_SOLVER_CHOLESKY) {
        if (s16) return hipErrorInvalidValue;
        hipLaunchKernelGGL((k_solve_cg_wave<F, PtrT, false, ALS_SOLVER_CHOLESKY, kExplicit>), dim3((unsigned)npos), dim3(64), 0, st,
                           perm, task_off, pos0, task0, (const PtrT *)ptr, slots, lambda, (const float *)nullptr, fs, eps, Xout, status);
    } else if (s16)
        hipLaunchKernelGGL((k_solve_cg_wave<F, PtrT, true, ALS_SOLVER_CG, kExplicit>), dim3((unsigned)npos), dim3(64), 0, st, perm,
                           task_off, pos0, task0, (const PtrT *)ptr, slots, lambda, (const float *)nullptr, fs, eps, Xout, status);
    else
        hipLaunchKernelGGL((k_solve_cg_wave<F, PtrT, false, ALS_SOLVER_CG, kExplicit>), dim3((unsigned)npos), dim3(64), 0, st, perm,
                           task_off, pos0, task0, (const PtrT *)ptr, slots, lambda, (const float *)nullptr, fs, eps, Xout, status);
    return hipGetLastError();
}

hipError_t launch_solve_cg_wave(int f, bool ptr64, bool s16, int solver, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                float lambda, int fs, float eps, float *Xout, int *status) {
#define CALL(FF)                                                                                                   \
    (ptr64 ? solve_wave_f<FF, int64_t>(s16, solver, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, fs, eps, Xout,  \
                                       status)                                                                     \
           : solve_wave_f<FF, int32_t>(s16, solver, st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, fs, eps, Xout,  \
                                       status))
    ALS_FOR_F(CALL)
#undef CALL
}

template <int F>
static hipError_t reduce_f(bool s16, hipStream_t st, const int32_t *task_off, int64_t pos0, int64_t npos,
                           int64_t task0, float *slots) {
    if (npos <= 0) return hipSuccess;
    if (s16)
        hipLaunchKernelGGL((k_reduce_slots<F, true>), dim3((unsigned)npos, (slot_words16(F) / 4 + 255) / 256),
                           dim3(256), 0, st, task_off, pos0, task0, slots);
    else
        hipLaunchKernelGGL((k_reduce_slots<F, false>), dim3((unsigned)npos, (slot_floats(F) / 4 + 255) / 256),
                           dim3(256), 0, st, task_off, pos0, task0, slots);
    return hipGetLastError();
}

hipError_t launch_reduce_slots(int f, bool s16, hipStream_t st, const int32_t *task_off, int64_t pos0, int64_t npos,
                               int64_t task0, float *slots) {
    if (f == 256) return reduce_f<256>(s16, st, task_off, pos0, npos, task0, slots);
#define CALL(FF) reduce_f<FF>(s16, st, task_off, pos0, npos, task0, slots)
    ALS_FOR_F(CALL)
#undef CALL
}

}  // namespace als
