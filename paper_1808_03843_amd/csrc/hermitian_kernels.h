// Kernel templates of get_hermitian + get_bias and of the two solvers that run on the accumulator tiles
// (instantiated by hermitian.hip for eq. (2)/(3) and by implicit.hip for Section 5.6).
#pragma once
#include "tiles.h"
#include "tiles16.h"
#include "tiles_x3.h"

namespace als {

// gather pipeline depth (register sets of theta operands in flight per wavefront)
#ifndef ALS_DEPTH_SLOTS
#define ALS_DEPTH_SLOTS 3
#endif
#ifndef ALS_DEPTH_FUSED
#define ALS_DEPTH_FUSED 3
#endif
#ifndef ALS_FUSED_WAVES
#define ALS_FUSED_WAVES 2
#endif
constexpr int kDepthSlots = ALS_DEPTH_SLOTS, kDepthFused = ALS_DEPTH_FUSED;
// wavefronts per SIMD the fused kernel is compiled for (register budget 512 / waves)
// (f = 128 with 16-bit inputs: the operand sets of 32 entries and the extra b_u tiles need the whole file)
constexpr int fused_waves(int F, int ET = ALS_F32, int MODE = kExplicit) {
    if (ET == ALS_F32X3) return F <= 100 ? 2 : 1;   // three operand sets of 32 entries beside the accumulators
    if (ET == ALS_F32X2) return F <= 100 ? 2 : 1;   // two operand sets (f = 128: 144 accumulator registers)
    if ((ET == ALS_BF16 || ET == ALS_F16) && MODE == kImplicit && F > 64) return 1;   // likewise: w * theta in three parts
    return F <= 100 ? ALS_FUSED_WAVES : (ET != ALS_F32 ? 1 : 2);
}

// 16-bit factor inputs go to the 16-bit matrix cores where the width allows it (tiles16.h)
constexpr bool use_tiles16(int F, int ET, int MODE) {
    return (ET == ALS_BF16 || ET == ALS_F16) && (MODE == kExplicit || MODE == kImplicit) && has_tiles16(F);
}

// least number of wavefronts per SIMD k_hermitian is compiled for: with 16-bit inputs at f = 100 the allocator
// otherwise lands just above the register budget of two and then spreads out to one
constexpr int slot_waves(int F, int ET, int MODE = kExplicit) {
    if (ET == ALS_F32X3) return F <= 100 ? 2 : 1;   // rows staged through LDS: two wavefronts fit
    if (ET == ALS_F32X2) return F <= 100 ? 2 : 1;
    return (F == 100 && (ET == ALS_BF16 || ET == ALS_F16) && MODE == kExplicit) ? 2 : 1;
}

// a value that is the same in every lane, moved to scalar registers
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// MODE: kExplicit (eq. (2)) or kImplicit (Section 5.6: every stored entry weighted by alpha * r_uv, b_u by
// 1 + alpha * r_uv; the dense Theta^T Theta term is added by the solver kernels).
template <int F, typename PtrT, bool WIDE, int ET, bool S16, int MODE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(slot_waves(F, ET, MODE)))) void k_hermitian(const int32_t *__restrict__ task_row,
                                                  const int32_t *__restrict__ task_chunk, const int32_t *__restrict__ task_order, int64_t task0, int chunk,
                                                  const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                  const float *__restrict__ val, const void *__restrict__ Theta,
                                                  float alpha, float *__restrict__ slots,
                                                  const uint32_t *__restrict__ absmax = nullptr) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = S16 ? slot_words16(F) : slot_floats(F);
    const int lane = threadIdx.x;
    // task_order (optional): the work item each workgroup of the launch takes (a permutation of the batch)
    const int64_t t = task_order ? (int64_t)task_order[task0 + blockIdx.x] - task0 : (int64_t)blockIdx.x;
    const int row = task_row[task0 + t];
    const int ch = task_chunk[task0 + t];
    const int64_t rs = (int64_t)ptr[row], re = (int64_t)ptr[row + 1];
    const int64_t s0 = rs + (int64_t)ch * chunk;
    const int64_t s1 = (s0 + chunk < re) ? s0 + chunk : re;
    // >= 1 with the plan of this matrix (rows without entries have no work items); a plan built from other row
    // offsets can name a chunk beyond the end of the row: then nothing is read
    const int len = s1 > s0 ? (int)(s1 - s0) : 0;

    v4f acc[NTILES];
#pragma unroll
    for (int q = 0; q < NTILES; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    float b[NT];
    if constexpr (ET == ALS_F32X3 || ET == ALS_F32X2) {   // fp32 rows cut into 16-bit parts, 16-bit matrix cores (tiles_x3.h)
        __shared__ __attribute__((aligned(16))) uint32_t fifo[x3_fifo_words(F)];   // one wavefront per workgroup
        // absmax (two-part route): the bits of max |Theta|, left by a reduction that ran before this launch
        const uint32_t mx = ET == ALS_F32X2 ? __builtin_amdgcn_readfirstlane(absmax[0]) : 0u;
        accumulate_tiles_x3<F, WIDE, true, rows_all(F), ET == ALS_F32X3 ? 3 : 2>(idx, val, Theta, uniform64(s0), len, acc, b,
                                                                                   fifo, mx);
    }
    else if constexpr (use_tiles16(F, ET, MODE))
        accumulate_tiles16<F, WIDE, ET, true, rows_all(F), MODE>(idx, val, Theta, uniform64(s0), len, acc, b, alpha);
    else
        accumulate_tiles<F, false, kDepthSlots, WIDE, ET, rows_all(F), true, MODE>(idx, val, Theta, uniform64(s0), len, acc,
                                                                                   b, alpha);

    float *out = slots + t * (int64_t)SLOT;
    if constexpr (S16) {
        uint32_t *out32 = reinterpret_cast<uint32_t *>(out);
#pragma unroll
        for (int q = 0; q < NTILES; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h) out32[(q * 2 + h) * 64 + lane] = pack_bf16(acc[q][2 * h], acc[q][2 * h + 1]);
#pragma unroll
        for (int q = 0; q < NT; ++q)
            if (lane < 16) out[NTILES * 128 + 16 * q + lane] = b[q];
    } else {
#pragma unroll
        for (int q = 0; q < NTILES; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[(q * 4 + r) * 64 + lane] = acc[q][r];
#pragma unroll
        for (int q = 0; q < NT; ++q)
            if (lane < 16) out[NTILES * 256 + 16 * q + lane] = b[q];
    }
}

// x (column layout, virtual coordinates) <-> a factor row in memory
template <int F>
__device__ __forceinline__ void load_vec(const float *__restrict__ src, float (&x)[tiles_1d(F)]) {
    const int c = threadIdx.x & 15;
#pragma unroll
    for (int q = 0; q < tiles_1d(F); ++q) {
        const int ft = feature_of(F, q, c);
        x[q] = ft >= 0 ? src[ft] : 0.f;
    }
}
template <int F>
__device__ __forceinline__ void store_vec(float *__restrict__ dst, const float (&x)[tiles_1d(F)], int *status) {
    const int lane = threadIdx.x & 63;
    bool bad = false;
#pragma unroll
    for (int q = 0; q < tiles_1d(F); ++q) {
        const int ft = feature_of(F, q, lane & 15);
        if (lane < 16 && ft >= 0) {
            dst[ft] = x[q];
            bad |= !isfinite(x[q]);
        }
    }
    if (bad) atomicOr(status, kStatusNonFinite);
}
template <int F>
__device__ __forceinline__ void store_zero_vec(float *__restrict__ dst) {
    for (int q = threadIdx.x; q < F; q += 64) dst[q] = 0.f;
}

// Tiles of a Gram matrix stored like a slot (tile q, register r, lane l at (4q+r)*64 + l)
template <int F>
__device__ __forceinline__ void load_tiles(const float *__restrict__ src, v4f (&acc)[tiles_tri(F)]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < tiles_tri(F); ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[q][r] = src[(q * 4 + r) * 64 + lane];
}

// gram (kImplicit only): tiles of Theta^T Theta, the starting value of the accumulators
template <int F, typename PtrT, bool WIDE, int ET, int SOLVER, int MODE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(fused_waves(F, ET, MODE), fused_waves(F, ET, MODE)))) void k_hermitian_cg(
    const int32_t *__restrict__ perm, int64_t pos0, const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
    const float *__restrict__ val, const void *__restrict__ Theta, float lambda, float alpha,
    const float *__restrict__ gram, int fs, float eps, float *__restrict__ Xout, int *__restrict__ status,
    const uint32_t *__restrict__ absmax = nullptr) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F);
    const int lane = threadIdx.x;
    const int row = perm[pos0 + blockIdx.x];
    const int64_t s0 = (int64_t)ptr[row];
    const int len = (int)((int64_t)ptr[row + 1] - s0);
    float *xg = Xout + (int64_t)row * F;
    if (len == 0) {   // no observation: x_u = 0
        store_zero_vec<F>(xg);
        return;
    }
    v4f acc[NTILES];
    if constexpr (MODE == kImplicit) {
        load_tiles<F>(gram, acc);
    } else {
#pragma unroll
        for (int q = 0; q < NTILES; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    }
    float b[NT];
    if constexpr (ET == ALS_F32X3 || ET == ALS_F32X2) {
        __shared__ __attribute__((aligned(16))) uint32_t fifo[x3_fifo_words(F)];   // one wavefront per workgroup
        const uint32_t mx = ET == ALS_F32X2 ? __builtin_amdgcn_readfirstlane(absmax[0]) : 0u;
        accumulate_tiles_x3<F, WIDE, true, rows_all(F), ET == ALS_F32X3 ? 3 : 2>(idx, val, Theta, uniform64(s0), len, acc, b,
                                                                                   fifo, mx);
    }
    else if constexpr (use_tiles16(F, ET, MODE))
        accumulate_tiles16<F, WIDE, ET, true, rows_all(F), MODE>(idx, val, Theta, uniform64(s0), len, acc, b, alpha);
    else
        accumulate_tiles<F, true, kDepthFused, WIDE, ET, rows_all(F), true, MODE>(idx, val, Theta, uniform64(s0), len, acc, b,
                                                                                  alpha);
    add_diagonal<F>(acc, MODE == kImplicit ? lambda : lambda * (float)len);
    float x[NT];
#ifdef ALS_TIMING_SKIP_SOLVER
    // Timing experiment only (wrong results): the fused kernel without its solver, to split its time into
    // get_hermitian and solve.  x_u = a bounded function of b_u and of every tile, so that nothing is optimised away
    // and the factors keep an ordinary magnitude over the sweeps of a timing run.
#pragma unroll
    for (int q = 0; q < NT; ++q) x[q] = b[q];
#pragma unroll
    for (int q = 0; q < NTILES; ++q) x[q % NT] += acc[q][0] + acc[q][1] + acc[q][2] + acc[q][3];
#pragma unroll
    for (int q = 0; q < NT; ++q) x[q] = x[q] / (1.f + fabsf(x[q]));
    (void)fs; (void)eps; (void)lane;
#else
    if constexpr (SOLVER == ALS_SOLVER_CG) {
        load_vec<F>(xg, x);
        cg_tiles<F>(acc, b, x, fs, eps);
    } else {
        __shared__ float tbuf[16 * 17];   // one wavefront per workgroup
        if (!ldlt_tiles<F>(acc, b, x, tbuf) && lane == 0) atomicOr(status, kStatusBadPivot);
    }
#endif
    store_vec<F>(xg, x, status);
}

template <int F, typename PtrT, bool S16, int SOLVER, int MODE>
__global__ __launch_bounds__(64) void k_solve_cg_wave(const int32_t *__restrict__ perm,
                                                      const int32_t *__restrict__ task_off, int64_t pos0,
                                                      int64_t task0, const PtrT *__restrict__ ptr,
                                                      const float *__restrict__ slots, float lambda,
                                                      const float *__restrict__ gram, int fs, float eps,
                                                      float *__restrict__ Xout, int *__restrict__ status) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = S16 ? slot_words16(F) : slot_floats(F);
    const int lane = threadIdx.x, c = lane & 15;
    const int64_t pos = pos0 + blockIdx.x;
    const int row = perm[pos];
    const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
    float *xg = Xout + (int64_t)row * F;
    if (n_u == 0) {
        store_zero_vec<F>(xg);
        return;
    }
    const float *slot = slots + (int64_t)(task_off[pos] - task0) * SLOT;
    v4f acc[NTILES];
    float b[NT];
    if constexpr (S16) {
        const uint32_t *slot32 = reinterpret_cast<const uint32_t *>(slot);
#pragma unroll
        for (int q = 0; q < NTILES; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t w = slot32[(q * 2 + h) * 64 + lane];
                acc[q][2 * h] = bits_to_float(w << 16);
                acc[q][2 * h + 1] = bits_to_float(w & 0xffff0000u);
            }
#pragma unroll
        for (int q = 0; q < NT; ++q) b[q] = slot[NTILES * 128 + 16 * q + c];
    } else {
#pragma unroll
        for (int q = 0; q < NTILES; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[q][r] = slot[(q * 4 + r) * 64 + lane];
#pragma unroll
        for (int q = 0; q < NT; ++q) b[q] = slot[NTILES * 256 + 16 * q + c];
    }
    if constexpr (MODE == kImplicit) {
#pragma unroll
        for (int q = 0; q < NTILES; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[q][r] += gram[(q * 4 + r) * 64 + lane];
    }
    add_diagonal<F>(acc, MODE == kImplicit ? lambda : lambda * (float)n_u);
    float x[NT];
    if constexpr (SOLVER == ALS_SOLVER_CG) {
        load_vec<F>(xg, x);
        cg_tiles<F>(acc, b, x, fs, eps);
    } else {
        __shared__ float tbuf[16 * 17];   // one wavefront per workgroup
        if (!ldlt_tiles<F>(acc, b, x, tbuf) && lane == 0) atomicOr(status, kStatusBadPivot);
    }
    store_vec<F>(xg, x, status);
}

}  // namespace als
