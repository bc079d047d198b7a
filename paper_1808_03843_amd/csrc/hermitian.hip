// get_hermitian + get_bias (Section 2, step (i); Section 3): the gathered, batched SYRK
//     A_u = sum_{v in Omega_u} theta_v theta_v^T,   b_u = sum_{v in Omega_u} r_uv theta_v
// on the fp32 matrix cores of gfx950.
//
// One wavefront owns one work item (a row, or a chunk of a long row) and keeps the whole lower
// triangle of A_u in MFMA accumulators: the paper keeps A_u in registers because it is the most
// reused operand (Section 3, Solution 1); here "registers" are the 16x16 accumulator tiles of
// v_mfma_f32_16x16x4_f32.  The K dimension of the MFMA runs over stored entries (4 per
// instruction), M and N both index features, so the A operand of tile row R and the B operand of
// tile column C are the same kind of register: lane l holds theta_{v(l/16)}[16*tile + l%16].
// theta rows are gathered straight into those operand registers (no staging buffer): every
// theta element is used by exactly one wavefront, so there is nothing to share through LDS, and a
// register double buffer hides the gather latency.
#include "als_internal.h"

namespace als {

typedef float v4f __attribute__((ext_vector_type(4)));

// acc += a (16x4, one stored entry per 16 lanes) * b (4x16).  Written as an in-place instruction on
// an accumulation register so that the 112 accumulators of f = 100 stay where they are across
// the loop (the builtin form let the register allocator shuffle them through copies).
__device__ __forceinline__ void mfma_16x16x4(v4f &acc, float a, float b) {
    asm("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

template <int F, typename PtrT>
__global__ __launch_bounds__(64) void k_hermitian(const int32_t *__restrict__ task_row,
                                                  const int32_t *__restrict__ task_chunk, int64_t task0, int chunk,
                                                  const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                  const float *__restrict__ val, const float *__restrict__ Theta,
                                                  float *__restrict__ slots) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = slot_floats(F);
    const int lane = threadIdx.x;
    const int i = lane & 15;   // feature inside a tile
    const int kq = lane >> 4;  // which of the 4 stored entries of a step
    const int64_t t = blockIdx.x;
    const int row = task_row[task0 + t];
    const int ch = task_chunk[task0 + t];
    const int64_t rs = (int64_t)ptr[row], re = (int64_t)ptr[row + 1];
    const int64_t s0 = rs + (int64_t)ch * chunk;
    const int64_t s1 = (s0 + chunk < re) ? s0 + chunk : re;
    const int len = (int)(s1 - s0);
    const int nsteps = (len + 3) >> 2;

    v4f acc[NTILES];
#pragma unroll
    for (int q = 0; q < NTILES; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    float bacc[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) bacc[q] = 0.f;

    // Software pipeline, every load unconditional (addresses clamped into the work item, the
    // values masked when they are consumed) so that the loop body is straight-line code:
    //   iteration s issues the (column id, rating) loads of step s+2, the theta gathers of
    //   step s+1, and runs the MFMAs of step s.
    const bool last_tile_ok = (16 * (NT - 1) + i) < F;
    const int fclamp = last_tile_ok ? 16 * (NT - 1) + i : F - 1;
    auto entry = [&](int step) {  // stored entry of this lane in a step, clamped
        const int e = 4 * step + kq;
        return e < len ? e : len - 1;
    };
    auto gather = [&](int c, float (&g)[NT]) {
        const float *p = Theta + (int64_t)c * F;
#pragma unroll
        for (int q = 0; q < NT - 1; ++q) g[q] = p[16 * q + i];
        g[NT - 1] = p[fclamp];
    };

    float gn[NT];
    int cn2;
    float rn, rn2;
    {
        const int e0 = entry(0);
        const int c0 = idx[s0 + e0];
        rn = val[s0 + e0];
        const int e1 = entry(1);
        cn2 = idx[s0 + e1];
        rn2 = val[s0 + e1];
        gather(c0, gn);
    }
    for (int s = 0; s < nsteps; ++s) {
        // (1) column id / rating of step s+2
        const int e2 = entry(s + 2);
        const int c_far = idx[s0 + e2];
        const float r_far = val[s0 + e2];
        // Keeps the two loads above in this iteration: without it the compiler folds the
        // loop-carried value into a load at the top of the NEXT iteration, which puts a full
        // memory latency in front of every gather.
        asm volatile("" ::: "memory");
        // (2) operands of step s (loaded one iteration ago), masked
        const bool ok = (4 * s + kq) < len;
        float g[NT];
#pragma unroll
        for (int q = 0; q < NT - 1; ++q) g[q] = ok ? gn[q] : 0.f;
        g[NT - 1] = (ok && last_tile_ok) ? gn[NT - 1] : 0.f;
        const float r = ok ? rn : 0.f;
        // (3) gathers of step s+1
        gather(cn2, gn);
        rn = rn2;
        cn2 = c_far;
        rn2 = r_far;
        // (4) MFMAs of step s, kept behind the loads issued above
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < NT; ++q) bacc[q] = fmaf(r, g[q], bacc[q]);
#pragma unroll
        for (int R = 0; R < NT; ++R)
#pragma unroll
            for (int C = 0; C <= R; ++C)
                mfma_16x16x4(acc[R * (R + 1) / 2 + C], g[R], g[C]);
    }

    // The MFMAs above are opaque to the compiler's hazard recogniser: leave the matrix pipeline
    // time to retire the last accumulator writes before they are read (8 passes = 32 cycles + margin).
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    float *out = slots + t * (int64_t)SLOT;
#pragma unroll
    for (int q = 0; q < NTILES; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) out[(q * 4 + r) * 64 + lane] = acc[q][r];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        float v = bacc[q];
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        if (kq == 0) out[NTILES * 256 + 16 * q + i] = v;
    }
}

template <int F>
static hipError_t launch_f(bool ptr64, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                           int64_t task0, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx,
                           const float *val, const float *Theta, float *slots) {
    if (ntasks <= 0) return hipSuccess;
    dim3 grid((unsigned)ntasks), block(64);
    if (ptr64)
        hipLaunchKernelGGL((k_hermitian<F, int64_t>), grid, block, 0, st, task_row, task_chunk, task0, chunk,
                           (const int64_t *)ptr, idx, val, Theta, slots);
    else
        hipLaunchKernelGGL((k_hermitian<F, int32_t>), grid, block, 0, st, task_row, task_chunk, task0, chunk,
                           (const int32_t *)ptr, idx, val, Theta, slots);
    return hipGetLastError();
}

hipError_t launch_hermitian(int f, bool ptr64, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                            int64_t task0, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx,
                            const float *val, const float *Theta, float *slots) {
    switch (f) {
        case 16: return launch_f<16>(ptr64, st, task_row, task_chunk, task0, ntasks, chunk, ptr, idx, val, Theta, slots);
        case 32: return launch_f<32>(ptr64, st, task_row, task_chunk, task0, ntasks, chunk, ptr, idx, val, Theta, slots);
        case 64: return launch_f<64>(ptr64, st, task_row, task_chunk, task0, ntasks, chunk, ptr, idx, val, Theta, slots);
        case 100: return launch_f<100>(ptr64, st, task_row, task_chunk, task0, ntasks, chunk, ptr, idx, val, Theta, slots);
        case 128: return launch_f<128>(ptr64, st, task_row, task_chunk, task0, ntasks, chunk, ptr, idx, val, Theta, slots);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace als
