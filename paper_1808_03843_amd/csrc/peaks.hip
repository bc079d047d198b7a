// What this machine sustains, measured with the simplest kernels that can reach it: the rate of back-to-back
// independent MFMAs (fp32 16x16x4, bf16 and fp16 16x16x32) and of a streaming copy.  bench.py reports the
// roofline fractions against the published peaks; these figures say how much of a published peak is reachable at
// the clocks the machine actually holds under load.
#include "als_internal.h"

namespace als {

typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf_t __attribute__((ext_vector_type(8)));
typedef _Float16 v8h_t __attribute__((ext_vector_type(8)));
typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));

// Every wavefront runs `iters` rounds of 8 MFMAs on 8 accumulator tiles of its own: consecutive MFMAs are
// independent, so the pipeline never waits for a result.  The operands are small enough for the sums to stay
// finite; the result is stored only if it has a value it cannot have, which keeps the loop alive.
template <int ET>
__global__ __launch_bounds__(256) void k_mfma_peak(int iters, float *__restrict__ sink) {
    v4f_t acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = (v4f_t){0.f, 0.f, 0.f, 0.f};
    const float x = 9.765625e-4f * (float)(1 + (threadIdx.x & 3));   // 2^-10 .. 2^-8
    if constexpr (ET == ALS_F32) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x, x, acc[q], 0, 0, 0);
        }
    } else {
        // 0x3a80 is 2^-10 in bf16, 0x1400 is 2^-10 in fp16
        const uint32_t w = ET == ALS_BF16 ? 0x3a803a80u : 0x14001400u;
        const v4u_t u = (v4u_t){w, w, w, w};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if constexpr (ET == ALS_BF16)
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf_t, u), __builtin_bit_cast(v8bf_t, u), acc[q], 0, 0, 0);
                else
                    acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h_t, u), __builtin_bit_cast(v8h_t, u), acc[q], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) s += acc[q][0] + acc[q][1] + acc[q][2] + acc[q][3];
    if (s == -1.f) sink[threadIdx.x] = s;   // the sums are positive: never taken
}

// four independent 16-byte loads in flight per thread, then the four stores
__global__ __launch_bounds__(256) void k_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 1024) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + 256 * k < n16) v[k] = src[i + 256 * k];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + 256 * k < n16) dst[i + 256 * k] = v[k];
    }
}

// flops of one launch: workgroups * 4 wavefronts * iters * 8 MFMAs * (2 * 16 * 16 * K)
hipError_t launch_mfma_peak(int et, hipStream_t st, int workgroups, int iters, float *sink, double *flops) {
    const dim3 grid((unsigned)workgroups), block(256);
    if (et == ALS_F32) hipLaunchKernelGGL(k_mfma_peak<ALS_F32>, grid, block, 0, st, iters, sink);
    else if (et == ALS_BF16) hipLaunchKernelGGL(k_mfma_peak<ALS_BF16>, grid, block, 0, st, iters, sink);
    else if (et == ALS_F16) hipLaunchKernelGGL(k_mfma_peak<ALS_F16>, grid, block, 0, st, iters, sink);
    else return hipErrorInvalidValue;
    *flops = (double)workgroups * 4.0 * (double)iters * 8.0 * 2.0 * 256.0 * (et == ALS_F32 ? 4.0 : 32.0);
    return hipGetLastError();
}

hipError_t launch_copy(hipStream_t st, int workgroups, const void *src, void *dst, int64_t bytes) {
    hipLaunchKernelGGL(k_copy, dim3((unsigned)workgroups), dim3(256), 0, st, (const uint4 *)src, (uint4 *)dst, bytes / 16);
    return hipGetLastError();
}

}  // namespace als
