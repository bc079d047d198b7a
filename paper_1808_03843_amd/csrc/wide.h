// Pieces shared by the kernels in which the wavefronts of one workgroup share a system (f = 256).
#pragma once
#include <utility>

#include "hermitian_kernels.h"

namespace als {

#ifndef ALS_WIDE_WAVES
#define ALS_WIDE_WAVES 8
#endif
constexpr int kWideWaves = ALS_WIDE_WAVES;   // 8: one pair of tile rows per wavefront; 4: two pairs
// 17 tiles per wavefront fit the vector registers beside the operand ring; 34 go to the accumulation
// registers (measured: the same speed)
constexpr bool kWideInVgpr = kWideWaves >= 8;
static_assert(64 * kWideWaves <= kWideThreads, "the host sizes its launches by kWideThreads");
// The fused kernel is built for four wavefronts per SIMD, i.e. two workgroups per CU, so that Algorithm 1 of
// one row (no MFMA work) overlaps the accumulation of another; that leaves registers for a gather pipeline
// of depth 1 only (depth 3 with one workgroup per CU was 19 % slower).
#ifndef ALS_DEPTH_WIDE
#define ALS_DEPTH_WIDE (ALS_WIDE_WAVES >= 8 ? 1 : 3)
#endif
#ifndef ALS_WIDE_EU
#define ALS_WIDE_EU (ALS_WIDE_WAVES >= 8 ? 4 : 1)
#endif
#ifndef ALS_DEPTH_WIDE_SLOTS
#define ALS_DEPTH_WIDE_SLOTS 3
#endif
constexpr int kDepthWideSlots = ALS_DEPTH_WIDE_SLOTS;
// wavefronts per SIMD the fused kernel is compiled for, and its gather pipeline depth
constexpr int kWideEu = ALS_WIDE_EU, kDepthWide = ALS_DEPTH_WIDE;
// (16-bit inputs and the weighted operands of implicit feedback need the register budget of two)
constexpr int wide_eu(int ET, int MODE = kExplicit) {
    return (ET == ALS_F32 && MODE == kExplicit) ? kWideEu : (kWideEu > 2 ? 2 : kWideEu);
}

// fn(integral_constant<w>) for the (wavefront-uniform) w == wave
template <int NW, typename Fn>
__device__ __forceinline__ void for_wave(int wave, Fn &&fn) {
    [&]<int... w>(std::integer_sequence<int, w...>) __attribute__((always_inline)) {
        ((wave == w ? fn(std::integral_constant<int, w>{}) : void()), ...);
    }(std::make_integer_sequence<int, NW>{});
}

// the tiles of the tile rows ROWS from a matrix stored like a slot (tile T, register r, lane l at (4T+r)*64 + l)
template <int F, uint32_t ROWS>
__device__ __forceinline__ void load_tiles_rows(const float *__restrict__ src, v4f (&acc)[tiles_in(ROWS)]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int R = 0; R < tiles_1d(F); ++R)
        if ((ROWS >> R) & 1u) {
#pragma unroll
            for (int C = 0; C <= R; ++C)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[tiles_below(ROWS, R) + C][r] = src[((R * (R + 1) / 2 + C) * 4 + r) * 64 + lane];
        }
}

}  // namespace als
