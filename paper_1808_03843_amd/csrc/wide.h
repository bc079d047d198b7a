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
constexpr int wide_eu(int ET) { return ET == ALS_F32 ? kWideEu : (kWideEu > 2 ? 2 : kWideEu); }   // 16-bit inputs: two

// fn(integral_constant<w>) for the (wavefront-uniform) w == wave
template <int NW, typename Fn>
__device__ __forceinline__ void for_wave(int wave, Fn &&fn) {
    [&]<int... w>(std::integer_sequence<int, w...>) __attribute__((always_inline)) {
        ((wave == w ? fn(std::integral_constant<int, w>{}) : void()), ...);
    }(std::make_integer_sequence<int, NW>{});
}

}  // namespace als
