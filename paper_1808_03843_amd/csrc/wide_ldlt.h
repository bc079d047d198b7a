// Exact solve (Section 2 step (ii), the baseline of Section 4.1) for f = 256, where the wavefronts of one
// workgroup share a system: blocked LDL^T directly on the register tiles each wavefront holds (tile rows
// w and 15-w, see wide.hip), only the current panel travels through LDS.
//
// Per panel K (tile column K), all indices compile-time so that every tile keeps its registers:
//   (A) the wavefront that owns the diagonal tile stages it to LDS, factors it with one lane per row (values
//       of other rows through v_readlane), forward-substitutes the panel's part of b, and writes
//       W = L_KK^-1 (row-major), 1/d and z/d;
//   (B) every panel tile (R, K), R > K, becomes X = A_RK W^T = (L d)_RK on the matrix cores: the tile goes
//       through LDS from the accumulator layout into the operand layout, four 16x16x4 MFMAs, and the result
//       is left row-major in LDS for everybody;
//   (C) trailing update, every wavefront on its own tiles: tile(R, C) -= X_RK D^-1 X_CK^T, four MFMAs with
//       operands read from the panel in LDS; b of the rows below is updated by one thread per row.  The owner
//       of the next diagonal tile updates that tile first and runs (A) for the next panel at once, while the
//       others work on their trailing tiles: two barriers per panel.
// Back substitution from the last tile row up: the owner of row R computes x_R = W_R^T D^-1 (...) and
// subtracts X_RC^T x_R from the blocks C < R (it holds all tiles of its row).
#pragma once
#include "wide.h"

// call operators of the generic lambdas below: the bodies hold register tiles and must not become functions
#define ALS_INLINE __attribute__((always_inline))

namespace als {

// wavefronts that share a system here (the slot layout does not depend on it), and where their tiles live
#ifndef ALS_LDLT_WAVES
#define ALS_LDLT_WAVES 8
#endif
constexpr int kLdltWaves = ALS_LDLT_WAVES;
constexpr bool kLdltInVgpr = kLdltWaves >= 8;   // 17 tiles in vector registers, 34 in accumulation registers

template <int N, typename Fn>
__device__ __forceinline__ void static_for(Fn &&fn) {
    [&]<int... k>(std::integer_sequence<int, k...>) ALS_INLINE { (fn(std::integral_constant<int, k>{}), ...); }(
        std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ float read_lane(float v, int l) {   // l: compile-time or wave-uniform
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

template <int F>
struct LdltShared {
    static constexpr int NT = tiles_1d(F), TS = 16 * 17;   // a 16x16 tile row-major with stride 17
    float P[NT][TS];      // the panel: X_RK = (L d)_RK of the current K
    float Winv[NT][TS];   // L_KK^-1 of every panel (kept for the back substitution)
    float D[TS];          // staging of the diagonal tile
    __attribute__((aligned(16))) float bs[F];   // b, then y (L y = b), then x; virtual order
    float dinv[F];        // 1 / d_j
    float zk[2][16];      // y_j / d_j of the current panel (even / odd K: the next panel's is written early)
};

// MFMA on operands that were written by LDS reads or the vector ALU a moment ago
template <bool IN_VGPR>
__device__ __forceinline__ void mfma4(v4f &acc, float (&a)[4], float (&b)[4]) {
    if constexpr (IN_VGPR) {
        asm volatile("s_nop 7" : "+v"(acc), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]),
                     "+v"(b[2]), "+v"(b[3]));
#pragma unroll
        for (int s = 0; s < 4; ++s) asm volatile(ALS_MFMA_PRE "v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+v"(acc) : "v"(a[s]), "v"(b[s]));
    } else {
        asm volatile("s_nop 7" : "+a"(acc), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]),
                     "+v"(b[2]), "+v"(b[3]));
#pragma unroll
        for (int s = 0; s < 4; ++s) asm volatile(ALS_MFMA_PRE "v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+a"(acc) : "v"(a[s]), "v"(b[s]));
    }
}
template <bool IN_VGPR>
__device__ __forceinline__ void tie(v4f &acc) {
    if constexpr (IN_VGPR) asm volatile("" : "+v"(acc));
    else asm volatile("" : "+a"(acc));
}

// The part of wavefront W.  acc: its tiles (regulariser already on the diagonal).  Returns false if a pivot was
// not positive (it is then replaced by 1).  Every wavefront of the workgroup runs its own instance; they meet
// at the same barriers.
template <int F, int NW, int W>
__device__ __forceinline__ bool ldlt_wide_wave(v4f (&acc)[tiles_tri(F) / NW], LdltShared<F> &sh) {
    constexpr int NT = tiles_1d(F), TS = LdltShared<F>::TS;
    constexpr uint32_t ROWS = wave_rows(NT, NW, W);
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = lane & 15, g = lane >> 4;   // accumulator layout: register r = element (4g + r, c);
                                              // operand layout: register s = element (c, 4g + s)
    bool bad = false;
    // (A) for panel K, run by the wavefront that owns the diagonal tile
    auto factor_diagonal = [&](auto kt) ALS_INLINE {
        constexpr int K = decltype(kt)::value;
        constexpr int q = tiles_below(ROWS, K) + K;
#pragma unroll
        for (int r = 0; r < 4; ++r) sh.D[(4 * g + r) * 17 + c] = acc[q][r];
        const int i = c;   // lane i (of every lane row) holds row i
        float a[16];
#pragma unroll
        for (int cc = 0; cc < 16; ++cc) a[cc] = sh.D[i * 17 + cc];
        float z = sh.bs[16 * K + i];
        float dinv_mine = 0.f;
        float lcol[16];   // lcol[j] = L[i][j] (lanes i > j; the other lanes hold values nobody reads)
        static_for<16>([&](auto jt) ALS_INLINE {
            constexpr int j = decltype(jt)::value;
            float d = read_lane(a[j], j);
            if (!(d > 0.f)) { bad = true; d = 1.f; }
            float inv = __builtin_amdgcn_rcpf(d);
            inv = fmaf(fmaf(-d, inv, 1.f), inv, inv);   // one Newton step: as accurate as a division here
            if (i == j) dinv_mine = inv;
            const float l = a[j] * inv;
            lcol[j] = l;
            const float zj = read_lane(z, j);
            if (i > j) z = fmaf(-l, zj, z);
            // rank-1 update of the columns behind j; rows above the diagonal pick up values that are never
            // read (row i only ever uses its columns <= i), which saves a select per element
            static_for<15 - j>([&](auto ct) ALS_INLINE {
                constexpr int cc = j + 1 + decltype(ct)::value;
                a[cc] = fmaf(-l, read_lane(a[j], cc), a[cc]);   // (L d)[cc][j] comes from lane cc
            });
            __builtin_amdgcn_sched_barrier(0);   // keeps the broadcasts of later steps out of scalar registers
        });
        // W = L^-1, lane i holds column i: W[r][i] = [r == i] - sum_{j < r} L[r][j] W[j][i]
        float w[16];
        static_for<16>([&](auto rt) ALS_INLINE {
            constexpr int r = decltype(rt)::value;
            float s = (r == i) ? 1.f : 0.f;
            static_for<r>([&](auto jt) ALS_INLINE {
                constexpr int j = decltype(jt)::value;
                s = fmaf(-read_lane(lcol[j], r), w[j], s);
            });
            w[r] = s;
            if (lane < 16) sh.Winv[K][r * 17 + i] = s;
            __builtin_amdgcn_sched_barrier(0);
        });
        if (lane < 16) {
            sh.bs[16 * K + i] = z;
            sh.dinv[16 * K + i] = dinv_mine;
            sh.zk[K & 1][i] = z * dinv_mine;
        }
    };
    // (C) for one tile: tile(R, C) -= X_RK D_K^-1 X_CK^T
    auto update_tile = [&](auto rt, auto ct, float (&aop)[4], const float (&ndk)[4]) ALS_INLINE {
        constexpr int R = decltype(rt)::value, C = decltype(ct)::value;
        float bop[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) bop[s] = sh.P[C][c * 17 + 4 * g + s] * ndk[s];
        mfma4<kLdltInVgpr>(acc[tiles_below(ROWS, R) + C], aop, bop);
    };

    if constexpr (ROWS & 1u) factor_diagonal(std::integral_constant<int, 0>{});
    __syncthreads();
    static_for<NT - 1>([&](auto kt) ALS_INLINE {
        constexpr int K = decltype(kt)::value;
        // ---- (B) panel tiles of this wavefront
        static_for<NT>([&](auto rt) ALS_INLINE {
            constexpr int R = decltype(rt)::value;
            if constexpr (((ROWS >> R) & 1u) && R > K) {
                constexpr int q = tiles_below(ROWS, R) + K;
                float *Pr = sh.P[R];
#pragma unroll
                for (int r = 0; r < 4; ++r) Pr[(4 * g + r) * 17 + c] = acc[q][r];
                float aop[4], wop[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    aop[s] = Pr[c * 17 + 4 * g + s];
                    wop[s] = sh.Winv[K][c * 17 + 4 * g + s];
                }
                v4f x = (v4f){0.f, 0.f, 0.f, 0.f};
                mfma4<true>(x, aop, wop);
                mfma_drain();
                asm volatile("" : "+v"(x));
                acc[q] = x;
#pragma unroll
                for (int r = 0; r < 4; ++r) Pr[(4 * g + r) * 17 + c] = x[r];
            }
        });
        __syncthreads();
        // ---- (C) trailing tiles of this wavefront and b of the rows below the panel.  The owner of the next
        // diagonal tile updates that tile first and factors it right away, while the others are still busy
        // with their trailing tiles: the serial step (A) leaves the critical path where there is trailing work.
        float ndk[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) ndk[s] = -sh.dinv[16 * K + 4 * g + s];
        constexpr bool NEXT_OWNER = ((ROWS >> (K + 1)) & 1u) != 0;
        if constexpr (NEXT_OWNER) {
            constexpr int R = K + 1;
            float aop[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) aop[s] = sh.P[R][c * 17 + 4 * g + s];
            update_tile(std::integral_constant<int, R>{}, std::integral_constant<int, R>{}, aop, ndk);
            mfma_drain();
            tie<kLdltInVgpr>(acc[tiles_below(ROWS, R) + R]);
            {   // b of the rows of the next panel (lane i = row i; every lane row computes the same)
                const float *xr = &sh.P[R][c * 17];
                float z = sh.bs[16 * R + c];
#pragma unroll
                for (int k = 0; k < 16; ++k) z = fmaf(-xr[k], sh.zk[K & 1][k], z);
                if (lane < 16) sh.bs[16 * R + c] = z;
            }
            factor_diagonal(std::integral_constant<int, R>{});
        }
        static_for<NT>([&](auto rt) ALS_INLINE {
            constexpr int R = decltype(rt)::value;
            if constexpr (((ROWS >> R) & 1u) && R > K + 1) {
                float aop[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) aop[s] = sh.P[R][c * 17 + 4 * g + s];
                static_for<R - K>([&](auto ct) ALS_INLINE {
                    update_tile(rt, std::integral_constant<int, K + 1 + decltype(ct)::value>{}, aop, ndk);
                });
            }
        });
        if (tid < F && tid >= 16 * (K + 2)) {
            const float *xr = &sh.P[tid >> 4][(tid & 15) * 17];
            float z = sh.bs[tid];
#pragma unroll
            for (int k = 0; k < 16; ++k) z = fmaf(-xr[k], sh.zk[K & 1][k], z);
            sh.bs[tid] = z;
        }
        mfma_drain();
#pragma unroll
        for (int t = 0; t < tiles_tri(F) / NW; ++t) tie<kLdltInVgpr>(acc[t]);
        __syncthreads();
    });
    // ---- back substitution
    static_for<NT>([&](auto it) ALS_INLINE {
        constexpr int R = NT - 1 - decltype(it)::value;
        if constexpr ((ROWS >> R) & 1u) {
            float x = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) x = fmaf(sh.Winv[R][r * 17 + c], sh.bs[16 * R + r] * sh.dinv[16 * R + r], x);
            if (lane < 16) sh.bs[16 * R + c] = x;
            if constexpr (R > 0) {
                const float4 xr = *reinterpret_cast<const float4 *>(&sh.bs[16 * R + 4 * g]);
                float part[R];
                static_for<R>([&](auto ct) ALS_INLINE {
                    constexpr int C = decltype(ct)::value;
                    const v4f t = acc[tiles_below(ROWS, R) + C];
                    part[C] = fmaf(t[3], xr.w, fmaf(t[2], xr.z, fmaf(t[1], xr.y, t[0] * xr.x)));
                });
#pragma unroll
                for (int C = 0; C < R; ++C) part[C] += __shfl_xor(part[C], 16);
#pragma unroll
                for (int C = 0; C < R; ++C) part[C] += __shfl_xor(part[C], 32);
                if (lane < 16) {
#pragma unroll
                    for (int C = 0; C < R; ++C) sh.bs[16 * C + c] -= part[C];
                }
            }
        }
        if constexpr (R > 0) __syncthreads();
    });
    return !bad;
}

// Solves the system held in acc (without the regulariser reg = lambda * n_u) and writes x to xg.
// bsrc: b_u in virtual order (global memory or LDS other than sh).  Every thread of the workgroup must call.
template <int F, int NW>
__device__ __forceinline__ void ldlt_wide(v4f (&acc)[tiles_tri(F) / NW], LdltShared<F> &sh, const float *bsrc,
                                          float reg, float *__restrict__ xg, int *status) {
    static_assert(F % 16 == 0 && F <= 64 * NW, "one thread per element");
    constexpr int NT = tiles_1d(F);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, g = lane >> 4;
    if (tid < F) sh.bs[tid] = bsrc[tid];
    bool ok = true;
    for_wave<NW>(wave, [&](auto wt) ALS_INLINE {
        constexpr int W = decltype(wt)::value;
        constexpr uint32_t ROWS = wave_rows(NT, NW, W);
        static_for<NT>([&](auto rt) ALS_INLINE {   // lambda * n_u on the diagonal: element (i, i) sits in lane (i, i/4), register i%4
            constexpr int R = decltype(rt)::value;
            if constexpr ((ROWS >> R) & 1u) {
                constexpr int q = tiles_below(ROWS, R) + R;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[q][r] += ((c >> 2) == g && (c & 3) == r) ? reg : 0.f;
            }
        });
        __syncthreads();
        ok = ldlt_wide_wave<F, NW, W>(acc, sh);
    });
    if (__syncthreads_or(ok ? 0 : 1) && tid == 0) atomicOr(status, kStatusBadPivot);
    if (tid < F) {
        const float x = sh.bs[tid];
        xg[feature_of(F, tid >> 4, tid & 15)] = x;
        if (!isfinite(x)) atomicOr(status, kStatusNonFinite);
    }
}

// short rows: built and solved without leaving the registers of the workgroup
#ifndef ALS_LDLT_WIDE_EU
#define ALS_LDLT_WIDE_EU 2
#endif
#ifndef ALS_LDLT_WIDE_DEPTH
#define ALS_LDLT_WIDE_DEPTH 3
#endif
// MODE kImplicit (Section 5.6): weighted entries, the accumulators start from the tiles of Theta^T Theta (gram),
// regulariser lambda instead of lambda * n_u
template <int F, int NW, typename PtrT, bool WIDE, int ET, int MODE = kExplicit>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(ALS_LDLT_WIDE_EU, ALS_LDLT_WIDE_EU))) void k_hermitian_ldlt_wide(const int32_t *__restrict__ perm, int64_t pos0,
                                                                  const PtrT *__restrict__ ptr,
                                                                  const int32_t *__restrict__ idx,
                                                                  const float *__restrict__ val,
                                                                  const void *__restrict__ Theta, float lambda,
                                                                  float alpha, const float *__restrict__ gram,
                                                                  float *__restrict__ Xout, int *__restrict__ status) {
    static_assert(MODE == kExplicit || ET == ALS_F32, "implicit feedback: fp32 factors");
    constexpr int NT = tiles_1d(F), NTW = tiles_tri(F) / NW;
    __shared__ LdltShared<F> sh;
    __shared__ float bsrc[F];
    __shared__ __attribute__((aligned(16))) uint32_t stage16[ET != ALS_F32 ? 2 * tiles_1d(F) * 256 : 4];   // operand staging, 16-bit inputs
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = perm[pos0 + blockIdx.x];
    const int64_t s0 = (int64_t)ptr[row];
    const int len = (int)((int64_t)ptr[row + 1] - s0);
    float *xg = Xout + (int64_t)row * F;
    if (len == 0) {   // no observation: x_u = 0
        for (int q = threadIdx.x; q < F; q += 64 * NW) xg[q] = 0.f;
        return;
    }
    v4f acc[NTW];
#pragma unroll
    for (int q = 0; q < NTW; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
    for_wave<NW>(wave, [&](auto wt) ALS_INLINE {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
        if constexpr (MODE == kImplicit) load_tiles_rows<F, ROWS>(gram, acc);
        float b[NT];
        // 16-bit inputs: on the 16-bit matrix cores, the rows gathered once per workgroup (tiles16.h)
        if constexpr (ET != ALS_F32)
            accumulate_tiles16_shared<F, NW, WIDE, ET, true, ROWS>(idx, val, Theta, uniform64(s0), len, acc, b, stage16, wave);
        else
            accumulate_tiles<F, kLdltInVgpr, ALS_LDLT_WIDE_DEPTH, WIDE, ET, ROWS, true, MODE>(idx, val, Theta, uniform64(s0),
                                                                                              len, acc, b, alpha);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if (((ROWS >> R) & 1u) && lane < 16) bsrc[16 * R + lane] = b[R];
    });
    __syncthreads();
    ldlt_wide<F, NW>(acc, sh, bsrc, MODE == kImplicit ? lambda : lambda * (float)len, xg, status);
}

// rows whose A_u sits in a (reduced) fp32 slot
template <int F, int NW, typename PtrT, int MODE = kExplicit>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(ALS_LDLT_WIDE_EU, ALS_LDLT_WIDE_EU))) void k_solve_ldlt_wide(const int32_t *__restrict__ perm,
                                                              const int32_t *__restrict__ task_off, int64_t pos0,
                                                              int64_t task0, const PtrT *__restrict__ ptr,
                                                              const float *__restrict__ slots, float lambda,
                                                              const float *__restrict__ gram,
                                                              float *__restrict__ Xout, int *__restrict__ status) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), NTW = NTILES / NW, SLOT = slot_floats(F);
    __shared__ LdltShared<F> sh;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t pos = pos0 + blockIdx.x;
    const int row = perm[pos];
    const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
    float *xg = Xout + (int64_t)row * F;
    if (n_u == 0) {
        for (int q = threadIdx.x; q < F; q += 64 * NW) xg[q] = 0.f;
        return;
    }
    const float *slot = slots + (int64_t)(task_off[pos] - task0) * SLOT;
    v4f acc[NTW];
    for_wave<NW>(wave, [&](auto wt) ALS_INLINE {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    const int T = R * (R + 1) / 2 + C, q = tiles_below(ROWS, R) + C;
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[q][r] = slot[(T * 4 + r) * 64 + lane];
                    if constexpr (MODE == kImplicit) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[q][r] += gram[(T * 4 + r) * 64 + lane];
                    }
                }
            }
    });
    ldlt_wide<F, NW>(acc, sh, slot + NTILES * 256, MODE == kImplicit ? lambda : lambda * (float)n_u, xg, status);
}

// launch of the fused kernel for one element type of the gathered factor (one translation unit each: the
// kernels are specialised per wavefront and unrolled over the panels, and take a while to compile)
template <int ET>
hipError_t launch_hermitian_ldlt_wide_et(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                         int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                         const void *Theta, float lambda, float *Xout, int *status) {
    constexpr int WF = 256, NW = kLdltWaves;
    const dim3 grid((unsigned)npos), block(64 * NW);
#define LAUNCH(P, W)                                                                                              \
    hipLaunchKernelGGL((k_hermitian_ldlt_wide<WF, NW, P, W, ET>), grid, block, 0, st, perm, pos0, (const P *)ptr, idx, \
                       val, Theta, lambda, 0.f, (const float *)nullptr, Xout, status)
    if (ptr64) { if (wide) LAUNCH(int64_t, true); else LAUNCH(int64_t, false); }
    else       { if (wide) LAUNCH(int32_t, true); else LAUNCH(int32_t, false); }
#undef LAUNCH
    return hipGetLastError();
}
hipError_t launch_hermitian_ldlt_wide_bf16(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                           int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                           const void *Theta, float lambda, float *Xout, int *status);
hipError_t launch_hermitian_ldlt_wide_f16(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                          int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                          const void *Theta, float lambda, float *Xout, int *status);

}  // namespace als
