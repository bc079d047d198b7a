// f = 256: the 136 tiles of A_u exceed one wavefront's registers, so the wavefronts of one workgroup share
// a system.  The 16 tile rows are dealt out in pairs (k, 15-k) of 17 tiles each, so that every wavefront
// holds the same number of tiles and runs the same number of MFMAs per gathered entry; each wavefront
// gathers the theta rows itself (the repeats hit the L1) and accumulates b_u for its own tile rows.
//
//   k_hermitian_wide      work items of long rows: tiles and b_u go to a slot (same slot layout as f <= 128).
//   k_hermitian_cg_wide   whole short rows (Section 3 + Section 4.1 fused): A_u stays in the registers of the
//                         workgroup and Algorithm 1 runs on it; only x_u is written.
//   k_solve_cg_wide       Algorithm 1 for rows whose A_u sits in a (reduced) slot.
//
// Algorithm 1 across wavefronts: thread t < f owns element t of x, r and p.  For A*p the vector is put in
// LDS; every wavefront multiplies its tiles (tile * p_C summed over the 16 lanes of a row gives rows of
// block R; tile^T * p_R gives per-lane-row partial sums of block C) and leaves the results in LDS, where
// the owner of each element adds them up in a fixed order.  Dot products: wavefront sums, then LDS.
#include "wide.h"

namespace als {

template <int F, int NW>
struct WideShared {
    static constexpr int YS = F + 16;   // stride of a row of partial sums: the 4 lane rows hit different banks
    __attribute__((aligned(16))) float ps[F];   // the vector A is applied to
    float yrow[F];                              // tile * p_C sums, complete
    float ylow[NW * 4][YS];                     // tile^T * p_R sums per wavefront and lane row
    float bs[F];                                // b_u (fused kernel)
    float red[2][NW];                           // wavefront sums of a dot product, two buffers in turn
};

// the share of one wavefront in A*p (p in sh.ps); ROWS = its tile rows
template <int F, int NW, uint32_t ROWS>
__device__ __forceinline__ void matvec_part(const v4f (&acc)[tiles_in(ROWS)], WideShared<F, NW> &sh, int wave) {
    constexpr int NT = tiles_1d(F);
    constexpr int RMAX = 31 - __builtin_clz(ROWS);
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    float pc[RMAX + 1], lower[RMAX + 1];
#pragma unroll
    for (int C = 0; C <= RMAX; ++C) {
        pc[C] = sh.ps[16 * C + c];
        lower[C] = 0.f;
    }
#pragma unroll
    for (int R = 0; R < NT; ++R)
        if ((ROWS >> R) & 1u) {
            const float4 pr = *reinterpret_cast<const float4 *>(&sh.ps[16 * R + 4 * g]);
            float row[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int C = 0; C <= R; ++C) {
                const v4f t = acc[tiles_below(ROWS, R) + C];
#pragma unroll
                for (int r = 0; r < 4; ++r) row[r] = fmaf(t[r], pc[C], row[r]);
                if (C < R) lower[C] = fmaf(t[3], pr.w, fmaf(t[2], pr.z, fmaf(t[1], pr.y, fmaf(t[0], pr.x, lower[C]))));
            }
            // lane c ends up with the sum of register c % 4, i.e. row 16R + 4g + c%4
            const float rs = rowsum16_sel4(row[0], row[1], row[2], row[3], (c & 1) != 0, (c & 2) != 0);
            if (c < 4) sh.yrow[16 * R + 4 * g + c] = rs;
        }
#pragma unroll
    for (int C = 0; C < RMAX; ++C) sh.ylow[wave * 4 + g][16 * C + c] = lower[C];   // columns >= RMAX stay zero
}

// Sum over the workgroup, the same value in every thread.  One barrier: consecutive calls alternate between
// two buffers, and a thread can only be two calls ahead of another one after a barrier in between.
template <int NW>
__device__ __forceinline__ float wide_sum(float v, float (&red)[2][NW], int &turn) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    float *buf = red[turn];
    turn ^= 1;
    if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += buf[w];
    return s;
}

// Algorithm 1 (CGSolve) for the system whose tiles the wavefronts of this workgroup hold in acc (without the
// regulariser: reg = lambda * n_u is applied as a diagonal term).  bsrc: b_u in virtual order (LDS or global).
// xg: the row of the factor matrix, warm start in, result out.  Every thread of the workgroup must call.
template <int F, int NW>
__device__ __forceinline__ void cg_wide(const v4f (&acc)[tiles_tri(F) / NW], WideShared<F, NW> &sh, const float *bsrc,
                                        float reg, int fs, float eps, float *__restrict__ xg, int *status) {
    static_assert(F % 16 == 0 && tiles_tri(F) % NW == 0 && F <= 64 * NW);
    constexpr int NT = tiles_1d(F);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool own = tid < F;   // owner of element tid of the vectors (virtual order)
    const int ft = feature_of(F, (tid >> 4) & (NT - 1), tid & 15);
    for (int k = tid; k < NW * 4 * WideShared<F, NW>::YS; k += 64 * NW) (&sh.ylow[0][0])[k] = 0.f;
    int turn = 0;
    // (no barrier in front: the last readers of ps passed the third barrier of the previous product, and the
    // owners' reads of yrow / ylow are followed by the barrier of a dot product before the next product)
    auto matvec = [&](float v) -> float {
        if (own) sh.ps[tid] = v;
        __syncthreads();
        for_wave<NW>(wave, [&](auto wt) {
            matvec_part<F, NW, wave_rows(NT, NW, decltype(wt)::value)>(acc, sh, wave);
        });
        __syncthreads();
        float y = 0.f;
        if (own) {
            y = sh.yrow[tid];
#pragma unroll
            for (int k = 0; k < NW * 4; ++k) y += sh.ylow[k][tid];
            y = fmaf(reg, v, y);
        }
        return y;
    };
    float x = own ? xg[ft] : 0.f;
    const float ax = matvec(x);
    float r = own ? bsrc[tid] - ax : 0.f;
    float p = r;
    float rs_old = wide_sum<NW>(r * r, sh.red, turn);
    if (rs_old != 0.f && !(rs_old > 0.f && isfinite(rs_old))) x = __builtin_nanf("");   // non-finite input: NaN, reported below
    if (rs_old > 0.f && isfinite(rs_old)) {
        for (int it = 0; it < fs; ++it) {
            const float ap = matvec(p);
            const float pap = wide_sum<NW>(p * ap, sh.red, turn);
            if (!(pap > 0.f) || !isfinite(pap)) break;
            const float alpha = rs_old / pap;
            x = fmaf(alpha, p, x);
            r = fmaf(-alpha, ap, r);
            const float rs_new = wide_sum<NW>(r * r, sh.red, turn);
            if (sqrtf(rs_new) < eps) break;
            p = fmaf(rs_new / rs_old, p, r);
            rs_old = rs_new;
        }
    }
    if (own) {
        xg[ft] = x;
        if (!isfinite(x)) atomicOr(status, kStatusNonFinite);
    }
}

// MODE: kExplicit, or kImplicit (Section 5.6: entries weighted by alpha * r_uv; the dense Theta^T Theta term is
// added by the solver kernels, as for f <= 128)
template <int F, int NW, typename PtrT, bool WIDE, int ET, bool S16, int MODE = kExplicit>
__global__ __launch_bounds__(64 * NW) void k_hermitian_wide(const int32_t *__restrict__ task_row,
                                                             const int32_t *__restrict__ task_chunk, const int32_t *__restrict__ task_order, int64_t task0,
                                                             int chunk, const PtrT *__restrict__ ptr,
                                                             const int32_t *__restrict__ idx,
                                                             const float *__restrict__ val,
                                                             const void *__restrict__ Theta, float alpha,
                                                             float *__restrict__ slots) {
    static_assert(MODE == kExplicit || ET == ALS_F32, "implicit feedback: fp32 factors");
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = S16 ? slot_words16(F) : slot_floats(F);
    __shared__ __attribute__((aligned(16))) uint32_t stage16[ET != ALS_F32 ? 2 * tiles_1d(F) * 256 : 4];   // operand staging, 16-bit inputs
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // task_order (optional): the work item each workgroup of the launch takes (a permutation of the batch)
    const int64_t t = task_order ? (int64_t)task_order[task0 + blockIdx.x] - task0 : (int64_t)blockIdx.x;
    const int row = task_row[task0 + t];
    const int ch = task_chunk[task0 + t];
    const int64_t rs = (int64_t)ptr[row], re = (int64_t)ptr[row + 1];
    const int64_t s0 = rs + (int64_t)ch * chunk;
    const int64_t s1 = (s0 + chunk < re) ? s0 + chunk : re;
    const int len = s1 > s0 ? (int)(s1 - s0) : 0;   // >= 1 with the plan of this matrix; 0 reads nothing
    float *out = slots + t * (int64_t)SLOT;
    for_wave<NW>(wave, [&](auto wt) {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
        v4f acc[tiles_in(ROWS)];
#pragma unroll
        for (int q = 0; q < tiles_in(ROWS); ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
        float b[NT];
        // 16-bit inputs: on the 16-bit matrix cores, the rows gathered once per workgroup (tiles16.h)
        if constexpr (ET != ALS_F32)
            accumulate_tiles16_shared<F, NW, WIDE, ET, true, ROWS>(idx, val, Theta, uniform64(s0), len, acc, b, stage16, wave);
        else
            accumulate_tiles<F, kWideInVgpr, kDepthWideSlots, WIDE, ET, ROWS, true, MODE>(idx, val, Theta, uniform64(s0), len,
                                                                                          acc, b, alpha);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    const v4f a = acc[tiles_below(ROWS, R) + C];
                    const int T = R * (R + 1) / 2 + C;
                    if constexpr (S16) {   // tiles as bf16 pairs (Section 4.2), b_u stays fp32
                        uint32_t *out32 = reinterpret_cast<uint32_t *>(out);
                        out32[(T * 2 + 0) * 64 + lane] = pack_bf16(a[0], a[1]);
                        out32[(T * 2 + 1) * 64 + lane] = pack_bf16(a[2], a[3]);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) out[(T * 4 + r) * 64 + lane] = a[r];
                    }
                }
                if (lane < 16) out[NTILES * (S16 ? 128 : 256) + 16 * R + lane] = b[R];
            }
    });
}

// gram (kImplicit only): tiles of Theta^T Theta in the slot layout, the starting value of the accumulators
template <int F, int NW, typename PtrT, bool WIDE, int ET, int MODE = kExplicit>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(wide_eu(ET, MODE), wide_eu(ET, MODE)))) void k_hermitian_cg_wide(const int32_t *__restrict__ perm, int64_t pos0,
                                                                const PtrT *__restrict__ ptr,
                                                                const int32_t *__restrict__ idx,
                                                                const float *__restrict__ val,
                                                                const void *__restrict__ Theta, float lambda,
                                                                float alpha, const float *__restrict__ gram, int fs,
                                                                float eps, float *__restrict__ Xout,
                                                                int *__restrict__ status) {
    static_assert(MODE == kExplicit || ET == ALS_F32, "implicit feedback: fp32 factors");
    constexpr int NT = tiles_1d(F), NTW = tiles_tri(F) / NW;
    __shared__ WideShared<F, NW> sh;
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
    for_wave<NW>(wave, [&](auto wt) {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
        static_assert(tiles_in(ROWS) == NTW);
        if constexpr (MODE == kImplicit) load_tiles_rows<F, ROWS>(gram, acc);
        float b[NT];
        // 16-bit inputs: on the 16-bit matrix cores, the rows gathered once per workgroup (tiles16.h)
        if constexpr (ET != ALS_F32)
            accumulate_tiles16_shared<F, NW, WIDE, ET, true, ROWS>(idx, val, Theta, uniform64(s0), len, acc, b, stage16, wave);
        else
            accumulate_tiles<F, kWideInVgpr, kDepthWide, WIDE, ET, ROWS, true, MODE>(idx, val, Theta, uniform64(s0), len, acc, b,
                                                                                     alpha);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if (((ROWS >> R) & 1u) && lane < 16) sh.bs[16 * R + lane] = b[R];
    });
    cg_wide<F, NW>(acc, sh, sh.bs, MODE == kImplicit ? lambda : lambda * (float)len, fs, eps, xg, status);
}

template <int F, int NW, typename PtrT, bool S16, int MODE = kExplicit>
__global__ __launch_bounds__(64 * NW) void k_solve_cg_wide(const int32_t *__restrict__ perm,
                                                            const int32_t *__restrict__ task_off, int64_t pos0,
                                                            int64_t task0, const PtrT *__restrict__ ptr,
                                                            const float *__restrict__ slots, float lambda,
                                                            const float *__restrict__ gram, int fs,
                                                            float eps, float *__restrict__ Xout,
                                                            int *__restrict__ status) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), NTW = NTILES / NW;
    constexpr int SLOT = S16 ? slot_words16(F) : slot_floats(F);
    __shared__ WideShared<F, NW> sh;
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
    for_wave<NW>(wave, [&](auto wt) {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    const int T = R * (R + 1) / 2 + C, q = tiles_below(ROWS, R) + C;
                    if constexpr (S16) {
                        const uint32_t *slot32 = reinterpret_cast<const uint32_t *>(slot);
                        const uint32_t w0 = slot32[(T * 2 + 0) * 64 + lane], w1 = slot32[(T * 2 + 1) * 64 + lane];
                        acc[q] = (v4f){bits_to_float(w0 << 16), bits_to_float(w0 & 0xffff0000u), bits_to_float(w1 << 16),
                                       bits_to_float(w1 & 0xffff0000u)};
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[q][r] = slot[(T * 4 + r) * 64 + lane];
                    }
                    if constexpr (MODE == kImplicit) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[q][r] += gram[(T * 4 + r) * 64 + lane];
                    }
                }
            }
    });
    cg_wide<F, NW>(acc, sh, slot + NTILES * (S16 ? 128 : 256), MODE == kImplicit ? lambda : lambda * (float)n_u, fs, eps,
                   xg, status);
}

// ---- launchers ---------------------------------------------------------------------------------------
namespace {
constexpr int WF = 256, NW = kWideWaves;

template <typename PtrT, bool WIDE>
hipError_t herm_wide_e(int et, bool s16, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk, const int32_t *task_order,
                       int64_t task0, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx, const float *val,
                       const void *Theta, float *slots) {
    const dim3 grid((unsigned)ntasks), block(64 * NW);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(E, S)                                                                                                \
    hipLaunchKernelGGL((k_hermitian_wide<WF, NW, PtrT, WIDE, E, S>), grid, block, 0, st, task_row, task_chunk, task_order, task0, \
                       chunk, p, idx, val, Theta, 0.f, slots)
    if (s16) {   // bf16 slots: fp32 factor inputs only
        if (et != ALS_F32) return hipErrorInvalidValue;
        LAUNCH(ALS_F32, true);
    } else if (et == ALS_F32) LAUNCH(ALS_F32, false);
    else if (et == ALS_BF16) LAUNCH(ALS_BF16, false);
    else LAUNCH(ALS_F16, false);
#undef LAUNCH
    return hipGetLastError();
}

template <int WF, int NW, typename PtrT, bool WIDE>
hipError_t herm_cg_wide_e(int et, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos, const void *ptr,
                          const int32_t *idx, const float *val, const void *Theta, float lambda, int fs, float eps,
                          float *Xout, int *status) {
    const dim3 grid((unsigned)npos), block(64 * NW);
    const PtrT *p = (const PtrT *)ptr;
#define LAUNCH(E)                                                                                                   \
    hipLaunchKernelGGL((k_hermitian_cg_wide<WF, NW, PtrT, WIDE, E>), grid, block, 0, st, perm, pos0, p, idx, val, Theta, \
                       lambda, 0.f, (const float *)nullptr, fs, eps, Xout, status)
    if (et == ALS_F32) LAUNCH(ALS_F32);
    else if (et == ALS_BF16) LAUNCH(ALS_BF16);
    else LAUNCH(ALS_F16);
#undef LAUNCH
    return hipGetLastError();
}
}  // namespace

hipError_t launch_hermitian_wide(bool ptr64, bool wide, int et, bool s16, hipStream_t st, const int32_t *task_row,
                                 const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                                 const int32_t *idx, const float *val, const void *Theta, float *slots) {
    if (ntasks <= 0) return hipSuccess;
#define ARGS et, s16, st, task_row, task_chunk, task_order, task0, ntasks, chunk, ptr, idx, val, Theta, slots
    if (ptr64) return wide ? herm_wide_e<int64_t, true>(ARGS) : herm_wide_e<int64_t, false>(ARGS);
    return wide ? herm_wide_e<int32_t, true>(ARGS) : herm_wide_e<int32_t, false>(ARGS);
#undef ARGS
}

hipError_t launch_hermitian_cg_wide(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                                    int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                    const void *Theta, float lambda, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
#define ARGS et, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, status
    if (f != 256) return hipErrorInvalidValue;
    if (ptr64) return wide ? herm_cg_wide_e<WF, NW, int64_t, true>(ARGS) : herm_cg_wide_e<WF, NW, int64_t, false>(ARGS);
    return wide ? herm_cg_wide_e<WF, NW, int32_t, true>(ARGS) : herm_cg_wide_e<WF, NW, int32_t, false>(ARGS);
#undef ARGS
}

hipError_t launch_solve_cg_wide(bool ptr64, bool s16, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                float lambda, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64 * NW);
#define LAUNCH(P, S)                                                                                               \
    hipLaunchKernelGGL((k_solve_cg_wide<WF, NW, P, S>), grid, block, 0, st, perm, task_off, pos0, task0, (const P *)ptr, \
                       slots, lambda, (const float *)nullptr, fs, eps, Xout, status)
    if (ptr64) { if (s16) LAUNCH(int64_t, true); else LAUNCH(int64_t, false); }
    else       { if (s16) LAUNCH(int32_t, true); else LAUNCH(int32_t, false); }
#undef LAUNCH
    return hipGetLastError();
}

// ---- implicit feedback at f = 256 (Section 5.6): Theta^T Theta and the launchers in kImplicit mode ----
// the rows [blockIdx.x * per, ...) of G as the "entries" of one work item (kGram mode), tiles to a slot
template <int F, int NW, bool WIDE>
__global__ __launch_bounds__(64 * NW) void k_gram_wide(const float *__restrict__ G, int64_t n, int per,
                                                        float *__restrict__ slots) {
    constexpr int NT = tiles_1d(F), SLOT = slot_floats(F);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t s0 = (int64_t)blockIdx.x * per;
    const int len = (int)((s0 + per < n) ? per : n - s0);   // >= 1 by the choice of the grid
    float *out = slots + (int64_t)blockIdx.x * SLOT;
    for_wave<NW>(wave, [&](auto wt) {
        constexpr uint32_t ROWS = wave_rows(NT, NW, decltype(wt)::value);
        v4f acc[tiles_in(ROWS)];
#pragma unroll
        for (int q = 0; q < tiles_in(ROWS); ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
        float b[NT];
        accumulate_tiles<F, kWideInVgpr, kDepthWideSlots, WIDE, ALS_F32, ROWS, false, kGram>(nullptr, nullptr, G, uniform64(s0),
                                                                                              len, acc, b);
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    const v4f a = acc[tiles_below(ROWS, R) + C];
                    const int T = R * (R + 1) / 2 + C;
#pragma unroll
                    for (int r = 0; r < 4; ++r) out[(T * 4 + r) * 64 + lane] = a[r];
                }
            }
    });
}

hipError_t launch_gram_wide(bool wide, hipStream_t st, const float *G, int64_t n, int per, int nslots, float *slots) {
    if (nslots <= 0) return hipSuccess;
    if (wide) hipLaunchKernelGGL((k_gram_wide<WF, NW, true>), dim3(nslots), dim3(64 * NW), 0, st, G, n, per, slots);
    else hipLaunchKernelGGL((k_gram_wide<WF, NW, false>), dim3(nslots), dim3(64 * NW), 0, st, G, n, per, slots);
    return hipGetLastError();
}

hipError_t launch_hermitian_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *task_row,
                                          const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk,
                                          const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                          float alpha, float *slots) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)ntasks), block(64 * NW);
#define LAUNCH(P, W)                                                                                               \
    hipLaunchKernelGGL((k_hermitian_wide<WF, NW, P, W, ALS_F32, false, kImplicit>), grid, block, 0, st, task_row,   \
                       task_chunk, task_order, task0, chunk, (const P *)ptr, idx, val, Theta, alpha, slots)
    if (ptr64) { if (wide) LAUNCH(int64_t, true); else LAUNCH(int64_t, false); }
    else       { if (wide) LAUNCH(int32_t, true); else LAUNCH(int32_t, false); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_hermitian_cg_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                             int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                             const void *Theta, float lambda, float alpha, const float *gram, int fs,
                                             float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64 * NW);
#define LAUNCH(P, W)                                                                                              \
    hipLaunchKernelGGL((k_hermitian_cg_wide<WF, NW, P, W, ALS_F32, kImplicit>), grid, block, 0, st, perm, pos0,    \
                       (const P *)ptr, idx, val, Theta, lambda, alpha, gram, fs, eps, Xout, status)
    if (ptr64) { if (wide) LAUNCH(int64_t, true); else LAUNCH(int64_t, false); }
    else       { if (wide) LAUNCH(int32_t, true); else LAUNCH(int32_t, false); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_solve_cg_wide_implicit(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                         int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                         float lambda, const float *gram, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    const dim3 grid((unsigned)npos), block(64 * NW);
    if (ptr64)
        hipLaunchKernelGGL((k_solve_cg_wide<WF, NW, int64_t, false, kImplicit>), grid, block, 0, st, perm, task_off, pos0,
                           task0, (const int64_t *)ptr, slots, lambda, gram, fs, eps, Xout, status);
    else
        hipLaunchKernelGGL((k_solve_cg_wide<WF, NW, int32_t, false, kImplicit>), grid, block, 0, st, perm, task_off, pos0,
                           task0, (const int32_t *)ptr, slots, lambda, gram, fs, eps, Xout, status);
    return hipGetLastError();
}

}  // namespace als
