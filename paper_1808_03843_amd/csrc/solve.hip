// Dense export of A_u and b_u from the work-item slots (als_hermitian: tests and breakdown runs).  The solvers
// themselves run on the accumulator tiles: tiles.h (one wavefront), wide.hip / wide_ldlt.h (f = 256).
#include "tiles.h"

namespace als {

// tile index -> (tile row R, tile column C), R >= C
__device__ __forceinline__ void tile_rc(int tile, int &R, int &C) {
    int r = 0;
    while ((r + 1) * (r + 2) / 2 <= tile) ++r;
    R = r;
    C = tile - r * (r + 1) / 2;
}

// packed lower triangle: element (i, k), k <= i, at i(i+1)/2 + k
__device__ __forceinline__ int tri(int i, int k) { return i * (i + 1) / 2 + k; }

// Sums the slots of one row into a packed lower triangle As[tri(row, col)] (col <= row < F, feature
// coordinates) and bs[0..F).  Adds reg to the diagonal.  Every thread of the block takes part.
template <int F>
__device__ __forceinline__ void load_system(const float *__restrict__ slots, int nslots, float reg, float *As,
                                            float *bs) {
    constexpr int NT = tiles_1d(F), NTILES = tiles_tri(F), SLOT = slot_floats(F);
    for (int o = threadIdx.x; o < NTILES * 256; o += blockDim.x) {
        const int tile = o >> 8, r = (o >> 6) & 3, l = o & 63;
        int R, C;
        tile_rc(tile, R, C);
        const int lr = 4 * (l >> 4) + r, lc = l & 15;          // position inside the tile
        const int fr = feature_of(F, R, lr), fc = feature_of(F, C, lc);
        if (fr >= 0 && fc >= 0 && (R > C || lc <= lr)) {        // each unordered pair once
            float v = 0.f;
            for (int s = 0; s < nslots; ++s) v += slots[(int64_t)s * SLOT + o];
            if (fr == fc) v += reg;
            const int hi = fr > fc ? fr : fc, lo = fr > fc ? fc : fr;
            As[tri(hi, lo)] = v;
        }
    }
    for (int o = threadIdx.x; o < NT * 16; o += blockDim.x) {
        const int ft = feature_of(F, o >> 4, o & 15);
        if (ft >= 0) {
            float v = 0.f;
            for (int s = 0; s < nslots; ++s) v += slots[(int64_t)s * SLOT + NTILES * 256 + o];
            bs[ft] = v;
        }
    }
}

// ---- dense export (tests, breakdown runs) -----------------------------------------------------
template <int F, typename PtrT>
__global__ __launch_bounds__(256) void k_export_dense(const int32_t *__restrict__ perm,
                                                      const int32_t *__restrict__ task_off, int64_t pos0,
                                                      int64_t task0, const PtrT *__restrict__ ptr,
                                                      const float *__restrict__ slots, float lambda, int64_t row0,
                                                      float *__restrict__ A_out, float *__restrict__ b_out) {
    constexpr int SLOT = slot_floats(F);
    __shared__ float As[F * (F + 1) / 2];
    __shared__ float bs[F];
    const int64_t pos = pos0 + blockIdx.x;
    const int row = perm[pos];
    const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
    const int first = task_off[pos] - (int)task0, nslots = task_off[pos + 1] - task_off[pos];
    load_system<F>(slots + (int64_t)first * SLOT, nslots, lambda * (float)n_u, As, bs);
    __syncthreads();
    float *A = A_out + (row - row0) * (int64_t)F * F;
    for (int o = threadIdx.x; o < F * F; o += blockDim.x) {
        const int r = o / F, c = o % F;
        A[o] = (c <= r) ? As[tri(r, c)] : As[tri(c, r)];
    }
    for (int o = threadIdx.x; o < F; o += blockDim.x) b_out[(row - row0) * (int64_t)F + o] = bs[o];
}

#define ALS_DISPATCH_F(CALL)                       \
    switch (f) {                                   \
        case 16: return CALL(16);                  \
        case 32: return CALL(32);                  \
        case 64: return CALL(64);                  \
        case 100: return CALL(100);                \
        case 128: return CALL(128);                \
        case 256: return CALL(256);                \
        default: return hipErrorInvalidValue;      \
    }

template <int F, typename PtrT>
static hipError_t export_f(hipStream_t st, const int32_t *perm, const int32_t *task_off, int64_t pos0, int64_t npos,
                           int64_t task0, const void *ptr, const float *slots, float lambda, int64_t row0,
                           float *A_out, float *b_out) {
    if (npos <= 0) return hipSuccess;
    hipLaunchKernelGGL((k_export_dense<F, PtrT>), dim3((unsigned)npos), dim3(256), 0, st, perm, task_off, pos0,
                       task0, (const PtrT *)ptr, slots, lambda, row0, A_out, b_out);
    return hipGetLastError();
}

hipError_t launch_export_dense(int f, bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                               int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                               float lambda, int64_t row0, float *A_out, float *b_out) {
#define CALL(FF)                                                                                                   \
    (ptr64 ? export_f<FF, int64_t>(st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, row0, A_out, b_out) \
           : export_f<FF, int32_t>(st, perm, task_off, pos0, npos, task0, ptr, slots, lambda, row0, A_out, b_out))
    ALS_DISPATCH_F(CALL)
#undef CALL
}

}  // namespace als
