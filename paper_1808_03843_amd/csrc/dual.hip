// Exact update of rows with fewer entries than features, in the dual form.  With G the n_u x f matrix of the
// gathered theta_v, eq. (2) reads x_u = (G^T G + lambda n_u I_f)^-1 G^T r_u, and the push-through identity
// gives the same vector as
//     x_u = G^T y,   (G G^T + lambda n_u I_n) y = r_u,
// an n_u x n_u system instead of an f x f one (Section 2's "solve" step on the smaller of the two Gram
// matrices; the paper always forms the f x f one).  On Netflix-shaped data most rows have n_u < f = 100.
//
// One wavefront per row, n_u <= 16 NTD - 1 (NTD = 1, 2, 3, 4, 6 or 8):
//   K = G G^T on the matrix cores: tile (R, C) of K is a 16 x 16 x f product of the theta rows of entries
//   16R.. and 16C..; lane (i, kq) supplies features 16s + 4kq .. + 3 of entry 16T + i (one 16-byte load per tile
//   and block s of 16 features), i.e. the contraction runs over the features;
//   lambda n_u on the diagonal (1 on the diagonal of the padding entries, whose rows and columns are zero);
//   the LDL^T solver of the one-wavefront path (tiles.h) on the NTD(NTD+1)/2 tiles;
//   x = G^T y with a second pass over the same theta rows (they are in the L1 / L2), reduced over the 16 lanes
//   of a row.
#include "hermitian_kernels.h"

namespace als {

// ET: element type of the gathered factor (16-bit rows are widened on load: the products are those of the fp32 path)
// One row of n <= 16 NTD - 1 entries starting at s0, by the calling wavefront.
template <int F, int NTD, int ET>
__device__ __forceinline__ void dual_row(int n, int64_t s0, const int32_t *__restrict__ idx, const float *__restrict__ val,
                                         const void *__restrict__ Theta, float lambda, float *__restrict__ xg,
                                         int *__restrict__ status, float *tbuf) {
    constexpr int N = 16 * NTD, NTILES = tiles_tri(N), NS = (F + 15) / 16;   // NS blocks of 16 features
    const int lane = threadIdx.x, i = lane & 15, kq = lane >> 4;
    // entry 16T + i of the row: its theta row (entries beyond n_u: row 0, masked) and its rating
    constexpr int ES = ET == ALS_F32 ? 4 : 2;
    const char *grow[NTD];
    bool live[NTD];
    float rhs[NTD];
#pragma unroll
    for (int T = 0; T < NTD; ++T) {
        const int e = 16 * T + i;
        live[T] = e < n;
        const int64_t at = s0 + (live[T] ? e : 0);
        const int c = idx[at];
        rhs[T] = live[T] ? val[at] : 0.f;
        grow[T] = reinterpret_cast<const char *>(Theta) + (int64_t)c * (F * ES);
    }
    auto features = [&](int T, int s) -> v4f {   // features 16s + 4kq .. + 3 of entry 16T + i, zero where there is none
        const int ft = 16 * s + 4 * kq;
        v4f g = (v4f){0.f, 0.f, 0.f, 0.f};
        if (live[T] && ft < F) {   // F % 4 == 0: whole or nothing
            if constexpr (ET == ALS_F32) {
                g = *reinterpret_cast<const v4f *>(grow[T] + 4 * ft);
            } else {
                const uint2 w = *reinterpret_cast<const uint2 *>(grow[T] + 2 * ft);
                g = (v4f){widen_lo<ET>(w.x), widen_hi<ET>(w.x), widen_lo<ET>(w.y), widen_hi<ET>(w.y)};
            }
        }
        return g;
    };
    static_assert(F % 4 == 0);

    v4f acc[NTILES];
#pragma unroll
    for (int q = 0; q < NTILES; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int s = 0; s < NS; ++s) {
        v4f g[NTD];
#pragma unroll
        for (int T = 0; T < NTD; ++T) g[T] = features(T, s);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int R = 0; R < NTD; ++R)
#pragma unroll
                for (int C = 0; C <= R; ++C)
                    acc[R * (R + 1) / 2 + C] = __builtin_amdgcn_mfma_f32_16x16x4f32(g[R][u], g[C][u], acc[R * (R + 1) / 2 + C], 0, 0, 0);
    }
    // regulariser: element (j, j) of the diagonal tile R sits in lane (c, g = c/4), register c % 4
    const float reg = lambda * (float)n;
#pragma unroll
    for (int R = 0; R < NTD; ++R)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (i == 4 * kq + r) acc[R * (R + 1) / 2 + R][r] += (16 * R + i < n) ? reg : 1.f;

    float y[NTD];
    if (!ldlt_tiles<N>(acc, rhs, y, tbuf) && lane == 0) atomicOr(status, kStatusBadPivot);

    // x = G^T y: lane (i, kq) adds up its entries' shares of features 16s + 4kq .. + 3, then the 16 lanes of the row
    bool bad = false;
#pragma unroll 1
    for (int s = 0; s < NS; ++s) {
        v4f part = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int T = 0; T < NTD; ++T) {
            const v4f g = features(T, s);
#pragma unroll
            for (int u = 0; u < 4; ++u) part[u] = fmaf(g[u], y[T], part[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) part[u] = rowsum16(part[u]);
        const int ft = 16 * s + 4 * kq;
        if (i == 0 && ft < F) {
            *reinterpret_cast<v4f *>(xg + ft) = part;
            bad |= !(isfinite(part[0]) && isfinite(part[1]) && isfinite(part[2]) && isfinite(part[3]));
        }
    }
    if (bad) atomicOr(status, kStatusNonFinite);
}

// One wavefront per row; the rows of a launch have fewer than 16 NTD entries, and those in the lower part of that
// range take a system of 3/4 (NTD >= 4) or 1/2 (NTD == 2) the size: the choice is uniform over the wavefront.
template <int F, int NTD, typename PtrT, int ET>
__global__ __launch_bounds__(64) void k_dual_exact(const int32_t *__restrict__ perm, int64_t pos0,
                                                   const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                   const float *__restrict__ val, const void *__restrict__ Theta,
                                                   float lambda, float *__restrict__ Xout, int *__restrict__ status) {
    __shared__ float tbuf[16 * 17];
    const int row = perm[pos0 + blockIdx.x];
    const int64_t s0 = (int64_t)ptr[row];
    const int n = (int)((int64_t)ptr[row + 1] - s0);   // <= 16 NTD - 1 by the caller's choice of rows
    float *xg = Xout + (int64_t)row * F;
    if (n == 0) {
        for (int q = threadIdx.x; q < F; q += 64) xg[q] = 0.f;
        return;
    }
    constexpr int SMALL = NTD >= 4 ? 3 * NTD / 4 : NTD / 2;
    if (n < 16 * SMALL)
        dual_row<F, SMALL, ET>(n, s0, idx, val, Theta, lambda, xg, status, tbuf);
    else
        dual_row<F, NTD, ET>(n, s0, idx, val, Theta, lambda, xg, status, tbuf);
}

template <int F, int NTD>
static hipError_t dual_n(bool ptr64, int et, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                         const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                         float *Xout, int *status) {
    const dim3 grid((unsigned)npos), block(64);
#define LAUNCH(P, E)                                                                                            \
    hipLaunchKernelGGL((k_dual_exact<F, NTD, P, E>), grid, block, 0, st, perm, pos0, (const P *)ptr, idx, val, Theta, \
                       lambda, Xout, status)
    if (ptr64) {
        if (et == ALS_F32) LAUNCH(int64_t, ALS_F32); else if (et == ALS_BF16) LAUNCH(int64_t, ALS_BF16); else LAUNCH(int64_t, ALS_F16);
    } else {
        if (et == ALS_F32) LAUNCH(int32_t, ALS_F32); else if (et == ALS_BF16) LAUNCH(int32_t, ALS_BF16); else LAUNCH(int32_t, ALS_F16);
    }
#undef LAUNCH
    return hipGetLastError();
}

bool has_dual_exact(int f, int ntd) {
    return (f == 100 || f == 128) ? (ntd == 2 || ntd == 4) : f == 256 ? (ntd == 2 || ntd == 4 || ntd == 8) : false;
}

hipError_t launch_dual_exact(int f, int ntd, bool ptr64, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                             int64_t npos, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                             float lambda, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    if (!has_dual_exact(f, ntd)) return hipErrorInvalidValue;
#define ARGS ptr64, et, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, Xout, status
    if (f == 100) return ntd == 2 ? dual_n<100, 2>(ARGS) : dual_n<100, 4>(ARGS);
    if (f == 128) return ntd == 2 ? dual_n<128, 2>(ARGS) : dual_n<128, 4>(ARGS);
    return ntd == 2 ? dual_n<256, 2>(ARGS) : ntd == 4 ? dual_n<256, 4>(ARGS) : dual_n<256, 8>(ARGS);
#undef ARGS
}

}  // namespace als
