// Batched RMSE (Section 5.2 metric): sum over stored entries of (r_uv - x_u^T theta_v)^2.
// In implicit mode (Section 5.6) the per-entry term is c (p - d)^2 - d^2 with d = x_u^T theta_v,
// p = [r > 0], c = 1 + alpha max(r, 0): the part of the all-pairs cost that depends on the stored entries.
// One wavefront per work item (the same row chunks as the update), 4 stored entries per step with
// 16 lanes sharing one dot product (each lane fetches its features of a theta row with one 16-, one 8- and one 4-byte
// load, as in the update kernels); the rows of four steps are in flight together and the column ids of the next four
// arrive meanwhile; fp32 dots, fp64 accumulation of the squared errors, per-item partial sums added in item order by
// a single block (deterministic).
#include "tiles.h"

namespace als {

template <int F, typename PtrT, int MODE>
__global__ __launch_bounds__(64) void k_sse(const int32_t *__restrict__ task_row,
                                            const int32_t *__restrict__ task_chunk, int chunk,
                                            const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                            const float *__restrict__ val, const float *__restrict__ X,
                                            const float *__restrict__ Theta, float alpha,
                                            double *__restrict__ partial) {
    constexpr int NT = tiles_1d(F), G = 4;   // G steps of 4 entries are in flight together
    const int lane = threadIdx.x, i = lane & 15, kq = lane >> 4;
    const int64_t t = blockIdx.x;
    const int row = task_row[t];
    const int ch = task_chunk[t];
    const int64_t rs = (int64_t)ptr[row], re = (int64_t)ptr[row + 1];
    const int64_t s0 = rs + (int64_t)ch * chunk;
    const int64_t s1 = (s0 + chunk < re) ? s0 + chunk : re;
    const int len = s1 > s0 ? (int)(s1 - s0) : 0;   // >= 1 with the plan of this matrix; 0 reads nothing
    // x_u with the lane -> feature map of the gathers (16-, 8- and 4-byte loads per lane)
    float xr[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        const int ft = feature_of(F, q, i);
        xr[q] = ft >= 0 ? X[(int64_t)row * F + ft] : 0.f;
    }
    // column ids and ratings of a group of 16 entries: step d of the group holds entry 4d + kq
    auto load_entries = [&](int e0, int (&c)[G], float (&r)[G]) {
#pragma unroll
        for (int d = 0; d < G; ++d) {
            const int e = e0 + 4 * d + kq;
            const int64_t at = s0 + (e < len ? e : len - 1);
            c[d] = idx[at];
            r[d] = val[at];
        }
    };
    double acc = 0.0;
    int cn[G];
    float rn[G];
    if (len > 0) load_entries(0, cn, rn);
    for (int e0 = 0; e0 < len; e0 += 4 * G) {
        int c[G];
        float r[G], g[G][NT];
#pragma unroll
        for (int d = 0; d < G; ++d) {
            c[d] = cn[d];
            r[d] = rn[d];
        }
#pragma unroll
        for (int d = 0; d < G; ++d) gather_lane_features<F, ALS_F32>(Theta, c[d], i, g[d]);
        if (e0 + 4 * G < len) load_entries(e0 + 4 * G, cn, rn);   // of the next group, while the rows arrive
#pragma unroll
        for (int d = 0; d < G; ++d) {
            const bool ok = e0 + 4 * d + kq < len;
            float dot = 0.f;
#pragma unroll
            for (int q = 0; q < NT; ++q) dot = fmaf(xr[q], g[d][q], dot);
            dot = rowsum16(dot);
            if constexpr (MODE == kImplicit) {
                const double rp = r[d] > 0.f ? (double)r[d] : 0.0, dd = (double)dot;
                const double pe = (r[d] > 0.f ? 1.0 : 0.0) - dd;
                if (ok && i == 0) acc += (1.0 + (double)alpha * rp) * pe * pe - dd * dd;
            } else {
                const float err = r[d] - dot;
                if (ok && i == 0) acc += (double)err * (double)err;
            }
        }
    }
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (lane == 0) partial[t] = acc;
}

__global__ __launch_bounds__(1024) void k_sum_partials(const double *__restrict__ partial, int64_t n,
                                                       double *__restrict__ total) {
    __shared__ double red[1024];
    // each thread sums a contiguous range, then a fixed tree: the order never depends on timing
    const int64_t per = (n + 1023) / 1024;
    const int64_t a = per * threadIdx.x, b = (a + per < n) ? a + per : n;
    double s = 0.0;
    for (int64_t q = a; q < b; ++q) s += partial[q];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *total = red[0];
}

template <int F, typename PtrT>
static hipError_t sse_f(bool implicit, float alpha, hipStream_t st, const int32_t *task_row, const int32_t *task_chunk,
                        int64_t ntasks, int chunk, const void *ptr, const int32_t *idx, const float *val,
                        const float *X, const float *Theta, double *partial, double *total) {
    constexpr int64_t kPiece = 0x7fffffff / 64;   // a launch holds fewer than 2^32 threads
    for (int64_t t0 = 0; t0 < ntasks; t0 += kPiece) {
        const dim3 grid((unsigned)(ntasks - t0 < kPiece ? ntasks - t0 : kPiece));
        if (implicit)
            hipLaunchKernelGGL((k_sse<F, PtrT, kImplicit>), grid, dim3(64), 0, st, task_row + t0, task_chunk + t0, chunk,
                               (const PtrT *)ptr, idx, val, X, Theta, alpha, partial + t0);
        else
            hipLaunchKernelGGL((k_sse<F, PtrT, kExplicit>), grid, dim3(64), 0, st, task_row + t0, task_chunk + t0, chunk,
                               (const PtrT *)ptr, idx, val, X, Theta, alpha, partial + t0);
    }
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(1024), 0, st, partial, ntasks, total);
    return hipGetLastError();
}

hipError_t launch_sse(int f, bool ptr64, bool implicit, float alpha, hipStream_t st, const int32_t *task_row,
                      const int32_t *task_chunk, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx,
                      const float *val, const float *X, const float *Theta, double *partial, double *total) {
#define CALL(FF)                                                                                                      \
    (ptr64 ? sse_f<FF, int64_t>(implicit, alpha, st, task_row, task_chunk, ntasks, chunk, ptr, idx, val, X, Theta,    \
                                partial, total)                                                                       \
           : sse_f<FF, int32_t>(implicit, alpha, st, task_row, task_chunk, ntasks, chunk, ptr, idx, val, X, Theta,    \
                                partial, total))
    switch (f) {
        case 16: return CALL(16);
        case 32: return CALL(32);
        case 64: return CALL(64);
        case 100: return CALL(100);
        case 128: return CALL(128);
        case 256: return CALL(256);
        default: return hipErrorInvalidValue;
    }
#undef CALL
}

}  // namespace als
