// Algorithm 1 (CGSolve, Section 4.1) for rows with fewer than 64 stored entries, without forming A_u.
// Algorithm 1 touches A_u only through the products A_u p, and with G the n_u x f matrix of the gathered theta_v
//     A_u p = G^T (G p) + lambda n_u p            (eq. (2): A_u = sum theta_v theta_v^T + lambda n_u I),
// 2 n_u f multiply-adds instead of f^2 -- and no get_hermitian at all (n_u f^2 multiply-adds) -- when G stays in
// registers.  The paper always builds the f x f matrix; on Netflix-shaped data more than half of the rows have fewer
// than 64 entries, and for those the build and the dense products are most of the work.  Same iteration, same
// stopping rules and guards as cg_tiles (tiles.h); the products differ from the dense ones by rounding order only.
//
// One wavefront per row.  Lane (i, kq) holds, for the entries 4j + kq (j = 0 .. 15), the features that lane i holds
// of every tile in the other kernels (feature_of: registers q = 0 .. NT-1), i.e. G[j][q]; vectors are in the column
// layout of cg_tiles (register q of lane (i, kq) = v[feature_of(q, i)], the same in the four lane rows).
//   t = G p:      per entry the lane's partial dot product, summed over the 16 lanes of its lane row;
//   y = G^T t:    per feature the sum over the lane's entries, then over the four lane rows.
// Steps j beyond the row's last entry are skipped (a wavefront-uniform branch), so the cost follows n_u.
// 16-bit factor rows are widened on load: the products are those of the fp32 path on the rounded factor.
#include "hermitian_kernels.h"

namespace als {


constexpr int kShortSteps = 16;   // steps the registers of a wavefront hold

// W: wavefronts that share a row (1; 2 at f = 256, where the 64 entries of a row are 256 registers per lane).  The
// entries are dealt out in blocks of 64 / W; every wavefront holds all vectors and runs the whole iteration, and
// the partial sums of G^T t meet through LDS: one barrier per product (two buffers used in turn -- a wavefront can
// only reach the write of product k+2 after every wavefront has passed the barrier of product k+1, i.e. has finished
// reading the buffer of product k).  The sums are formed in the same order everywhere, so the wavefronts of a row
// hold identical vectors and take the same branches.
// NJ: steps of 4 entries one wavefront holds (16; 8 at f = 256): rows of fewer than 4 NJ W entries.
template <int F, typename PtrT, int ET, int W, int NJ>
__global__ __launch_bounds__(64 * W) void k_cg_gathered(const int32_t *__restrict__ perm, int64_t pos0,
                                                        const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                        const float *__restrict__ val, const void *__restrict__ Theta,
                                                        float lambda, int fs, float eps, float *__restrict__ Xout,
                                                        int *__restrict__ status) {
    static_assert(W == 1 || W == 2);
    constexpr int NT = tiles_1d(F), CAPW = 4 * NJ;   // entries of one wavefront
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, i = lane & 15, kq = lane >> 4;
    const int row = perm[pos0 + blockIdx.x];
    const int64_t r0 = (int64_t)ptr[row];
    // fewer than CAPW * W by the caller's choice of rows; clamped so that a plan built from other row offsets cannot
    // make the kernel read more than it holds
    int nrow = (int)((int64_t)ptr[row + 1] - r0);
    nrow = __builtin_amdgcn_readfirstlane(nrow < 0 ? 0 : (nrow > CAPW * W ? CAPW * W : nrow));
    float *xg = Xout + (int64_t)row * F;
    if (nrow == 0) {   // (the whole workgroup leaves here, before any barrier)
        store_zero_vec<F>(xg);
        return;
    }
    // this wavefront's entries: CAPW * wv .. of the row
    const int64_t s0 = r0 + CAPW * wv;
    const int n = __builtin_amdgcn_readfirstlane(nrow - CAPW * wv < 0 ? 0 : (nrow - CAPW * wv > CAPW ? CAPW : nrow - CAPW * wv));
    const int nj = (n + 3) >> 2;   // steps that hold an entry

    // Column ids and ratings: lane l fetches those of entry l (one coalesced load each), then every lane picks up
    // those of its own entries 4j + kq through the LDS crossbar -- one memory round trip for the whole row, so that the
    // gathers below can all be in flight together (loads complete in order: a second round of id loads behind the
    // first gathers would wait for them).
    const bool mine = lane < n;
    const int64_t at = mine ? s0 + lane : r0;
    const int my_col = idx[at];                      // (entries beyond the end: the row's first column, masked below)
    const float my_r = mine ? val[at] : 0.f;
    // the gathered rows and their ratings; entries beyond the end count as zero rows
    float G[NJ][NT], rt[NJ];
    int col[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int src = 4 * (4 * j + kq);            // byte address of lane 4j + kq
        col[j] = __builtin_amdgcn_ds_bpermute(src, my_col);
        rt[j] = bperm(src, my_r);
    }
#pragma unroll
    for (int j0 = 0; j0 < NJ; j0 += 4) {
#pragma unroll
        for (int j = j0; j < j0 + 4; ++j)
#pragma unroll
            for (int q = 0; q < NT; ++q) G[j][q] = 0.f;
        if (j0 < nj) {   // (four steps per branch)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const bool ok = 4 * (j0 + d) + kq < n;
                float g[NT];
                gather_lane_features<F, ET>(Theta, col[j0 + d], i, g);
#pragma unroll
                for (int q = 0; q < NT; ++q) G[j0 + d][q] = ok ? g[q] : 0.f;
            }
        }
    }

    // Sum of a per-lane partial vector over the four lane rows and, with W > 1, over the wavefronts of the row
    __shared__ float xch[W > 1 ? 2 * W * 16 * NT : 1];
    int buf = 0;
    auto allsum = [&](float (&y)[NT]) {
#pragma unroll
        for (int q = 0; q < NT; ++q) y[q] = colsum4(y[q]);
        if constexpr (W > 1) {
            // (element (q, i) at q * 16 + i: the 16 lanes of a lane row touch consecutive words, the four lane rows
            // read the same ones)
            float *mine_out = xch + (buf * W + wv) * 16 * NT + i;
            if (kq == 0) {
#pragma unroll
                for (int q = 0; q < NT; ++q) mine_out[16 * q] = y[q];
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < NT; ++q) y[q] = 0.f;
#pragma unroll
            for (int k = 0; k < W; ++k) {   // the same order in every wavefront
                const float *part = xch + (buf * W + k) * 16 * NT + i;
#pragma unroll
                for (int q = 0; q < NT; ++q) y[q] += part[16 * q];
            }
            buf ^= 1;
        }
    };

    // b_u = G^T r_u (get_bias, Section 2 step (i))
    float b[NT], x[NT];
    {
#pragma unroll
        for (int q = 0; q < NT; ++q) b[q] = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            if (j < nj) {
#pragma unroll
                for (int q = 0; q < NT; ++q) b[q] = fmaf(rt[j], G[j][q], b[q]);
            }
        allsum(b);
    }
    load_vec<F>(xg, x);   // warm start

    const float reg = lambda * (float)nrow;
    auto matvec = [&](const float (&p)[NT], float (&ap)[NT]) {
        float y[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) y[q] = 0.f;
#pragma unroll
        for (int j0 = 0; j0 < NJ; j0 += 2)
            if (j0 < nj) {   // (two steps per branch: a step without entries holds zeros)
                float t[2];
#pragma unroll
                for (int d = 0; d < 2; ++d) {
                    t[d] = 0.f;
#pragma unroll
                    for (int q = 0; q < NT; ++q) t[d] = fmaf(G[j0 + d][q], p[q], t[d]);
                }
#pragma unroll
                for (int d = 0; d < 2; ++d) t[d] = rowsum16(t[d]);   // theta_v . p of entry 4j + kq
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int q = 0; q < NT; ++q) y[q] = fmaf(G[j0 + d][q], t[d], y[q]);
            }
        allsum(y);
#pragma unroll
        for (int q = 0; q < NT; ++q) ap[q] = fmaf(reg, p[q], y[q]);
    };
    auto dot = [&](const float (&u)[NT], const float (&v)[NT]) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) s = fmaf(u[q], v[q], s);
        return rowsum16(s);   // the 4 lane rows hold the same values
    };

    // Algorithm 1, as in cg_tiles
    float r[NT], p[NT], ap[NT];
    matvec(x, ap);
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        r[q] = b[q] - ap[q];
        p[q] = r[q];
    }
    float rs_old = dot(r, r);
    if (rs_old != 0.f && !(rs_old > 0.f && isfinite(rs_old))) {   // non-finite input: the row gets NaN, reported by the store
#pragma unroll
        for (int q = 0; q < NT; ++q) x[q] = __builtin_nanf("");
    }
    if (rs_old > 0.f && isfinite(rs_old)) {
        for (int it = 0; it < fs; ++it) {
            matvec(p, ap);
            const float pap = dot(p, ap);
            if (!(pap > 0.f) || !isfinite(pap)) break;
            const float alpha = rs_old / pap;
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                x[q] = fmaf(alpha, p[q], x[q]);
                r[q] = fmaf(-alpha, ap[q], r[q]);
            }
            const float rs_new = dot(r, r);
            if (sqrtf(rs_new) < eps) break;
            const float beta = rs_new / rs_old;
#pragma unroll
            for (int q = 0; q < NT; ++q) p[q] = fmaf(beta, p[q], r[q]);
            rs_old = rs_new;
        }
    }
    if (wv == 0) store_vec<F>(xg, x, status);
}

// The same for rows of fewer than 64 / R entries, R = 2 or 4 of them per wavefront: a row of a dozen entries leaves
// most of a wavefront's lanes idle in the steps above, and what does not depend on n_u (the reductions over the lane
// rows, the dot products, the vector updates, the divisions: about 110 of the vector instructions of an iteration)
// is then paid once per R rows.  Row slot rs = kq / (4 / R) of the wavefront takes row pos0 + R * blockIdx + rs
// (none beyond pos_end); its 4 / R lane rows hold the entries (4 / R) j + kq % (4 / R), j = 0 .. 15.  Everything that
// is wavefront-uniform above (n_u, the row's pointers, lambda n_u, the scalars of Algorithm 1, its stopping tests) is
// a per-lane value here, the same in the lanes of a row slot; a row that has stopped keeps its x (select), the loop
// ends when every row of the wavefront has stopped.
template <int F, typename PtrT, int ET, int R>
__global__ __launch_bounds__(64) void k_cg_gathered_packed(const int32_t *__restrict__ perm, int64_t pos0, int64_t pos_end,
                                                           const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                           const float *__restrict__ val, const void *__restrict__ Theta,
                                                           float lambda, int fs, float eps, float *__restrict__ Xout,
                                                           int *__restrict__ status) {
    static_assert(R == 2 || R == 4);
    constexpr int NT = tiles_1d(F), NJ = kShortSteps, EPS = 4 / R, CAP = NJ * EPS;   // entries per step and per row
    const int lane = threadIdx.x, i = lane & 15, kq = lane >> 4;
    const int rs = kq / EPS, sub = kq % EPS;
    const int64_t pos = pos0 + (int64_t)R * blockIdx.x + rs;
    const bool valid = pos < pos_end;
    const int row = perm[valid ? pos : pos0];
    const int64_t s0 = (int64_t)ptr[row];
    int n = (int)((int64_t)ptr[row + 1] - s0);   // fewer than CAP by the caller's choice of rows (clamped: see above)
    n = !valid ? 0 : (n < 0 ? 0 : (n > CAP ? CAP : n));
    float *xg = Xout + (int64_t)row * F;
    // steps that hold an entry of some row of the wavefront (uniform)
    int nmax = 0;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int nk = __builtin_amdgcn_readlane(n, 16 * EPS * k);
        nmax = nk > nmax ? nk : nmax;
    }
    const int nj = (nmax + EPS - 1) / EPS;

    // column ids and ratings: lane l of a row slot fetches those of entry l of its row, then every lane picks up those
    // of its own entries
    const int lr = lane - 16 * EPS * rs;             // lane within the row slot, 0 .. 16 EPS - 1
    const bool mine = lr < n;
    const int64_t at = s0 + (mine ? lr : 0);
    const int my_col = (valid && n > 0) ? idx[at] : 0;   // (no entry: row 0 of the factor, masked below)
    const float my_r = mine ? val[at] : 0.f;
    float G[NJ][NT], rt[NJ];
    int col[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int src = 4 * (16 * EPS * rs + EPS * j + sub);
        col[j] = __builtin_amdgcn_ds_bpermute(src, my_col);
        rt[j] = bperm(src, my_r);
    }
#pragma unroll
    for (int j0 = 0; j0 < NJ; j0 += 4) {
#pragma unroll
        for (int j = j0; j < j0 + 4; ++j)
#pragma unroll
            for (int q = 0; q < NT; ++q) G[j][q] = 0.f;
        if (j0 < nj) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const bool ok = EPS * (j0 + d) + sub < n;
                float g[NT];
                gather_lane_features<F, ET>(Theta, col[j0 + d], i, g);
#pragma unroll
                for (int q = 0; q < NT; ++q) G[j0 + d][q] = ok ? g[q] : 0.f;
            }
        }
    }
    // sum over the lane rows of a row slot (R = 4: one lane row, nothing to add)
    auto slotsum = [&](float v) { return R == 2 ? v + __shfl_xor(v, 16) : v; };

    float b[NT], x[NT];
    {
        float s[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) s[q] = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            if (j < nj) {
#pragma unroll
                for (int q = 0; q < NT; ++q) s[q] = fmaf(rt[j], G[j][q], s[q]);
            }
#pragma unroll
        for (int q = 0; q < NT; ++q) b[q] = slotsum(s[q]);
    }
#pragma unroll
    for (int q = 0; q < NT; ++q) {   // warm start; a row without entries gets x = 0
        const int ft = feature_of(F, q, i);
        x[q] = (ft >= 0 && n > 0) ? xg[ft] : 0.f;
    }

    const float reg = lambda * (float)n;
    auto matvec = [&](const float (&p)[NT], float (&ap)[NT]) {
        float y[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) y[q] = 0.f;
#pragma unroll
        for (int j0 = 0; j0 < NJ; j0 += 2)
            if (j0 < nj) {
                float t[2];
#pragma unroll
                for (int d = 0; d < 2; ++d) {
                    t[d] = 0.f;
#pragma unroll
                    for (int q = 0; q < NT; ++q) t[d] = fmaf(G[j0 + d][q], p[q], t[d]);
                }
#pragma unroll
                for (int d = 0; d < 2; ++d) t[d] = rowsum16(t[d]);
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int q = 0; q < NT; ++q) y[q] = fmaf(G[j0 + d][q], t[d], y[q]);
            }
#pragma unroll
        for (int q = 0; q < NT; ++q) ap[q] = fmaf(reg, p[q], slotsum(y[q]));
    };
    auto dot = [&](const float (&u)[NT], const float (&v)[NT]) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) s = fmaf(u[q], v[q], s);
        return rowsum16(s);   // the lane rows of a row slot hold the same values
    };

    // Algorithm 1 with per-row stopping
    float r[NT], p[NT], ap[NT];
    matvec(x, ap);
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        r[q] = b[q] - ap[q];
        p[q] = r[q];
    }
    float rs_old = dot(r, r);
    bool live = n > 0 && rs_old > 0.f && isfinite(rs_old);
    if (n > 0 && !live && rs_old != 0.f) {   // non-finite input: the row gets NaN, reported by the store
#pragma unroll
        for (int q = 0; q < NT; ++q) x[q] = __builtin_nanf("");
    }
    for (int it = 0; it < fs; ++it) {
        if (__ballot(live) == 0ull) break;
        matvec(p, ap);
        const float pap = dot(p, ap);
        live = live && pap > 0.f && isfinite(pap);
        const float alpha = live ? rs_old / pap : 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            x[q] = live ? fmaf(alpha, p[q], x[q]) : x[q];
            r[q] = fmaf(-alpha, ap[q], r[q]);
        }
        const float rs_new = dot(r, r);
        live = live && !(sqrtf(rs_new) < eps);
        const float beta = live ? rs_new / rs_old : 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) p[q] = fmaf(beta, p[q], r[q]);
        rs_old = live ? rs_new : rs_old;
    }
    bool bad = false;
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        const int ft = feature_of(F, q, i);
        if (valid && sub == 0 && ft >= 0) {
            xg[ft] = x[q];
            bad |= !isfinite(x[q]);
        }
    }
    if (bad) atomicOr(status, kStatusNonFinite);
}

// rows: rows per wavefront (1, 2, 4)
template <int F, typename PtrT, int ROWS>
static hipError_t cg_gathered_f(int et, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos, const void *ptr,
                                const int32_t *idx, const float *val, const void *Theta, float lambda, int fs, float eps,
                                float *Xout, int *status) {
    // ROWS: 4, 2, 1 rows per wavefront; -2: two wavefronts per row (rows of 64 .. 127 entries, f <= 128).  At f = 256 a
    // wavefront holds 8 steps, so ROWS == 1 already means two wavefronts per row.
    constexpr int W = (F > 128 || ROWS == -2) ? 2 : 1, NJ = F > 128 ? kShortSteps / 2 : kShortSteps;
    constexpr int PER = ROWS > 0 ? ROWS : 1;
    const dim3 grid((unsigned)((npos + PER - 1) / PER)), block(ROWS > 1 ? 64 : 64 * W);
#define LAUNCH(E)                                                                                                           \
    if constexpr (ROWS <= 1)                                                                                                \
        hipLaunchKernelGGL((k_cg_gathered<F, PtrT, E, W, NJ>), grid, block, 0, st, perm, pos0, (const PtrT *)ptr, idx, val, \
                           Theta, lambda, fs, eps, Xout, status);                                                           \
    else                                                                                                                    \
        hipLaunchKernelGGL((k_cg_gathered_packed<F, PtrT, E, ROWS>), grid, block, 0, st, perm, pos0, pos0 + npos,           \
                           (const PtrT *)ptr, idx, val, Theta, lambda, fs, eps, Xout, status)
    if (et == ALS_F32) { LAUNCH(ALS_F32); } else if (et == ALS_BF16) { LAUNCH(ALS_BF16); } else { LAUNCH(ALS_F16); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_cg_gathered(int f, int rows_per_wave, bool ptr64, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                              int64_t npos, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                              float lambda, int fs, float eps, float *Xout, int *status) {
    if (npos <= 0) return hipSuccess;
    if ((et != ALS_F32 && et != ALS_BF16 && et != ALS_F16) ||
        (rows_per_wave != 1 && rows_per_wave != 2 && rows_per_wave != 4 && rows_per_wave != -2))
        return hipErrorInvalidValue;
#define ARGS et, st, perm, pos0, npos, ptr, idx, val, Theta, lambda, fs, eps, Xout, status
#define CALL_P(FF, PP) \
    (rows_per_wave == 4 ? cg_gathered_f<FF, PP, 4>(ARGS) : rows_per_wave == 2 ? cg_gathered_f<FF, PP, 2>(ARGS)   \
     : rows_per_wave == 1 ? cg_gathered_f<FF, PP, 1>(ARGS) : cg_gathered_f<FF, PP, -2>(ARGS))
    if (f == 256)   // one row per workgroup of two wavefronts only
        return rows_per_wave != 1 ? hipErrorInvalidValue
                                  : (ptr64 ? cg_gathered_f<256, int64_t, 1>(ARGS) : cg_gathered_f<256, int32_t, 1>(ARGS));
#define CALL(FF) (ptr64 ? CALL_P(FF, int64_t) : CALL_P(FF, int32_t))
    switch (f) {
        case 16: return CALL(16);
        case 32: return CALL(32);
        case 64: return CALL(64);
        case 100: return CALL(100);
        case 128: return CALL(128);
        default: return hipErrorInvalidValue;
    }
#undef CALL
#undef CALL_P
#undef ARGS
}

}  // namespace als
