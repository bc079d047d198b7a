// Device code shared by the get_hermitian kernels: the gathered SYRK main loop on fp32 MFMA
// accumulator tiles, and Algorithm 1 (CGSolve) run by one wavefront directly on those tiles.
#pragma once
#include "als_internal.h"

namespace als {

typedef float v4f __attribute__((ext_vector_type(4)));

// acc += a (16x4, one stored entry per 16 lanes) * b (4x16).  Written as an in-place instruction so
// that the accumulators stay where they are across the loop (the builtin form let the register
// allocator shuffle them through copies).  IN_VGPR picks architectural registers (needed when the
// tiles are read by vector ALU code afterwards) instead of accumulation registers.
template <bool IN_VGPR>
__device__ __forceinline__ void mfma_16x16x4(v4f &acc, float a, float b) {
    if constexpr (IN_VGPR)
        asm("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
    else
        asm("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// The MFMAs above are opaque to the compiler's hazard recogniser: leave the matrix pipeline time to
// retire the last accumulator writes before they are read (8 passes = 32 cycles, plus margin).
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory"); }

// A_u (lower-triangle tiles) and b_u (per-lane partial sums, one stored entry slot kq per 16 lanes)
// of the stored entries [s0, s0+len) of one row.  Section 2 step (i): get_hermitian and get_bias.
//
// Software pipeline with every load unconditional (addresses clamped into the work item, values
// masked when consumed) so that the loop body is straight-line code: iteration s issues the
// (column id, rating) loads of step s+2 and the theta gathers of step s+1, and runs the MFMAs of
// step s.  Lane l supplies theta_{v(l/16)}[16*tile + l%16] both as the A operand of tile row
// `tile` and as the B operand of tile column `tile`.
template <int F, bool IN_VGPR>
__device__ __forceinline__ void accumulate_tiles(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                 const float *__restrict__ Theta, int64_t s0, int len,
                                                 v4f (&acc)[tiles_tri(F)], float (&bacc)[tiles_1d(F)]) {
    constexpr int NT = tiles_1d(F);
    const int lane = threadIdx.x & 63;
    const int i = lane & 15;   // feature inside a tile
    const int kq = lane >> 4;  // which of the 4 stored entries of a step
    const int nsteps = (len + 3) >> 2;
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
        // Keeps the two loads above in this iteration: without it the compiler folds the loop-carried
        // value into a load at the top of the NEXT iteration, which puts a full memory latency in
        // front of every gather.
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
            for (int C = 0; C <= R; ++C) mfma_16x16x4<IN_VGPR>(acc[R * (R + 1) / 2 + C], g[R], g[C]);
    }
    mfma_drain();
}

// ---- cross-lane helpers -----------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// sum over the 16 lanes of a DPP row, result in every lane of the row
__device__ __forceinline__ float rowsum16(float v) {
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror
    return v;
}
// sum over the 4 rows of 16 lanes (lanes l, l+16, l+32, l+48), result in all of them
__device__ __forceinline__ float colsum4(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}
__device__ __forceinline__ float bperm(int byte_addr, float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(byte_addr, __builtin_bit_cast(int, v)));
}

// Algorithm 1 (CGSolve) on one system held by one wavefront.
//   acc   lower-triangle tiles of the symmetric A (register layout of the 16x16 MFMA result:
//         lane (c = l%16, g = l/16), register r of tile (R,C) is A[16R+4g+r][16C+c]); rows and
//         columns >= F are zero; the diagonal already carries lambda*n_u.
//   b, x  vectors in "column layout": register T of lane (c, g) holds v[16T + c] (the same in the 4
//         lane rows g); entries >= F are zero.  x is the warm start on entry, the result on exit.
// A*p is formed per tile row R: tile(R,C)*p_C (summed over the 16 lanes of a row with DPP) gives the
// rows of block R, tile(R,C)^T*p_R (summed over the 4 lane rows) the rows of block C.
template <int F>
__device__ __forceinline__ void cg_tiles(const v4f (&acc)[tiles_tri(F)], const float (&b)[tiles_1d(F)],
                                         float (&x)[tiles_1d(F)], int fs, float eps) {
    constexpr int NT = tiles_1d(F);
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    // lane (c,g) fetches p[16R + 4g + r] from the lane of its own row that holds column 4g+r
    int addr_rl[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) addr_rl[r] = 4 * (16 * g + 4 * g + r);
    // lane (c,g) fetches y[16T + c] from lane row c/4, where register c%4 holds it
    const int addr_cl = 4 * (16 * (c >> 2) + c);
    const int csel = c & 3;

    auto matvec = [&](const float (&p)[NT], float (&ap)[NT]) {
        float lower[NT];  // tile^T * p_R contributions, per-lane partial sums over the lane rows
#pragma unroll
        for (int q = 0; q < NT; ++q) lower[q] = 0.f;
#pragma unroll
        for (int R = 0; R < NT; ++R) {
            float pr[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) pr[r] = bperm(addr_rl[r], p[R]);
            float row[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int C = 0; C <= R; ++C) {
                const v4f t = acc[R * (R + 1) / 2 + C];
#pragma unroll
                for (int r = 0; r < 4; ++r) row[r] = fmaf(t[r], p[C], row[r]);
                if (C < R) {
                    float s = lower[C];
#pragma unroll
                    for (int r = 0; r < 4; ++r) s = fmaf(t[r], pr[r], s);
                    lower[C] = s;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) row[r] = rowsum16(row[r]);
            const float sel = csel == 0 ? row[0] : csel == 1 ? row[1] : csel == 2 ? row[2] : row[3];
            ap[R] = bperm(addr_cl, sel);
        }
#pragma unroll
        for (int q = 0; q < NT - 1; ++q) ap[q] += colsum4(lower[q]);
    };
    auto dot = [&](const float (&u)[NT], const float (&v)[NT]) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) s = fmaf(u[q], v[q], s);
        return rowsum16(s);   // the 4 lane rows hold the same values
    };

    float r[NT], p[NT], ap[NT];
    matvec(x, ap);
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        r[q] = b[q] - ap[q];
        p[q] = r[q];
    }
    float rs_old = dot(r, r);
    if (!(rs_old > 0.f)) return;
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

// adds reg to the diagonal entries (feature < F) of the diagonal tiles
template <int F>
__device__ __forceinline__ void add_diagonal(v4f (&acc)[tiles_tri(F)], float reg) {
    constexpr int NT = tiles_1d(F);
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int R = 0; R < NT; ++R)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (c == 4 * g + r && 16 * R + c < F) acc[R * (R + 1) / 2 + R][r] += reg;
}

}  // namespace als
