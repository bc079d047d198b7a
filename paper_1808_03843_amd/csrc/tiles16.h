// get_hermitian + get_bias (Section 2 step (i), Section 3) on the 16-bit matrix cores, for factor matrices
// that are gathered as bf16 or fp16 (the reduced-precision route of Section 4.2 taken one step further: the
// products of two 16-bit values are exact in fp32, so v_mfma_f32_16x16x32_{bf16,f16} with its fp32
// accumulators computes the same sums as widening the inputs and multiplying in fp32 -- at 16 times the rate).
//
// One step consumes 32 stored entries: lane (i, kq) supplies, for every tile, the value of "its" feature in
// the 8 entries 8kq .. 8kq+7 of the step, packed in pairs (4 registers per tile).  The contraction index of the
// MFMA is the entry, and since the A and B operands of tile (R, C) are the same registers g[R], g[C], any
// assignment of entries to (lane row, register half) is as good as any other.
// Rows are gathered entry by entry with the widest loads the feature permutation allows (4, 2, 1 features per
// lane, the same lane -> feature map as the fp32 path, so that everything downstream is unchanged) and
// repacked with one byte-permute per register.
//
// b_u rides along: the rating is split into three 16-bit parts (hi + mid + lo = the fp32 rating up to 2^-24, or
// better; fp16 parts cannot go below the spacing 2^-24 of the smallest fp16 numbers, so with fp16 factors that bound
// is an absolute one for |r_uv| < 1).  When f is not a multiple of 16, three spare lanes of the last tile (features f, f+1, f+2 of the
// padded row) carry them, so rows f .. f+2 of the accumulated matrix add up to b_u; they and the remaining
// padding are zeroed at the end.  When f is a multiple of 16 there is no spare lane: the parts form an operand of
// their own (lanes 0..2, the others zero) and one more row of NT tiles is accumulated, whose rows 0..2 add up to
// b_u (NT more MFMAs per step).
#pragma once
#include "tiles.h"

namespace als {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// widths for which this route exists (one wavefront per system; up to 13 features in a partial last tile)
constexpr bool has_tiles16(int F) { return (F % 16) <= 13; }

template <int ET>
__device__ __forceinline__ void mfma_16x16x32(v4f &acc, const v4u &a, const v4u &b) {
    if constexpr (ET == ALS_BF16)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), acc, 0, 0, 0);
    else
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), acc, 0, 0, 0);
}

// two fp32 values -> their leading 16-bit parts packed (first in the low half), and the remainders
template <int ET>
__device__ __forceinline__ uint32_t split16(float &x0, float &x1) {
    if constexpr (ET == ALS_BF16) {   // truncation: the remainder is exact
        const uint32_t u0 = __builtin_bit_cast(uint32_t, x0), u1 = __builtin_bit_cast(uint32_t, x1);
        const uint32_t packed = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
        x0 -= bits_to_float(u0 & 0xffff0000u);
        x1 -= bits_to_float(u1 & 0xffff0000u);
        return packed;
    } else {
        typedef _Float16 v2h __attribute__((ext_vector_type(2)));
        const v2h h = __builtin_bit_cast(v2h, __builtin_amdgcn_cvt_pkrtz(x0, x1));
        x0 -= (float)h.x;
        x1 -= (float)h.y;
        return __builtin_bit_cast(uint32_t, h);
    }
}

// Same contract as accumulate_tiles<F, ..., ROWS, WANT_B, kExplicit>: acc += the tiles of the tile rows ROWS of
// sum theta theta^T over the entries [s0, s0+len), b = sum r theta in column layout (tile rows of ROWS; zero
// elsewhere), padding zeroed.
//
// MODE = kImplicit (Section 5.6): entry (u, v) enters A_u with the weight w = alpha * max(r_uv, 0) and b_u with
// c = 1 + w if r_uv > 0.  A weight does not fit into 16 bits together with the value, so the two operands of a tile
// differ: its columns get the plain 16-bit theta, its rows w * theta -- an fp32 product, cut into three 16-bit parts
// that add up to it (three MFMAs per tile instead of one).  The rating lanes (rows) carry the parts of c.
template <int F, bool WIDE, int ET, bool WANT_B, uint32_t ROWS = rows_all(F), int MODE = kExplicit>
__device__ __forceinline__ void accumulate_tiles16(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                   const void *__restrict__ Theta, int64_t s0, int len,
                                                   v4f (&acc)[tiles_in(ROWS)], float (&b)[tiles_1d(F)],
                                                   float alpha = 0.f) {
    static_assert(ET == ALS_BF16 || ET == ALS_F16);
    static_assert(MODE == kExplicit || MODE == kImplicit);
    constexpr bool IMP = MODE == kImplicit;
    static_assert(has_tiles16(F));
    static_assert(ROWS == rows_all(F) || (F % 16) == 0, "partial sets of tile rows need f to be a multiple of 16");
    constexpr int NT = tiles_1d(F), RI = F % 16;
    constexpr bool BX = RI == 0;   // the rating parts are an operand of their own
    constexpr int N4 = loads16(F), N2 = loads8(F), N1 = loads4(F);
    constexpr int base1 = 64 * N4 + 32 * N2;
    constexpr int RWE = 2 * N4 + N2 + N1;   // raw registers per gathered row
    constexpr int LB = (NT - 1) * NT / 2;
    const int lane = threadIdx.x & 63, i = lane & 15, kq = lane >> 4;
    const int32_t *__restrict__ ib = idx + s0;
    const float *__restrict__ vb = val + s0;
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t ids_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ib), 0, 4 * len, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vb), 0, 4 * len, kRsrcFlags);
    const int nsteps = (len + 31) >> 5;
    // lane offsets of the three kinds of loads inside a row (bytes)
    const uint32_t lane_a = 8u * (uint32_t)i;
    const uint32_t lane_b = 128u * N4 + 4u * (uint32_t)i;
    const uint32_t lane_c = 2u * (uint32_t)(base1 + i);
    const uint32_t lane_l = 2u * (uint32_t)((base1 + 16 * (N1 - 1) + i < F) ? base1 + 16 * (N1 - 1) + i : F - 1);
    const uint32_t eoff0 = 32u * (uint32_t)kq;   // this lane's 8 entries inside a step (bytes into idx / val)

    struct Ids { v4u lo, hi; };
    auto load_ids = [&](int t) -> Ids {
        const uint32_t o = eoff0 + 128u * (uint32_t)t;
        Ids r;
        r.lo = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(ids_rsrc, o, 0, 0));
        r.hi = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(ids_rsrc, o + 16u, 0, 0));
        return r;
    };
    auto load_ratings = [&](int t, float (&r)[8]) {
        const uint32_t o = eoff0 + 128u * (uint32_t)t;
        const v4u a = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o, 0, 0));
        const v4u c = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o + 16u, 0, 0));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r[j] = bits_to_float(a[j]);
            r[4 + j] = bits_to_float(c[j]);
        }
    };
    // one gathered row -> raw registers (entries beyond the work item read row 0 and are masked later)
    const uint32_t d_ab = lane_b - lane_a, d_ac = lane_c - lane_a, d_al = lane_l - lane_a;
    auto gather = [&](uint32_t c, uint32_t (&w)[RWE]) {
        const char *p;
        uint32_t oa;
        if constexpr (WIDE) {
            p = reinterpret_cast<const char *>(Theta) + (int64_t)c * (2 * F);
            oa = lane_a;
        } else {
            p = reinterpret_cast<const char *>(Theta);
            oa = row_offset<(uint32_t)(2 * F)>(c, lane_a);
        }
#pragma unroll
        for (int q = 0; q < N4; ++q) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p + oa + 128 * q);
            w[2 * q] = v.x;
            w[2 * q + 1] = v.y;
        }
        if constexpr (N2 > 0) w[2 * N4] = *reinterpret_cast<const uint32_t *>(p + (oa + d_ab));
        if constexpr (N1 > 1) {
            const uint32_t oc = oa + d_ac;
#pragma unroll
            for (int k = 0; k < N1 - 1; ++k) w[2 * N4 + N2 + k] = *reinterpret_cast<const unsigned short *>(p + oc + 32 * k);
        }
        if constexpr (N1 > 0) w[2 * N4 + N2 + N1 - 1] = *reinterpret_cast<const unsigned short *>(p + (oa + d_al));
    };
    auto gather8 = [&](const Ids &ids, uint32_t (&raw)[8][RWE]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            gather(ids.lo[j], raw[j]);
            gather(ids.hi[j], raw[4 + j]);
        }
    };
    // operands of one step: g[T] = 4 registers, pair m holds (entry 2m in the low half, entry 2m+1 in the high half)
    constexpr uint32_t kLoLo = 0x05040100u, kHiHi = 0x07060302u;
    auto pack = [&](const uint32_t (&raw)[8][RWE], v4u (&g)[NT]) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t (&e0)[RWE] = raw[2 * m];
            const uint32_t (&e1)[RWE] = raw[2 * m + 1];
#pragma unroll
            for (int q = 0; q < N4; ++q) {
                g[4 * q][m] = __builtin_amdgcn_perm(e1[2 * q], e0[2 * q], kLoLo);
                g[4 * q + 1][m] = __builtin_amdgcn_perm(e1[2 * q], e0[2 * q], kHiHi);
                g[4 * q + 2][m] = __builtin_amdgcn_perm(e1[2 * q + 1], e0[2 * q + 1], kLoLo);
                g[4 * q + 3][m] = __builtin_amdgcn_perm(e1[2 * q + 1], e0[2 * q + 1], kHiHi);
            }
            if constexpr (N2 > 0) {
                g[4 * N4][m] = __builtin_amdgcn_perm(e1[2 * N4], e0[2 * N4], kLoLo);
                g[4 * N4 + 1][m] = __builtin_amdgcn_perm(e1[2 * N4], e0[2 * N4], kHiHi);
            }
#pragma unroll
            for (int k = 0; k < N1; ++k)
                g[4 * N4 + 2 * N2 + k][m] = __builtin_amdgcn_perm(e1[2 * N4 + N2 + k], e0[2 * N4 + N2 + k], kLoLo);
        }
    };

    const bool is_r0 = i == RI, is_r1 = i == RI + 1, is_r2 = i == RI + 2, is_feat = i < RI;
    v4f bt[BX ? NT : 1];   // BX: rows 0..2 of these tiles are the three parts of b_u
#pragma unroll
    for (int T = 0; T < (BX ? NT : 1); ++T) bt[T] = (v4f){0.f, 0.f, 0.f, 0.f};
    // operands of step t from the gathered rows and ratings; gw (implicit mode): the three parts of w * theta
    auto operands = [&](const uint32_t (&raw)[8][RWE], float (&r)[8], int t, v4u (&g)[NT], v4u &gr,
                        v4u (&gw)[IMP ? 3 : 1][IMP ? NT : 1]) {
        pack(raw, g);
        float wv[8];
        if constexpr (IMP) {   // the rating becomes the weight of b_u, c = 1 + w for r > 0 (0 beyond the work item: r = 0)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                wv[j] = alpha * fmaxf(r[j], 0.f);
                r[j] = r[j] > 0.f ? 1.f + wv[j] : 0.f;
            }
        }
        // the rating lanes: of the last tile, or of the extra operand
        gr = (v4u){0u, 0u, 0u, 0u};
        uint32_t rp[4] = {0u, 0u, 0u, 0u};
        if constexpr (WANT_B) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t p0 = split16<ET>(r[2 * m], r[2 * m + 1]);
                const uint32_t p1 = split16<ET>(r[2 * m], r[2 * m + 1]);
                const uint32_t p2 = split16<ET>(r[2 * m], r[2 * m + 1]);
                rp[m] = is_r0 ? p0 : (is_r1 ? p1 : (is_r2 ? p2 : 0u));
                if constexpr (BX) gr[m] = rp[m];
            }
        }
        if constexpr (!BX) {   // (implicit mode: the columns of the padding stay zero, the rating lanes are rows only)
#pragma unroll
            for (int m = 0; m < 4; ++m) g[NT - 1][m] = is_feat ? g[NT - 1][m] : (IMP ? 0u : rp[m]);
        }
        if (t == nsteps - 1) {   // the last step may hold fewer than 32 entries: zero the others
            const int e0 = 32 * t + 8 * kq;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t mask = ((e0 + 2 * m < len) ? 0x0000ffffu : 0u) | ((e0 + 2 * m + 1 < len) ? 0xffff0000u : 0u);
#pragma unroll
                for (int T = 0; T < NT; ++T) g[T][m] &= mask;
            }
        }
        if constexpr (IMP) {
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int T = 0; T < NT; ++T) {
                    float x0 = widen_lo<ET>(g[T][m]) * wv[2 * m], x1 = widen_hi<ET>(g[T][m]) * wv[2 * m + 1];
                    const uint32_t q0 = split16<ET>(x0, x1);
                    const uint32_t q1 = split16<ET>(x0, x1);
                    const uint32_t q2 = split16<ET>(x0, x1);
                    const bool keep = BX || T < NT - 1 || is_feat;
                    gw[0][T][m] = keep ? q0 : rp[m];   // rows f .. f+2 of the last tile row: the parts of c
                    gw[1][T][m] = keep ? q1 : 0u;
                    gw[2][T][m] = keep ? q2 : 0u;
                }
        }
    };
    auto multiply = [&](const v4u (&g)[NT], const v4u &gr, const v4u (&gw)[IMP ? 3 : 1][IMP ? NT : 1]) {
        if constexpr (BX && WANT_B) {
#pragma unroll
            for (int C = 0; C < NT; ++C)
                if ((ROWS >> C) & 1u) mfma_16x16x32<ET>(bt[C], gr, g[C]);
        }
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    if constexpr (IMP) {
#pragma unroll
                        for (int k = 2; k >= 0; --k) mfma_16x16x32<ET>(acc[tiles_below(ROWS, R) + C], gw[k][R], g[C]);
                    } else {
                        mfma_16x16x32<ET>(acc[tiles_below(ROWS, R) + C], g[R], g[C]);
                    }
                }
            }
    };

    // One set of row registers: the rows of step t are repacked into operands as soon as they have arrived,
    // the gathers of step t+1 are issued into the same registers and are in flight during the MFMAs of step t;
    // the column ids run one step further ahead.
    uint32_t raw[8][RWE];
    float rat[8];
    Ids ids = load_ids(0);
    gather8(ids, raw);
    load_ratings(0, rat);
    ids = load_ids(1);
    for (int t = 0; t < nsteps; ++t) {
        v4u g[NT], gr, gw[IMP ? 3 : 1][IMP ? NT : 1];
        operands(raw, rat, t, g, gr, gw);
        if (t + 1 < nsteps) {
            gather8(ids, raw);
            load_ratings(t + 1, rat);
            ids = load_ids(t + 2);   // (beyond the end: zeros, never used)
        }
        multiply(g, gr, gw);
    }

    // b_u = rows RI .. RI+2 of the last tile row (or rows 0 .. 2 of the extra tiles), then zero the padding
    const int c = i, g4 = kq;
    if constexpr (WANT_B) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const int row = RI + k;   // row of the tile (compile-time after unrolling): lane row row/4, register row%4
                s += bperm(4 * (16 * (row / 4) + c), BX ? bt[T][row % 4] : acc[LB + T][row % 4]);
            }
            b[T] = (((ROWS >> T) & 1u) && (BX || T < NT - 1 || c < RI)) ? s : 0.f;
        }
    }
    if constexpr (!BX) {
#pragma unroll
        for (int T = 0; T < NT; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool keep = (4 * g4 + r < RI) && (T < NT - 1 || c < RI);
                acc[LB + T][r] = keep ? acc[LB + T][r] : 0.f;
            }
    }
}

}  // namespace als

namespace als {

// The same for a system shared by the NW wavefronts of a workgroup (f = 256, tile rows ROWS per wavefront):
// instead of every wavefront gathering every row, the rows of a step are gathered once -- wavefront w fetches
// entries 4w .. 4w+3 of the 32 -- repacked, and put into LDS in the operand layout, from where every wavefront
// reads the operand registers of the tiles it needs (16 bytes per lane and tile, conflict-free).  Two staging
// buffers in turn, one barrier per step.  Every wavefront of the workgroup must call, with the same s0 and len.
//   stage: 2 * tiles_1d(F) * 256 words of LDS.
// Producer lane (i, kq): entry pair p = kq % 2 of the wavefront's four entries, feature half kq / 2 (tiles
// 8*(kq/2) .. +7, the usual lane -> feature map), so that both entries of an operand word are in one lane.
template <int F, int NW, bool WIDE, int ET, bool WANT_B, uint32_t ROWS>
__device__ __forceinline__ void accumulate_tiles16_shared(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                          const void *__restrict__ Theta, int64_t s0, int len,
                                                          v4f (&acc)[tiles_in(ROWS)], float (&b)[tiles_1d(F)],
                                                          uint32_t *stage, int wave) {
    static_assert(ET == ALS_BF16 || ET == ALS_F16);
    static_assert(F == 256 && NW == 8, "16 tiles, four 8-byte loads per row and lane pair, 8 wavefronts x 4 entries");
    constexpr int NT = tiles_1d(F);
    constexpr int RMAX = 31 - __builtin_clz(ROWS);
    constexpr int STAGE = NT * 256;   // words per staging buffer
    const int lane = threadIdx.x & 63, i = lane & 15, kq = lane >> 4;
    const int p = kq & 1, hf = kq >> 1;
    const int32_t *__restrict__ ib = idx + s0;
    const float *__restrict__ vb = val + s0;
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t ids_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ib), 0, 4 * len, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vb), 0, 4 * len, kRsrcFlags);
    const int nsteps = (len + 31) >> 5;
    const int e_in_step = 4 * wave + 2 * p;                 // first of this lane's two entries inside a step
    const uint32_t id_off = 4u * (uint32_t)e_in_step;
    const uint32_t lane_a = 8u * (uint32_t)i + 256u * (uint32_t)hf;   // bytes into the row: tiles 8hf .. 8hf+7
    // word of (tile T, this lane's pair) in a staging buffer: lane (i, kq') of the consumers, register m
    const int P = 2 * wave + p;
    const int w_base = (16 * (P >> 2) + i) * 4 + (P & 3);

    struct Pair { uint32_t a, b; };
    auto load_pair_ids = [&](int t) -> Pair {
        Pair r;
        r.a = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(ids_rsrc, id_off + 128u * (uint32_t)t, 0, 0);
        r.b = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(ids_rsrc, id_off + 4u + 128u * (uint32_t)t, 0, 0);
        return r;
    };
    auto gather = [&](uint32_t c, uint32_t (&w)[4]) {   // 8 features of one row: two 8-byte loads
        const char *q;
        uint32_t o;
        if constexpr (WIDE) {
            q = reinterpret_cast<const char *>(Theta) + (int64_t)c * (2 * F);
            o = lane_a;
        } else {
            q = reinterpret_cast<const char *>(Theta);
            o = row_offset<(uint32_t)(2 * F)>(c, lane_a);
        }
        const uint2 v0 = *reinterpret_cast<const uint2 *>(q + o);
        const uint2 v1 = *reinterpret_cast<const uint2 *>(q + o + 128);
        w[0] = v0.x; w[1] = v0.y; w[2] = v1.x; w[3] = v1.y;
    };
    constexpr uint32_t kLoLo = 0x05040100u, kHiHi = 0x07060302u;
    // rows of step t (raw registers e0, e1) -> staging buffer; entries beyond the work item become zeros
    auto stage_rows = [&](const uint32_t (&e0)[4], const uint32_t (&e1)[4], int t, uint32_t *buf) {
        const int e = 32 * t + e_in_step;
        const uint32_t mask = ((e < len) ? 0x0000ffffu : 0u) | ((e + 1 < len) ? 0xffff0000u : 0u);
#pragma unroll
        for (int k = 0; k < 4; ++k) {   // register k holds the features of tiles 8hf + 2k (low half) and 8hf + 2k + 1 (high)
            const uint32_t lo = __builtin_amdgcn_perm(e1[k], e0[k], kLoLo) & mask;
            const uint32_t hi = __builtin_amdgcn_perm(e1[k], e0[k], kHiHi) & mask;
            buf[(8 * hf + 2 * k) * 256 + w_base] = lo;
            buf[(8 * hf + 2 * k + 1) * 256 + w_base] = hi;
        }
    };
    auto load_ratings = [&](int t, float (&r)[8]) {
        const uint32_t o = 32u * (uint32_t)kq + 128u * (uint32_t)t;
        const v4u a = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o, 0, 0));
        const v4u c = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o + 16u, 0, 0));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r[j] = bits_to_float(a[j]);
            r[4 + j] = bits_to_float(c[j]);
        }
    };

    v4f bt[NT];   // rows 0..2 of these tiles are the three parts of b_u (tile rows of ROWS only)
#pragma unroll
    for (int T = 0; T < NT; ++T) bt[T] = (v4f){0.f, 0.f, 0.f, 0.f};
    const bool is_r0 = i == 0, is_r1 = i == 1, is_r2 = i == 2;

    // Gathers run PD steps ahead of their use (a step's rows are 8 registers per lane here, and with one workgroup
    // per CU nothing else hides the memory latency); the column ids one step further.
    constexpr int PD = 4;
    uint32_t raw[PD][2][4];
    float rat[8];
    Pair ids;
    auto fetch = [&](auto slot, int step) {   // ids must hold the column ids of `step`
        gather(ids.a, raw[decltype(slot)::value][0]);
        gather(ids.b, raw[decltype(slot)::value][1]);
        (void)step;
    };
    [&]<int... u>(std::integer_sequence<int, u...>) {
        ((u < nsteps ? (ids = load_pair_ids(u), fetch(std::integral_constant<int, u>{}, u)) : void()), ...);
    }(std::make_integer_sequence<int, PD>{});
    stage_rows(raw[0][0], raw[0][1], 0, stage);
    if (PD < nsteps) {
        ids = load_pair_ids(PD);
        fetch(std::integral_constant<int, 0>{}, PD);
    }
    ids = load_pair_ids(PD + 1);   // (beyond the end: zeros, never used)
    if constexpr (WANT_B) load_ratings(0, rat);
    __syncthreads();
    auto step = [&](auto utag, int t) {
        constexpr int U = decltype(utag)::value;     // t % PD
        constexpr int S = (U + 1) % PD;              // register set of step t+1, reused for step t+1+PD
        const uint32_t *cur = stage + (t & 1) * STAGE;
        v4u g[RMAX + 1];
#pragma unroll
        for (int T = 0; T <= RMAX; ++T) g[T] = *reinterpret_cast<const v4u *>(cur + T * 256 + 4 * lane);
        v4u gr = (v4u){0u, 0u, 0u, 0u};
        if constexpr (WANT_B) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t p0 = split16<ET>(rat[2 * m], rat[2 * m + 1]);
                const uint32_t p1 = split16<ET>(rat[2 * m], rat[2 * m + 1]);
                const uint32_t p2 = split16<ET>(rat[2 * m], rat[2 * m + 1]);
                gr[m] = is_r0 ? p0 : (is_r1 ? p1 : (is_r2 ? p2 : 0u));
            }
        }
        if (t + 1 < nsteps) {   // rows of the next step into the other buffer, then its registers take new gathers
            stage_rows(raw[S][0], raw[S][1], t + 1, stage + ((t + 1) & 1) * STAGE);
            if constexpr (WANT_B) load_ratings(t + 1, rat);
            if (t + 1 + PD < nsteps) fetch(std::integral_constant<int, S>{}, t + 1 + PD);
            ids = load_pair_ids(t + 2 + PD);
        }
        if constexpr (WANT_B) {
#pragma unroll
            for (int C = 0; C < NT; ++C)
                if ((ROWS >> C) & 1u) mfma_16x16x32<ET>(bt[C], gr, g[C]);
        }
#pragma unroll
        for (int R = 0; R < NT; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) mfma_16x16x32<ET>(acc[tiles_below(ROWS, R) + C], g[R], g[C]);
            }
        __syncthreads();   // the next buffer is complete; everybody is done reading this one
    };
    for (int t0 = 0; t0 < nsteps; t0 += PD) {
        [&]<int... u>(std::integer_sequence<int, u...>) {
            ((t0 + u < nsteps ? step(std::integral_constant<int, u>{}, t0 + u) : void()), ...);
        }(std::make_integer_sequence<int, PD>{});
    }
    if constexpr (WANT_B) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            float s = 0.f;
            if ((ROWS >> T) & 1u) {
#pragma unroll
                for (int k = 0; k < 3; ++k) s += bperm(4 * i, bt[T][k]);   // rows 0..2: lane row 0, registers 0..2
            }
            b[T] = s;
        }
    }
}

}  // namespace als
