// get_hermitian + get_bias (Section 2 step (i), Section 3) for fp32 factor matrices on the 16-bit matrix cores:
// every gathered fp32 value x is cut into three bf16 parts by truncation, x = h + m + l EXACTLY (8 + 8 + 8
// significant bits), and a product x*y is formed as the six bf16 products
//     h*h' + h*m' + m*h' + m*m' + h*l' + l*h'
// on v_mfma_f32_16x16x32_bf16 with fp32 accumulation.  Each of them is exact in fp32; what is left out
// (m*l' + l*m' + l*l') is below 2^-23 |x*y|, the size of one fp32 rounding.  Six 16-bit MFMAs per tile and 32
// entries stand against eight fp32 MFMAs (16x16x4) that take twice as long each.
//
// Layout as in tiles16.h: one step consumes 32 stored entries, lane (i, kq) supplies its feature of the 8 entries
// 8kq .. 8kq+7, packed in pairs; the three parts of a value sit at the same place of three operand registers.
// Rows are gathered entry by entry as fp32 with the lane -> feature map and load widths of the fp32 path.
//
// b_u: when f is not a multiple of 16 the lane i = f % 16 of the last tile carries the fp32 rating instead of a
// feature and is cut into parts like everything else, so row f of the accumulated matrix is b_u to the same
// accuracy; the lanes beyond it carry zeros.  When f is a multiple of 16 the three parts of the rating form an
// operand of their own (lanes 0..2) that is multiplied with all three parts of every tile column: 3 NT more MFMAs
// per step, whose rows 0..2 add up to b_u.
#pragma once
#include "tiles16.h"

namespace als {

// Same contract as accumulate_tiles16 for ET = fp32 rows in memory.
template <int F, bool WIDE, bool WANT_B, uint32_t ROWS = rows_all(F)>
__device__ __forceinline__ void accumulate_tiles_x3(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                    const void *__restrict__ Theta, int64_t s0, int len,
                                                    v4f (&acc)[tiles_in(ROWS)], float (&b)[tiles_1d(F)]) {
    static_assert(ROWS == rows_all(F) || (F % 16) == 0, "partial sets of tile rows need f to be a multiple of 16");
    constexpr int NT = tiles_1d(F), RI = F % 16;
    constexpr bool BX = RI == 0;   // the rating parts are an operand of their own
    constexpr int N4 = loads16(F), N2 = loads8(F), N1 = loads4(F);
    constexpr int base1 = 64 * N4 + 32 * N2;
    constexpr int LB = (NT - 1) * NT / 2;
    const int lane = threadIdx.x & 63, i = lane & 15, kq = lane >> 4;
    const int32_t *__restrict__ ib = idx + s0;
    const float *__restrict__ vb = val + s0;
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t ids_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ib), 0, 4 * len, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vb), 0, 4 * len, kRsrcFlags);
    const int nsteps = (len + 31) >> 5;
    // lane offsets of the three kinds of loads inside a row (bytes)
    const uint32_t lane_a = 16u * (uint32_t)i;
    const uint32_t lane_b = 256u * N4 + 8u * (uint32_t)i;
    const uint32_t lane_c = 4u * (uint32_t)(base1 + i);
    const uint32_t lane_l = 4u * (uint32_t)((base1 + 16 * (N1 - 1) + i < F) ? base1 + 16 * (N1 - 1) + i : F - 1);
    const uint32_t lane_first = N4 > 0 ? lane_a : N2 > 0 ? lane_b : N1 > 1 ? lane_c : lane_l;
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
        if constexpr (!WANT_B) return;
        const uint32_t o = eoff0 + 128u * (uint32_t)t;
        const v4u a = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o, 0, 0));
        const v4u c = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(val_rsrc, o + 16u, 0, 0));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            r[j] = bits_to_float(a[j]);
            r[4 + j] = bits_to_float(c[j]);
        }
    };
    // The loads of one gathered fp32 row come in three groups -- 16 bytes per lane (tiles 0 .. 4 N4 - 1), 8 bytes (the
    // next 2 N2 tiles), 4 bytes (the last N1 tiles) -- and a group of the next step is issued as soon as the last
    // tile it fills has been cut into parts.  (Entries beyond the work item read row 0 and are masked later.)
    constexpr int first1 = 4 * N4 + 2 * N2;
    constexpr int endA = N4 > 0 ? 4 * N4 - 1 : -1, endB = N2 > 0 ? first1 - 1 : -1, endC = N1 > 0 ? NT - 1 : -1;
    auto row_base = [&](uint32_t c, const char *&p, uint32_t &ro) {
        if constexpr (WIDE) {
            p = reinterpret_cast<const char *>(Theta) + (int64_t)c * (4 * F);
            ro = lane_first;
        } else {
            p = reinterpret_cast<const char *>(Theta);
            ro = row_offset<(uint32_t)(4 * F)>(c, lane_first);
        }
    };
    auto gather_group = [&](auto gtag, uint32_t c, uint32_t (&w)[NT]) {
        constexpr int G = decltype(gtag)::value;
        const char *p;
        uint32_t ro;
        row_base(c, p, ro);
        if constexpr (G == 0 && N4 > 0) {
            const uint32_t o = ro + (lane_a - lane_first);
#pragma unroll
            for (int q = 0; q < N4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4 *>(p + o + 256 * q);
                w[4 * q] = v.x; w[4 * q + 1] = v.y; w[4 * q + 2] = v.z; w[4 * q + 3] = v.w;
            }
        }
        if constexpr (G == 1 && N2 > 0) {
            const uint2 v = *reinterpret_cast<const uint2 *>(p + (ro + (lane_b - lane_first)));
            w[4 * N4] = v.x; w[4 * N4 + 1] = v.y;
        }
        if constexpr (G == 2 && N1 > 0) {
            if constexpr (N1 > 1) {
                const uint32_t o = ro + (lane_c - lane_first);
#pragma unroll
                for (int k = 0; k < N1 - 1; ++k) w[first1 + k] = *reinterpret_cast<const uint32_t *>(p + o + 64 * k);
            }
            w[first1 + N1 - 1] = *reinterpret_cast<const uint32_t *>(p + (ro + (lane_l - lane_first)));
        }
    };
    auto gather8_group = [&](auto gtag, const Ids &ids, uint32_t (&raw)[8][NT]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            gather_group(gtag, ids.lo[j], raw[j]);
            gather_group(gtag, ids.hi[j], raw[4 + j]);
        }
    };
    using G0 = std::integral_constant<int, 0>;
    using G1 = std::integral_constant<int, 1>;
    using G2 = std::integral_constant<int, 2>;

    const bool is_rating = i == RI, is_feat = i < RI;
    const bool is_r0 = i == 0, is_r1 = i == 1, is_r2 = i == 2;
    v4f bt[BX ? NT : 1];   // BX: rows 0..2 of these tiles are the three parts of b_u
#pragma unroll
    for (int T = 0; T < (BX ? NT : 1); ++T) bt[T] = (v4f){0.f, 0.f, 0.f, 0.f};

    // the last step may hold fewer than 32 entries: the others count as zero (a wave-uniform branch)
    auto mask_tail = [&](uint32_t (&raw)[8][NT], float (&r)[8], int t) {
        const int e0 = 32 * t + 8 * kq;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool ok = e0 + e < len;
#pragma unroll
            for (int T = 0; T < NT; ++T) raw[e][T] = ok ? raw[e][T] : 0u;
            r[e] = ok ? r[e] : 0.f;
        }
    };
    // operands of one tile: the leading (h), middle (m) and trailing (l) bf16 parts of the lane's 8 entries
    auto split_tile = [&](auto ttag, const uint32_t (&raw)[8][NT], const float (&r)[8], v4u &h, v4u &m, v4u &l) {
        constexpr int T = decltype(ttag)::value;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            float x0 = bits_to_float(raw[2 * pr][T]), x1 = bits_to_float(raw[2 * pr + 1][T]);
            if constexpr (!BX && T == NT - 1) {   // the rating lane and the zero lanes of the last tile
                x0 = is_feat ? x0 : ((WANT_B && is_rating) ? r[2 * pr] : 0.f);
                x1 = is_feat ? x1 : ((WANT_B && is_rating) ? r[2 * pr + 1] : 0.f);
            }
            h[pr] = split16<ALS_BF16>(x0, x1);
            m[pr] = split16<ALS_BF16>(x0, x1);
            l[pr] = split16<ALS_BF16>(x0, x1);
        }
    };
    auto rating_operand = [&](const float (&r)[8], v4u &gr) {
        gr = (v4u){0u, 0u, 0u, 0u};
        if constexpr (BX && WANT_B) {
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                float r0 = r[2 * pr], r1 = r[2 * pr + 1];
                const uint32_t p0 = split16<ALS_BF16>(r0, r1);
                const uint32_t p1 = split16<ALS_BF16>(r0, r1);
                const uint32_t p2 = split16<ALS_BF16>(r0, r1);
                gr[pr] = is_r0 ? p0 : (is_r1 ? p1 : (is_r2 ? p2 : 0u));
            }
        }
    };

    // One step, tile row by tile row: the MFMAs of tile row T (six per tile, 16 matrix-pipeline cycles each) need the
    // parts of the tiles 0 .. T only, so the vector-ALU work that cuts tile T+1 into parts is placed among them and
    // runs in their shadow; only tile 0 is cut with the matrix pipeline idle.  The scheduling barriers keep the
    // compiler from collecting the vector-ALU work of a step in front of its MFMAs.
    uint32_t raw[8][NT];
    float rat[8];
    Ids ids = load_ids(0);
    gather8_group(G0{}, ids, raw);
    gather8_group(G1{}, ids, raw);
    gather8_group(G2{}, ids, raw);
    load_ratings(0, rat);
    ids = load_ids(1);
    for (int t = 0; t < nsteps; ++t) {
        v4u h[NT], m[NT], l[NT], gr;
        if (t == nsteps - 1) mask_tail(raw, rat, t);
        rating_operand(rat, gr);
        split_tile(std::integral_constant<int, 0>{}, raw, rat, h[0], m[0], l[0]);
        [&]<int... T>(std::integer_sequence<int, T...>) {
            ([&] {
                __builtin_amdgcn_sched_barrier(0);
                if constexpr ((ROWS >> T) & 1u) {
#pragma unroll
                    for (int C = 0; C <= T; ++C) {
                        v4f &a = acc[tiles_below(ROWS, T) + C];
                        mfma_16x16x32<ALS_BF16>(a, h[T], l[C]);
                        mfma_16x16x32<ALS_BF16>(a, l[T], h[C]);
                        mfma_16x16x32<ALS_BF16>(a, m[T], m[C]);
                        mfma_16x16x32<ALS_BF16>(a, h[T], m[C]);
                        mfma_16x16x32<ALS_BF16>(a, m[T], h[C]);
                        mfma_16x16x32<ALS_BF16>(a, h[T], h[C]);
                    }
                    if constexpr (BX && WANT_B) {
                        mfma_16x16x32<ALS_BF16>(bt[T], gr, l[T]);
                        mfma_16x16x32<ALS_BF16>(bt[T], gr, m[T]);
                        mfma_16x16x32<ALS_BF16>(bt[T], gr, h[T]);
                    }
                }
                if constexpr (T + 1 < NT) split_tile(std::integral_constant<int, T + 1>{}, raw, rat, h[T + 1], m[T + 1], l[T + 1]);
                // rows of the next step: a group of loads goes out once the last tile it fills is in parts (tile T+1
                // has just been cut; tile 0 was cut before the first tile row)
                constexpr auto due = [](int end_tile, int T_) { return (end_tile == T_ + 1 && T_ + 1 < NT) || (end_tile == 0 && T_ == 0); };
                if constexpr (due(endA, T)) gather8_group(G0{}, ids, raw);
                if constexpr (due(endB, T)) gather8_group(G1{}, ids, raw);
                if constexpr (due(endC, T)) gather8_group(G2{}, ids, raw);
                // the ratings are last used by the rating operand (at the start of the step) or by the last tile
                if constexpr (BX ? T == 0 : T == NT - 1) load_ratings(t + 1, rat);
                if constexpr (T == NT - 1) ids = load_ids(t + 2);   // (beyond the end: zeros, never used)
            }(), ...);
        }(std::make_integer_sequence<int, NT>{});
        __builtin_amdgcn_sched_barrier(0);
    }

    // b_u = row RI of the last tile row (or rows 0 .. 2 of the extra tiles), then zero the padding
    const int c = i, g4 = kq;
    if constexpr (WANT_B) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            float s = 0.f;
            if constexpr (BX) {
#pragma unroll
                for (int k = 0; k < 3; ++k) s += bperm(4 * c, bt[T][k]);   // rows 0..2: lane row 0, registers 0..2
            } else {
                s = bperm(4 * (16 * (RI / 4) + c), acc[LB + T][RI % 4]);   // row RI: lane row RI/4, register RI%4
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
