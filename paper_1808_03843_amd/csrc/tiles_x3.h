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
// Measured (Mid shape, f = 100): the slot kernel issues 1.3 PFLOP/s of bf16 MFMA work, 94 % of what this chip
// sustains on back-to-back bf16 MFMAs (it lowers its clock under that load), i.e. 135-155 TFLOP/s of Gram work.
//
// b_u: when f is not a multiple of 16 the lane i = f % 16 of the last tile carries the fp32 rating instead of a
// feature and is cut into parts like everything else, so row f of the accumulated matrix is b_u to the same
// accuracy; the lanes beyond it carry zeros.  When f is a multiple of 16 the three parts of the rating form an
// operand of their own (lanes 0..2) that is multiplied with all three parts of every tile column: 3 NT more MFMAs
// per step, whose rows 0..2 add up to b_u.
//
// The gathered rows are staged through LDS (Section 3: the rows of Theta that a row of R refers to are staged on
// chip in batches; here the staging buffer is a per-wavefront FIFO).
// Why: the operands of a step (three parts of 32 entries: 84 registers at f = 100) and the 112 accumulator registers
// leave no room for the 56 registers of the next step's rows in flight if two wavefronts are to share a SIMD -- and
// with one wavefront per SIMD nothing hides the memory latency or the vector-ALU work of cutting the values into
// parts.  So the rows of the next step travel by direct global-to-LDS loads (no destination registers), and are read
// back, 8 registers at a time, just before they are cut.  Every lane reads back exactly what it loaded: the buffer
// is laid out load instruction by load instruction, lane by lane (bank-conflict free both ways).
//
// The buffer of one wavefront holds the rows of one step, in three regions that follow the three kinds of loads of a
// row (16 bytes per lane for tiles 0 .. 4 N4 - 1; two 4-byte loads for the next 2 N2 tiles; 4 bytes for the last N1
// tiles).  A region is refilled for step t+1 as soon as step t has read it.
#pragma once
#include "tiles16.h"

namespace als {

constexpr int x3_fifo_words(int F) { return 8 * 64 * (4 * loads16(F) + 2 * loads8(F) + loads4(F)); }

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// PARTS = 2 (factor_dtype = ALS_F32X2): the value is cut into two fp16 parts instead, h = fp16(s x) and
// l = fp16(s x - h), both rounded to nearest, so |s x - (h + l)| <= 2^-22 |s x|; a product is the three fp16 products
//     h*h' + h*l' + l*h'      (what is dropped, l*l', is below 2^-22 |x*y|)
// on v_mfma_f32_16x16x32_f16: half the matrix-core work and well under half the cutting work of the three-part route,
// at a representation error of the size of fp32 accumulation rounding instead of none.  fp16 has a narrow exponent
// range, so the factor is scaled by a power of two s with 2^14 <= s * max|Theta| < 2^15 (absmax_bits: the bits of
// max |Theta|, found by a reduction before the launch); the sums are scaled back exactly at the end.  The rating is
// not scaled: |r_uv| must stay below 65504, and a rating that is no fp16 number carries an absolute error of up to
// 2^-25 beside the relative 2^-22.
//
// Every wavefront of the kernel must call with its own fifo (x3_fifo_words(F) words, 16-byte aligned).
template <int F, bool WIDE, bool WANT_B, uint32_t ROWS = rows_all(F), int PARTS = 3>
__device__ __forceinline__ void accumulate_tiles_x3(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                        const void *__restrict__ Theta, int64_t s0, int len,
                                                        v4f (&acc)[tiles_in(ROWS)], float (&b)[tiles_1d(F)],
                                                        uint32_t *fifo, uint32_t absmax_bits = 0u) {
    static_assert(ROWS == rows_all(F) || (F % 16) == 0, "partial sets of tile rows need f to be a multiple of 16");
    static_assert(PARTS == 2 || PARTS == 3, "two fp16 parts or three bf16 parts");
    constexpr int PT = PARTS == 3 ? ALS_BF16 : ALS_F16;   // element type of the parts
    // the power-of-two scale of the two-part route (uniform: scalar registers)
    float scale = 1.f, inv_scale = 1.f;
    if constexpr (PARTS == 2) {
        const uint32_t e = (absmax_bits >> 23) & 0xffu;
        uint32_t se = (e == 0u || e == 255u) ? 127u : 268u - e;   // s * max in [2^14, 2^15)
        se = se > 187u ? 187u : se;                               // (a factor of all-tiny values: s stays at 2^60)
        scale = bits_to_float(se << 23);
        inv_scale = bits_to_float((254u - se) << 23);
    }
    constexpr int NT = tiles_1d(F), RI = F % 16;
    constexpr bool BX = RI == 0;   // the rating parts are an operand of their own
    constexpr int N4 = loads16(F), N2 = loads8(F), N1 = loads4(F);
    constexpr int base1 = 64 * N4 + 32 * N2, first1 = 4 * N4 + 2 * N2;
    constexpr int LB = (NT - 1) * NT / 2;
    constexpr int baseA = 0, baseB = 8 * N4 * 256, baseC = baseB + 8 * N2 * 128;   // word offsets of the regions
    const int lane = threadIdx.x & 63, i = lane & 15, kq = lane >> 4;
    const int32_t *__restrict__ ib = idx + s0;
    const float *__restrict__ vb = val + s0;
    constexpr int kRsrcFlags = 0x00020000;
    const __amdgpu_buffer_rsrc_t ids_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ib), 0, 4 * len, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t val_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vb), 0, 4 * len, kRsrcFlags);
    const int nsteps = (len + 31) >> 5;
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
    auto row_base = [&](uint32_t c, const char *&p, uint32_t &ro) {
        if constexpr (WIDE) {
            p = reinterpret_cast<const char *>(Theta) + (int64_t)c * (4 * F);
            ro = lane_first;
        } else {
            p = reinterpret_cast<const char *>(Theta);
            ro = row_offset<(uint32_t)(4 * F)>(c, lane_first);
        }
    };
    // the loads of group G (0: 16-byte, 1: the 8-byte pair as two 4-byte loads, 2: 4-byte) of entry j, global -> LDS
    auto dma_group = [&](auto gtag, int j, uint32_t c) {
        constexpr int G = decltype(gtag)::value;
        const char *p;
        uint32_t ro;
        row_base(c, p, ro);
        if constexpr (G == 0 && N4 > 0) {
            const uint32_t o = ro + (lane_a - lane_first);
#pragma unroll
            for (int q = 0; q < N4; ++q)
                __builtin_amdgcn_global_load_lds((global_void *)(p + o + 256 * q), (lds_void *)(fifo + baseA + (j * N4 + q) * 256), 16, 0, 0);
        }
        if constexpr (G == 1 && N2 > 0) {
            const uint32_t o = ro + (lane_b - lane_first);
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                __builtin_amdgcn_global_load_lds((global_void *)(p + o + 4 * hh), (lds_void *)(fifo + baseB + (j * 2 + hh) * 64), 4, 0, 0);
        }
        if constexpr (G == 2 && N1 > 0) {
            if constexpr (N1 > 1) {
                const uint32_t o = ro + (lane_c - lane_first);
#pragma unroll
                for (int k = 0; k < N1 - 1; ++k)
                    __builtin_amdgcn_global_load_lds((global_void *)(p + o + 64 * k), (lds_void *)(fifo + baseC + (j * N1 + k) * 64), 4, 0, 0);
            }
            __builtin_amdgcn_global_load_lds((global_void *)(p + (ro + (lane_l - lane_first))),
                                             (lds_void *)(fifo + baseC + (j * N1 + N1 - 1) * 64), 4, 0, 0);
        }
    };
    auto dma8_group = [&](auto gtag, const Ids &ids) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dma_group(gtag, j, ids.lo[j]);
            dma_group(gtag, 4 + j, ids.hi[j]);
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

    typedef _Float16 v2h __attribute__((ext_vector_type(2)));
    typedef float v2f __attribute__((ext_vector_type(2)));
    auto round_pair = [](float a, float c) -> v2h { return __builtin_convertvector((v2f){a, c}, v2h); };   // to nearest
    v4u h[NT], m[PARTS == 3 ? NT : 1], l[NT], gr;
    // tile T, entry pair pr: the two fp32 values -> three packed part pairs.  ok0 / ok1: entry inside the work item
    auto cut = [&](auto ttag, int pr, float x0, float x1, const float (&r)[8], bool ok0, bool ok1, auto lasttag) {
        constexpr int T = decltype(ttag)::value;
        if constexpr (!BX && T == NT - 1) {   // the rating lane and the zero lanes of the last tile
            // (two parts: r / s here, so that the scaling below gives the rating back exactly; applied here and not
            // where the rating is loaded, which would make the load wait)
            const float rs0 = PARTS == 2 ? r[2 * pr] * inv_scale : r[2 * pr];
            const float rs1 = PARTS == 2 ? r[2 * pr + 1] * inv_scale : r[2 * pr + 1];
            x0 = is_feat ? x0 : ((WANT_B && is_rating) ? rs0 : 0.f);
            x1 = is_feat ? x1 : ((WANT_B && is_rating) ? rs1 : 0.f);
        }
        if constexpr (decltype(lasttag)::value) {
            x0 = ok0 ? x0 : 0.f;
            x1 = ok1 ? x1 : 0.f;
        }
        if constexpr (PARTS == 3) {
            h[T][pr] = split16<ALS_BF16>(x0, x1);
            m[T][pr] = split16<ALS_BF16>(x0, x1);
            l[T][pr] = split16<ALS_BF16>(x0, x1);
        } else {
            x0 *= scale;
            x1 *= scale;
            const v2h hh = round_pair(x0, x1);
            h[T][pr] = __builtin_bit_cast(uint32_t, hh);
            l[T][pr] = __builtin_bit_cast(uint32_t, round_pair(x0 - (float)hh.x, x1 - (float)hh.y));
        }
    };
    // reads a region back, one entry pair at a time, and cuts its tiles into parts
    auto read_group = [&](auto gtag, const float (&r)[8], int t, auto lasttag) {
        constexpr int G = decltype(gtag)::value;
        const int e0 = 32 * t + 8 * kq;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const bool ok0 = e0 + 2 * pr < len, ok1 = e0 + 2 * pr + 1 < len;
            if constexpr (G == 0 && N4 > 0) {
                [&]<int... q>(std::integer_sequence<int, q...>) {
                    ([&] {
                        const v4u v0 = *reinterpret_cast<const v4u *>(fifo + baseA + ((2 * pr) * N4 + q) * 256 + 4 * lane);
                        const v4u v1 = *reinterpret_cast<const v4u *>(fifo + baseA + ((2 * pr + 1) * N4 + q) * 256 + 4 * lane);
                        cut(std::integral_constant<int, 4 * q>{}, pr, bits_to_float(v0[0]), bits_to_float(v1[0]), r, ok0, ok1, lasttag);
                        cut(std::integral_constant<int, 4 * q + 1>{}, pr, bits_to_float(v0[1]), bits_to_float(v1[1]), r, ok0, ok1, lasttag);
                        cut(std::integral_constant<int, 4 * q + 2>{}, pr, bits_to_float(v0[2]), bits_to_float(v1[2]), r, ok0, ok1, lasttag);
                        cut(std::integral_constant<int, 4 * q + 3>{}, pr, bits_to_float(v0[3]), bits_to_float(v1[3]), r, ok0, ok1, lasttag);
                    }(), ...);
                }(std::make_integer_sequence<int, N4>{});
            }
            if constexpr (G == 1 && N2 > 0) {
                const uint32_t a0 = fifo[baseB + ((2 * pr) * 2 + 0) * 64 + lane], a1 = fifo[baseB + ((2 * pr) * 2 + 1) * 64 + lane];
                const uint32_t c0 = fifo[baseB + ((2 * pr + 1) * 2 + 0) * 64 + lane], c1 = fifo[baseB + ((2 * pr + 1) * 2 + 1) * 64 + lane];
                cut(std::integral_constant<int, 4 * N4>{}, pr, bits_to_float(a0), bits_to_float(c0), r, ok0, ok1, lasttag);
                cut(std::integral_constant<int, 4 * N4 + 1>{}, pr, bits_to_float(a1), bits_to_float(c1), r, ok0, ok1, lasttag);
            }
            if constexpr (G == 2 && N1 > 0) {
                [&]<int... k>(std::integer_sequence<int, k...>) {
                    ([&] {
                        const uint32_t a0 = fifo[baseC + ((2 * pr) * N1 + k) * 64 + lane];
                        const uint32_t c0 = fifo[baseC + ((2 * pr + 1) * N1 + k) * 64 + lane];
                        cut(std::integral_constant<int, first1 + k>{}, pr, bits_to_float(a0), bits_to_float(c0), r, ok0, ok1, lasttag);
                    }(), ...);
                }(std::make_integer_sequence<int, N1>{});
            }
        }
    };
    auto rating_operand = [&](const float (&r)[8]) {
        gr = (v4u){0u, 0u, 0u, 0u};
        if constexpr (BX && WANT_B) {
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                float r0 = r[2 * pr], r1 = r[2 * pr + 1];
                if constexpr (PARTS == 3) {
                    const uint32_t p0 = split16<ALS_BF16>(r0, r1);
                    const uint32_t p1 = split16<ALS_BF16>(r0, r1);
                    const uint32_t p2 = split16<ALS_BF16>(r0, r1);
                    gr[pr] = is_r0 ? p0 : (is_r1 ? p1 : (is_r2 ? p2 : 0u));
                } else {   // (the rating itself: this operand is not scaled)
                    const v2h hh = round_pair(r0, r1);
                    const uint32_t p0 = __builtin_bit_cast(uint32_t, hh);
                    const uint32_t p1 = __builtin_bit_cast(uint32_t, round_pair(r0 - (float)hh.x, r1 - (float)hh.y));
                    gr[pr] = is_r0 ? p0 : (is_r1 ? p1 : 0u);
                }
            }
        }
    };
    // the MFMAs of the tile rows [R0, R1): six per tile (three with two parts)
    auto rows_mfma = [&](auto r0tag, auto r1tag) {
        constexpr int R0 = decltype(r0tag)::value, R1 = decltype(r1tag)::value;
#pragma unroll
        for (int R = R0; R < R1; ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) {
                    v4f &a = acc[tiles_below(ROWS, R) + C];
                    mfma_16x16x32<PT>(a, h[R], l[C]);
                    mfma_16x16x32<PT>(a, l[R], h[C]);
                    if constexpr (PARTS == 3) {
                        mfma_16x16x32<PT>(a, m[R], m[C]);
                        mfma_16x16x32<PT>(a, h[R], m[C]);
                        mfma_16x16x32<PT>(a, m[R], h[C]);
                    }
                    mfma_16x16x32<PT>(a, h[R], h[C]);
                }
                if constexpr (BX && WANT_B) {
                    mfma_16x16x32<PT>(bt[R], gr, l[R]);
                    if constexpr (PARTS == 3) mfma_16x16x32<PT>(bt[R], gr, m[R]);
                    mfma_16x16x32<PT>(bt[R], gr, h[R]);
                }
            }
    };
    constexpr int endA = 4 * N4, endB = first1;   // first tile beyond group A / groups A and B
    using T0 = std::integral_constant<int, 0>;
    using TA = std::integral_constant<int, endA>;
    using TB = std::integral_constant<int, endB>;
    using TN = std::integral_constant<int, NT>;

    float rat[8];
    Ids ids = load_ids(0);
    dma8_group(G0{}, ids);
    dma8_group(G1{}, ids);
    dma8_group(G2{}, ids);
    load_ratings(0, rat);
    ids = load_ids(1);   // of the next step: the loads of step t+1 go out during step t
    // one step; LAST: the final step of the work item -- entries beyond its end count as zero, nothing is prefetched
    auto step = [&](auto lasttag, int t) {
        constexpr bool LAST = decltype(lasttag)::value;
        // everything this step reads from the buffer was issued a step ago
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        rating_operand(rat);
        // (a region is refilled only after its values have been read AND used: the scheduling barrier keeps the
        // loads that overwrite it behind the instructions that wait for the reads)
        read_group(G0{}, rat, t, lasttag);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (!LAST) dma8_group(G0{}, ids);
        rows_mfma(T0{}, TA{});
        read_group(G1{}, rat, t, lasttag);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (!LAST) dma8_group(G1{}, ids);
        rows_mfma(TA{}, TB{});
        read_group(G2{}, rat, t, lasttag);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (!LAST) {
            dma8_group(G2{}, ids);
            load_ratings(t + 1, rat);
            ids = load_ids(t + 2);   // (beyond the end: zeros -> row 0, read but never used)
        }
        __builtin_amdgcn_sched_barrier(0);
        rows_mfma(TB{}, TN{});
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int t = 0; t + 1 < nsteps; ++t) step(std::false_type{}, t);
    step(std::true_type{}, nsteps - 1);

    // b_u = row RI of the last tile row (or rows 0 .. 2 of the extra tiles), then zero the padding
    const int c = i, g4 = kq;
    if constexpr (WANT_B) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            float s = 0.f;
            if constexpr (BX) {
#pragma unroll
                for (int k = 0; k < PARTS; ++k) s += bperm(4 * c, bt[T][k]);   // rows 0..2: lane row 0, registers 0..2
            } else {
                s = bperm(4 * (16 * (RI / 4) + c), acc[LB + T][RI % 4]);   // row RI: lane row RI/4, register RI%4
            }
            if constexpr (PARTS == 2) s *= inv_scale;   // sum of r * (s theta)
            b[T] = (((ROWS >> T) & 1u) && (BX || T < NT - 1 || c < RI)) ? s : 0.f;
        }
    }
    if constexpr (PARTS == 2) {   // sums of (s theta)(s theta'): back to the caller's scale, exactly
        const float inv2 = inv_scale * inv_scale;
#pragma unroll
        for (int q = 0; q < tiles_in(ROWS); ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[q][r] *= inv2;
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
