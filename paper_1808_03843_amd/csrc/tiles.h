// Device code shared by the get_hermitian kernels: the gathered SYRK main loop on fp32 MFMA
// accumulator tiles, and Algorithm 1 (CGSolve) run by one wavefront directly on those tiles.
#pragma once
#include <type_traits>
#include <utility>

#include "als_internal.h"

namespace als {

typedef float v4f __attribute__((ext_vector_type(4)));

// The fp32 MFMAs below are inline asm: the compiler inserts none of the wait states that the hardware needs between
// a vector-ALU write and an MFMA read of the same register, or between an MFMA and a read of its result; the code
// keeps those distances by hand (mfma_settle, mfma_drain, the s_nop tied to operands).  ALS_DRAINED_MFMA builds a
// canary library in which every hand-written MFMA waits for its operands before it issues and for its result
// after: several times slower, but free of any hazard by construction.  A test compares the two libraries bit for bit.
#ifdef ALS_DRAINED_MFMA
#define ALS_MFMA_PRE "s_nop 7\n\ts_nop 7\n\t"
#define ALS_MFMA_POST "\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15"
#else
#define ALS_MFMA_PRE ""
#define ALS_MFMA_POST ""
#endif

// acc += a (16x4, one stored entry per 16 lanes) * b (4x16).  Written as an in-place instruction so
// that the accumulators stay where they are across the loop (the builtin form let the register
// allocator shuffle them through copies).  IN_VGPR picks architectural registers (needed when the
// tiles are read by vector ALU code afterwards) instead of accumulation registers.
template <bool IN_VGPR>
__device__ __forceinline__ void mfma_16x16x4(v4f &acc, float a, float b) {
    if constexpr (IN_VGPR)
        asm(ALS_MFMA_PRE "v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+v"(acc) : "v"(a), "v"(b));
    else
        asm(ALS_MFMA_PRE "v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+a"(acc) : "v"(a), "v"(b));
}

// acc (16 blocks of 4x4) += a (4x1 per block) * b (1x4 per block): block q = lanes 4q..4q+3, register r of
// lane 4q+j holds element (r, j) of block q.  Used for a last tile row that has only 4 feature rows: with
// the 16-lane operand layout above, block q = 4*kq + cg multiplies theta_{v(kq)}[4 feature rows] by
// theta_{v(kq)}[columns 4cg..4cg+3 of a tile], i.e. lane (i, kq) accumulates the part of rows 0..3 x
// column i that comes from the entries of lane row kq -- a quarter of the matrix-pipeline time of a full
// 16x16x4 tile.  The four lane rows are summed once, after the loop.
template <bool IN_VGPR>
__device__ __forceinline__ void mfma_4x4x1(v4f &acc, float a, float b) {
    if constexpr (IN_VGPR)
        asm(ALS_MFMA_PRE "v_mfma_f32_4x4x1_16b_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+v"(acc) : "v"(a), "v"(b));
    else
        asm(ALS_MFMA_PRE "v_mfma_f32_4x4x1_16b_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+a"(acc) : "v"(a), "v"(b));
}

// The MFMAs above are opaque to the compiler's hazard recogniser: leave the matrix pipeline time to
// retire the last accumulator writes before they are read (8 passes = 32 cycles, plus margin).
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory"); }
// The same wait at the end of a block of MFMAs that is followed by a control-flow edge (loop back edge or
// exit, end of a conditional step): the register copies the compiler places on such edges read the
// accumulators, and it cannot know that they are still being written.  16 wait states cover the 8 passes
// of the last 16x16x4 instruction.
// Every tile is an operand of the (otherwise empty) statements, so that none of the MFMAs, which the
// compiler may reorder, can be placed after the wait.
template <bool IN_VGPR, int N>
__device__ __forceinline__ void mfma_settle(v4f (&acc)[N]) {
    constexpr int G = 8;   // operands per statement (the limit is 30)
#pragma unroll
    for (int q = 0; q + G <= N; q += G) {
        if constexpr (IN_VGPR)
            asm volatile("" : "+v"(acc[q]), "+v"(acc[q + 1]), "+v"(acc[q + 2]), "+v"(acc[q + 3]), "+v"(acc[q + 4]),
                         "+v"(acc[q + 5]), "+v"(acc[q + 6]), "+v"(acc[q + 7]));
        else
            asm volatile("" : "+a"(acc[q]), "+a"(acc[q + 1]), "+a"(acc[q + 2]), "+a"(acc[q + 3]), "+a"(acc[q + 4]),
                         "+a"(acc[q + 5]), "+a"(acc[q + 6]), "+a"(acc[q + 7]));
    }
#pragma unroll
    for (int q = N - N % G; q < N; ++q) {
        if constexpr (IN_VGPR) asm volatile("" : "+v"(acc[q]));
        else asm volatile("" : "+a"(acc[q]));
    }
    asm volatile("s_nop 15" ::: "memory");
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

// m ? b : a per lane, m a 64-bit lane mask.  Written as the instruction: the optimiser turns chains of
// per-lane selects on values that come back from LDS permutes into divergent branches.
__device__ __forceinline__ float lane_select(float a, float b, uint64_t m) {
    float d;
    asm("v_cndmask_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "s"(m));
    return d;
}
// v[k] with k = 2*[lane in m1] + [lane in m0]
__device__ __forceinline__ float lane_select4(float v0, float v1, float v2, float v3, uint64_t m0, uint64_t m1) {
    return lane_select(lane_select(v0, v1, m0), lane_select(v2, v3, m0), m1);
}

// Sums of four registers over the 16 lanes of a DPP row, "transposed": lane c ends up with the sum of
// register c % 4 (b0, b1: bits 0 and 1 of c).  The first two levels halve the number
// of live registers instead of reducing each one separately: 11 instructions instead of 16 + 3 selects.
__device__ __forceinline__ float rowsum16_sel4(float r0, float r1, float r2, float r3, bool b0, bool b1) {
    // (plain selects, not the asm form: their results feed DPP instructions, and the wait states a DPP read
    // of a freshly written register needs are only inserted for instructions the compiler can see)
    // level 1, partner lane c ^ 1: even lanes keep r0 / r2, odd lanes r1 / r3
    const float s01 = (b0 ? r1 : r0) + dpp_mov<0xB1>(b0 ? r0 : r1);
    const float s23 = (b0 ? r3 : r2) + dpp_mov<0xB1>(b0 ? r2 : r3);
    // level 2, partner lane c ^ 2
    float t = (b1 ? s23 : s01) + dpp_mov<0x4E>(b1 ? s01 : s23);
    // the four quads of the row hold the same register at the same position: rotate by 4 and by 8
    t += dpp_mov<0x124>(t);   // row_ror:4
    t += dpp_mov<0x128>(t);   // row_ror:8
    return t;
}

// A_u (lower-triangle tiles) and b_u of the stored entries [s0, s0+len) of one row (len >= 1).
// Section 2 step (i): get_hermitian and get_bias.
//
// Lane l = (i = l%16, kq = l/16) supplies theta_{v(kq)}[16*tile + i] both as the A operand of tile
// row `tile` and as the B operand of tile column `tile`; one step consumes 4 stored entries.
//
// When F is not a multiple of 16 the last tile has spare lanes: lane i = F%16 carries the rating
// r_uv, so row F of the accumulated matrix is b_u and get_bias costs no instruction; lanes beyond
// it carry a finite filler (a clamped theta element) whose rows and columns are zeroed at the end.
// Otherwise b_u is accumulated with one FMA per tile and step.
// When F%16 == 4 (f = 100) the last tile row is a strip of 4 feature rows and is accumulated with the
// 4x4x1 instruction instead (a quarter of the time of 16x16x4 tiles that would be 3/4 padding); every
// lane then loads feature 16(NT-1) + i%4 for the last tile, and b_u takes the FMA route.
//
// Software pipeline: a ring of D+1 operand register sets.  Step t runs its MFMAs directly on set
// t mod (D+1) while the gathers of step t+D land in the set that step t-1 used, and the
// (column id, rating) loads run two steps further ahead.  Every load is unconditional (entries
// are clamped into the work item); only the last steps of a work item, which may hold fewer than
// 4 entries, go through a masked copy of the operands.  The vector ALU shares the issue port with
// the matrix pipeline, so the full steps carry almost no ALU work: addresses are a scalar base
// plus a 32-bit lane offset (WIDE = false; the factor matrix must be smaller than 4 GiB).
template <int F>
struct TileGeom {
    static constexpr int NT = tiles_1d(F);
    static constexpr bool STRIP = (F % 16) == 4 && tiles_1d(F) > 1;   // last tile row as a 4-row strip
    static constexpr bool RIT = (F % 16) != 0 && !STRIP;   // rating rides in the last tile
    static constexpr int RI = F % 16;            // its lane (RIT); number of valid rows / columns of the last tile
};

// (a << SH) + b in one full-rate instruction
template <int SH>
__device__ __forceinline__ uint32_t lshl_add(uint32_t a, uint32_t b) {
    uint32_t d;
    asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "n"(SH), "v"(b));
    return d;
}
// c * M + add for the row pitches that occur (a power of two, or 25 times one: f = 100), without the
// quarter-rate 32-bit multiply
template <uint32_t M>
__device__ __forceinline__ uint32_t row_offset(uint32_t c, uint32_t add) {
    constexpr int tz = __builtin_ctz(M);
    if constexpr ((M >> tz) == 1) {
        return lshl_add<tz>(c, add);
    } else if constexpr ((M >> tz) == 25) {
        // one full-rate 24-bit multiply-add: the row index is below 2^24 whenever the matrix is below 4 GiB
        // (M >= 200 bytes per row)
        uint32_t d;
        asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(d) : "v"(c), "v"(M), "v"(add));
        return d;
    } else {
        return c * M + add;
    }
}

// ET: element type of the gathered factor matrix (ALS_F32 / ALS_BF16 / ALS_F16).  16-bit elements are
// fetched with loads of half the width and widened to fp32 in registers; the MFMAs stay fp32.
__device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
template <int ET>
__device__ __forceinline__ float widen_lo(uint32_t w) {   // low 16 bits of w
    if constexpr (ET == ALS_BF16) return bits_to_float(w << 16);
    else return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xffffu));
}
template <int ET>
__device__ __forceinline__ float widen_hi(uint32_t w) {   // high 16 bits of w
    if constexpr (ET == ALS_BF16) return bits_to_float(w & 0xffff0000u);
    else return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16));
}

// The features of lane i (register q: feature_of(F, q, i), filler lanes 0) of row c of the factor matrix, as fp32, with
// the widest loads the feature map allows and a 64-bit row address.  For the kernels that keep gathered rows as
// plain fp32 registers (Algorithm 1 on the gathered rows, the RMSE).
template <int F, int ET>
__device__ __forceinline__ void gather_lane_features(const void *__restrict__ Theta, int c, int i, float (&g)[tiles_1d(F)]) {
    constexpr int NT = tiles_1d(F), N4 = loads16(F), N2 = loads8(F), N1 = loads4(F);
    static_assert(4 * N4 + 2 * N2 + N1 == NT);
    constexpr int ES = ET == ALS_F32 ? 4 : 2;
    const char *row = reinterpret_cast<const char *>(Theta) + (int64_t)c * (F * ES);
#pragma unroll
    for (int q = 0; q < N4; ++q) {   // features 64q + 4i .. + 3
        if constexpr (ET == ALS_F32) {
            const v4f v = *reinterpret_cast<const v4f *>(row + 4 * (64 * q + 4 * i));
            g[4 * q] = v[0]; g[4 * q + 1] = v[1]; g[4 * q + 2] = v[2]; g[4 * q + 3] = v[3];
        } else {
            const uint2 w = *reinterpret_cast<const uint2 *>(row + 2 * (64 * q + 4 * i));
            g[4 * q] = widen_lo<ET>(w.x); g[4 * q + 1] = widen_hi<ET>(w.x);
            g[4 * q + 2] = widen_lo<ET>(w.y); g[4 * q + 3] = widen_hi<ET>(w.y);
        }
    }
    if constexpr (N2 > 0) {          // features 64 N4 + 2i, + 1
        if constexpr (ET == ALS_F32) {
            const float2 v = *reinterpret_cast<const float2 *>(row + 4 * (64 * N4 + 2 * i));
            g[4 * N4] = v.x; g[4 * N4 + 1] = v.y;
        } else {
            const uint32_t w = *reinterpret_cast<const uint32_t *>(row + 2 * (64 * N4 + 2 * i));
            g[4 * N4] = widen_lo<ET>(w); g[4 * N4 + 1] = widen_hi<ET>(w);
        }
    }
#pragma unroll
    for (int k = 0; k < N1; ++k) {   // feature 64 N4 + 32 N2 + 16k + i, if there is one
        const int ft = 64 * N4 + 32 * N2 + 16 * k + i;
        float v = 0.f;
        if (ft < F) {
            if constexpr (ET == ALS_F32) v = *reinterpret_cast<const float *>(row + 4 * ft);
            else v = widen_lo<ET>((uint32_t)*reinterpret_cast<const unsigned short *>(row + 2 * ft));
        }
        g[4 * N4 + 2 * N2 + k] = v;
    }
}

// ROWS: the wavefront accumulates the tile rows of this set only (acc[tiles_below(ROWS, R) + C]); the
// default is the whole triangle.  WANT_B: also produce b_u, for the tile rows of the set.
// MODE: kExplicit as described above.  kImplicit (Section 5.6): the entry (u, v) enters A_u with weight
// w = alpha * max(r_uv, 0) (both operands are scaled by sqrt(w)) and b_u with weight 1 + w if r_uv > 0.
// kGram: the "entries" are the rows s0 .. s0+len-1 of Theta themselves (idx and val are not read),
// unit weights, for Theta^T Theta.
template <int F, bool IN_VGPR, int D, bool WIDE, int ET, uint32_t ROWS = rows_all(F), bool WANT_B = true,
          int MODE = kExplicit>
__device__ __forceinline__ void accumulate_tiles(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                 const void *__restrict__ Theta, int64_t s0, int len,
                                                 v4f (&acc)[tiles_in(ROWS)], float (&b)[tiles_1d(F)],
                                                 float alpha = 0.f) {
    static_assert(ROWS == rows_all(F) || (F % 16) == 0, "partial sets of tile rows need f to be a multiple of 16");
    static_assert(ROWS != 0 && (ROWS & ~rows_all(F)) == 0, "tile rows out of range");
    static_assert(MODE == kExplicit || !TileGeom<F>::RIT, "the rating lane carries the plain rating only");
    static_assert(MODE != kGram || !WANT_B, "a Gram matrix has no right-hand side");
    constexpr int NT = TileGeom<F>::NT, NB = D + 1;
    constexpr bool RIT = TileGeom<F>::RIT, STRIP = TileGeom<F>::STRIP;
    constexpr int RI = TileGeom<F>::RI;
    const int lane = threadIdx.x & 63;
    const int i = lane & 15;
    const int kq = lane >> 4;
    const int32_t *__restrict__ ib = idx + s0;   // wave-uniform bases
    const float *__restrict__ vb = val + s0;
    const int nsteps = (len + 3) >> 2;
    const int nmain = ((len >> 2) / NB) * NB;    // full steps handled by the unmasked rounds
    const int last = len - 1;
    constexpr int N4 = loads16(F), N2 = loads8(F), N1 = loads4(F);
    constexpr int base1 = 64 * N4 + 32 * N2;       // first feature fetched by the single-element loads
    constexpr int ES = ET == ALS_F32 ? 4 : 2;       // bytes per element
    constexpr int RW = ET == ALS_F32 ? NT : 2 * N4 + N2 + N1;   // 32-bit registers one gathered row needs
    // Column ids and ratings are fetched through buffer resources that span exactly this work item: a fetch
    // beyond its end (the prefetches of the last rounds, the padding of the last step) returns 0 instead of
    // touching memory outside it, so no index needs clamping.  Lane (i, kq) reads entry 4*step + kq, i.e. byte
    // offset 16*step + 4*kq: a lane offset plus a compile-time constant in every unrolled step.
    constexpr int kRsrcFlags = 0x00020000;   // raw buffer, dword elements (gfx9 family encoding)
    __amdgpu_buffer_rsrc_t ids_rsrc, val_rsrc;
    if constexpr (MODE != kGram) {
        ids_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(ib), 0, 4 * len, kRsrcFlags);
        val_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vb), 0, 4 * len, kRsrcFlags);
    }
    const int row0 = (int)s0;   // kGram: entry e is row s0 + e of the factor matrix
    // eoff: byte offset of this lane's entry in step `base` (base = first step of the current round)
    auto load_id = [&](uint32_t eoff, int step_rel) -> int32_t {
        if constexpr (MODE == kGram) {
            const int e = (int)(eoff >> 2) + 4 * step_rel;
            return row0 + (e < last ? e : last);
        } else {
            return __builtin_amdgcn_raw_buffer_load_b32(ids_rsrc, eoff + 16u * (uint32_t)step_rel, 0, 0);
        }
    };
    auto load_rating = [&](uint32_t eoff, int step_rel) -> float {
        if constexpr (MODE == kGram) return 1.f;
        else return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(val_rsrc, eoff + 16u * (uint32_t)step_rel, 0, 0));
    };
    // One theta row -> raw registers, with the widest loads the feature permutation allows: 4, 2 and 1
    // elements per lane.  Addresses are (scalar base) + (32-bit lane offset) + (immediate) unless WIDE.
    const uint32_t lane_a = (uint32_t)(4 * ES) * (uint32_t)i;
    const uint32_t lane_b = (uint32_t)(64 * ES * N4) + (uint32_t)(2 * ES) * (uint32_t)i;
    const uint32_t lane_c = (uint32_t)ES * (uint32_t)(base1 + i);
    const uint32_t lane_l = STRIP ? (uint32_t)ES * (uint32_t)(base1 + 16 * (N1 - 1) + (i & 3))
                                  : (uint32_t)ES * (uint32_t)((base1 + 16 * (N1 - 1) + i < F) ? base1 + 16 * (N1 - 1) + i : F - 1);
    const uint32_t lane_first = N4 > 0 ? lane_a : N2 > 0 ? lane_b : N1 > 1 ? lane_c : lane_l;
    auto gather = [&](int c, uint32_t (&w)[RW]) {
        const char *p;
        uint32_t ro = 0;   // offset of the lane's first load: row offset + lane_first
        if constexpr (WIDE) {
            p = reinterpret_cast<const char *>(Theta) + (int64_t)c * (ES * F);
            ro = lane_first;
        } else {
            p = reinterpret_cast<const char *>(Theta);
            ro = row_offset<(uint32_t)(ES * F)>((uint32_t)c, lane_first);
        }
        if constexpr (N4 > 0) {
            const uint32_t o = ro + (lane_a - lane_first);
#pragma unroll
            for (int q = 0; q < N4; ++q) {
                if constexpr (ET == ALS_F32) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(p + o + 256 * q);
                    w[4 * q] = v.x; w[4 * q + 1] = v.y; w[4 * q + 2] = v.z; w[4 * q + 3] = v.w;
                } else {
                    const uint2 v = *reinterpret_cast<const uint2 *>(p + o + 128 * q);
                    w[2 * q] = v.x; w[2 * q + 1] = v.y;
                }
            }
        }
        if constexpr (N2 > 0) {
            const uint32_t o = ro + (lane_b - lane_first);
            if constexpr (ET == ALS_F32) {
                const uint2 v = *reinterpret_cast<const uint2 *>(p + o);
                w[4 * N4] = v.x; w[4 * N4 + 1] = v.y;
            } else {
                w[2 * N4] = *reinterpret_cast<const uint32_t *>(p + o);
            }
        }
        constexpr int first1 = ET == ALS_F32 ? 4 * N4 + 2 * N2 : 2 * N4 + N2;
        if constexpr (N1 > 1) {
            const uint32_t o = ro + (lane_c - lane_first);
#pragma unroll
            for (int k = 0; k < N1 - 1; ++k) {
                if constexpr (ET == ALS_F32) w[first1 + k] = *reinterpret_cast<const uint32_t *>(p + o + 64 * k);
                else w[first1 + k] = *reinterpret_cast<const unsigned short *>(p + o + 32 * k);
            }
        }
        if constexpr (N1 > 0) {
            const uint32_t o = ro + (lane_l - lane_first);
            if constexpr (ET == ALS_F32) w[first1 + N1 - 1] = *reinterpret_cast<const uint32_t *>(p + o);
            else w[first1 + N1 - 1] = *reinterpret_cast<const unsigned short *>(p + o);
        }
    };
    // raw registers -> fp32 operands, one per tile
    auto unpack = [&](const uint32_t (&w)[RW], float (&g)[NT]) {
        if constexpr (ET == ALS_F32) {
#pragma unroll
            for (int q = 0; q < NT; ++q) g[q] = bits_to_float(w[q]);
        } else {
#pragma unroll
            for (int q = 0; q < N4; ++q) {
                g[4 * q] = widen_lo<ET>(w[2 * q]); g[4 * q + 1] = widen_hi<ET>(w[2 * q]);
                g[4 * q + 2] = widen_lo<ET>(w[2 * q + 1]); g[4 * q + 3] = widen_hi<ET>(w[2 * q + 1]);
            }
            if constexpr (N2 > 0) { g[4 * N4] = widen_lo<ET>(w[2 * N4]); g[4 * N4 + 1] = widen_hi<ET>(w[2 * N4]); }
#pragma unroll
            for (int k = 0; k < N1; ++k) g[4 * N4 + 2 * N2 + k] = widen_lo<ET>(w[2 * N4 + N2 + k]);
        }
    };

    // Rings with compile-time slots (step j lives in slot j mod NB), so that no register is ever
    // moved: a move of a value that is still in flight would make the compiler wait for it.
    //   gbuf/rbuf  operands and rating of a step, loaded D steps ahead
    //   cbuf       column id of a step, loaded IDA steps before its gather is issued
    constexpr int IDA = D >= 2 ? 2 : 1, K = D + IDA;
    uint32_t gbuf[NB][RW];
    float rbuf[NB];
    int cbuf[NB];
    float bacc[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) bacc[q] = 0.f;
    // The caller has just written the accumulators (zeros, or a starting matrix) with vector-ALU or memory
    // instructions, which the compiler is free to sink to just before their first use -- the first MFMA,
    // which must not read a register written in the previous few cycles.  Pin those writes here.
    mfma_settle<IN_VGPR>(acc);
    // Prologue in the order of the loop body (far ids first, then the gathers, oldest step first): the
    // compiler's wait-count bookkeeping merges both paths at the loop head, and any other order makes
    // it drain the outstanding gathers at the top of every round.
    uint32_t eoff = 4u * (uint32_t)kq;   // this lane's entry offset in the first step of the current round
#pragma unroll
    for (int j = D; j < K; ++j) cbuf[j % NB] = load_id(eoff, j);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int d = 0; d < D; ++d) {
        rbuf[d] = load_rating(eoff, d);
        gather(load_id(eoff, d), gbuf[d]);
        asm volatile("" ::: "memory");
    }

    // one step; MASKED = the step may hold fewer than 4 entries (or none)
    auto step = [&](auto dtag, auto mtag, int t) {
        constexpr int d = decltype(dtag)::value;
        constexpr bool MASKED = decltype(mtag)::value;
        constexpr int dn = (d + D) % NB;
        // (1) column id of step t+K
        cbuf[(d + K) % NB] = load_id(eoff, d + K);
        // keeps the load above here: the compiler would otherwise fold the carried value into a load
        // at its use, putting a full memory latency in front of a gather
        asm volatile("" ::: "memory");
        // (2) gathers and rating of step t+D into the set that step t-1 has finished with
        gather(cbuf[dn], gbuf[dn]);
        rbuf[dn] = load_rating(eoff, d + D);
        __builtin_amdgcn_sched_barrier(0);
        // (3) MFMAs of step t
        float g[NT];
        float r = rbuf[d];
        unpack(gbuf[d], g);
        if constexpr (MASKED) {
            const bool ok = (4 * t + kq) < len;
#pragma unroll
            for (int q = 0; q < NT; ++q) g[q] = ok ? g[q] : 0.f;
            r = ok ? r : 0.f;
        }
        if constexpr (MODE == kImplicit) {
            const float w = alpha * fmaxf(r, 0.f);
            const float bw = r > 0.f ? 1.f + w : 0.f;
            const float sw = __builtin_amdgcn_sqrtf(w);
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                if constexpr (WANT_B) bacc[q] = fmaf(bw, g[q], bacc[q]);
                g[q] *= sw;
            }
        } else if constexpr (RIT) {
            g[NT - 1] = (i == RI) ? r : g[NT - 1];
        } else if constexpr (WANT_B) {
#pragma unroll
            for (int q = 0; q < NT; ++q)
                if ((ROWS >> q) & 1u) bacc[q] = fmaf(r, g[q], bacc[q]);
        }
        if constexpr (MASKED || ET != ALS_F32 || (RIT && NT < 3) || MODE == kImplicit) {
            // An operand written by the vector ALU must not be read by an MFMA in the next few cycles,
            // and the compiler, to which the MFMAs are opaque, does not keep that distance: wait here,
            // and tie every operand to the wait so that no MFMA can be moved in front of it.
            asm volatile("s_nop 7" : "+v"(g[0]));
#pragma unroll
            for (int q = 1; q < NT; ++q) asm volatile("" : "+v"(g[q]), "+v"(g[0]));
        }
#pragma unroll
        for (int R = 0; R < (STRIP ? NT - 1 : NT); ++R)
            if ((ROWS >> R) & 1u) {
#pragma unroll
                for (int C = 0; C <= R; ++C) mfma_16x16x4<IN_VGPR>(acc[tiles_below(ROWS, R) + C], g[R], g[C]);
            }
        if constexpr (STRIP) {
#pragma unroll
            for (int C = 0; C < NT; ++C) mfma_4x4x1<IN_VGPR>(acc[(NT - 1) * NT / 2 + C], g[NT - 1], g[C]);
        }
        if constexpr (MASKED) mfma_settle<IN_VGPR>(acc);   // masked steps are conditional
    };
    auto round = [&](auto mtag, int s, int limit) {
        [&]<int... d>(std::integer_sequence<int, d...>) {
            ((s + d < limit ? step(std::integral_constant<int, d>{}, mtag, s + d) : void()), ...);
        }(std::make_integer_sequence<int, NB>{});
    };
    for (int s = 0; s < nmain; s += NB) {
        // opaque to the optimiser: it would otherwise re-base the offsets of the round on other induction
        // variables and spend an addition per load instead of using the instruction's immediate offset
        asm volatile("" : "+v"(eoff));
        [&]<int... d>(std::integer_sequence<int, d...>) {
            (step(std::integral_constant<int, d>{}, std::false_type{}, s + d), ...);
        }(std::make_integer_sequence<int, NB>{});
#ifndef ALS_NO_ROUND_SETTLE
        mfma_settle<IN_VGPR>(acc);
#endif
        eoff += 16u * NB;
    }
    asm volatile("" : "+v"(eoff));
    round(std::true_type{}, nmain, nsteps);   // at most NB steps remain
    mfma_drain();

    // b_u in column layout, and the filler rows / columns of the last tile zeroed
    const int c = i, g4 = kq;
    if constexpr (RIT) {
        const int src = 4 * (16 * (RI / 4) + c);   // lane (c, g = RI/4) holds row RI of the last tile row
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            const float v = bperm(src, acc[(NT - 1) * NT / 2 + T][RI % 4]);
            b[T] = (T < NT - 1 || c < RI) ? v : 0.f;
        }
#pragma unroll
        for (int T = 0; T < NT; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool keep = (4 * g4 + r < RI) && (T < NT - 1 || c < RI);
                acc[(NT - 1) * NT / 2 + T][r] = keep ? acc[(NT - 1) * NT / 2 + T][r] : 0.f;
            }
    } else if constexpr (WANT_B) {
#pragma unroll
        for (int q = 0; q < NT; ++q) b[q] = ((ROWS >> q) & 1u) ? colsum4(bacc[q]) : 0.f;
    }
    if constexpr (STRIP) {
        // lane (c, kq) register r holds the share of lane row kq in element (row r, column c) of the strip:
        // summed over kq this is the ordinary tile layout of lane row 0; the other lane rows are padding
        if constexpr (WANT_B) b[NT - 1] = (c < RI) ? b[NT - 1] : 0.f;
        // The permutes of a stage are issued before the first result is used (LDS round trips are long).  With
        // the tiles in accumulation registers the batches are short: the temporaries must not push the
        // kernel over the register budget of two wavefronts per SIMD.
        const int a16 = 4 * (lane ^ 16), a32 = 4 * (lane ^ 32);
        constexpr int BT = IN_VGPR ? NT : 2;   // tiles per batch
#pragma unroll
        for (int T0 = 0; T0 < NT; T0 += BT) {
            constexpr int LB = (NT - 1) * NT / 2;
            float t[BT][4];
#pragma unroll
            for (int T = T0; T < T0 + BT && T < NT; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) t[T - T0][r] = bperm(a16, acc[LB + T][r]);
#pragma unroll
            for (int T = T0; T < T0 + BT && T < NT; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[LB + T][r] += t[T - T0][r];
#pragma unroll
            for (int T = T0; T < T0 + BT && T < NT; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) t[T - T0][r] = bperm(a32, acc[LB + T][r]);
#pragma unroll
            for (int T = T0; T < T0 + BT && T < NT; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool keep = (g4 == 0) && (T < NT - 1 || c < RI);
                    acc[LB + T][r] = keep ? acc[LB + T][r] + t[T - T0][r] : 0.f;
                }
        }
    }
}

// fp32 -> bf16 bits, round to nearest even; two values packed in one word (first in the low half)
__device__ __forceinline__ uint32_t bf16_bits(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }

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
    const uint64_t csel0 = __ballot((c & 1) != 0), csel1 = __ballot((c & 2) != 0);   // bits of c & 3 as lane masks
    const int a16 = 4 * (lane ^ 16), a32 = 4 * (lane ^ 32);

    // LDS permutes have a long latency: all permutes of a stage are issued before the first result is used
    auto matvec = [&](const float (&p)[NT], float (&ap)[NT]) {
        float lower[NT];  // tile^T * p_R contributions, per-lane partial sums over the lane rows
#pragma unroll
        for (int q = 0; q < NT; ++q) lower[q] = 0.f;
        float prs[NT][4];
#pragma unroll
        for (int R = 1; R < NT; ++R)
#pragma unroll
            for (int r = 0; r < 4; ++r) prs[R][r] = bperm(addr_rl[r], p[R]);
#pragma unroll
        for (int R = 0; R < NT; ++R) {
            const float (&pr)[4] = prs[R];
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
            ap[R] = bperm(addr_cl, rowsum16_sel4(row[0], row[1], row[2], row[3], (c & 1) != 0, (c & 2) != 0));
        }
        if constexpr (NT > 1) {
            float t[NT - 1];
#pragma unroll
            for (int q = 0; q < NT - 1; ++q) t[q] = bperm(a16, lower[q]);
#pragma unroll
            for (int q = 0; q < NT - 1; ++q) lower[q] += t[q];
#pragma unroll
            for (int q = 0; q < NT - 1; ++q) t[q] = bperm(a32, lower[q]);
#pragma unroll
            for (int q = 0; q < NT - 1; ++q) ap[q] += lower[q] + t[q];
        }
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
    if (!(rs_old > 0.f) || !isfinite(rs_old)) {
        // r = 0: x solves the system already.  Anything else here is a non-finite A_u, b_u or warm start: the row
        // gets that value instead of silently keeping its warm start, and the store reports it
        if (rs_old != 0.f) {
#pragma unroll
            for (int q = 0; q < NT; ++q) x[q] = __builtin_nanf("");   // NaN
        }
        return;
    }
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

// Exact solve (Section 2 step (ii), Section 4.1 baseline) of one system held by one wavefront: LDL^T
// without square roots, right-looking, blocked by tile columns, directly on the accumulator tiles; then
// the two triangular solves, blocked the same way.  Same argument layout as cg_tiles; acc is overwritten
// (column j ends up holding L[:,j]*d_j).  Returns false if a pivot was not positive (the pivot is then
// replaced by 1).
//   Panel (tile column K), column by column: the pivot, z_j and the column in the "row layout" of every
//   tile row of the panel (4 permutes each) are fetched in one batch; the diagonal tile's part is turned
//   into the "column layout" (one more permute) and scaled by 1/d_j; the remaining columns of the panel
//   tiles get their rank-1 update (4 FMAs per tile); z of the panel is forward-substituted.
//   Once per panel, on the matrix cores: tile (R, C) -= (L_RK D_K) (L_CK)^T as four 16x16x4 MFMAs.  The
//   operands are the panel tiles transposed into the operand layout (lane (i, kq), register s = element
//   (i, 4kq+s)) through `tbuf`, 272 floats of LDS private to the wavefront; the same transposed tiles
//   carry the panel's z into the tile rows below (4 FMAs per tile).
//   Back substitution: per panel, column by column inside the diagonal tile, then one tile-times-vector
//   product per tile to its left.
template <bool IN_VGPR>
__device__ __forceinline__ void mfma_16x16x4_ordered(v4f &acc, float a, float b) {
    asm volatile(ALS_MFMA_PRE "v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" ALS_MFMA_POST : "+v"(acc) : "v"(a), "v"(b));
}

template <int F>
__device__ __forceinline__ bool ldlt_tiles(v4f (&acc)[tiles_tri(F)], const float (&b)[tiles_1d(F)],
                                           float (&x)[tiles_1d(F)], float *tbuf) {
    constexpr int NT = tiles_1d(F);
    constexpr int LASTCOLS = (F % 16) ? (F % 16) : 16;   // feature columns of the last tile
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int addr_cl = 4 * (16 * (c >> 2) + c);
    const uint64_t csel0 = __ballot((c & 1) != 0), csel1 = __ballot((c & 2) != 0);   // bits of c & 3 as lane masks
    const int a16 = 4 * (lane ^ 16), a32 = 4 * (lane ^ 32);
    float z[NT], dinv[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        z[q] = b[q];
        dinv[q] = 0.f;
    }
    bool ok = true;
    auto pick = [](const v4f &t, int r) { return r == 0 ? t[0] : r == 1 ? t[1] : r == 2 ? t[2] : t[3]; };
    // The trailing updates below are MFMAs that accumulate into the tiles.  The caller's last vector-ALU
    // writes to them (the regulariser on the diagonal, an added Gram matrix) may be delayed by the compiler
    // until just before that first use, too close for the MFMA to see them: pin them here.  Afterwards a
    // tile is written by MFMAs only until its own panel comes up.
    mfma_settle<true>(acc);
#pragma unroll
    for (int K = 0; K < NT; ++K) {
        const int ncol = (K == NT - 1) ? LASTCOLS : 16;
        const int DK = K * (K + 1) / 2 + K;   // the diagonal tile of the panel
#pragma unroll 1
        for (int jl = 0; jl < ncol; ++jl) {
            const int jr = jl & 3, jg = jl >> 2;
            // one LDS round trip: the pivot, z_j and the column in row layout
            float d = bperm(4 * (16 * jg + jl), pick(acc[DK], jr));
            const float zj = bperm(4 * jl, z[K]);
            float colv[NT][4];
            const int addr_rl = 4 * (16 * g + jl);
#pragma unroll
            for (int R = K; R < NT; ++R)
#pragma unroll
                for (int r = 0; r < 4; ++r) colv[R][r] = bperm(addr_rl, acc[R * (R + 1) / 2 + K][r]);
            // second round trip: the diagonal tile's part of the column in column layout
            float rowk = bperm(addr_cl, lane_select4(colv[K][0], colv[K][1], colv[K][2], colv[K][3], csel0, csel1));
            if (!(d > 0.f)) {
                ok = false;
                d = 1.f;
            }
            float inv = __builtin_amdgcn_rcpf(d);
            inv = inv * fmaf(-d, inv, 2.f);        // one Newton step: relative error ~1e-7
            rowk = (c > jl) ? rowk * inv : 0.f;    // columns up to j of this tile column are final
            dinv[K] = (c == jl) ? inv : dinv[K];
            z[K] = fmaf(-rowk, zj, z[K]);
#pragma unroll
            for (int R = K; R < NT; ++R)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[R * (R + 1) / 2 + K][r] = fmaf(-colv[R][r], rowk, acc[R * (R + 1) / 2 + K][r]);
        }
        if (K < NT - 1) {
            // T[R][s] = (L_RK D_K)(i, 4kq+s); V[R][s] = -T[R][s] / d_(4kq+s); zs[s] = z_(4kq+s) / d_(4kq+s)
            float T[NT][4], V[NT][4], dk[4], zs[4];
            const float zd = z[K] * dinv[K];
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                dk[s4] = -bperm(4 * (4 * g + s4), dinv[K]);
                zs[s4] = bperm(4 * (4 * g + s4), zd);
            }
#pragma unroll
            for (int R = K + 1; R < NT; ++R) {
#pragma unroll
                for (int r = 0; r < 4; ++r) tbuf[(4 * g + r) * 17 + c] = acc[R * (R + 1) / 2 + K][r];
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    T[R][s4] = tbuf[c * 17 + 4 * g + s4];
                    V[R][s4] = T[R][s4] * dk[s4];
                }
            }
            // a register written by the vector ALU must not be read by an MFMA within the next few cycles
#pragma unroll
            for (int R = K + 1; R < NT; ++R)
                asm volatile("" : "+v"(V[R][0]), "+v"(V[R][1]), "+v"(V[R][2]), "+v"(V[R][3]), "+v"(T[R][0]), "+v"(T[R][1]),
                             "+v"(T[R][2]), "+v"(T[R][3]));
            asm volatile("s_nop 7" ::: "memory");
#pragma unroll
            for (int R = K + 1; R < NT; ++R)
#pragma unroll
                for (int C = K + 1; C <= R; ++C)
#pragma unroll
                    for (int s4 = 0; s4 < 4; ++s4) {
                        mfma_16x16x4_ordered<true>(acc[R * (R + 1) / 2 + C], T[R][s4], V[C][s4]);
#ifdef ALS_DEBUG_SERIAL_MFMA
                        mfma_drain();
#endif
                    }
            // forward substitution of the tile rows below, while the MFMAs run: z_R -= (L_RK D_K) (z_K / d_K)
            float part[NT];
#pragma unroll
            for (int R = K + 1; R < NT; ++R) {
                float p4 = T[R][0] * zs[0];
#pragma unroll
                for (int s4 = 1; s4 < 4; ++s4) p4 = fmaf(T[R][s4], zs[s4], p4);
                part[R] = p4;
            }
            float t[NT];
#pragma unroll
            for (int R = K + 1; R < NT; ++R) t[R] = bperm(a16, part[R]);
#pragma unroll
            for (int R = K + 1; R < NT; ++R) part[R] += t[R];
#pragma unroll
            for (int R = K + 1; R < NT; ++R) t[R] = bperm(a32, part[R]);
#pragma unroll
            for (int R = K + 1; R < NT; ++R) z[R] -= part[R] + t[R];
            mfma_drain();
            // nothing may read the updated tiles before the wait above
#pragma unroll
            for (int R = K + 1; R < NT; ++R)
#pragma unroll
                for (int C = K + 1; C <= R; ++C) asm volatile("" : "+v"(acc[R * (R + 1) / 2 + C]));
        }
    }
    // back substitution, panels from the last to the first: x_j = z_j/d_j, then z_i -= (L[j][i] d_i) x_j, i < j
#pragma unroll
    for (int q = 0; q < NT; ++q) x[q] = 0.f;
#pragma unroll
    for (int K = NT - 1; K >= 0; --K) {
        const int ncol = (K == NT - 1) ? LASTCOLS : 16;
        const int DK = K * (K + 1) / 2 + K;
#pragma unroll 1
        for (int jl = ncol - 1; jl >= 0; --jl) {
            const int jr = jl & 3, jg = jl >> 2;
            const float xj = bperm(4 * jl, z[K] * dinv[K]);
            // lane (c, jg) holds row j of the diagonal tile
            const float lrow = bperm(4 * (16 * jg + c), pick(acc[DK], jr));
            x[K] = (c == jl) ? xj : x[K];
            z[K] -= (c < jl) ? lrow * xj : 0.f;
        }
        if (K > 0) {
            // tiles to the left of the diagonal: z_C -= (tile (K, C))^T x_K, rows of the tile = lane rows x registers
            float xr[4], part[NT], t[NT];
#pragma unroll
            for (int r = 0; r < 4; ++r) xr[r] = bperm(4 * (4 * g + r), x[K]);
#pragma unroll
            for (int C = 0; C < K; ++C) {
                const v4f tile = acc[K * (K + 1) / 2 + C];
                float p4 = tile[0] * xr[0];
#pragma unroll
                for (int r = 1; r < 4; ++r) p4 = fmaf(tile[r], xr[r], p4);
                part[C] = p4;
            }
#pragma unroll
            for (int C = 0; C < K; ++C) t[C] = bperm(a16, part[C]);
#pragma unroll
            for (int C = 0; C < K; ++C) part[C] += t[C];
#pragma unroll
            for (int C = 0; C < K; ++C) t[C] = bperm(a32, part[C]);
#pragma unroll
            for (int C = 0; C < K; ++C) z[C] -= part[C] + t[C];
        }
    }
    return ok;
}

// adds reg to the diagonal entries of the diagonal tiles that belong to a feature
template <int F>
__device__ __forceinline__ void add_diagonal(v4f (&acc)[tiles_tri(F)], float reg) {
    constexpr int NT = tiles_1d(F);
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int R = 0; R < NT; ++R)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (c == 4 * g + r && feature_of(F, R, c) >= 0) acc[R * (R + 1) / 2 + R][r] += reg;
}

}  // namespace als
