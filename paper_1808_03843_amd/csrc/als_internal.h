// Internal declarations shared by the translation units of libals_gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/als.h"

namespace als {

// ---- geometry of one work item's output ("slot") --------------------------------------------
// A_u is accumulated as 16x16 tiles of the lower triangle (tile row R >= tile column C) in the
// register layout of v_mfma_f32_16x16x4_f32: lane l, register r of a tile holds the element
// (row 4*(l/16)+r, column l%16).  A slot stores tile t = R(R+1)/2+C at float offset
// (4t+r)*64 + l, followed by b_u padded to 16*NT floats.
//
// Tile coordinates are "virtual" indices v = 16*tile + lane: the features are permuted so that a
// lane can fetch the operands of several tiles with one wide load.  With N4 = F/64 16-byte loads,
// N2 = (F%64)/32 8-byte loads and N1 4-byte loads per theta row,
//   tiles 4q..4q+3      (q < N4)   lane i holds features 64q + 4i + (0..3)
//   the next 2*N2 tiles            lane i holds features 64*N4 + 2i + (0..1)
//   the last N1 tiles              lane i holds feature  64*N4 + 32*N2 + 16k + i
// A symmetric permutation of the Gram matrix: the solvers work in virtual coordinates, and only
// the code that reads or writes factor rows and dense matrices converts.
constexpr int tiles_1d(int F) { return (F + 15) / 16; }
constexpr int tiles_tri(int F) { return tiles_1d(F) * (tiles_1d(F) + 1) / 2; }
constexpr int slot_floats(int F) { return tiles_tri(F) * 256 + tiles_1d(F) * 16; }
// A set of tile rows as a bit mask (bit R = tile row R): what one wavefront holds when a system is shared by
// several.  Its tiles are numbered row by row in ascending R, C = 0..R inside a row.
constexpr uint32_t rows_all(int F) { return (1u << tiles_1d(F)) - 1u; }
constexpr int tiles_in(uint32_t rows) {
    int n = 0;
    for (int R = 0; R < 32; ++R)
        if ((rows >> R) & 1u) n += R + 1;
    return n;
}
constexpr int tiles_below(uint32_t rows, int R) { return tiles_in(rows & ((1u << R) - 1u)); }
// NW wavefronts share the NT tile rows in pairs (k, NT-1-k) of NT+1 tiles each: equal tile counts
constexpr uint32_t wave_rows(int NT, int NW, int w) {
    const int NP = NT / 2;   // pairs
    uint32_t m = 0;
    for (int k = 0; k < NP; ++k) {
        const bool mine = (NW == NP) ? (k == w) : (k == w || k == NP - 1 - w);   // NW == NP or NW == NP/2
        if (mine) m |= (1u << k) | (1u << (NT - 1 - k));
    }
    return m;
}
// slot with the tiles stored as packed bf16 pairs (registers 2h, 2h+1 of a tile in one 32-bit word at
// word offset (2t+h)*64 + l), b_u still fp32: the reduced-precision storage of Section 4.2
constexpr int slot_words16(int F) { return tiles_tri(F) * 128 + tiles_1d(F) * 16; }
constexpr int loads16(int F) { return F / 64; }
constexpr int loads8(int F) { return (F % 64) / 32; }
constexpr int loads4(int F) { return tiles_1d(F) - 4 * loads16(F) - 2 * loads8(F); }
// feature held by lane i of tile t, or -1 (filler / rating lane)
__host__ __device__ constexpr int feature_of(int F, int t, int i) {
    if (t < 4 * loads16(F)) return 64 * (t / 4) + 4 * i + (t % 4);
    t -= 4 * loads16(F);
    if (t < 2 * loads8(F)) return 64 * loads16(F) + 2 * i + t;
    t -= 2 * loads8(F);
    const int f = 64 * loads16(F) + 32 * loads8(F) + 16 * t + i;
    return f < F ? f : -1;
}

constexpr int kWave = 64;

// what the gathered accumulation computes (template parameter MODE of the kernels)
constexpr int kExplicit = 0;   // eq. (2): sum theta theta^T, b = sum r theta
constexpr int kImplicit = 1;   // Section 5.6: sum alpha*r theta theta^T, b = sum (1 + alpha*r) theta over r > 0
constexpr int kGram = 2;       // rows s0..s0+len of the factor matrix itself, unit weights, no b

struct Plan {                     // per sparse matrix, built once and cached
    const void *key_ptr = nullptr;
    int64_t nrows = 0, nnz = 0;
    int chunk = 0;
    int32_t *perm = nullptr;      // DEVICE [nrows] rows grouped by degree class, heaviest first
    int32_t *task_off = nullptr;  // DEVICE [nrows+1] first work item of the row at each perm position
    int32_t *task_row = nullptr;  // DEVICE [ntasks]
    int32_t *task_chunk = nullptr;// DEVICE [ntasks]
    unsigned long long *fingerprint = nullptr;   // DEVICE: fingerprint of the row offsets the plan was built from
    int32_t *task_order = nullptr;// DEVICE [work items of the slot path]: launch order inside every batch (see build_order)
    int32_t *task_off_host = nullptr; // HOST copy of task_off
    int64_t ntasks = 0;
    int64_t split_pos = 0;        // perm positions [0, split_pos): rows with >= chunk entries (slot path)
    int64_t rows_ge[33] = {};     // rows_ge[c]: rows with at least 2^(c-1) entries (class >= c) = perm positions [0, rows_ge[c]); rows_ge[0] = nrows
};

constexpr int kWideThreads = 512;   // threads of the largest workgroup any kernel here uses (f = 256: 8 wavefronts)

// status word bits set by kernels
constexpr int kStatusBadPivot = 1;
constexpr int kStatusNonFinite = 2;
constexpr int kStatusStalePlan = 4;   // the row offsets of a matrix differ from those its cached plan was built from

// ---- launchers (each defined next to its kernels) --------------------------------------------
// wide: the gathered factor matrix is 4 GiB or larger (64-bit lane addresses)
// et: element type of the gathered factor matrix (ALS_F32 / ALS_BF16 / ALS_F16; ALS_F32X3: fp32 in memory; ALS_F32X2 has launchers of its own)
// s16: slots hold bf16 tiles (slot_words16) instead of fp32 tiles (slot_floats)
hipError_t launch_hermitian(int f, bool ptr64, bool wide, int et, bool s16, hipStream_t st, const int32_t *task_row,
                            const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                            const int32_t *idx, const float *val, const void *Theta, float *slots);

// factor_dtype = ALS_F32X3, f <= 128 (hermitian_x3.hip); launch_hermitian and launch_hermitian_cg forward to these
hipError_t launch_hermitian_x3(int f, bool ptr64, bool wide, bool s16, hipStream_t st, const int32_t *task_row,
                               const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                               int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                               float *slots);
hipError_t launch_hermitian_cg_x3(int f, bool ptr64, bool wide, int solver, hipStream_t st, const int32_t *perm,
                                  int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                  const void *Theta, float lambda, int fs, float eps, float *Xout, int *status);

// factor_dtype = ALS_F32X2, f <= 128 (hermitian_x2.hip): as above with two fp16 parts.  absmax: DEVICE, one word,
// the bits of max |Theta| (launch_absmax on the same stream, before these)
hipError_t launch_absmax(hipStream_t st, const float *x, int64_t n, uint32_t *absmax);
hipError_t launch_hermitian_x2(int f, bool ptr64, bool wide, bool s16, hipStream_t st, const int32_t *task_row,
                               const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                               int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                               float *slots, const uint32_t *absmax);
hipError_t launch_hermitian_cg_x2(int f, bool ptr64, bool wide, int solver, hipStream_t st, const int32_t *perm,
                                  int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                  const void *Theta, float lambda, int fs, float eps, float *Xout, int *status,
                                  const uint32_t *absmax);

// cg_short.hip: Algorithm 1 on the gathered rows themselves (A_u p = G^T (G p) + lambda n_u p), one wavefront per
// row, or 2 or 4 rows per wavefront, for the rows perm[pos0 .. pos0+npos) which must have fewer than
// 64 / rows_per_wave entries (f = 256: rows_per_wave = 1, two wavefronts per row); rows_per_wave = -2 (f <= 128): two
// wavefronts per row, fewer than 128 entries.  et: ALS_F32 / ALS_BF16 / ALS_F16, the element type in memory
hipError_t launch_cg_gathered(int f, int rows_per_wave, bool ptr64, int et, hipStream_t st, const int32_t *perm, int64_t pos0, int64_t npos,
                              const void *ptr, const int32_t *idx, const float *val, const void *Theta, float lambda,
                              int fs, float eps, float *Xout, int *status);

// solver: ALS_SOLVER_CG or ALS_SOLVER_CHOLESKY
hipError_t launch_hermitian_cg(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st, const int32_t *perm,
                               int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                               const void *Theta, float lambda, int fs, float eps, float *Xout, int *status);
hipError_t launch_solve_cg_wave(int f, bool ptr64, bool s16, int solver, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                float lambda, int fs, float eps, float *Xout, int *status);
// f = 256 (wide.hip): a system is shared by the wavefronts of one workgroup.  Same arguments as the
// launchers above; Algorithm 1 only (the exact solver at this width is in wide_ldlt.hip, declared below).
hipError_t launch_hermitian_wide(bool ptr64, bool wide, int et, bool s16, hipStream_t st, const int32_t *task_row,
                                 const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk, const void *ptr,
                                 const int32_t *idx, const float *val, const void *Theta, float *slots);
hipError_t launch_hermitian_cg_wide(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                                    int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                    const void *Theta, float lambda, int fs, float eps, float *Xout, int *status);
// exact solver at f = 256 (wide_ldlt.hip): fused with the build for short rows, from fp32 slots otherwise
hipError_t launch_hermitian_ldlt_wide(bool ptr64, bool wide, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                                      int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                      const void *Theta, float lambda, float *Xout, int *status);
hipError_t launch_solve_ldlt_wide(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                  int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                  float lambda, float *Xout, int *status);
// implicit feedback at f = 256 (wide.hip, wide_ldlt_implicit.hip): the f = 256 counterparts of launch_gram's
// first stage and of the three implicit launchers below
hipError_t launch_gram_wide(bool wide, hipStream_t st, const float *G, int64_t n, int per, int nslots, float *slots);
hipError_t launch_hermitian_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *task_row,
                                          const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk,
                                          const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                          float alpha, float *slots);
hipError_t launch_hermitian_cg_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                             int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                             const void *Theta, float lambda, float alpha, const float *gram, int fs,
                                             float eps, float *Xout, int *status);
hipError_t launch_solve_cg_wide_implicit(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                         int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                         float lambda, const float *gram, int fs, float eps, float *Xout, int *status);
hipError_t launch_hermitian_ldlt_wide_implicit(bool ptr64, bool wide, hipStream_t st, const int32_t *perm, int64_t pos0,
                                               int64_t npos, const void *ptr, const int32_t *idx, const float *val,
                                               const void *Theta, float lambda, float alpha, const float *gram,
                                               float *Xout, int *status);
hipError_t launch_solve_ldlt_wide_implicit(bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                           int64_t pos0, int64_t npos, int64_t task0, const void *ptr,
                                           const float *slots, float lambda, const float *gram, float *Xout,
                                           int *status);
// exact update in the dual form for rows with fewer than 16 * ntd entries (dual.hip)
bool has_dual_exact(int f, int ntd);
hipError_t launch_dual_exact(int f, int ntd, bool ptr64, int et, hipStream_t st, const int32_t *perm, int64_t pos0,
                             int64_t npos, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                             float lambda, float *Xout, int *status);
hipError_t launch_solve_cg_wide(bool ptr64, bool s16, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                                int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                                float lambda, int fs, float eps, float *Xout, int *status);
hipError_t launch_reduce_slots(int f, bool s16, hipStream_t st, const int32_t *task_off, int64_t pos0, int64_t npos,
                               int64_t task0, float *slots);

hipError_t launch_export_dense(int f, bool ptr64, hipStream_t st, const int32_t *perm, const int32_t *task_off,
                               int64_t pos0, int64_t npos, int64_t task0, const void *ptr, const float *slots,
                               float lambda, int64_t row0, float *A_out, float *b_out);

hipError_t launch_sse(int f, bool ptr64, bool implicit, float alpha, hipStream_t st, const int32_t *task_row,
                      const int32_t *task_chunk, int64_t ntasks, int chunk, const void *ptr, const int32_t *idx,
                      const float *val, const float *X, const float *Theta, double *partial, double *total);

// implicit feedback (Section 5.6), f <= 128, fp32 slots; et: element type of the gathered factor
// G^T G of the n x f matrix G: nslots work items of `per` rows each (per a multiple of 4) -> slots -> out (tile layout)
// et: element type of G (16-bit only for f <= 128)
hipError_t launch_gram(int f, bool wide, int et, hipStream_t st, const void *G, int64_t n, int per, int nslots,
                       float *slots, float *out);
hipError_t launch_tiles_to_dense(int f, hipStream_t st, const float *tiles, float *out);
// als_gram_static: a file-scope device array of kGramStaticFloats floats (16 MiB) holds the slots and, after
// them, the summed tiles.  gram_static_scratch returns its address on the CURRENT device.
constexpr size_t kGramStaticFloats = (size_t)4 << 20;
constexpr int kGramStaticMaxSlots = 512;
hipError_t gram_static_scratch(float **ptr);
hipError_t launch_gram_dot(int f, hipStream_t st, const float *A, const float *B, double *out3);
// 16-bit factor inputs, f <= 128 (implicit16.hip); the two launchers below forward to these
hipError_t launch_hermitian_implicit16(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *task_row,
                                       const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks,
                                       int chunk, const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                       float alpha, float *slots);
hipError_t launch_hermitian_cg_implicit16(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st,
                                          const int32_t *perm, int64_t pos0, int64_t npos, const void *ptr,
                                          const int32_t *idx, const float *val, const void *Theta, float lambda,
                                          float alpha, const float *gram, int fs, float eps, float *Xout, int *status);
hipError_t launch_hermitian_implicit(int f, bool ptr64, bool wide, int et, hipStream_t st, const int32_t *task_row,
                                     const int32_t *task_chunk, const int32_t *task_order, int64_t task0, int64_t ntasks, int chunk,
                                     const void *ptr, const int32_t *idx, const float *val, const void *Theta,
                                     float alpha, float *slots);
hipError_t launch_hermitian_cg_implicit(int f, bool ptr64, bool wide, int et, int solver, hipStream_t st, const int32_t *perm,
                                        int64_t pos0, int64_t npos, const void *ptr, const int32_t *idx,
                                        const float *val, const void *Theta, float lambda, float alpha,
                                        const float *gram, int fs, float eps, float *Xout, int *status);
hipError_t launch_solve_wave_implicit(int f, bool ptr64, int solver, hipStream_t st, const int32_t *perm,
                                      const int32_t *task_off, int64_t pos0, int64_t npos, int64_t task0,
                                      const void *ptr, const float *slots, float lambda, const float *gram, int fs,
                                      float eps, float *Xout, int *status);

// plan.hip
// scratch: a buffer the two calls below grow on demand (hipFree + hipMalloc), unless scratch_fixed: then it is part
// of a caller's workspace, and a buffer smaller than plan_scratch_bytes(nrows, nclass) gives hipErrorOutOfMemory
size_t plan_scratch_bytes(int64_t nrows, int nclass);
hipError_t ensure_scratch(void **scratch, size_t *have, size_t need, bool fixed);
hipError_t plan_bin_rows(bool ptr64, hipStream_t st, int64_t nrows, const void *ptr, int nclass, int32_t *perm,
                         int32_t *class_start_dev /*nclass+1*/, void **scratch, size_t *scratch_bytes, bool scratch_fixed);
hipError_t plan_tasks(bool ptr64, hipStream_t st, int64_t nrows, const void *ptr, const int32_t *perm, int chunk,
                      int32_t *task_off /*nrows+1*/, void **scratch, size_t *scratch_bytes, bool scratch_fixed);
// order[first .. first+count) = the work items first .. first+count-1 sorted by key (stable); batches of more than
// kMaxRankedItems items keep their natural order
constexpr int64_t kMaxRankedItems = 1 << 18;
hipError_t plan_rank_order(hipStream_t st, const int32_t *key, int64_t first, int64_t count, int32_t *order);
hipError_t plan_emit(bool ptr64, hipStream_t st, int64_t nrows, const void *ptr, const int32_t *perm, int chunk,
                     const int32_t *task_off, int32_t *task_row, int32_t *task_chunk);
hipError_t fill_iota(hipStream_t st, int32_t *p, int64_t n, int32_t first);
// data[0 .. n) -> its exclusive prefix sums, in place (DEVICE; unsigned 32-bit sums); scratch: DEVICE,
// scan_scratch_ints(n) words
size_t scan_scratch_ints(int64_t n);
hipError_t exclusive_scan_u32(hipStream_t st, uint32_t *data, int64_t n, uint32_t *scratch);
hipError_t fill_zero(hipStream_t st, void *p, int64_t n);   // n 32-bit words, by a kernel
// validation of a matrix: bits ORed into *flags (DEVICE): 1 row offsets not 0 .. nnz ascending, 2 column id out of
// range, 4 column ids of a row not strictly ascending.  check_idx needs offsets that passed check_ptr.
hipError_t check_ptr(bool ptr64, hipStream_t st, const void *ptr, int64_t nrows, int64_t nnz, int *flags);
hipError_t check_idx(bool ptr64, hipStream_t st, const void *ptr, const int32_t *idx, int64_t nrows, int64_t ncols,
                     int64_t nnz, int *flags);
// *sum (DEVICE) += fingerprint of the n row offsets: a sum of mixed (position, offset) pairs, so the order of the
// additions does not matter.  *done (DEVICE, zero between launches) counts the finished workgroups.  With `want`
// (DEVICE): the last workgroup sets kStatusStalePlan in *status if the sum differs from *want, and clears *sum.
hipError_t plan_fingerprint(bool ptr64, hipStream_t st, const void *ptr, int64_t n, unsigned long long *sum,
                            unsigned int *done, const unsigned long long *want, int *status);
// key[t] = index of the first stored entry of work item t, t < ntasks (DEVICE arrays)
hipError_t plan_task_keys(bool ptr64, hipStream_t st, const void *ptr, const int32_t *idx, const int32_t *task_row,
                          const int32_t *task_chunk, int64_t ntasks, int chunk, int32_t *key);

// peaks.hip: the rates this machine sustains (see als_measure_peak)
hipError_t launch_mfma_peak(int et, hipStream_t st, int workgroups, int iters, float *sink, double *flops);
hipError_t launch_copy(hipStream_t st, int workgroups, const void *src, void *dst, int64_t bytes);

// transpose.hip
hipError_t transpose_csr(bool ptr64, hipStream_t st, int64_t nrows, int64_t ncols, int64_t nnz, const void *ptr,
                         const int32_t *idx, const float *val, void *cptr, int32_t *cidx, float *cval);

inline bool supported_f(int f) { return f == 16 || f == 32 || f == 64 || f == 100 || f == 128 || f == 256; }
// f whose lower triangle fits the registers of one wavefront (fused build+solve, wave-per-row CG)
inline bool single_wave_f(int f) { return f <= 128; }

}  // namespace als
