// Compressed columns of R from its compressed rows: the CSC that "Update Theta" (eq. (3)) walks.
// A stable sort of the stored entries by column id keeps the rows of every column ascending, so the result is the
// canonical CSC and is reproducible bit for bit.  The sort is a least-significant-digit radix sort of (column id,
// position of the entry) pairs, one to three passes of up to 11 bits: per pass a digit histogram of every tile, one
// prefix sum over (digit, tile), and a scatter in which one wavefront walks its tile in order and ranks equal digits
// with ballots (no atomics whose order could matter).  Off the per-sweep path: once per matrix.
#include <cstring>

#include "als_internal.h"

namespace als {

template <typename PtrT>
__device__ __forceinline__ int64_t row_of_entry(const PtrT *__restrict__ ptr, int64_t nrows, int64_t q) {
    // largest row with ptr[row] <= q
    int64_t lo = 0, hi = nrows;  // ptr[lo] <= q < ptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)ptr[mid] <= q) lo = mid; else hi = mid;
    }
    return lo;
}

constexpr int kMaxDigitBits = 11;
constexpr int64_t kMinTile = 2048;            // keys per tile, a power of two, doubled until ...
constexpr int64_t kMaxCounts = 1ll << 25;     // ... (tiles x digits) stays below this many counters (128 MB)

// counts[d * ntiles + t] = number of keys of tile t whose digit (bits shift .. shift+bits-1) is d
__global__ __launch_bounds__(256) void k_digit_hist(const uint32_t *__restrict__ keys, int64_t n, int64_t tile, int shift,
                                                    int bits, int64_t ntiles, uint32_t *__restrict__ counts) {
    __shared__ uint32_t cnt[1 << kMaxDigitBits];
    const int nd = 1 << bits;
    for (int d = threadIdx.x; d < nd; d += 256) cnt[d] = 0u;
    __syncthreads();
    const int64_t t = blockIdx.x, lo = t * tile, hi = lo + tile < n ? lo + tile : n;
    for (int64_t q = lo + threadIdx.x; q < hi; q += 256) atomicAdd(&cnt[(keys[q] >> shift) & (uint32_t)(nd - 1)], 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < nd; d += 256) counts[(int64_t)d * ntiles + t] = cnt[d];
}

// One wavefront per tile.  offsets[d * ntiles + t]: where the keys of tile t with digit d start in the output (the
// prefix sums of the counts).  The wavefront takes its keys 64 at a time, in order; lanes with the same digit find
// each other with one ballot per digit bit, and the lower lanes of such a group come first: the pass is stable.
// vals == nullptr: the value of a key is its position (first pass).
__global__ __launch_bounds__(64) void k_digit_scatter(const uint32_t *__restrict__ keys, const uint32_t *__restrict__ vals,
                                                      int64_t n, int64_t tile, int shift, int bits, int64_t ntiles,
                                                      const uint32_t *__restrict__ offsets,
                                                      uint32_t *__restrict__ keys_out, uint32_t *__restrict__ vals_out) {
    __shared__ uint32_t next[1 << kMaxDigitBits];   // next free output position of every digit, for this tile
    const int lane = threadIdx.x, nd = 1 << bits;
    const int64_t t = blockIdx.x, lo = t * tile, hi = lo + tile < n ? lo + tile : n;
    for (int d = lane; d < nd; d += 64) next[d] = offsets[(int64_t)d * ntiles + t];
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int64_t q0 = lo; q0 < hi; q0 += 64) {
        const int64_t q = q0 + lane;
        const bool ok = q < hi;
        const uint32_t key = ok ? keys[q] : 0u;
        const uint32_t val = ok ? (vals ? vals[q] : (uint32_t)q) : 0u;
        const uint32_t d = (key >> shift) & (uint32_t)(nd - 1);
        unsigned long long same = __ballot(ok);
        for (int k = 0; k < bits; ++k) {
            const bool bit = ((d >> k) & 1u) != 0u;
            const unsigned long long m = __ballot(bit);
            same &= bit ? m : ~m;
        }
        // (one wavefront: its LDS reads and writes are performed in program order, so every lane of a group has read
        // next[d] before the first lane of the group moves it on)
        uint32_t base = 0u;
        if (ok) base = next[d];
        const uint32_t rank = (uint32_t)__popcll(same & below);
        if (ok) {
            keys_out[base + rank] = key;
            vals_out[base + rank] = val;
            if (rank == 0u) next[d] = base + (uint32_t)__popcll(same);
        }
        __syncthreads();   // (a single wavefront: orders the LDS write above before the next round's reads)
    }
}

template <typename PtrT>
__global__ __launch_bounds__(256) void k_gather_entries(const PtrT *__restrict__ ptr, int64_t nrows, int64_t nnz,
                                                        const uint32_t *__restrict__ order,
                                                        const float *__restrict__ val, int32_t *__restrict__ cidx,
                                                        float *__restrict__ cval) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= nnz) return;
    const int64_t q = order[j];
    cidx[j] = (int32_t)row_of_entry(ptr, nrows, q);
    cval[j] = val[q];
}

template <typename PtrT>
__global__ __launch_bounds__(256) void k_column_starts(const uint32_t *__restrict__ sorted_cols, int64_t nnz,
                                                       int64_t ncols, PtrT *__restrict__ cptr) {
    const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (v > ncols) return;
    int64_t lo = 0, hi = nnz;  // first position whose column id is >= v
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)sorted_cols[mid] < v) lo = mid + 1; else hi = mid;
    }
    cptr[v] = (PtrT)lo;
}

template <typename PtrT>
static hipError_t transpose_t(hipStream_t st, int64_t nrows, int64_t ncols, int64_t nnz, const PtrT *ptr,
                              const int32_t *idx, const float *val, PtrT *cptr, int32_t *cidx, float *cval) {
    hipError_t e = hipSuccess;
    uint32_t *keys[2] = {nullptr, nullptr}, *vals[2] = {nullptr, nullptr}, *counts = nullptr;
    auto cleanup = [&]() {
        for (int k = 0; k < 2; ++k) { (void)hipFree(keys[k]); (void)hipFree(vals[k]); }
        (void)hipFree(counts);
    };
    int key_bits = 1;   // bits of the largest column id
    while (key_bits < 32 && (1ll << key_bits) < ncols) ++key_bits;
    const int npass = (key_bits + kMaxDigitBits - 1) / kMaxDigitBits, bits = (key_bits + npass - 1) / npass;
    const uint32_t *sorted_cols = nullptr;
    if (nnz > 0) {
        int64_t tile = kMinTile;
        while ((((nnz + tile - 1) / tile) << bits) > kMaxCounts) tile *= 2;
        const int64_t ntiles = (nnz + tile - 1) / tile, ncount = ntiles << bits;
        for (int k = 0; k < (npass > 1 ? 2 : 1); ++k) {
            if ((e = hipMalloc(&keys[k], sizeof(uint32_t) * nnz)) != hipSuccess) { cleanup(); return e; }
            if ((e = hipMalloc(&vals[k], sizeof(uint32_t) * nnz)) != hipSuccess) { cleanup(); return e; }
        }
        if ((e = hipMalloc(&counts, sizeof(uint32_t) * (ncount + scan_scratch_ints(ncount)))) != hipSuccess) { cleanup(); return e; }
        const uint32_t *kin = reinterpret_cast<const uint32_t *>(idx), *vin = nullptr;   // first pass: value = position
        for (int p = 0; p < npass; ++p) {
            uint32_t *kout = keys[p & 1], *vout = vals[p & 1];
            hipLaunchKernelGGL(k_digit_hist, dim3((unsigned)ntiles), dim3(256), 0, st, kin, nnz, tile, p * bits, bits, ntiles, counts);
            if ((e = hipGetLastError()) != hipSuccess) { cleanup(); return e; }
            if ((e = exclusive_scan_u32(st, counts, ncount, counts + ncount)) != hipSuccess) { cleanup(); return e; }
            hipLaunchKernelGGL(k_digit_scatter, dim3((unsigned)ntiles), dim3(64), 0, st, kin, vin, nnz, tile, p * bits, bits, ntiles,
                               counts, kout, vout);
            if ((e = hipGetLastError()) != hipSuccess) { cleanup(); return e; }
            kin = kout;
            vin = vout;
        }
        sorted_cols = kin;
        hipLaunchKernelGGL((k_gather_entries<PtrT>), dim3((unsigned)((nnz + 255) / 256)), dim3(256), 0, st, ptr, nrows, nnz, vin, val,
                           cidx, cval);
    }
    hipLaunchKernelGGL((k_column_starts<PtrT>), dim3((unsigned)((ncols + 1 + 255) / 256)), dim3(256), 0, st,
                       sorted_cols, nnz, ncols, cptr);
    e = hipGetLastError();
    hipError_t e2 = hipStreamSynchronize(st);  // the temporaries are freed below
    cleanup();
    return e != hipSuccess ? e : e2;
}

hipError_t transpose_csr(bool ptr64, hipStream_t st, int64_t nrows, int64_t ncols, int64_t nnz, const void *ptr,
                         const int32_t *idx, const float *val, void *cptr, int32_t *cidx, float *cval) {
    if (ptr64)
        return transpose_t<int64_t>(st, nrows, ncols, nnz, (const int64_t *)ptr, idx, val, (int64_t *)cptr, cidx,
                                    cval);
    return transpose_t<int32_t>(st, nrows, ncols, nnz, (const int32_t *)ptr, idx, val, (int32_t *)cptr, cidx, cval);
}

}  // namespace als
