// Compressed columns of R from its compressed rows: the CSC that "Update Theta" (eq. (3)) walks.
// A stable radix sort of the stored entries by column id (rocPRIM, a library primitive for a step
// that is not on the per-sweep path) keeps the rows of every column ascending, so the result is
// the canonical CSC and is reproducible bit for bit.
#include <cstring>

#include <rocprim/rocprim.hpp>

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

__global__ __launch_bounds__(256) void k_iota_u32(uint32_t *__restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (uint32_t)i;
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
    hipError_t e;
    uint32_t *keys_out = nullptr, *vals_in = nullptr, *vals_out = nullptr;
    void *temp = nullptr;
    size_t temp_bytes = 0;
    unsigned end_bit = 1;
    while (end_bit < 32 && (1ll << end_bit) < ncols) ++end_bit;
    const uint32_t *keys_in = reinterpret_cast<const uint32_t *>(idx);
    auto cleanup = [&]() {
        (void)hipFree(keys_out); (void)hipFree(vals_in); (void)hipFree(vals_out); (void)hipFree(temp);
    };
    if (nnz > 0) {
        if ((e = hipMalloc(&keys_out, sizeof(uint32_t) * nnz)) != hipSuccess) { cleanup(); return e; }
        if ((e = hipMalloc(&vals_in, sizeof(uint32_t) * nnz)) != hipSuccess) { cleanup(); return e; }
        if ((e = hipMalloc(&vals_out, sizeof(uint32_t) * nnz)) != hipSuccess) { cleanup(); return e; }
        e = rocprim::radix_sort_pairs(nullptr, temp_bytes, keys_in, keys_out, vals_in, vals_out, (size_t)nnz, 0u,
                                      end_bit, st);
        if (e != hipSuccess) { cleanup(); return e; }
        if ((e = hipMalloc(&temp, temp_bytes ? temp_bytes : 16)) != hipSuccess) { cleanup(); return e; }
        const unsigned nb = (unsigned)((nnz + 255) / 256);
        hipLaunchKernelGGL(k_iota_u32, dim3(nb), dim3(256), 0, st, vals_in, nnz);
        e = rocprim::radix_sort_pairs(temp, temp_bytes, keys_in, keys_out, vals_in, vals_out, (size_t)nnz, 0u,
                                      end_bit, st);
        if (e != hipSuccess) { cleanup(); return e; }
        hipLaunchKernelGGL((k_gather_entries<PtrT>), dim3(nb), dim3(256), 0, st, ptr, nrows, nnz, vals_out, val,
                           cidx, cval);
    }
    hipLaunchKernelGGL((k_column_starts<PtrT>), dim3((unsigned)((ncols + 1 + 255) / 256)), dim3(256), 0, st,
                       keys_out, nnz, ncols, cptr);
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
