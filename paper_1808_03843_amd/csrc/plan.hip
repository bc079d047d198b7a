// Load balancing of the per-row work (not in the paper, which launches one thread block per row
// whatever its length, Section 3): rows are grouped by degree class, heaviest first, and rows
// longer than `chunk` stored entries are split into several work items.  Integer work only; the
// results are deterministic (stable counting sort built from ballots and prefix sums, no atomics).
#include "als_internal.h"

namespace als {

// ---- exclusive prefix sum of 32-bit counts, in place (unsigned: sums up to 2^32 - 1) -----------------
constexpr int kScanThreads = 256, kScanItems = 8, kScanBlock = kScanThreads * kScanItems;

__global__ __launch_bounds__(kScanThreads) void k_scan_block(uint32_t *__restrict__ data, int64_t n,
                                                             uint32_t *__restrict__ block_sums) {
    __shared__ uint32_t wave_tot[kScanThreads / 64];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems];
    uint32_t sum = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        v[q] = (base + q < n) ? data[base + q] : 0u;
        sum += v[q];
    }
    // inclusive scan of `sum` across the wavefront
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = (uint32_t)__shfl_up((int)inc, o);
        if (lane >= o) inc += t;
    }
    if (lane == 63) wave_tot[w] = inc;
    __syncthreads();
    uint32_t woff = 0, total = 0;
#pragma unroll
    for (int q = 0; q < kScanThreads / 64; ++q) {
        if (q < w) woff += wave_tot[q];
        total += wave_tot[q];
    }
    uint32_t run = woff + inc - sum;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q) {
        if (base + q < n) data[base + q] = run;
        run += v[q];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_add(uint32_t *__restrict__ data, int64_t n,
                                                           const uint32_t *__restrict__ block_offsets) {
    const uint32_t off = block_offsets[blockIdx.x];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
#pragma unroll
    for (int q = 0; q < kScanItems; ++q)
        if (base + q < n) data[base + q] += off;
}

size_t scan_scratch_ints(int64_t n) {
    size_t total = 0;
    while (n > 1) {
        n = (n + kScanBlock - 1) / kScanBlock;
        total += (size_t)n;
        if (n == 1) break;
    }
    return total + 1;
}

hipError_t exclusive_scan_u32(hipStream_t st, uint32_t *data, int64_t n, uint32_t *scratch) {
    if (n <= 0) return hipSuccess;
    const int64_t nb = (n + kScanBlock - 1) / kScanBlock;
    hipLaunchKernelGGL(k_scan_block, dim3((unsigned)nb), dim3(kScanThreads), 0, st, data, n, scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || nb == 1) return e;
    e = exclusive_scan_u32(st, scratch, nb, scratch + nb);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scan_add, dim3((unsigned)nb), dim3(kScanThreads), 0, st, data, n, scratch);
    return hipGetLastError();
}

// (the counts of the plans are non-negative int32: same bits)
static hipError_t exclusive_scan(hipStream_t st, int32_t *data, int64_t n, int32_t *scratch) {
    return exclusive_scan_u32(st, reinterpret_cast<uint32_t *>(data), n, reinterpret_cast<uint32_t *>(scratch));
}

size_t plan_scratch_bytes(int64_t nrows, int nclass) {
    const int64_t nseg = (nrows + 63) / 64;
    const int64_t ncount = (int64_t)nclass * nseg + 1;
    const size_t bin = (size_t)(ncount + scan_scratch_ints(ncount)) * sizeof(int32_t);
    const size_t tasks = scan_scratch_ints(nrows + 1) * sizeof(int32_t);
    return bin > tasks ? bin : tasks;
}

// fixed: the buffer belongs to a caller's workspace and can neither grow nor be freed here
hipError_t ensure_scratch(void **scratch, size_t *have, size_t need, bool fixed) {
    if (*have >= need) return hipSuccess;
    if (fixed) return hipErrorOutOfMemory;
    if (*scratch) {
        hipError_t e = hipFree(*scratch);
        if (e != hipSuccess) return e;
        *scratch = nullptr;
        *have = 0;
    }
    hipError_t e = hipMalloc(scratch, need);
    if (e == hipSuccess) *have = need;
    return e;
}

// ---- degree classes -----------------------------------------------------------------------------
__device__ __forceinline__ int degree_class(int64_t n_u, int nclass) {
    if (n_u <= 0) return 0;
    const int c = 1 + (63 - __clzll((long long)n_u));
    return c < nclass ? c : nclass - 1;
}

// counts[slot * nseg + seg] = rows of the 64-row segment whose class is nclass-1-slot
template <typename PtrT>
__global__ __launch_bounds__(256) void k_class_hist(const PtrT *__restrict__ ptr, int64_t nrows, int nclass,
                                                    int64_t nseg, int32_t *__restrict__ counts) {
    const int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (seg >= nseg) return;
    const int lane = threadIdx.x & 63;
    const int64_t row = seg * 64 + lane;
    const int slot = (row < nrows) ? nclass - 1 - degree_class((int64_t)ptr[row + 1] - (int64_t)ptr[row], nclass) : -1;
    int32_t mine = 0;
    for (int s = 0; s < nclass; ++s) {
        const unsigned long long m = __ballot(slot == s);
        if (lane == s) mine = __popcll(m);
    }
    if (lane < nclass) counts[(int64_t)lane * nseg + seg] = mine;
}

template <typename PtrT>
__global__ __launch_bounds__(256) void k_class_scatter(const PtrT *__restrict__ ptr, int64_t nrows, int nclass,
                                                       int64_t nseg, const int32_t *__restrict__ offsets,
                                                       int32_t *__restrict__ perm) {
    const int64_t seg = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (seg >= nseg) return;
    const int lane = threadIdx.x & 63;
    const int64_t row = seg * 64 + lane;
    const int slot = (row < nrows) ? nclass - 1 - degree_class((int64_t)ptr[row + 1] - (int64_t)ptr[row], nclass) : -1;
    unsigned long long same = 0;
    for (int s = 0; s < nclass; ++s) {
        const unsigned long long m = __ballot(slot == s);
        if (slot == s) same = m;
    }
    if (slot >= 0) {
        const int rank = __popcll(same & ((1ull << lane) - 1ull));
        perm[offsets[(int64_t)slot * nseg + seg] + rank] = (int32_t)row;
    }
}

__global__ void k_class_start(const int32_t *__restrict__ offsets, int nclass, int64_t nseg,
                              int32_t *__restrict__ class_start) {
    const int s = threadIdx.x;
    if (s <= nclass) class_start[s] = offsets[(int64_t)s * nseg];  // entry nclass*nseg holds the total
}

__global__ void k_set_zero(int32_t *p) { *p = 0; }

hipError_t plan_bin_rows(bool ptr64, hipStream_t st, int64_t nrows, const void *ptr, int nclass, int32_t *perm,
                         int32_t *class_start_dev, void **scratch, size_t *scratch_bytes, bool scratch_fixed) {
    if (nclass < 2 || nclass > 64) return hipErrorInvalidValue;
    const int64_t nseg = (nrows + 63) / 64;
    const int64_t ncount = (int64_t)nclass * nseg + 1;
    const size_t need = (size_t)(ncount + scan_scratch_ints(ncount)) * sizeof(int32_t);
    hipError_t e = ensure_scratch(scratch, scratch_bytes, need, scratch_fixed);
    if (e != hipSuccess) return e;
    int32_t *counts = (int32_t *)*scratch;
    if (nseg > 0) {
        const unsigned nb = (unsigned)((nseg + 3) / 4);
        if (ptr64)
            hipLaunchKernelGGL((k_class_hist<int64_t>), dim3(nb), dim3(256), 0, st, (const int64_t *)ptr, nrows,
                               nclass, nseg, counts);
        else
            hipLaunchKernelGGL((k_class_hist<int32_t>), dim3(nb), dim3(256), 0, st, (const int32_t *)ptr, nrows,
                               nclass, nseg, counts);
    }
    hipLaunchKernelGGL(k_set_zero, dim3(1), dim3(1), 0, st, counts + ncount - 1);
    e = exclusive_scan(st, counts, ncount, counts + ncount);
    if (e != hipSuccess) return e;
    if (nseg > 0) {
        const unsigned nb = (unsigned)((nseg + 3) / 4);
        if (ptr64)
            hipLaunchKernelGGL((k_class_scatter<int64_t>), dim3(nb), dim3(256), 0, st, (const int64_t *)ptr, nrows,
                               nclass, nseg, counts, perm);
        else
            hipLaunchKernelGGL((k_class_scatter<int32_t>), dim3(nb), dim3(256), 0, st, (const int32_t *)ptr, nrows,
                               nclass, nseg, counts, perm);
    }
    if (class_start_dev)
        hipLaunchKernelGGL(k_class_start, dim3(1), dim3(128), 0, st, counts, nclass, nseg, class_start_dev);
    return hipGetLastError();
}

// ---- work items -----------------------------------------------------------------------------------
template <typename PtrT>
__global__ __launch_bounds__(256) void k_count_items(const PtrT *__restrict__ ptr, const int32_t *__restrict__ perm,
                                                     int64_t nrows, int chunk, int32_t *__restrict__ task_off) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > nrows) return;
    int32_t nt = 0;
    if (i < nrows) {
        const int row = perm[i];
        const int64_t n_u = (int64_t)ptr[row + 1] - (int64_t)ptr[row];
        nt = (int32_t)((n_u + chunk - 1) / chunk);
    }
    task_off[i] = nt;
}

hipError_t plan_tasks(bool ptr64, hipStream_t st, int64_t nrows, const void *ptr, const int32_t *perm, int chunk,
                      int32_t *task_off, void **scratch, size_t *scratch_bytes, bool scratch_fixed) {
    const size_t need = scan_scratch_ints(nrows + 1) * sizeof(int32_t);
    hipError_t e = ensure_scratch(scratch, scratch_bytes, need, scratch_fixed);
    if (e != hipSuccess) return e;
    const unsigned nb = (unsigned)((nrows + 1 + 255) / 256);
    if (ptr64)
        hipLaunchKernelGGL((k_count_items<int64_t>), dim3(nb), dim3(256), 0, st, (const int64_t *)ptr, perm, nrows,
                           chunk, task_off);
    else
        hipLaunchKernelGGL((k_count_items<int32_t>), dim3(nb), dim3(256), 0, st, (const int32_t *)ptr, perm, nrows,
                           chunk, task_off);
    return exclusive_scan(st, task_off, nrows + 1, (int32_t *)*scratch);
}

__global__ __launch_bounds__(256) void k_emit_items(const int32_t *__restrict__ perm,
                                                    const int32_t *__restrict__ task_off, int64_t nrows,
                                                    int32_t *__restrict__ task_row, int32_t *__restrict__ task_chunk) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nrows) return;
    const int row = perm[i];
    const int32_t a = task_off[i], b = task_off[i + 1];
    for (int32_t t = a; t < b; ++t) {
        task_row[t] = row;
        task_chunk[t] = t - a;
    }
}

hipError_t plan_emit(bool, hipStream_t st, int64_t nrows, const void *, const int32_t *perm, int,
                     const int32_t *task_off, int32_t *task_row, int32_t *task_chunk) {
    if (nrows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_emit_items, dim3((unsigned)((nrows + 255) / 256)), dim3(256), 0, st, perm, task_off, nrows,
                       task_row, task_chunk);
    return hipGetLastError();
}

// key[t] = index of the first stored entry of work item t (its position in the gathered factor matrix)
template <typename PtrT>
__global__ __launch_bounds__(256) void k_task_keys(const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                   const int32_t *__restrict__ task_row,
                                                   const int32_t *__restrict__ task_chunk, int64_t ntasks, int chunk,
                                                   int32_t *__restrict__ key) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntasks) return;
    key[t] = idx[(int64_t)ptr[task_row[t]] + (int64_t)task_chunk[t] * chunk];
}

hipError_t plan_task_keys(bool ptr64, hipStream_t st, const void *ptr, const int32_t *idx, const int32_t *task_row,
                          const int32_t *task_chunk, int64_t ntasks, int chunk, int32_t *key) {
    if (ntasks <= 0) return hipSuccess;
    const dim3 grid((unsigned)((ntasks + 255) / 256)), block(256);
    if (ptr64)
        hipLaunchKernelGGL(k_task_keys<int64_t>, grid, block, 0, st, (const int64_t *)ptr, idx, task_row, task_chunk, ntasks,
                           chunk, key);
    else
        hipLaunchKernelGGL(k_task_keys<int32_t>, grid, block, 0, st, (const int32_t *)ptr, idx, task_row, task_chunk, ntasks,
                           chunk, key);
    return hipGetLastError();
}

// Stable sort of the work items [first, first + count) of one batch by key, by counting: the rank of item t is the
// number of items with a smaller key, or the same key and a smaller index.  order[first + rank] = first + t.
// Quadratic, but a batch has at most a few hundred thousand items, it runs once per matrix, and it needs no
// temporary memory and no atomics.
constexpr int kRankTile = 1024;
__global__ __launch_bounds__(256) void k_rank_order(const int32_t *__restrict__ key, int64_t first, int count,
                                                    int32_t *__restrict__ order) {
    __shared__ int32_t tile[kRankTile];
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int32_t mine = t < count ? key[first + t] : 0;
    int rank = 0;
    for (int base = 0; base < count; base += kRankTile) {
        __syncthreads();
        for (int q = threadIdx.x; q < kRankTile; q += 256) tile[q] = base + q < count ? key[first + base + q] : 0;
        __syncthreads();
        const int lim = count - base < kRankTile ? count - base : kRankTile;
        for (int q = 0; q < lim; ++q) {
            const int32_t k = tile[q];
            rank += (k < mine || (k == mine && base + q < t)) ? 1 : 0;
        }
    }
    if (t < count) order[first + rank] = (int32_t)(first + t);
}

hipError_t plan_rank_order(hipStream_t st, const int32_t *key, int64_t first, int64_t count, int32_t *order) {
    if (count <= 0) return hipSuccess;
    if (count > kMaxRankedItems) return fill_iota(st, order + first, count, (int32_t)first);   // too many to rank: batch order
    hipLaunchKernelGGL(k_rank_order, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, key, first, (int)count, order);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_iota(int32_t *__restrict__ p, int64_t n, int32_t first) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = first + (int32_t)i;
}

hipError_t fill_iota(hipStream_t st, int32_t *p, int64_t n, int32_t first) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_iota, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, first);
    return hipGetLastError();
}

// ---- validation of a caller's matrix (als_check_matrix) ----
constexpr int kBadPtr = 1, kBadIndex = 2, kBadOrder = 4;

template <typename PtrT>
__global__ __launch_bounds__(256) void k_check_ptr(const PtrT *__restrict__ ptr, int64_t nrows, int64_t nnz,
                                                   int *__restrict__ flags) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool bad = false;
    if (i < nrows) bad = (int64_t)ptr[i] > (int64_t)ptr[i + 1] || (int64_t)ptr[i] < 0;
    if (i == 0) bad = bad || (int64_t)ptr[0] != 0 || (int64_t)ptr[nrows] != nnz;
    if (bad) atomicOr(flags, kBadPtr);
}

// ptr has passed k_check_ptr.  Every column id in range; ids ascending inside a row: where idx[e+1] <= idx[e],
// entry e+1 must be the first of a row, i.e. some ptr[i] == e+1 (binary search, needed about once per row).
template <typename PtrT>
__global__ __launch_bounds__(256) void k_check_idx(const PtrT *__restrict__ ptr, const int32_t *__restrict__ idx,
                                                   int64_t nrows, int64_t ncols, int64_t nnz, int *__restrict__ flags) {
    int bad = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
        const int32_t c = idx[e];
        if (c < 0 || c >= ncols) bad |= kBadIndex;
        if (e + 1 < nnz && idx[e + 1] <= c) {
            int64_t lo = 0, hi = nrows;   // first i with ptr[i] >= e + 1
            while (lo < hi) {
                const int64_t mid = (lo + hi) >> 1;
                if ((int64_t)ptr[mid] < e + 1) lo = mid + 1; else hi = mid;
            }
            if ((int64_t)ptr[lo] != e + 1) bad |= kBadOrder;
        }
    }
    if (bad) atomicOr(flags, bad);
}

hipError_t check_ptr(bool ptr64, hipStream_t st, const void *ptr, int64_t nrows, int64_t nnz, int *flags) {
    const dim3 grid((unsigned)((nrows + 256) / 256)), block(256);   // at least one workgroup: thread 0 checks the ends
    if (ptr64) hipLaunchKernelGGL(k_check_ptr<int64_t>, grid, block, 0, st, (const int64_t *)ptr, nrows, nnz, flags);
    else hipLaunchKernelGGL(k_check_ptr<int32_t>, grid, block, 0, st, (const int32_t *)ptr, nrows, nnz, flags);
    return hipGetLastError();
}

hipError_t check_idx(bool ptr64, hipStream_t st, const void *ptr, const int32_t *idx, int64_t nrows, int64_t ncols,
                     int64_t nnz, int *flags) {
    if (nnz <= 0) return hipSuccess;
    int64_t nb = (nnz + 255) / 256;
    if (nb > 65536) nb = 65536;
    const dim3 grid((unsigned)nb), block(256);
    if (ptr64)
        hipLaunchKernelGGL(k_check_idx<int64_t>, grid, block, 0, st, (const int64_t *)ptr, idx, nrows, ncols, nnz, flags);
    else
        hipLaunchKernelGGL(k_check_idx<int32_t>, grid, block, 0, st, (const int32_t *)ptr, idx, nrows, ncols, nnz, flags);
    return hipGetLastError();
}

// finaliser of a 64-bit hash (xor-shift and odd multipliers): spreads every input bit over the word
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x ^= x >> 33;
    x *= 0xff51afd7ed558ccdull;
    x ^= x >> 33;
    x *= 0xc4ceb9fe1a85ec53ull;
    x ^= x >> 33;
    return x;
}

// *sum += fingerprint of ptr[0 .. n).  The workgroup that finishes last (a ticket counter, *done, which it puts back
// to zero) sees the complete sum: with `want` given it compares, flags a mismatch in *status and clears *sum for the
// next call; without, the sum stays where it is (the fingerprint a plan is built with).
template <typename PtrT>
__global__ __launch_bounds__(256) void k_fingerprint(const PtrT *__restrict__ ptr, int64_t n,
                                                     unsigned long long *__restrict__ sum, unsigned int *__restrict__ done,
                                                     const unsigned long long *__restrict__ want,
                                                     int *__restrict__ status) {
    __shared__ unsigned long long part[4];
    uint64_t h = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        h += mix64((uint64_t)ptr[i] + 0x9e3779b97f4a7c15ull * (uint64_t)(i + 1));
    for (int o = 32; o > 0; o >>= 1) h += (uint64_t)__shfl_down((unsigned long long)h, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
    __syncthreads();
    if (threadIdx.x != 0) return;
    // one atomic per workgroup (many on one address would queue up); an integer sum: any order gives the same word
    atomicAdd(sum, part[0] + part[1] + part[2] + part[3]);
    __threadfence();
    if (atomicAdd(done, 1u) != gridDim.x - 1) return;
    __threadfence();
    *done = 0u;
    if (want) {
        const unsigned long long total = atomicExch(sum, 0ull);
        if (total != *want) atomicOr(status, kStatusStalePlan);
    }
}

hipError_t plan_fingerprint(bool ptr64, hipStream_t st, const void *ptr, int64_t n, unsigned long long *sum,
                            unsigned int *done, const unsigned long long *want, int *status) {
    if (n <= 0) return hipSuccess;
    int64_t nb = (n + 1023) / 1024;   // at least four offsets per thread; few workgroups, since each ends in an atomic
    if (nb > 1024) nb = 1024;
    if (ptr64)
        hipLaunchKernelGGL(k_fingerprint<int64_t>, dim3((unsigned)nb), dim3(256), 0, st, (const int64_t *)ptr, n, sum, done,
                           want, status);
    else
        hipLaunchKernelGGL(k_fingerprint<int32_t>, dim3((unsigned)nb), dim3(256), 0, st, (const int32_t *)ptr, n, sum, done,
                           want, status);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_fill_zero(uint32_t *__restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// n 32-bit words set to zero by a kernel (a memset node in a captured graph is avoided on purpose)
hipError_t fill_zero(hipStream_t st, void *p, int64_t n) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t *)p, n);
    return hipGetLastError();
}

}  // namespace als
