// C ABI of libals_gfx950 (see include/als.h): argument checks, the cached per-matrix plan, the
// batch loop of an update half-sweep, error bookkeeping.  No arithmetic of the method lives here.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "als_internal.h"

using namespace als;

namespace {

// 32-bit byte offsets into the gathered factor matrix are enough below 4 GiB; row pitches that are not a power
// of two are multiplied with a 24-bit instruction, which also limits the row index
bool needs_wide_offsets(int64_t rows, int f, size_t esize) {
    const uint64_t pitch = (uint64_t)f * esize;
    if ((uint64_t)rows * pitch >= (1ull << 32)) return true;
    return (pitch & (pitch - 1)) != 0 && rows >= (1 << 24);
}
bool fp32_in_memory(int factor_dtype) { return factor_dtype == ALS_F32 || factor_dtype == ALS_F32X3 || factor_dtype == ALS_F32X2; }
size_t factor_bytes(int factor_dtype) { return fp32_in_memory(factor_dtype) ? 4 : 2; }
constexpr int kPlanClasses = 24;
constexpr int kMaxPlans = 4;

// ---- layout of a caller's workspace ---------------------------------------------------------------------------
constexpr size_t kAlign = 256;
constexpr size_t aligned(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }
// upper bounds that hold for every matrix with `rows` rows and `nnz` stored entries: a row of n_u entries has
// ceil(n_u / chunk) work items, and only rows with n_u >= chunk (fewer than 2 n_u / chunk items each) use slots
int64_t max_tasks(int64_t rows, int64_t nnz, int chunk) { return rows + nnz / chunk; }
int64_t max_slot_tasks(int64_t rows, int64_t nnz, int chunk) {
    const int64_t a = max_tasks(rows, nnz, chunk), b = 2 * nnz / chunk;
    return a < b ? a : b;
}
size_t plan_bytes_bound(int64_t rows, int64_t nnz, int chunk) {
    const size_t t = (size_t)max_tasks(rows, nnz, chunk), s = (size_t)max_slot_tasks(rows, nnz, chunk);
    return aligned(4 * (size_t)(rows > 0 ? rows : 1)) + aligned(4 * (size_t)(rows + 1)) + 2 * aligned(4 * (t > 0 ? t : 1)) +
           aligned(4 * (s > 0 ? s : 1)) + aligned(16);
}
size_t slot_bytes(const als_config &c) {
    return sizeof(float) * (size_t)(c.herm_dtype == ALS_BF16 ? slot_words16(c.f) : slot_floats(c.f));
}
struct WorkspaceLayout {   // byte offsets of the pieces; `total` is what als_workspace_bytes returns
    size_t fixed_words, gram0, gram1, sse_partial, scratch, scratch_bytes, slots, arena, arena_bytes, total;
    int64_t slot_capacity;
};
// cfg: chunk and batch_slots already resolved (no zeros)
WorkspaceLayout workspace_layout(const als_config &c, int64_t rows, int64_t nnz) {
    WorkspaceLayout L{};
    size_t o = 0;
    L.fixed_words = o; o += aligned(1024);   // status, check flags, fingerprint + counter, sums, class starts
    L.gram0 = o; o += aligned(sizeof(float) * (size_t)slot_floats(c.f));
    L.gram1 = o; o += aligned(sizeof(float) * (size_t)slot_floats(c.f));
    L.sse_partial = o; o += aligned(sizeof(double) * (size_t)(max_tasks(rows, nnz, c.chunk) + 1));
    // plan scratch; also holds the sort keys of the slot work items (one int each)
    L.scratch_bytes = plan_scratch_bytes(rows, kPlanClasses);
    const size_t keys = 4 * (size_t)(max_slot_tasks(rows, nnz, c.chunk) + 1);
    if (keys > L.scratch_bytes) L.scratch_bytes = keys;
    L.scratch_bytes = aligned(L.scratch_bytes);
    L.scratch = o; o += L.scratch_bytes;
    L.slot_capacity = max_slot_tasks(rows, nnz, c.chunk) + 1;
    if (L.slot_capacity > c.batch_slots) L.slot_capacity = c.batch_slots;
    L.slots = o; o += aligned((size_t)L.slot_capacity * slot_bytes(c));
    L.arena_bytes = 2 * plan_bytes_bound(rows, nnz, c.chunk);
    L.arena = o; o += L.arena_bytes;
    L.total = o;
    return L;
}
#ifndef ALS_TASK_ORDER
#define ALS_TASK_ORDER 1
#endif
constexpr bool kTaskOrder = ALS_TASK_ORDER != 0;   // band order of the work items of a batch (build_order)
#ifndef ALS_DUAL_EXACT
#define ALS_DUAL_EXACT 1
#endif
constexpr bool kDualExact = ALS_DUAL_EXACT != 0;   // dual-form exact solve of rows with n_u < f (dual.hip)

// Rows with fewer stored entries than this run Algorithm 1 on their gathered rows (cg_short.hip) instead of building
// A_u; 0: no row does.  64 entries fit the registers of one wavefront (two at f = 256).  On the fp32 MFMA path at
// f >= 100, where building A_u is the expensive part, rows of 64 .. 127 entries go the same way with two wavefronts
// per row (Mid shape: 19.1 -> 18.7 ms per sweep; with 16-bit matrix cores or a narrower A_u the dense route is as fast).
int short_row_limit(const als_config &c) {
    if (c.solver != ALS_SOLVER_CG || c.dense_short_rows) return 0;
    return (c.factor_dtype == ALS_F32 && (c.f == 100 || c.f == 128)) ? 128 : 64;
}

struct TimedLaunch { hipEvent_t a, b; int kernel; };
}  // namespace

struct als_ctx {
    als_config cfg;
    hipStream_t stream = nullptr;
    std::string err;
    Plan plans[kMaxPlans];
    int next_plan = 0;
    float *slots = nullptr;
    size_t slots_bytes = 0;
    void *scratch = nullptr;
    size_t scratch_bytes = 0;
    int *status = nullptr;       // DEVICE status word
    int *check_flags = nullptr;  // DEVICE: result word of als_check_matrix
    unsigned long long *fp_now = nullptr;   // DEVICE: fingerprint of the row offsets of the current call (zero between calls),
                                            // followed by the 32-bit count of finished workgroups (fp_done)
    unsigned int *fp_done = nullptr;
    uint32_t *absmax = nullptr;  // DEVICE: bits of max |gathered factor| of the current update (factor_dtype ALS_F32X2)
    double *sse_partial = nullptr;
    size_t sse_partial_bytes = 0;
    double *sse_total = nullptr; // DEVICE
    float *gram[2] = {nullptr, nullptr};   // DEVICE, tile layout: G^T G of the gathered factor (implicit mode)
    double *gram_dot = nullptr;            // DEVICE, 3 doubles
    float *gram_static = nullptr;          // DEVICE: this device's copy of the file-scope scratch of als_gram_static
    // caller-owned workspace (cfg.workspace != nullptr): every device buffer above is a piece of it
    bool fixed = false;                    // true: nothing here is ever hipMalloc'ed or hipFree'd
    int32_t *class_start_dev = nullptr;    // DEVICE [kPlanClasses + 1] (workspace mode; a temporary otherwise)
    char *arena = nullptr;                 // the part of the workspace that holds the plans, filled front to back
    size_t arena_bytes = 0, arena_used = 0;
    int64_t slot_capacity = 0;             // workspace mode: slots the slot region holds (of the configured storage type)
    std::vector<TimedLaunch> timed;
    std::vector<hipEvent_t> free_events;
};

namespace {

// Makes the context's device current for the duration of a call and puts the caller's device back afterwards.
struct DeviceGuard {
    int prev = -1;
    hipError_t enter(int device) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess || cur == device) return e;
        prev = cur;
        return hipSetDevice(device);
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int fail(als_ctx *ctx, int code, const std::string &msg) {
    if (ctx) ctx->err = msg;
    return code;
}
int fail_hip(als_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, e == hipErrorOutOfMemory ? ALS_ENOMEM : ALS_EHIP,
                std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(ctx, expr)                                   \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return fail_hip(ctx, e_, #expr); \
    } while (0)

void free_plan(als_ctx *ctx, Plan &p) {
    if (!ctx->fixed) {
        hipFree(p.perm); hipFree(p.task_off); hipFree(p.task_row); hipFree(p.task_chunk); hipFree(p.task_order); hipFree(p.fingerprint);
    }
    delete[] p.task_off_host;
    p = Plan();
}

// device memory of a plan: a piece of the arena (workspace mode; the caller has made sure the plan fits) or hipMalloc
template <typename T>
hipError_t plan_alloc(als_ctx *ctx, T **out, size_t bytes) {
    if (!ctx->fixed) return hipMalloc(out, bytes);
    if (ctx->arena_used + aligned(bytes) > ctx->arena_bytes) return hipErrorOutOfMemory;
    *out = reinterpret_cast<T *>(ctx->arena + ctx->arena_used);
    ctx->arena_used += aligned(bytes);
    return hipSuccess;
}

std::string workspace_needed(als_ctx *ctx, int64_t rows, int64_t nnz) {
    const int64_t r = rows > ctx->cfg.workspace_max_rows ? rows : ctx->cfg.workspace_max_rows;
    const int64_t z = nnz > ctx->cfg.workspace_max_nnz ? nnz : ctx->cfg.workspace_max_nnz;
    return "the workspace was sized for " + std::to_string(ctx->cfg.workspace_max_rows) + " rows and " +
           std::to_string(ctx->cfg.workspace_max_nnz) + " entries; this matrix has " + std::to_string(rows) + " rows and " +
           std::to_string(nnz) + " entries and needs " + std::to_string(workspace_layout(ctx->cfg, r, z).total) + " bytes";
}

int check_sparse(als_ctx *ctx, const als_sparse *a) {
    if (!a) return fail(ctx, ALS_EINVAL, "sparse matrix descriptor is null");
    if (a->nrows < 0 || a->ncols < 0 || a->nnz < 0) return fail(ctx, ALS_EINVAL, "negative matrix size");
    if (a->nrows > 0x7fffffff || a->ncols > 0x7fffffff) return fail(ctx, ALS_EINVAL, "more than 2^31-1 rows or columns");
    if (!a->ptr) return fail(ctx, ALS_EINVAL, "ptr is null");
    if (a->nnz > 0 && (!a->idx || !a->val)) return fail(ctx, ALS_EINVAL, "idx or val is null");
    if (!a->ptr_is_64 && a->nnz > 0x7fffffff) return fail(ctx, ALS_EINVAL, "nnz >= 2^31 needs 64-bit ptr");
    if (ctx && ctx->fixed && (a->nrows > ctx->cfg.workspace_max_rows || a->nnz > ctx->cfg.workspace_max_nnz))
        return fail(ctx, ALS_EINVAL, "workspace too small: " + workspace_needed(ctx, a->nrows, a->nnz));
    return ALS_OK;
}

hipEvent_t get_event(als_ctx *ctx) {
    if (!ctx->free_events.empty()) {
        hipEvent_t e = ctx->free_events.back();
        ctx->free_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct Timed {   // brackets one launch with events when profiling is on
    als_ctx *ctx; int kernel; hipEvent_t a = nullptr, b = nullptr;
    Timed(als_ctx *c, int k) : ctx(c), kernel(k) {
        if (ctx->cfg.profile) {
            a = get_event(ctx); b = get_event(ctx);
            if (a && b) hipEventRecord(a, ctx->stream);
        }
    }
    ~Timed() {
        if (a && b) {
            hipEventRecord(b, ctx->stream);
            try {
                ctx->timed.push_back({a, b, kernel});
            } catch (...) {   // a destructor must not throw: this launch goes untimed
                hipEventDestroy(a);
                hipEventDestroy(b);
            }
        }
    }
};

int build_plan(als_ctx *ctx, const als_sparse *a, Plan &p);

// Finds or builds the plan of a matrix: degree-class permutation, work items, launch order of the slot work items.
int get_plan(als_ctx *ctx, const als_sparse *a, Plan **out) {
    for (auto &p : ctx->plans)
        if (p.key_ptr == a->ptr && p.nrows == a->nrows && p.nnz == a->nnz && p.chunk == ctx->cfg.chunk) {
            *out = &p;
            return ALS_OK;
        }
    if (ctx->fixed) {
        // Plans fill the arena front to back.  When the table or the arena is full, every cached plan is dropped;
        // the arena holds two plans of the largest matrix the workspace was sized for.  Kernels of earlier calls
        // that still read the old plans are ahead of the new plan's kernels on the stream.
        const bool table_full = ctx->plans[kMaxPlans - 1].key_ptr != nullptr;
        if (table_full || ctx->arena_used + plan_bytes_bound(a->nrows, a->nnz, ctx->cfg.chunk) > ctx->arena_bytes) {
            for (auto &p : ctx->plans) free_plan(ctx, p);
            ctx->arena_used = 0;
            ctx->next_plan = 0;
        }
    }
    Plan &p = ctx->plans[ctx->next_plan];
    ctx->next_plan = (ctx->next_plan + 1) % kMaxPlans;
    if (p.key_ptr) {   // (never in workspace mode: the table was emptied above)
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        free_plan(ctx, p);
    }
    const size_t arena_mark = ctx->arena_used;
    const int rc = build_plan(ctx, a, p);
    if (rc != ALS_OK) {   // nothing of a half-built plan stays behind
        (void)hipStreamSynchronize(ctx->stream);
        free_plan(ctx, p);
        ctx->arena_used = arena_mark;
        ctx->next_plan = (ctx->next_plan + kMaxPlans - 1) % kMaxPlans;
        return rc;
    }
    *out = &p;
    return ALS_OK;
}

// largest end with off[end] - off[pos] <= cap (at least pos + 1): the rows of one batch of the slot path
int64_t batch_end(const int32_t *off, int64_t pos, int64_t slot_rows, int64_t cap) {
    int64_t lo = pos + 1, hi = slot_rows;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if ((int64_t)off[mid] - off[pos] <= cap) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// work items whose partial Gram matrices are held at once
int64_t batch_capacity(const als_ctx *ctx) {
    return ctx->fixed && ctx->slot_capacity < ctx->cfg.batch_slots ? ctx->slot_capacity : ctx->cfg.batch_slots;
}

// Launch order of the work items inside every batch of the slot path.  The entries of a row are sorted by
// index, so a work item (a chunk of a long row) gathers from a band of the factor matrix that starts at its first
// index; workgroups are dispatched in launch order, and ordering the work items of a batch by that first index
// (instead of row by row, which puts disjoint bands side by side) makes the work items in flight gather from the
// same band, which then stays in the L2.  The slot of a work item is still its index in the batch.  Sorted on the
// device, batch by batch (the batches are those of update(): the capacity is fixed for the life of the context).
int build_order(als_ctx *ctx, const als_sparse *a, Plan &p) {
    const int32_t *off = p.task_off_host;
    const int64_t slot_rows = p.split_pos, n = slot_rows > 0 ? off[slot_rows] : 0;
    HIP_TRY(ctx, plan_alloc(ctx, &p.task_order, sizeof(int32_t) * (size_t)(n > 0 ? n : 1)));
    if (n == 0) return ALS_OK;
    HIP_TRY(ctx, ensure_scratch(&ctx->scratch, &ctx->scratch_bytes, sizeof(int32_t) * (size_t)n, ctx->fixed));
    int32_t *key = static_cast<int32_t *>(ctx->scratch);
    HIP_TRY(ctx, plan_task_keys(a->ptr_is_64 != 0, ctx->stream, a->ptr, a->idx, p.task_row, p.task_chunk, n, p.chunk, key));
    const int64_t cap = batch_capacity(ctx);
    for (int64_t pos = 0; pos < slot_rows;) {
        const int64_t end = batch_end(off, pos, slot_rows, cap);
        HIP_TRY(ctx, plan_rank_order(ctx->stream, key, off[pos], (int64_t)off[end] - off[pos], p.task_order));
        pos = end;
    }
    return ALS_OK;
}

int build_plan(als_ctx *ctx, const als_sparse *a, Plan &p) {
    Timed timed(ctx, ALS_K_PLAN);
    const int64_t m = a->nrows;
    const bool p64 = a->ptr_is_64 != 0;
    HIP_TRY(ctx, plan_alloc(ctx, &p.perm, sizeof(int32_t) * (size_t)(m > 0 ? m : 1)));
    HIP_TRY(ctx, plan_alloc(ctx, &p.task_off, sizeof(int32_t) * (size_t)(m + 1)));
    int32_t *class_start_dev = ctx->class_start_dev;
    if (!ctx->fixed) HIP_TRY(ctx, hipMalloc(&class_start_dev, sizeof(int32_t) * (kPlanClasses + 1)));
    hipError_t eb = plan_bin_rows(p64, ctx->stream, m, a->ptr, kPlanClasses, p.perm, class_start_dev, &ctx->scratch,
                                  &ctx->scratch_bytes, ctx->fixed);
    int32_t class_start[kPlanClasses + 1];
    if (eb == hipSuccess)
        eb = hipMemcpyAsync(class_start, class_start_dev, sizeof(class_start), hipMemcpyDeviceToHost, ctx->stream);
    if (eb == hipSuccess) eb = hipStreamSynchronize(ctx->stream);
    if (!ctx->fixed) (void)hipFree(class_start_dev);
    HIP_TRY(ctx, eb);
    {   // rows with >= chunk = 2^j entries are the classes >= j+1, i.e. the first class_start[...] positions
        int j = 0;
        while ((1 << j) < ctx->cfg.chunk) ++j;
        p.split_pos = class_start[kPlanClasses - 1 - j];
    }
    for (int c = 0; c <= 32; ++c)   // class c = 1 + floor(log2 n_u) (0 for empty rows), heaviest class first in perm
        p.rows_ge[c] = c == 0 ? m : (c < kPlanClasses ? class_start[kPlanClasses - c] : 0);
    HIP_TRY(ctx, plan_tasks(p64, ctx->stream, m, a->ptr, p.perm, ctx->cfg.chunk, p.task_off, &ctx->scratch,
                            &ctx->scratch_bytes, ctx->fixed));
    p.task_off_host = new (std::nothrow) int32_t[(size_t)m + 1];
    if (!p.task_off_host) return fail(ctx, ALS_ENOMEM, "host allocation of the work-item offsets failed");
    HIP_TRY(ctx, hipMemcpyAsync(p.task_off_host, p.task_off, sizeof(int32_t) * (size_t)(m + 1), hipMemcpyDeviceToHost,
                                ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    p.ntasks = p.task_off_host[m];
    HIP_TRY(ctx, plan_alloc(ctx, &p.task_row, sizeof(int32_t) * (size_t)(p.ntasks > 0 ? p.ntasks : 1)));
    HIP_TRY(ctx, plan_alloc(ctx, &p.task_chunk, sizeof(int32_t) * (size_t)(p.ntasks > 0 ? p.ntasks : 1)));
    HIP_TRY(ctx, plan_emit(p64, ctx->stream, m, a->ptr, p.perm, ctx->cfg.chunk, p.task_off, p.task_row, p.task_chunk));
    p.chunk = ctx->cfg.chunk;
    const int rc = build_order(ctx, a, p);
    if (rc != ALS_OK) return rc;
    HIP_TRY(ctx, plan_alloc(ctx, &p.fingerprint, 2 * sizeof(unsigned long long)));
    HIP_TRY(ctx, fill_zero(ctx->stream, p.fingerprint, 2));
    HIP_TRY(ctx, plan_fingerprint(p64, ctx->stream, a->ptr, m + 1, p.fingerprint, ctx->fp_done, nullptr, ctx->status));
    p.key_ptr = a->ptr; p.nrows = m; p.nnz = a->nnz;
    return ALS_OK;
}

// The plan of a matrix is found by address and sizes.  Every call that uses it recomputes the fingerprint of the row
// offsets on the device and compares it with the plan's: a matrix that changed under its plan sets
// kStatusStalePlan, which the next als_synchronize reports (kernels only: nothing here waits or allocates).
int check_plan(als_ctx *ctx, const als_sparse *a, const Plan *p) {
    HIP_TRY(ctx, plan_fingerprint(a->ptr_is_64 != 0, ctx->stream, a->ptr, a->nrows + 1, ctx->fp_now, ctx->fp_done,
                                  p->fingerprint, ctx->status));
    return ALS_OK;
}

// A launch holds fewer than 2^32 threads.  The kernels that take one workgroup per row (or per work item) are
// launched over pieces of at most this many workgroups.
int64_t max_workgroups(int threads) { return (int64_t)0x7fffffff / threads; }

template <typename L>
int in_pieces(int64_t pos0, int64_t n, int64_t piece, L launch) {   // launch(first position, count) -> status
    for (int64_t done = 0; done < n; done += piece) {
        const int rc = launch(pos0 + done, n - done < piece ? n - done : piece);
        if (rc != ALS_OK) return rc;
    }
    return ALS_OK;
}

int ensure_slots(als_ctx *ctx, int64_t nslots, bool s16) {
    const size_t need = (size_t)nslots * (s16 ? slot_words16(ctx->cfg.f) : slot_floats(ctx->cfg.f)) * sizeof(float);
    if (ctx->slots_bytes >= need) return ALS_OK;
    if (ctx->fixed)
        return fail(ctx, ALS_EINVAL, "workspace too small: " + std::to_string(nslots) + " partial Gram matrices (" +
                                         std::to_string(need) + " bytes) are needed at once, the workspace holds " +
                                         std::to_string(ctx->slots_bytes) + " bytes of them");
    if (ctx->slots) {
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        HIP_TRY(ctx, hipFree(ctx->slots));
        ctx->slots = nullptr; ctx->slots_bytes = 0;
    }
    HIP_TRY(ctx, hipMalloc(&ctx->slots, need));
    ctx->slots_bytes = need;
    return ALS_OK;
}

// G^T G (n x f fp32 rows) into ctx->gram[which], tile layout.  Uses the slot workspace.
int compute_gram(als_ctx *ctx, const void *G, int et, int64_t n, int which) {
    const int f = ctx->cfg.f;
    if (!ctx->gram[which]) HIP_TRY(ctx, hipMalloc(&ctx->gram[which], sizeof(float) * (size_t)slot_floats(f)));
    if (n == 0) {
        HIP_TRY(ctx, fill_zero(ctx->stream, ctx->gram[which], slot_floats(f)));
        return ALS_OK;
    }
    // work items of `per` rows (a multiple of 4): enough of them to fill the chip, few enough to sum quickly
    int64_t items = (n + 255) / 256;
    if (items > 2048) items = 2048;
    if (ctx->fixed) {   // no more work items than the workspace holds fp32 slots for
        const int64_t room = (int64_t)(ctx->slots_bytes / (sizeof(float) * (size_t)slot_floats(f)));
        if (room < 1) return fail(ctx, ALS_EINVAL, "workspace too small for one partial Gram matrix");
        if (items > room) items = room;
    }
    int64_t per = ((n + items - 1) / items + 3) & ~(int64_t)3;
    if (per > (1 << 28)) return fail(ctx, ALS_EINVAL, "factor matrix too tall for the Gram kernel");
    const int nslots = (int)((n + per - 1) / per);
    int rc = ensure_slots(ctx, nslots, false);
    if (rc != ALS_OK) return rc;
    const bool wide = needs_wide_offsets(n, f, factor_bytes(et));
    Timed t(ctx, ALS_K_GRAM);
    HIP_TRY(ctx, launch_gram(f, wide, et, ctx->stream, G, n, (int)per, nslots, ctx->slots, ctx->gram[which]));
    return ALS_OK;
}

// gathered: the call gathers a factor of the configured element type (the updates; not the cost, which takes fp32)
int check_implicit(als_ctx *ctx, float alpha, bool gathered) {
    const int et = ctx->cfg.factor_dtype;
    const bool sixteen = (et == ALS_BF16 || et == ALS_F16) && single_wave_f(ctx->cfg.f);
    if ((et != ALS_F32 && !(gathered && sixteen)) || ctx->cfg.herm_dtype != ALS_F32)
        return fail(ctx, ALS_EINVAL, "implicit feedback needs fp32 factors (bf16 / fp16 for the updates at f <= 128) and "
                                     "fp32 storage of A_u");
    if (!(alpha >= 0.f)) return fail(ctx, ALS_EINVAL, "alpha must be >= 0");
    return ALS_OK;
}

// One half-sweep: rows of `a` updated from the gathered factor `G` into `Out`.
// mode kExplicit: eq. (2)/(3); kImplicit: Section 5.6 with confidence scale alpha.
int update(als_ctx *ctx, const als_sparse *a, const void *G, float lambda, int f, float *Out, int mode = kExplicit,
           float alpha = 0.f) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, a);
    if (rc != ALS_OK) return rc;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (!(lambda >= 0.f)) return fail(ctx, ALS_EINVAL, "lambda must be >= 0");
    if (a->nrows == 0) return ALS_OK;   // nothing to write
    if (!Out || (a->nnz > 0 && !G)) return fail(ctx, ALS_EINVAL, "factor pointer is null");
    if (!aligned16(Out) || !aligned16(G)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    const bool implicit = mode == kImplicit;
    if (implicit) {
        rc = check_implicit(ctx, alpha, true);
        if (rc != ALS_OK) return rc;
        if (!G) return fail(ctx, ALS_EINVAL, "factor pointer is null");
        rc = compute_gram(ctx, G, ctx->cfg.factor_dtype, a->ncols, 0);
        if (rc != ALS_OK) return rc;
    }
    const float *gram = ctx->gram[0];
    Plan *p = nullptr;
    rc = get_plan(ctx, a, &p);
    if (rc != ALS_OK) return rc;
    rc = check_plan(ctx, a, p);
    if (rc != ALS_OK) return rc;
    const int64_t cap = batch_capacity(ctx);
    const bool p64 = a->ptr_is_64 != 0;
    const int32_t *off = p->task_off_host;
    const int64_t m = a->nrows;
    const bool cg = ctx->cfg.solver == ALS_SOLVER_CG;
    const bool s16 = ctx->cfg.herm_dtype == ALS_BF16;
    const size_t esize = factor_bytes(ctx->cfg.factor_dtype);
    const bool wide = needs_wide_offsets(a->ncols, f, esize);
    // Rows with fewer than `chunk` entries are one work item each; with the CG solver they are built
    // and solved by one wavefront without leaving the registers.  Everything else goes through slots.
    const bool one_wave = single_wave_f(f);   // larger f: the wavefronts of a workgroup share a system
    // rows shorter than a chunk are built and solved without leaving the registers (both solvers); longer
    // rows go through slots
    const int64_t slot_rows = p->split_pos;
    const int32_t *order = kTaskOrder ? p->task_order : nullptr;
    const bool x2 = ctx->cfg.factor_dtype == ALS_F32X2;
    if (x2 && !implicit)   // the power-of-two scale of the two-part route follows max |G|
        HIP_TRY(ctx, launch_absmax(ctx->stream, static_cast<const float *>(G), a->ncols * (int64_t)f, ctx->absmax));
    int64_t pos = 0;
    while (pos < slot_rows) {
        // rows [pos, end): as many as fit in `cap` slots, at least one row
        const int64_t end = batch_end(off, pos, slot_rows, cap);
        const int64_t task0 = off[pos], ntasks = (int64_t)off[end] - off[pos];
        rc = ensure_slots(ctx, ntasks > 0 ? ntasks : 1, s16);
        if (rc != ALS_OK) return rc;
        {
            Timed t(ctx, ALS_K_HERMITIAN);
            if (implicit)
                HIP_TRY(ctx, launch_hermitian_implicit(f, p64, wide, ctx->cfg.factor_dtype, ctx->stream, p->task_row, p->task_chunk, order, task0,
                                                       ntasks, ctx->cfg.chunk, a->ptr, a->idx, a->val, G, alpha,
                                                       ctx->slots));
            else if (x2)
                HIP_TRY(ctx, launch_hermitian_x2(f, p64, wide, s16, ctx->stream, p->task_row, p->task_chunk, order, task0,
                                                 ntasks, ctx->cfg.chunk, a->ptr, a->idx, a->val, G, ctx->slots, ctx->absmax));
            else
                HIP_TRY(ctx, launch_hermitian(f, p64, wide, ctx->cfg.factor_dtype, s16, ctx->stream, p->task_row,
                                              p->task_chunk, order, task0, ntasks, ctx->cfg.chunk, a->ptr, a->idx, a->val, G,
                                              ctx->slots));
        }
        {
            Timed t(ctx, ALS_K_SOLVE);
            if (ntasks > end - pos)   // some row of the batch has several slots
                HIP_TRY(ctx, launch_reduce_slots(f, s16, ctx->stream, p->task_off, pos, end - pos, task0, ctx->slots));
            if (implicit)
                HIP_TRY(ctx, launch_solve_wave_implicit(f, p64, ctx->cfg.solver, ctx->stream, p->perm, p->task_off, pos,
                                                        end - pos, task0, a->ptr, ctx->slots, lambda, gram,
                                                        ctx->cfg.cg_iters, ctx->cfg.cg_eps, Out, ctx->status));
            else if (!cg && !one_wave)
                HIP_TRY(ctx, launch_solve_ldlt_wide(p64, ctx->stream, p->perm, p->task_off, pos, end - pos, task0, a->ptr,
                                                    ctx->slots, lambda, Out, ctx->status));
            else if (cg && !one_wave)
                HIP_TRY(ctx, launch_solve_cg_wide(p64, s16, ctx->stream, p->perm, p->task_off, pos, end - pos, task0,
                                                  a->ptr, ctx->slots, lambda, ctx->cfg.cg_iters, ctx->cfg.cg_eps,
                                                  Out, ctx->status));
            else
                HIP_TRY(ctx, launch_solve_cg_wave(f, p64, s16, ctx->cfg.solver, ctx->stream, p->perm, p->task_off, pos, end - pos, task0,
                                                  a->ptr, ctx->slots, lambda, ctx->cfg.cg_iters, ctx->cfg.cg_eps,
                                                  Out, ctx->status));
        }
        pos = end;
    }
    // Exact solver: rows with fewer entries than features are solved in the dual form, an
    // n_u x n_u system (dual.hip).  They are the tail of perm: fewer than 2^(c-1) entries from rows_ge[c] on.
    int64_t fused_end = m;
    const int64_t piece = max_workgroups(one_wave ? 64 : kWideThreads);
    if (kDualExact && !implicit && !cg) {
        Timed t(ctx, ALS_K_FUSED);
        for (int c = 6; c <= 8; ++c) {   // fewer than 32, 64, 128 entries: 2, 4, 8 tiles of 16 entries
            const int ntd = 1 << (c - 5);
            if (16 * ntd > f || !has_dual_exact(f, ntd)) break;
            const int64_t lo = p->rows_ge[c] > slot_rows ? p->rows_ge[c] : slot_rows;
            if (lo < fused_end) {
                rc = in_pieces(lo, fused_end - lo, max_workgroups(64), [&](int64_t pos0, int64_t npos) {
                    HIP_TRY(ctx, launch_dual_exact(f, ntd, p64, fp32_in_memory(ctx->cfg.factor_dtype) ? ALS_F32 : ctx->cfg.factor_dtype, ctx->stream, p->perm, pos0, npos, a->ptr,
                                                   a->idx, a->val, G, lambda, Out, ctx->status));
                    return (int)ALS_OK;
                });
                if (rc != ALS_OK) return rc;
                fused_end = lo;
            }
        }
    }
    // Algorithm 1, explicit feedback: rows with fewer than 64 entries (classes below 7, the tail of perm) iterate on
    // the gathered rows themselves and never form A_u (cg_short.hip)
    if (cg && !implicit && !ctx->cfg.dense_short_rows) {
        const int et = fp32_in_memory(ctx->cfg.factor_dtype) ? ALS_F32 : ctx->cfg.factor_dtype;
        // one launch per group of classes, shortest rows first: fewer than 16, 32, 64 entries as 4, 2, 1 rows per
        // wavefront (f = 256: one row per pair of wavefronts throughout)
        // c = 8: rows of 64 .. 127 entries, two wavefronts per row, where short_row_limit says so
        const int cmax = short_row_limit(ctx->cfg) > 64 ? 8 : 7;
        for (int c = one_wave ? 5 : 7; c <= cmax; ++c) {
            const int64_t lo = p->rows_ge[c] > slot_rows ? p->rows_ge[c] : slot_rows;
            if (lo < fused_end) {
                Timed t(ctx, ALS_K_SHORT);
                rc = in_pieces(lo, fused_end - lo, max_workgroups(128), [&](int64_t pos0, int64_t npos) {
                    HIP_TRY(ctx, launch_cg_gathered(f, c == 8 ? -2 : 1 << (7 - c), p64, et, ctx->stream, p->perm, pos0, npos, a->ptr, a->idx,
                                                    a->val, G, lambda, ctx->cfg.cg_iters, ctx->cfg.cg_eps, Out, ctx->status));
                    return (int)ALS_OK;
                });
                if (rc != ALS_OK) return rc;
                fused_end = lo;
            }
        }
    }
    if (slot_rows < fused_end) {
        Timed t(ctx, ALS_K_FUSED);
        rc = in_pieces(slot_rows, fused_end - slot_rows, piece, [&](int64_t pos0, int64_t npos) {
            if (implicit)
                HIP_TRY(ctx, launch_hermitian_cg_implicit(f, p64, wide, ctx->cfg.factor_dtype, ctx->cfg.solver, ctx->stream, p->perm,
                                                          pos0, npos, a->ptr, a->idx, a->val, G, lambda, alpha, gram,
                                                          ctx->cfg.cg_iters, ctx->cfg.cg_eps, Out, ctx->status));
            else if (x2)
                HIP_TRY(ctx, launch_hermitian_cg_x2(f, p64, wide, ctx->cfg.solver, ctx->stream, p->perm, pos0, npos, a->ptr,
                                                    a->idx, a->val, G, lambda, ctx->cfg.cg_iters, ctx->cfg.cg_eps, Out,
                                                    ctx->status, ctx->absmax));
            else
                HIP_TRY(ctx, launch_hermitian_cg(f, p64, wide, ctx->cfg.factor_dtype, ctx->cfg.solver, ctx->stream, p->perm,
                                                 pos0, npos, a->ptr, a->idx, a->val, G, lambda, ctx->cfg.cg_iters,
                                                 ctx->cfg.cg_eps, Out, ctx->status));
            return (int)ALS_OK;
        });
        if (rc != ALS_OK) return rc;
    }
    return ALS_OK;
}

// Runs the body of an entry point; a C++ exception (host containers running out of memory) becomes a status.
template <typename L>
int guarded(als_ctx *ctx, L body) {
    try {
        return body();
    } catch (const std::bad_alloc &) {
        try { if (ctx) ctx->err = "host allocation failed"; } catch (...) {}
        return ALS_ENOMEM;
    } catch (...) {
        try { if (ctx) ctx->err = "unexpected C++ exception"; } catch (...) {}
        return ALS_EHIP;
    }
}

}  // namespace

extern "C" {

// Checks a configuration and fills in its defaults (chunk, batch_slots).  false: als_create refuses it.
static bool resolve_config(const als_config *in, als_config *c) {
    *c = *in;
    if (!supported_f(c->f)) return false;
    if (c->solver != ALS_SOLVER_CHOLESKY && c->solver != ALS_SOLVER_CG) return false;
    if (c->solver == ALS_SOLVER_CG && c->cg_iters < 0) return false;
    if (c->dense_short_rows != 0 && c->dense_short_rows != 1) return false;
    if (c->factor_dtype != ALS_F32 && c->factor_dtype != ALS_BF16 && c->factor_dtype != ALS_F16 &&
        c->factor_dtype != ALS_F32X3 && c->factor_dtype != ALS_F32X2)
        return false;
    // the routes through 16-bit parts exist for f <= 128
    if ((c->factor_dtype == ALS_F32X3 || c->factor_dtype == ALS_F32X2) && !single_wave_f(c->f)) return false;
    // reduced-precision storage of A_u only makes sense with the approximate solver; fp16 cannot hold the
    // sums of 10^5 squares that heavy rows reach, so bf16 is the reduced type
    if (c->herm_dtype != ALS_F32 &&
        !(c->herm_dtype == ALS_BF16 && c->solver == ALS_SOLVER_CG &&
          (single_wave_f(c->f) || c->factor_dtype == ALS_F32)))   // f = 256: with fp32 factor inputs only
        return false;
    if (c->chunk < 0 || c->batch_slots < 0) return false;
    if (c->chunk != 0 && (c->chunk < 64 || c->chunk > (1 << 20) || (c->chunk & (c->chunk - 1)))) return false;
    if (c->chunk == 0) c->chunk = 4096;
    if (c->batch_slots > max_workgroups(kWideThreads)) c->batch_slots = max_workgroups(kWideThreads);
    if (c->batch_slots == 0) {   // about 4 GB of slots
        c->batch_slots = 131072;
        while (c->batch_slots > 1024 && (size_t)c->batch_slots * slot_floats(c->f) * 4 > (4ull << 30)) c->batch_slots /= 2;
    }
    return true;
}

size_t als_workspace_bytes(const als_config *cfg, int64_t max_rows, int64_t max_nnz) {
    als_config c;
    if (!cfg || max_rows < 0 || max_nnz < 0 || max_rows > 0x7fffffff || !resolve_config(cfg, &c)) return 0;
    return workspace_layout(c, max_rows, max_nnz).total;
}

int als_create(als_ctx **out, const als_config *cfg) {
    if (!out || !cfg) return ALS_EINVAL;
    *out = nullptr;
    als_config c;
    if (!resolve_config(cfg, &c)) return ALS_EINVAL;
    const bool fixed = c.workspace != nullptr;
    WorkspaceLayout L{};
    if (fixed) {
        if (c.workspace_max_rows < 0 || c.workspace_max_rows > 0x7fffffff || c.workspace_max_nnz < 0) return ALS_EINVAL;
        if (reinterpret_cast<uintptr_t>(c.workspace) % kAlign != 0) return ALS_EINVAL;
        L = workspace_layout(c, c.workspace_max_rows, c.workspace_max_nnz);
        if (c.workspace_bytes < L.total) return ALS_EINVAL;
    } else if (c.workspace_bytes != 0 || c.workspace_max_rows != 0 || c.workspace_max_nnz != 0) {
        return ALS_EINVAL;
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || c.device < 0 || c.device >= ndev) return ALS_EHIP;
    als_ctx *ctx = new (std::nothrow) als_ctx();
    if (!ctx) return ALS_ENOMEM;
    ctx->cfg = c;
    ctx->fixed = fixed;
    ctx->stream = (hipStream_t)c.stream;
    DeviceGuard on_device;
    bool ok = on_device.enter(c.device) == hipSuccess;
    if (ok && fixed) {
        char *w = static_cast<char *>(c.workspace);
        char *fw = w + L.fixed_words;                       // 1 KiB of small words, 16 bytes apart at least
        ctx->status = reinterpret_cast<int *>(fw);
        ctx->check_flags = reinterpret_cast<int *>(fw + 16);
        ctx->fp_now = reinterpret_cast<unsigned long long *>(fw + 32);   // fingerprint, then the counter
        ctx->sse_total = reinterpret_cast<double *>(fw + 64);
        ctx->gram_dot = reinterpret_cast<double *>(fw + 96);             // 3 doubles
        ctx->absmax = reinterpret_cast<uint32_t *>(fw + 128);
        ctx->class_start_dev = reinterpret_cast<int32_t *>(fw + 256);    // kPlanClasses + 1 ints
        ctx->gram[0] = reinterpret_cast<float *>(w + L.gram0);
        ctx->gram[1] = reinterpret_cast<float *>(w + L.gram1);
        ctx->sse_partial = reinterpret_cast<double *>(w + L.sse_partial);
        ctx->sse_partial_bytes = L.scratch - L.sse_partial;
        ctx->scratch = w + L.scratch;
        ctx->scratch_bytes = L.scratch_bytes;
        ctx->slots = reinterpret_cast<float *>(w + L.slots);
        ctx->slots_bytes = L.arena - L.slots;
        ctx->slot_capacity = L.slot_capacity;
        ctx->arena = w + L.arena;
        ctx->arena_bytes = L.arena_bytes;
        ok = fill_zero(ctx->stream, fw, 256) == hipSuccess;   // status, flags, fingerprint and counter start at zero
    } else if (ok) {
        ok = hipMalloc(&ctx->status, sizeof(int)) == hipSuccess && hipMalloc(&ctx->sse_total, sizeof(double)) == hipSuccess &&
             hipMalloc(&ctx->fp_now, 3 * sizeof(unsigned long long)) == hipSuccess &&   // + the word of absmax
             hipMemsetAsync(ctx->status, 0, sizeof(int), ctx->stream) == hipSuccess &&
             hipMemsetAsync(ctx->fp_now, 0, 2 * sizeof(unsigned long long), ctx->stream) == hipSuccess;
    }
    if (ok) ok = gram_static_scratch(&ctx->gram_static) == hipSuccess;   // the context's device is current here
    if (!ok) {
        if (!fixed) { hipFree(ctx->status); hipFree(ctx->sse_total); hipFree(ctx->fp_now); }
        delete ctx;
        return ALS_EHIP;
    }
    ctx->fp_done = reinterpret_cast<unsigned int *>(ctx->fp_now + 1);
    if (!fixed) ctx->absmax = reinterpret_cast<uint32_t *>(ctx->fp_now + 2);
    *out = ctx;
    return ALS_OK;
}

void als_destroy(als_ctx *ctx) {
    if (!ctx) return;
    DeviceGuard on_device;
    (void)on_device.enter(ctx->cfg.device);
    hipStreamSynchronize(ctx->stream);
    for (auto &p : ctx->plans) free_plan(ctx, p);
    if (!ctx->fixed) {
        hipFree(ctx->slots); hipFree(ctx->scratch); hipFree(ctx->status); hipFree(ctx->sse_partial);
        hipFree(ctx->sse_total); hipFree(ctx->fp_now); hipFree(ctx->check_flags); hipFree(ctx->gram[0]); hipFree(ctx->gram[1]); hipFree(ctx->gram_dot);
    }
    for (auto &t : ctx->timed) { hipEventDestroy(t.a); hipEventDestroy(t.b); }
    for (auto e : ctx->free_events) hipEventDestroy(e);
    delete ctx;
}

const char *als_last_error(const als_ctx *ctx) { return ctx ? ctx->err.c_str() : "context is null"; }

static int als_update_rows_impl(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f, float *X) {
    return update(ctx, csr, Theta, lambda, f, X);
}

static int als_update_cols_impl(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, int f, float *Theta) {
    return update(ctx, csc, X, lambda, f, Theta);
}

static int als_update_rows_implicit_impl(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, float alpha,
                             int f, float *X) {
    return update(ctx, csr, Theta, lambda, f, X, kImplicit, alpha);
}

static int als_update_cols_implicit_impl(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, float alpha, int f,
                             float *Theta) {
    return update(ctx, csc, X, lambda, f, Theta, kImplicit, alpha);
}

static int als_gram_impl(als_ctx *ctx, const float *G, int64_t n, int f, float *out) {
    if (!ctx) return ALS_EINVAL;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (n < 0 || n > 0x7fffffff || !out || (n > 0 && !G)) return fail(ctx, ALS_EINVAL, "bad argument");
    if (!aligned16(G)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    int rc = compute_gram(ctx, G, ALS_F32, n, 0);
    if (rc != ALS_OK) return rc;
    HIP_TRY(ctx, launch_tiles_to_dense(f, ctx->stream, ctx->gram[0], out));
    return ALS_OK;
}

// als_gram without any allocation: slots and summed tiles live in the file-scope device array (implicit.hip).
static int als_gram_static_impl(als_ctx *ctx, const float *G, int64_t n, int f, float *out) {
    if (!ctx) return ALS_EINVAL;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (n < 0 || !out || (n > 0 && !G)) return fail(ctx, ALS_EINVAL, "bad argument");
    if (n > ALS_GRAM_STATIC_MAX_ROWS)
        return fail(ctx, ALS_EINVAL, "als_gram_static takes at most ALS_GRAM_STATIC_MAX_ROWS (2^30) rows");
    if (!aligned16(G)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    const size_t tile_part = (size_t)tiles_tri(f) * 256;
    float *slots = ctx->gram_static, *tiles = ctx->gram_static + (kGramStaticFloats - tile_part);
    if (n == 0) {
        HIP_TRY(ctx, fill_zero(ctx->stream, tiles, (int64_t)tile_part));
    } else {
        // as many work items as the array holds slots for (at most kGramStaticMaxSlots), each of `per` rows
        int64_t cap = (int64_t)((kGramStaticFloats - tile_part) / (size_t)slot_floats(f));
        if (cap > kGramStaticMaxSlots) cap = kGramStaticMaxSlots;
        int64_t items = (n + 255) / 256;
        if (items > cap) items = cap;
        const int64_t per = ((n + items - 1) / items + 3) & ~(int64_t)3;   // <= 2^30 / 116 + 3 rows
        const int nslots = (int)((n + per - 1) / per);
        HIP_TRY(ctx, launch_gram(f, needs_wide_offsets(n, f, 4), ALS_F32, ctx->stream, G, n, (int)per, nslots, slots, tiles));
    }
    HIP_TRY(ctx, launch_tiles_to_dense(f, ctx->stream, tiles, out));
    return ALS_OK;
}

static int sum_over_entries(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, int f,
                            bool implicit, float alpha, double *sum_out);

static int als_implicit_loss_impl(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, float lambda,
                      float alpha, int f, double *loss_out) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, csr);
    if (rc != ALS_OK) return rc;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (!loss_out || !X || !Theta) return fail(ctx, ALS_EINVAL, "null pointer");
    if (!aligned16(X) || !aligned16(Theta)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    rc = check_implicit(ctx, alpha, false);
    if (rc != ALS_OK) return rc;
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    double entries = 0.0;
    if (csr->nnz > 0) {
        rc = sum_over_entries(ctx, csr, X, Theta, f, true, alpha, &entries);
        if (rc != ALS_OK) return rc;
    }
    rc = compute_gram(ctx, X, ALS_F32, csr->nrows, 0);
    if (rc != ALS_OK) return rc;
    rc = compute_gram(ctx, Theta, ALS_F32, csr->ncols, 1);
    if (rc != ALS_OK) return rc;
    if (!ctx->gram_dot) HIP_TRY(ctx, hipMalloc(&ctx->gram_dot, 3 * sizeof(double)));
    HIP_TRY(ctx, launch_gram_dot(f, ctx->stream, ctx->gram[0], ctx->gram[1], ctx->gram_dot));
    double d3[3] = {0, 0, 0};
    HIP_TRY(ctx, hipMemcpyAsync(d3, ctx->gram_dot, sizeof(d3), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    *loss_out = entries + d3[0] + (double)lambda * (d3[1] + d3[2]);
    return ALS_OK;
}

static int als_rmse_impl(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, int f, double *rmse_out) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, csr);
    if (rc != ALS_OK) return rc;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (!rmse_out || (csr->nnz > 0 && (!X || !Theta))) return fail(ctx, ALS_EINVAL, "null pointer");
    if (!aligned16(X) || !aligned16(Theta)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    if (csr->nnz == 0) { *rmse_out = 0.0; return ALS_OK; }
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    double sse = 0.0;
    rc = sum_over_entries(ctx, csr, X, Theta, f, false, 0.f, &sse);
    if (rc != ALS_OK) return rc;
    *rmse_out = sqrt(sse / (double)csr->nnz);
    return ALS_OK;
}

// sum over the stored entries of the squared error (explicit) or of the entry part of the implicit cost
static int sum_over_entries(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, int f,
                            bool implicit, float alpha, double *sum_out) {
    int rc;
    Plan *p = nullptr;
    rc = get_plan(ctx, csr, &p);
    if (rc != ALS_OK) return rc;
    rc = check_plan(ctx, csr, p);
    if (rc != ALS_OK) return rc;
    const size_t need = sizeof(double) * (size_t)(p->ntasks > 0 ? p->ntasks : 1);
    if (ctx->sse_partial_bytes < need) {
        if (ctx->fixed) return fail(ctx, ALS_EINVAL, "workspace too small for the partial sums of this matrix");
        if (ctx->sse_partial) { HIP_TRY(ctx, hipStreamSynchronize(ctx->stream)); HIP_TRY(ctx, hipFree(ctx->sse_partial)); }
        ctx->sse_partial = nullptr; ctx->sse_partial_bytes = 0;
        HIP_TRY(ctx, hipMalloc(&ctx->sse_partial, need));
        ctx->sse_partial_bytes = need;
    }
    {
        Timed t(ctx, ALS_K_RMSE);
        HIP_TRY(ctx, launch_sse(f, csr->ptr_is_64 != 0, implicit, alpha, ctx->stream, p->task_row, p->task_chunk,
                                p->ntasks, ctx->cfg.chunk, csr->ptr, csr->idx, csr->val, X, Theta, ctx->sse_partial,
                                ctx->sse_total));
    }
    double sse = 0.0;
    HIP_TRY(ctx, hipMemcpyAsync(&sse, ctx->sse_total, sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    *sum_out = sse;
    return ALS_OK;
}

static int als_hermitian_impl(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f, int64_t row0,
                  int64_t nrows, float *A_out, float *b_out) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, csr);
    if (rc != ALS_OK) return rc;
    if (f != ctx->cfg.f) return fail(ctx, ALS_EINVAL, "f differs from the f given at als_create");
    if (row0 < 0 || nrows < 0 || row0 + nrows > csr->nrows) return fail(ctx, ALS_EINVAL, "row range outside the matrix");
    if (!A_out || !b_out || !Theta) return fail(ctx, ALS_EINVAL, "null pointer");
    if (!aligned16(Theta)) return fail(ctx, ALS_EINVAL, "factor matrices must be 16-byte aligned");
    if (nrows == 0) return ALS_OK;
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    // a throw-away plan over the row range, in natural order
    const bool p64 = csr->ptr_is_64 != 0;
    const size_t esize = factor_bytes(ctx->cfg.factor_dtype);
    const bool wide = needs_wide_offsets(csr->ncols, f, esize);
    int32_t *perm = nullptr, *task_off = nullptr, *task_row = nullptr, *task_chunk = nullptr;
    auto cleanup = [&]() { hipFree(perm); hipFree(task_off); hipFree(task_row); hipFree(task_chunk); };
    hipError_t e;
    if ((e = hipMalloc(&perm, sizeof(int32_t) * (size_t)nrows)) != hipSuccess ||
        (e = hipMalloc(&task_off, sizeof(int32_t) * (size_t)(nrows + 1))) != hipSuccess) {
        cleanup();
        return fail_hip(ctx, e, "hipMalloc");
    }
    std::vector<int32_t> off((size_t)nrows + 1);
    void *tmp = nullptr;     // scan scratch of this call (the context's may be a fixed piece of a workspace)
    size_t tmp_bytes = 0;
    auto cleanup_tmp = [&]() { hipFree(tmp); tmp = nullptr; };
    if ((e = fill_iota(ctx->stream, perm, nrows, (int32_t)row0)) != hipSuccess ||
        (e = plan_tasks(p64, ctx->stream, nrows, csr->ptr, perm, ctx->cfg.chunk, task_off, &tmp, &tmp_bytes, false)) !=
            hipSuccess ||
        (e = hipMemcpyAsync(off.data(), task_off, sizeof(int32_t) * (size_t)(nrows + 1), hipMemcpyDeviceToHost,
                            ctx->stream)) != hipSuccess ||
        (e = hipStreamSynchronize(ctx->stream)) != hipSuccess) {
        cleanup();
        cleanup_tmp();
        return fail_hip(ctx, e, "plan of the row range");
    }
    cleanup_tmp();
    const int64_t ntasks = off[(size_t)nrows];
    if ((e = hipMalloc(&task_row, sizeof(int32_t) * (size_t)(ntasks > 0 ? ntasks : 1))) != hipSuccess ||
        (e = hipMalloc(&task_chunk, sizeof(int32_t) * (size_t)(ntasks > 0 ? ntasks : 1))) != hipSuccess ||
        (e = plan_emit(p64, ctx->stream, nrows, csr->ptr, perm, ctx->cfg.chunk, task_off, task_row, task_chunk)) !=
            hipSuccess) {
        cleanup();
        return fail_hip(ctx, e, "work items of the row range");
    }
    rc = ensure_slots(ctx, ntasks > 0 ? ntasks : 1, false);
    if (rc != ALS_OK) { cleanup(); return rc; }
    {
        Timed t(ctx, ALS_K_HERMITIAN);
        if (ctx->cfg.factor_dtype == ALS_F32X2) {
            e = launch_absmax(ctx->stream, static_cast<const float *>(Theta), csr->ncols * (int64_t)f, ctx->absmax);
            if (e == hipSuccess)
                e = launch_hermitian_x2(f, p64, wide, false, ctx->stream, task_row, task_chunk, nullptr, 0, ntasks,
                                        ctx->cfg.chunk, csr->ptr, csr->idx, csr->val, Theta, ctx->slots, ctx->absmax);
        } else {
            e = launch_hermitian(f, p64, wide, ctx->cfg.factor_dtype, false, ctx->stream, task_row, task_chunk, nullptr, 0,
                                 ntasks, ctx->cfg.chunk, csr->ptr, csr->idx, csr->val, Theta, ctx->slots);
        }
    }
    if (e == hipSuccess)
        e = launch_export_dense(f, p64, ctx->stream, perm, task_off, 0, nrows, 0, csr->ptr, ctx->slots, lambda, row0,
                                A_out, b_out);
    hipError_t e2 = hipStreamSynchronize(ctx->stream);
    cleanup();
    if (e != hipSuccess) return fail_hip(ctx, e, "get_hermitian launch");
    if (e2 != hipSuccess) return fail_hip(ctx, e2, "get_hermitian");
    return ALS_OK;
}

static int als_bin_rows_impl(als_ctx *ctx, const als_sparse *csr, int nclass, int32_t *perm_out, int64_t *class_start_out) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, csr);
    if (rc != ALS_OK) return rc;
    if (nclass < 2 || nclass > 64) return fail(ctx, ALS_EINVAL, "nclass must be in [2, 64]");
    if (!perm_out || !class_start_out) return fail(ctx, ALS_EINVAL, "null pointer");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    int32_t *cs_dev = nullptr;
    HIP_TRY(ctx, hipMalloc(&cs_dev, sizeof(int32_t) * 65));
    void *tmp = nullptr;     // scratch of this call (the context's may be a fixed piece of a workspace)
    size_t tmp_bytes = 0;
    hipError_t e = plan_bin_rows(csr->ptr_is_64 != 0, ctx->stream, csr->nrows, csr->ptr, nclass, perm_out, cs_dev,
                                 &tmp, &tmp_bytes, false);
    int32_t cs[65];
    if (e == hipSuccess)
        e = hipMemcpyAsync(cs, cs_dev, sizeof(int32_t) * (size_t)(nclass + 1), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    hipFree(cs_dev);
    hipFree(tmp);
    if (e != hipSuccess) return fail_hip(ctx, e, "als_bin_rows");
    for (int c = 0; c <= nclass; ++c) class_start_out[c] = cs[c];
    return ALS_OK;
}

static int als_csr_to_csc_impl(als_ctx *ctx, const als_sparse *csr, void *cptr_out, int32_t *cidx_out, float *cval_out) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, csr);
    if (rc != ALS_OK) return rc;
    if (csr->nnz > 0xffffffffll) return fail(ctx, ALS_EINVAL, "als_csr_to_csc needs nnz < 2^32");
    if (!cptr_out || (csr->nnz > 0 && (!cidx_out || !cval_out))) return fail(ctx, ALS_EINVAL, "null pointer");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    hipError_t e = transpose_csr(csr->ptr_is_64 != 0, ctx->stream, csr->nrows, csr->ncols, csr->nnz, csr->ptr,
                                 csr->idx, csr->val, cptr_out, cidx_out, cval_out);
    if (e != hipSuccess) return fail_hip(ctx, e, "als_csr_to_csc");
    return ALS_OK;
}

static int als_synchronize_impl(als_ctx *ctx) {
    if (!ctx) return ALS_EINVAL;
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    int st = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&st, ctx->status, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (st != 0) {
        HIP_TRY(ctx, fill_zero(ctx->stream, ctx->status, 1));
        std::string msg;
        if (st & kStatusBadPivot) msg += "non-positive pivot in the exact solver; ";
        if (st & kStatusNonFinite) msg += "non-finite value in a solution; ";
        if (st & kStatusStalePlan)
            msg += "the row offsets of a matrix changed after its work plan was built: results are invalid, call als_drop_plans; ";
        return fail(ctx, (st & kStatusStalePlan) ? ALS_EINVAL : ALS_ENUMERIC, msg);
    }
    return ALS_OK;
}

static int als_kernel_time_impl(als_ctx *ctx, int kernel_id, double *ms_out, int64_t *launches_out) {
    if (!ctx || !ms_out || !launches_out) return ALS_EINVAL;
    if (kernel_id < 0 || kernel_id >= ALS_K_COUNT) return fail(ctx, ALS_EINVAL, "unknown kernel id");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    double ms = 0.0;
    int64_t n = 0;
    for (auto &t : ctx->timed)
        if (t.kernel == kernel_id) {
            float dt = 0.f;
            HIP_TRY(ctx, hipEventElapsedTime(&dt, t.a, t.b));
            ms += dt;
            ++n;
        }
    *ms_out = ms;
    *launches_out = n;
    return ALS_OK;
}

static int als_profile_reset_impl(als_ctx *ctx) {
    if (!ctx) return ALS_EINVAL;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (auto &t : ctx->timed) { ctx->free_events.push_back(t.a); ctx->free_events.push_back(t.b); }
    ctx->timed.clear();
    return ALS_OK;
}

static int als_check_matrix_impl(als_ctx *ctx, const als_sparse *a) {
    if (!ctx) return ALS_EINVAL;
    int rc = check_sparse(ctx, a);
    if (rc != ALS_OK) return rc;
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    if (!ctx->check_flags) HIP_TRY(ctx, hipMalloc(&ctx->check_flags, sizeof(int)));
    const bool p64 = a->ptr_is_64 != 0;
    int flags = 0;
    HIP_TRY(ctx, fill_zero(ctx->stream, ctx->check_flags, 1));
    HIP_TRY(ctx, check_ptr(p64, ctx->stream, a->ptr, a->nrows, a->nnz, ctx->check_flags));
    HIP_TRY(ctx, hipMemcpyAsync(&flags, ctx->check_flags, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (flags == 0) {   // the index check walks ptr: only with sound offsets
        HIP_TRY(ctx, check_idx(p64, ctx->stream, a->ptr, a->idx, a->nrows, a->ncols, a->nnz, ctx->check_flags));
        HIP_TRY(ctx, hipMemcpyAsync(&flags, ctx->check_flags, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    if (flags == 0) return ALS_OK;
    std::string msg;
    if (flags & 1) msg += "row offsets are not an ascending sequence from 0 to nnz; ";
    if (flags & 2) msg += "a column id lies outside [0, ncols); ";
    if (flags & 4) msg += "the column ids of a row are not strictly ascending; ";
    return fail(ctx, ALS_EINVAL, msg);
}

static int als_measure_peak_impl(als_ctx *ctx, int what, double *rate_out) {
    if (!ctx) return ALS_EINVAL;
    if (!rate_out) return fail(ctx, ALS_EINVAL, "null pointer");
    if (what < ALS_PEAK_MFMA_F32 || what > ALS_PEAK_COPY) return fail(ctx, ALS_EINVAL, "unknown peak id");
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    int cus = 0;
    HIP_TRY(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->cfg.device));
    const int workgroups = 8 * cus;   // 8 wavefronts per SIMD
    const int64_t bytes = 1ll << 30;
    char *buf = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    double work = 0.0;
    hipError_t e = hipMalloc(&buf, what == ALS_PEAK_COPY ? (size_t)(2 * bytes) : (size_t)4096);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    float ms = 0.f;
    for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {   // the first pass warms up (clocks, code, pages)
        e = hipEventRecord(e0, ctx->stream);
        if (e != hipSuccess) break;
        if (what == ALS_PEAK_COPY) {
            for (int k = 0; k < 10 && e == hipSuccess; ++k) e = launch_copy(ctx->stream, 32 * cus, buf, buf + bytes, bytes);
            work = 10.0 * 2.0 * (double)bytes;   // read + written
        } else {
            const int et = what == ALS_PEAK_MFMA_F32 ? ALS_F32 : what == ALS_PEAK_MFMA_BF16 ? ALS_BF16 : ALS_F16;
            e = launch_mfma_peak(et, ctx->stream, workgroups, 20000, (float *)buf, &work);
        }
        if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    }
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    hipFree(buf);
    if (e != hipSuccess) return fail_hip(ctx, e, "als_measure_peak");
    *rate_out = work / ((double)ms * 1e-3);
    return ALS_OK;
}

static int als_drop_plans_impl(als_ctx *ctx) {
    if (!ctx) return ALS_EINVAL;
    DeviceGuard on_device;
    HIP_TRY(ctx, on_device.enter(ctx->cfg.device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (auto &p : ctx->plans) free_plan(ctx, p);
    ctx->next_plan = 0;
    ctx->arena_used = 0;
    return ALS_OK;
}

// The entry points proper: nothing is thrown across the C boundary.
int als_update_rows(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f, float *X) {
    return guarded(ctx, [&] { return als_update_rows_impl(ctx, csr, Theta, lambda, f, X); });
}

int als_update_cols(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, int f, float *Theta) {
    return guarded(ctx, [&] { return als_update_cols_impl(ctx, csc, X, lambda, f, Theta); });
}

int als_update_rows_implicit(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, float alpha, int f, float *X) {
    return guarded(ctx, [&] { return als_update_rows_implicit_impl(ctx, csr, Theta, lambda, alpha, f, X); });
}

int als_update_cols_implicit(als_ctx *ctx, const als_sparse *csc, const void *X, float lambda, float alpha, int f, float *Theta) {
    return guarded(ctx, [&] { return als_update_cols_implicit_impl(ctx, csc, X, lambda, alpha, f, Theta); });
}

int als_gram(als_ctx *ctx, const float *G, int64_t n, int f, float *out) {
    return guarded(ctx, [&] { return als_gram_impl(ctx, G, n, f, out); });
}

int als_gram_static(als_ctx *ctx, const float *G, int64_t n, int f, float *out) {
    return guarded(ctx, [&] { return als_gram_static_impl(ctx, G, n, f, out); });
}

int als_implicit_loss(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, float lambda, float alpha, int f, double *loss_out) {
    return guarded(ctx, [&] { return als_implicit_loss_impl(ctx, csr, X, Theta, lambda, alpha, f, loss_out); });
}

int als_rmse(als_ctx *ctx, const als_sparse *csr, const float *X, const float *Theta, int f, double *rmse_out) {
    return guarded(ctx, [&] { return als_rmse_impl(ctx, csr, X, Theta, f, rmse_out); });
}

int als_hermitian(als_ctx *ctx, const als_sparse *csr, const void *Theta, float lambda, int f, int64_t row0, int64_t nrows, float *A_out, float *b_out) {
    return guarded(ctx, [&] { return als_hermitian_impl(ctx, csr, Theta, lambda, f, row0, nrows, A_out, b_out); });
}

int als_bin_rows(als_ctx *ctx, const als_sparse *csr, int nclass, int32_t *perm_out, int64_t *class_start_out) {
    return guarded(ctx, [&] { return als_bin_rows_impl(ctx, csr, nclass, perm_out, class_start_out); });
}

int als_csr_to_csc(als_ctx *ctx, const als_sparse *csr, void *cptr_out, int32_t *cidx_out, float *cval_out) {
    return guarded(ctx, [&] { return als_csr_to_csc_impl(ctx, csr, cptr_out, cidx_out, cval_out); });
}

int als_synchronize(als_ctx *ctx) {
    return guarded(ctx, [&] { return als_synchronize_impl(ctx); });
}

int als_kernel_time(als_ctx *ctx, int kernel_id, double *ms_out, int64_t *launches_out) {
    return guarded(ctx, [&] { return als_kernel_time_impl(ctx, kernel_id, ms_out, launches_out); });
}

int als_profile_reset(als_ctx *ctx) {
    return guarded(ctx, [&] { return als_profile_reset_impl(ctx); });
}

int als_drop_plans(als_ctx *ctx) {
    return guarded(ctx, [&] { return als_drop_plans_impl(ctx); });
}

int als_check_matrix(als_ctx *ctx, const als_sparse *a) {
    return guarded(ctx, [&] { return als_check_matrix_impl(ctx, a); });
}

int als_short_row_limit(const als_ctx *ctx) { return ctx ? short_row_limit(ctx->cfg) : 0; }

int als_measure_peak(als_ctx *ctx, int what, double *rate_out) {
    return guarded(ctx, [&] { return als_measure_peak_impl(ctx, what, rate_out); });
}

}  // extern "C"
