// Handle, device-memory cache, options, statistics, error strings.
#include "common.hpp"

#include <chrono>
#include "chain.hpp"

#include <algorithm>
#include <new>

namespace tsp {

static void *default_alloc(void *, size_t bytes, void *) {
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return p;
}
static void default_free(void *, void *p, void *) { (void)hipFree(p); }

int hip_fail(tsp_context *ctx, hipError_t e) {
    if (ctx) ctx->last_hip = (int)e;
    (void)hipGetLastError();
    return TSP_ERR_HIP;
}

// Canaries (TSP_OPT_WORKSPACE_CANARIES): every block gets a guard zone of kGuardBytes in front of the caller's
// part and one behind it, filled with a pattern when the block is handed out and compared when it comes back;
// words that changed are counted in the slot behind the handle's scalar block.
constexpr size_t kGuardBytes = 256;
constexpr uint32_t kGuardWord = 0xA5C3965Au;
__global__ void k_guard_fill(uint32_t *front, uint32_t *back) {
    front[threadIdx.x] = kGuardWord;
    back[threadIdx.x] = kGuardWord;
}
__global__ void k_guard_check(const uint32_t *front, const uint32_t *back, unsigned long long *violations) {
    const unsigned bad = (front[threadIdx.x] != kGuardWord) + (back[threadIdx.x] != kGuardWord);
    if (bad) atomicAdd(violations, (unsigned long long)bad);
}

// Best fit from the cache; a cached block is taken only if it wastes at most half of itself.
void *ctx_alloc(tsp_context *ctx, size_t bytes, hipStream_t s) {
    bytes = (bytes + 255) & ~size_t(255);
    if (bytes == 0) bytes = 256;
    const size_t user_bytes = bytes;
    const bool guarded = ctx->canaries != 0;
    if (guarded) bytes += 2 * kGuardBytes;
    int best = -1;
    for (int i = 0; i < (int)ctx->cache.size(); ++i) {
        size_t b = ctx->cache[i].bytes;
        if (b >= bytes && b <= 2 * bytes + 4096 && (best < 0 || b < ctx->cache[best].bytes)) best = i;
    }
    void *p;
    size_t got;
    if (best >= 0) {
        p = ctx->cache[best].ptr;
        got = ctx->cache[best].bytes;
        ctx->cache[best] = ctx->cache.back();
        ctx->cache.pop_back();
    } else {
        p = ctx->allocator.alloc(ctx->allocator.user, bytes, (void *)s);
        if (!p) {
            // give cached memory back and retry once
            for (auto &b : ctx->cache) {
                ctx->allocator.free(ctx->allocator.user, b.ptr, (void *)s);
                ctx->held_bytes -= (int64_t)b.bytes;
            }
            ctx->cache.clear();
            p = ctx->allocator.alloc(ctx->allocator.user, bytes, (void *)s);
            if (!p) return nullptr;
        }
        got = bytes;
        ctx->held_bytes += (int64_t)got;
        ctx->peak_bytes = std::max(ctx->peak_bytes, ctx->held_bytes);
    }
    void *user = p;
    if (guarded) {
        user = static_cast<char *>(p) + kGuardBytes;
        hipLaunchKernelGGL(k_guard_fill, dim3(1), dim3(kGuardBytes / 4), 0, s, static_cast<uint32_t *>(p),
                           reinterpret_cast<uint32_t *>(static_cast<char *>(user) + user_bytes));
    }
    ctx->live.emplace(user, LiveBlock{p, got, user_bytes, guarded});
    return user;
}

void ctx_free(tsp_context *ctx, void *p, hipStream_t s) {
    if (!p) return;
    auto it = ctx->live.find(p);
    if (it == ctx->live.end()) return;   // not ours: ignore
    const LiveBlock b = it->second;
    if (b.guarded)
        hipLaunchKernelGGL(k_guard_check, dim3(1), dim3(kGuardBytes / 4), 0, s, static_cast<const uint32_t *>(b.base),
                           reinterpret_cast<const uint32_t *>(static_cast<char *>(p) + b.user_bytes),
                           reinterpret_cast<unsigned long long *>(ctx->d_scalars + kScalars));
    ctx->cache.push_back({b.base, b.bytes});
    ctx->live.erase(it);
}

int read_scalars(tsp_context *ctx, hipStream_t s) {
    TSP_HIP_CHECK(ctx, hipMemcpyAsync(ctx->h_scalars, ctx->d_scalars, sizeof(int64_t) * kScalars,
                                      hipMemcpyDeviceToHost, s));
    TSP_HIP_CHECK(ctx, hipStreamSynchronize(s));
    return TSP_OK;
}

int wait_published_scalars(tsp_context *ctx, int64_t tag, hipStream_t s) {
    // The kernel is short (tens of microseconds after the launch): poll the mirror for a while before
    // falling back to a blocking wait, whose wake-up alone costs several microseconds.  The publication is
    // complete when every slot carries its tag; the tags are then taken off.
    const uint64_t want = publish_tag16(tag);
    auto complete = [&]() {
        for (int i = 0; i < kScalars; ++i)
            if (((uint64_t)__atomic_load_n(&ctx->h_scalars[i], __ATOMIC_ACQUIRE) >> kPublishTagShift) != want) return false;
        return true;
    };
    auto strip = [&]() {
        for (int i = 0; i < kScalars; ++i) ctx->h_scalars[i] &= (int64_t)((1ull << kPublishTagShift) - 1u);
        return TSP_OK;
    };
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spins = 0;; ++spins) {
        if (complete()) return strip();
        if ((spins & 1023) == 1023 &&
            std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(500)) break;
    }
    TSP_HIP_CHECK(ctx, hipStreamSynchronize(s));
    if (!complete()) return hip_fail(ctx, hipErrorUnknown);
    return strip();
}

void *chain_prepare(tsp_context *ctx, int64_t blocks, unsigned *epoch, hipStream_t s) {
    if (blocks > ctx->chain_capacity || ctx->chain_epoch >= (1u << 29)) {
        const int64_t want = blocks > ctx->chain_capacity ? (blocks < 1024 ? 1024 : 2 * blocks) : ctx->chain_capacity;
        if (want != ctx->chain_capacity) {
            if (ctx->chain_slots) ctx_free(ctx, ctx->chain_slots, s);
            ctx->chain_slots = ctx_alloc(ctx, (size_t)want * sizeof(ChainSlot), s);
            ctx->chain_capacity = ctx->chain_slots ? want : 0;
            if (!ctx->chain_slots) return nullptr;
        }
        // all flags to "no epoch"; epochs restart at 1
        if (hipMemsetAsync(ctx->chain_slots, 0, (size_t)ctx->chain_capacity * sizeof(ChainSlot), s) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        ctx->chain_epoch = 0;
    }
    *epoch = ++ctx->chain_epoch;
    return ctx->chain_slots;
}

static void ensure_events(tsp_context *ctx) {
    if (ctx->ev_created) return;
    for (auto &e : ctx->ev) (void)hipEventCreate(&e);
    for (auto &e : ctx->kev) (void)hipEventCreate(&e);
    ctx->ev_created = true;
}
void phase_begin(tsp_context *ctx, int phase, hipStream_t s) {
    if (!ctx->timers) return;
    ensure_events(ctx);
    // a phase entered more than once in a call (conversion of A, then of B) keeps its first begin
    if (!ctx->ev_recorded[2 * phase]) {
        (void)hipEventRecord(ctx->ev[2 * phase], s);
        ctx->ev_recorded[2 * phase] = true;
    }
}
void phase_end(tsp_context *ctx, int phase, hipStream_t s) {
    if (!ctx->timers) return;
    ensure_events(ctx);
    (void)hipEventRecord(ctx->ev[2 * phase + 1], s);
    ctx->ev_recorded[2 * phase + 1] = true;
}
void total_begin(tsp_context *ctx, hipStream_t s) {
    if (!ctx->timers) return;
    ensure_events(ctx);
    for (auto &r : ctx->ev_recorded) r = false;
    for (auto &r : ctx->kev_recorded) r = false;
    (void)hipEventRecord(ctx->ev[2 * TSP_PHASE_COUNT_], s);
    ctx->ev_recorded[2 * TSP_PHASE_COUNT_] = true;
}
void total_end(tsp_context *ctx, hipStream_t s) {
    if (!ctx->timers) return;
    (void)hipEventRecord(ctx->ev[2 * TSP_PHASE_COUNT_ + 1], s);
    ctx->ev_recorded[2 * TSP_PHASE_COUNT_ + 1] = true;
}
void collect_timers(tsp_context *ctx) {
    if (!ctx->timers || !ctx->ev_created) return;
    for (int p = 0; p <= TSP_PHASE_COUNT_; ++p) {
        float ms = 0.f;
        float *dst = p < TSP_PHASE_COUNT_ ? &ctx->stats.phase_us[p] : &ctx->stats.total_us;
        *dst = 0.f;
        if (ctx->ev_recorded[2 * p] && ctx->ev_recorded[2 * p + 1] &&
            hipEventElapsedTime(&ms, ctx->ev[2 * p], ctx->ev[2 * p + 1]) == hipSuccess)
            *dst = ms * 1000.f;
        else
            (void)hipGetLastError();
    }
    for (int k = 0; k < TSP_KERNEL_COUNT_; ++k) {
        float ms = 0.f;
        ctx->stats.kernel_us[k] = 0.f;
        if (ctx->kev_recorded[k] && hipEventElapsedTime(&ms, ctx->kev[2 * k], ctx->kev[2 * k + 1]) == hipSuccess)
            ctx->stats.kernel_us[k] = ms * 1000.f;
        else
            (void)hipGetLastError();
    }
}

KernelTimer::KernelTimer(tsp_context *c, int kernel_id, hipStream_t stream) : ctx(c), id(kernel_id), s(stream) {
    if (!ctx->timers) return;
    ensure_events(ctx);
    (void)hipEventRecord(ctx->kev[2 * id], s);
}
KernelTimer::~KernelTimer() {
    if (!ctx->timers) return;
    (void)hipEventRecord(ctx->kev[2 * id + 1], s);
    ctx->kev_recorded[id] = true;
}

}  // namespace tsp

using namespace tsp;

extern "C" int tsp_create(tsp_handle *handle, const tsp_allocator *allocator) {
    if (!handle) return TSP_ERR_INVALID_ARG;
    *handle = nullptr;
    if (allocator && (!allocator->alloc || !allocator->free)) return TSP_ERR_INVALID_ARG;
    tsp_context *ctx = new (std::nothrow) tsp_context();
    if (!ctx) return TSP_ERR_ALLOC_FAILED;
    if (allocator) {
        ctx->allocator = *allocator;
        ctx->user_allocator = true;
    } else {
        ctx->allocator = {default_alloc, default_free, nullptr};
    }
    hipError_t e = hipGetDevice(&ctx->device);
    // (one slot behind the scalar block counts the words of guard zones found changed; no kernel clears it)
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->d_scalars, sizeof(int64_t) * (kScalars + 1));
    if (e == hipSuccess) e = hipMemset(ctx->d_scalars, 0, sizeof(int64_t) * (kScalars + 1));
    if (e == hipSuccess) e = hipHostMalloc((void **)&ctx->h_scalars, sizeof(int64_t) * kScalars,
                                             hipHostMallocCoherent | hipHostMallocMapped);   // polled: fine-grained whatever the environment says
    if (e == hipSuccess) e = hipHostGetDevicePointer((void **)&ctx->h_scalars_dev, ctx->h_scalars, 0);
    if (e == hipSuccess) std::memset(ctx->h_scalars, 0, sizeof(int64_t) * kScalars);
    if (e != hipSuccess) {
        if (ctx->h_scalars) (void)hipHostFree(ctx->h_scalars);
        if (ctx->d_scalars) (void)hipFree(ctx->d_scalars);
        (void)hipGetLastError();
        delete ctx;
        return TSP_ERR_HIP;
    }
    if (static_scratch_setup(ctx, nullptr) != TSP_OK) {      // address of the no-allocation scratch on this device
        (void)hipHostFree(ctx->h_scalars);
        (void)hipFree(ctx->d_scalars);
        delete ctx;
        return TSP_ERR_HIP;
    }
    *handle = ctx;
    return TSP_OK;
}

extern "C" int tsp_destroy(tsp_handle ctx) {
    if (!ctx) return TSP_ERR_INVALID_ARG;
    (void)hipDeviceSynchronize();
    for (auto &b : ctx->cache) ctx->allocator.free(ctx->allocator.user, b.ptr, nullptr);
    for (auto &kv : ctx->live) ctx->allocator.free(ctx->allocator.user, kv.second.base, nullptr);
    if (ctx->ev_created)
    {
        for (auto &e : ctx->ev) (void)hipEventDestroy(e);
        for (auto &e : ctx->kev) (void)hipEventDestroy(e);
    }
    (void)hipFree(ctx->d_scalars);
    (void)hipHostFree(ctx->h_scalars);
    delete ctx;
    return TSP_OK;
}

extern "C" int tsp_set_option(tsp_handle ctx, int key, int64_t value) {
    if (!ctx) return TSP_ERR_INVALID_ARG;
    switch (key) {
        case TSP_OPT_VALIDATE: ctx->validate = value != 0; return TSP_OK;
        case TSP_OPT_PHASE_TIMERS: ctx->timers = value != 0; return TSP_OK;
        case TSP_OPT_WIDE_INDEX: ctx->force_wide = value != 0; return TSP_OK;
        case TSP_OPT_COMPACT_ZEROS: ctx->compact = value != 0; return TSP_OK;
        case TSP_OPT_MATRIX_CORES: ctx->matrix_cores = value != 0; return TSP_OK;
        case TSP_OPT_WORK_ORDER:
            if (value < 0 || value > 2) return TSP_ERR_INVALID_ARG;
            ctx->work_order = (int)value;
            return TSP_OK;
        case TSP_OPT_COUNT_PRODUCTS: ctx->count_products = value != 0; return TSP_OK;
        case TSP_OPT_WORKSPACE_CANARIES:
            ctx->canaries = value != 0;
            ctx->canaries_used = ctx->canaries_used || value != 0;
            return TSP_OK;
        case TSP_OPT_STRIP_ORDER:
            if (value < 0 || (value > 2 && value < 16) || value > (1 << 30)) return TSP_ERR_INVALID_ARG;
            ctx->strip_order = (int)value;
            return TSP_OK;
        case TSP_OPT_NUMERIC_RUN:
            if (value != 0 && value != 4 && value != 8) return TSP_ERR_INVALID_ARG;
            ctx->numeric_run_len = (int)value;
            return TSP_OK;
        default: return TSP_ERR_INVALID_ARG;
    }
}

extern "C" int tsp_trim(tsp_handle ctx, void *stream) {
    if (!ctx) return TSP_ERR_INVALID_ARG;
    TSP_HIP_CHECK(ctx, hipStreamSynchronize((hipStream_t)stream));
    for (auto &b : ctx->cache) {
        ctx->allocator.free(ctx->allocator.user, b.ptr, stream);
        ctx->held_bytes -= (int64_t)b.bytes;
    }
    ctx->cache.clear();
    return TSP_OK;
}

extern "C" int tsp_get_stats(tsp_handle ctx, tsp_stats *out) {
    if (!ctx || !out) return TSP_ERR_INVALID_ARG;
    ctx->stats.workspace_bytes = ctx->held_bytes;
    ctx->stats.workspace_peak_bytes = ctx->peak_bytes;
    int64_t changed = 0;
    if (ctx->canaries_used)                                // (a blocking copy: the checks enqueued so far have run)
        TSP_HIP_CHECK(ctx, hipMemcpy(&changed, ctx->d_scalars + kScalars, sizeof(int64_t), hipMemcpyDeviceToHost));
    ctx->stats.workspace_violations = changed;
    *out = ctx->stats;
    return TSP_OK;
}

extern "C" int tsp_last_hip_error(tsp_handle ctx) { return ctx ? ctx->last_hip : 0; }

extern "C" const char *tsp_strerror(int status) {
    switch (status) {
        case TSP_OK: return "success";
        case TSP_ERR_INVALID_ARG: return "invalid argument";
        case TSP_ERR_SHAPE_MISMATCH: return "inner dimensions differ (A.cols != B.rows)";
        case TSP_ERR_NOT_CANONICAL: return "input CSR is not canonical";
        case TSP_ERR_ALLOC_FAILED: return "device allocation failed";
        case TSP_ERR_INDEX_OVERFLOW: return "a size exceeds the index width of the format";
        case TSP_ERR_HIP: return "HIP runtime error";
        case TSP_ERR_UNSUPPORTED: return "a limit of this build is exceeded";
        default: return "unknown status";
    }
}

extern "C" int tsp_csr_free(tsp_handle ctx, tsp_csr *C, void *stream) {
    if (!ctx || !C) return TSP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    ctx_free(ctx, C->row_ptr, s);
    ctx_free(ctx, C->col_idx, s);
    ctx_free(ctx, C->val, s);
    std::memset(C, 0, sizeof(*C));
    return TSP_OK;
}
