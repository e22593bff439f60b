// Compaction of zeros (paper Section 4.4; the two compaction steps that end Algorithm 1): the multiplication pass writes
// every structural position of C; numerical cancellation (and stored zeros in the inputs) leaves
// some of them with the value 0.  This pass removes them, so that the result is strictly sparse:
// count the survivors per row, prefix-sum into the new row_ptr, copy the survivors in order.
// The paper compacts the element array with a library primitive and drops empty tiles; here the
// output is already CSR, so a row-wise stream compaction does both.
#include "common.hpp"

#include <mutex>

namespace tsp {

constexpr int kCompactThreads = 256;
constexpr int kCompactLanes = 16;              // lanes that share one CSR row

template <typename RP>
struct CompactArgs {
    const RP *row_ptr;
    const int32_t *col;
    const float *val;
    int64_t rows, nnz;
};

// Entry range of a row, clamped so that a row_ptr that is not monotone or runs past nnz cannot
// take a read or a write out of bounds (count and copy see the same ranges).
template <typename RP>
__device__ __forceinline__ void row_range(const CompactArgs<RP> &a, int64_t row, int64_t &e0, int64_t &e1) {
    e0 = min(max((int64_t)a.row_ptr[row], (int64_t)0), a.nnz);
    e1 = min(max((int64_t)a.row_ptr[row + 1], e0), a.nnz);
}

// +0.0 and -0.0 are zeros, NaN is not
__device__ __forceinline__ bool survives(float v) { return !(v == 0.0f); }

// A block counts 16 consecutive rows; their sum goes to group_keep (what row_ptr_in_one_launch wants).
// Rows of a few hundred entries at most: 16 lanes each.  Where the block's 16 rows hold more than
// kCompactLongSpan entries together (products of graphs: thousands of entries per row, a hundred thousand in
// a hub's), the whole block takes the rows one after the other, 256 consecutive entries per step, so that a
// long row is not left to 16 lanes.
static_assert(kCompactThreads / kCompactLanes == T, "a block covers one group of 16 rows");
constexpr int64_t kCompactLongSpan = 4096;

// entries of the block's rows [r0, r1) together (block-uniform)
template <typename RP>
__device__ __forceinline__ int64_t block_span(const CompactArgs<RP> &a, int64_t r0, int64_t r1) {
    int64_t b0, b1, e0, e1;
    row_range(a, r0, b0, e0);
    row_range(a, r1 - 1, b1, e1);
    return e1 - b0;
}

template <typename RP>
__global__ __launch_bounds__(kCompactThreads) void k_compact_count(CompactArgs<RP> a, int32_t *__restrict__ keep,
                                                                  uint32_t *__restrict__ group_keep) {
    __shared__ int s_rows[T];
    const int64_t r0 = (int64_t)blockIdx.x * T, r1 = min(r0 + T, a.rows);
    if (r0 < a.rows && block_span(a, r0, r1) > kCompactLongSpan) {       // (whole block)
        if (threadIdx.x < T) s_rows[threadIdx.x] = 0;
        __syncthreads();
        for (int64_t row = r0; row < r1; ++row) {
            int64_t e0, e1;
            row_range(a, row, e0, e1);
            int n = 0;
            for (int64_t e = e0 + threadIdx.x; e < e1; e += kCompactThreads) n += survives(a.val[e]) ? 1 : 0;
            n = (int)wave_sum((uint32_t)n);
            if ((threadIdx.x & 63) == 0 && n) atomicAdd(&s_rows[row - r0], n);
        }
        __syncthreads();
        if (threadIdx.x < T && r0 + threadIdx.x < a.rows) keep[r0 + threadIdx.x] = s_rows[threadIdx.x];
    } else {
        const int64_t row = r0 + threadIdx.x / kCompactLanes;
        const int l = threadIdx.x % kCompactLanes;
        int n = 0;
        if (row < a.rows) {                        // whole 16-lane groups
            int64_t e0, e1;
            row_range(a, row, e0, e1);
            for (int64_t e = e0 + l; e < e1; e += kCompactLanes) n += survives(a.val[e]) ? 1 : 0;
        }
#pragma unroll
        for (int d = kCompactLanes / 2; d > 0; d >>= 1) n += __shfl_xor(n, d, kCompactLanes);
        if (l == 0) {
            if (row < a.rows) keep[row] = n;
            s_rows[threadIdx.x / kCompactLanes] = n;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        uint32_t sum = 0;
        for (int r = 0; r < T; ++r) sum += r0 + r < a.rows ? (uint32_t)s_rows[r] : 0u;
        group_keep[blockIdx.x] = sum;
    }
    // zeros behind the last group, up to a multiple of four entries (the array has four spare ones)
    if (blockIdx.x == 0 && threadIdx.x < 4) group_keep[gridDim.x + threadIdx.x] = 0;
}

template <typename RP>
__global__ __launch_bounds__(kCompactThreads) void k_compact_fill(CompactArgs<RP> a,
                                                                 const int64_t *__restrict__ new_row_ptr,
                                                                 int32_t *__restrict__ out_col,
                                                                 float *__restrict__ out_val) {
    const int64_t r0 = (int64_t)blockIdx.x * T, r1 = min(r0 + T, a.rows);
    if (r0 >= a.rows) return;
    if (block_span(a, r0, r1) > kCompactLongSpan) {                      // (whole block)
        __shared__ uint32_t s_wave[2][kCompactThreads / 64];              // survivors per wave, two steps in flight
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        int step = 0;
        for (int64_t row = r0; row < r1; ++row) {
            int64_t e0, e1;
            row_range(a, row, e0, e1);
            int64_t at = new_row_ptr[row];
            for (int64_t base = e0; base < e1; base += kCompactThreads, step ^= 1) {   // the whole block runs every trip
                const int64_t e = base + threadIdx.x;
                const bool in = e < e1;
                const float v = in ? a.val[e] : 0.0f;
                const bool on = in && survives(v);
                const unsigned long long mine = __ballot(on);
                if (lane == 0) s_wave[step][wave] = (uint32_t)__popcll(mine);
                __syncthreads();                   // (the other buffer is free again: every wave has passed the barrier of the step before)
                uint32_t before = 0, all = 0;
#pragma unroll
                for (int w = 0; w < kCompactThreads / 64; ++w) {
                    const uint32_t n = s_wave[step][w];
                    before += w < wave ? n : 0u;
                    all += n;
                }
                if (on) {
                    const int64_t p = at + before + __popcll(mine & ((1ull << lane) - 1ull));
                    out_col[p] = a.col[e];
                    out_val[p] = v;
                }
                at += all;
            }
        }
        return;
    }
    const int64_t row = r0 + threadIdx.x / kCompactLanes;
    const int l = threadIdx.x % kCompactLanes;
    if (row >= a.rows) return;
    int64_t e0, e1;
    row_range(a, row, e0, e1);
    int64_t at = new_row_ptr[row];
    const int shift = (threadIdx.x & 63) / kCompactLanes * kCompactLanes;   // this group's bits in the wave ballot
    for (int64_t e = e0; e < e1; e += kCompactLanes) {                     // the 16 lanes run the same trip count
        const bool in = e + l < e1;
        const float v = in ? a.val[e + l] : 0.0f;
        const bool on = in && survives(v);
        const uint32_t mine = (uint32_t)(__ballot(on) >> shift) & 0xFFFFu;
        if (on) {
            const int64_t p = at + __popc(mine & ((1u << l) - 1u));
            out_col[p] = a.col[e + l];
            out_val[p] = v;
        }
        at += __popc(mine);
    }
}

__global__ void k_compact_clear(int64_t *d_scalars) {
    if (threadIdx.x == 0) {
        d_scalars[S_INTERNAL] = 0;
        d_scalars[S_C_NNZ] = 0;
    }
}

template <typename RP>
static int compact_run(tsp_context *ctx, const tsp_csr *C, tsp_csr *out, hipStream_t s, bool *taken) {
    const int64_t rows = C->rows;
    CompactArgs<RP> a{static_cast<const RP *>(C->row_ptr), C->col_idx, static_cast<const float *>(C->val), rows, C->nnz};
    int32_t *keep = ctx_alloc_n<int32_t>(ctx, (size_t)rows + 1, s);
    int64_t *new_row_ptr = ctx_alloc_n<int64_t>(ctx, (size_t)rows + 1, s);
    int32_t *col = nullptr;
    float *val = nullptr;
    const int64_t row_blocks = (rows * kCompactLanes + kCompactThreads - 1) / kCompactThreads;   // groups of 16 rows
    uint32_t *group_keep = ctx_alloc_n<uint32_t>(ctx, (size_t)row_blocks + 4, s);
    auto fail = [&](int code) {
        ctx_free(ctx, keep, s);
        ctx_free(ctx, group_keep, s);
        ctx_free(ctx, new_row_ptr, s);
        ctx_free(ctx, col, s);
        ctx_free(ctx, val, s);
        return code;
    };
    if (!keep || !new_row_ptr || !group_keep) return fail(TSP_ERR_ALLOC_FAILED);
    if (!ctx->scalars_clean) hipLaunchKernelGGL(k_compact_clear, dim3(1), dim3(64), 0, s, ctx->d_scalars);
    ctx->scalars_clean = false;
    if (rows > 0)
        hipLaunchKernelGGL(k_compact_count<RP>, dim3((unsigned)row_blocks), dim3(kCompactThreads), 0, s, a, keep,
                           group_keep);
    // new row_ptr = exclusive prefix of the survivor counts, the total to the scalar block and on to the host:
    // one launch that writes the scalars into the host's mirror itself, or three and a copy for very many rows
    int rc = TSP_OK;
    if (row_ptr_in_one_launch(ctx, keep, rows, group_keep, new_row_ptr, s)) {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(hip_fail(ctx, e));
        rc = wait_published_scalars(ctx, ctx->publish_tag, s);   // host synchronisation: the new nnz
    } else {
        int64_t *tmp = ctx_alloc_n<int64_t>(ctx, scan_tmp_entries(rows), s);
        if (!tmp) return fail(TSP_ERR_ALLOC_FAILED);
        rc = scan_exclusive_i32_to_i64(ctx, keep, new_row_ptr, rows, ctx->d_scalars + S_C_NNZ, nullptr, tmp, s);
        ctx_free(ctx, tmp, s);
        if (rc) return fail(rc);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(hip_fail(ctx, e));
        rc = read_scalars(ctx, s);                           // host synchronisation: the new nnz
    }
    if (rc) return fail(rc);
    if (ctx->h_scalars[S_INTERNAL]) return fail(TSP_ERR_HIP);
    const int64_t nnz = ctx->h_scalars[S_C_NNZ];
    if (taken && nnz == C->nnz) {                        // nothing to drop: the caller's arrays are the result
        fail(TSP_OK);                                    // (releases the scratch arrays)
        *out = *C;
        *taken = true;
        return TSP_OK;
    }
    col = ctx_alloc_n<int32_t>(ctx, (size_t)nnz, s);
    val = ctx_alloc_n<float>(ctx, (size_t)nnz, s);
    if (!col || !val) return fail(TSP_ERR_ALLOC_FAILED);
    if (rows > 0 && nnz > 0) {
        hipLaunchKernelGGL(k_compact_fill<RP>, dim3((unsigned)row_blocks), dim3(kCompactThreads), 0, s, a, new_row_ptr,
                           col, val);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(hip_fail(ctx, e));
    }
    ctx_free(ctx, keep, s);
    ctx_free(ctx, group_keep, s);
    out->rows = C->rows;
    out->cols = C->cols;
    out->nnz = nnz;
    out->row_ptr = new_row_ptr;
    out->col_idx = col;
    out->val = val;
    out->row_ptr_type = TSP_I64;
    out->val_type = TSP_F32;
    return TSP_OK;
}

int compact_zeros(tsp_context *ctx, const tsp_csr *C, tsp_csr *out, hipStream_t s, bool *taken) {
    std::memset(out, 0, sizeof(*out));
    if (taken) *taken = false;
    if (C->rows < 0 || C->cols < 0 || C->nnz < 0 || !C->row_ptr) return TSP_ERR_INVALID_ARG;
    if (C->val_type != TSP_F32) return TSP_ERR_INVALID_ARG;
    if (C->nnz > 0 && (!C->col_idx || !C->val)) return TSP_ERR_INVALID_ARG;
    if (C->rows >= INT32_MAX - 16) return TSP_ERR_INDEX_OVERFLOW;
    if (C->row_ptr_type == TSP_I64) return compact_run<int64_t>(ctx, C, out, s, taken);
    if (C->row_ptr_type == TSP_I32) return compact_run<int32_t>(ctx, C, out, s, taken);
    return TSP_ERR_INVALID_ARG;
}

// ---- the same compaction without any allocation (tsp_compact_zeros_static) -----------------------
// The survivor counts per row and their sums per 16 rows, which compact_run takes from the handle's
// allocator, live in a file-scope device array instead.  Every device the library runs on holds its own
// copy of the array, at its own address, until the process ends; the address is looked up once per device
// (static_scratch_setup) and only that pointer is ever handed to kernels.
constexpr int64_t kStaticMaxRows = TSP_COMPACT_STATIC_MAX_ROWS;
constexpr size_t kStaticKeepBytes = ((size_t)(kStaticMaxRows + 1) * sizeof(int32_t) + 255) & ~size_t(255);
constexpr size_t kStaticGroupBytes = ((size_t)(kStaticMaxRows / T + 4) * sizeof(uint32_t) + 255) & ~size_t(255);
static __device__ __align__(256) unsigned char scratch[kStaticKeepBytes + kStaticGroupBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static unsigned char *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on every device seen so far

// Device address of the scratch array on the current device (looked up on the first call per device).
int static_scratch_setup(tsp_context *ctx, unsigned char **ptr) {
    int device = -1;
    TSP_HIP_CHECK(ctx, hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return TSP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        TSP_HIP_CHECK(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return hip_fail(ctx, hipErrorInvalidSymbol);
        g_scratch_ptr[device] = static_cast<unsigned char *>(p);
    }
    if (ptr) *ptr = g_scratch_ptr[device];
    return TSP_OK;
}

template <typename RP>
static int compact_run_static(tsp_context *ctx, const tsp_csr *C, tsp_csr *out, hipStream_t s) {
    const int64_t rows = C->rows;
    unsigned char *base = nullptr;
    int rc = static_scratch_setup(ctx, &base);
    if (rc) return rc;
    int32_t *keep = reinterpret_cast<int32_t *>(base);
    uint32_t *group_keep = reinterpret_cast<uint32_t *>(base + kStaticKeepBytes);
    int64_t *new_row_ptr = static_cast<int64_t *>(out->row_ptr);
    CompactArgs<RP> a{static_cast<const RP *>(C->row_ptr), C->col_idx, static_cast<const float *>(C->val), rows, C->nnz};
    const int64_t row_blocks = (rows * kCompactLanes + kCompactThreads - 1) / kCompactThreads;
    if (!ctx->scalars_clean) hipLaunchKernelGGL(k_compact_clear, dim3(1), dim3(64), 0, s, ctx->d_scalars);
    ctx->scalars_clean = false;
    // (nothing in the scratch array has to start at zero: the count kernel writes every word the prefix sum reads)
    hipLaunchKernelGGL(k_compact_count<RP>, dim3((unsigned)row_blocks), dim3(kCompactThreads), 0, s, a, keep, group_keep);
    if (!row_ptr_in_one_launch(ctx, keep, rows, group_keep, new_row_ptr, s)) return TSP_ERR_UNSUPPORTED;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(ctx, e);
    rc = wait_published_scalars(ctx, ctx->publish_tag, s);       // host synchronisation: the new nnz
    if (rc) return rc;
    if (ctx->h_scalars[S_INTERNAL]) return TSP_ERR_HIP;
    const int64_t nnz = ctx->h_scalars[S_C_NNZ];
    if (nnz > 0) {
        hipLaunchKernelGGL(k_compact_fill<RP>, dim3((unsigned)row_blocks), dim3(kCompactThreads), 0, s, a, new_row_ptr,
                           out->col_idx, static_cast<float *>(out->val));
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(ctx, e);
    }
    out->rows = C->rows;
    out->cols = C->cols;
    out->nnz = nnz;
    out->row_ptr_type = TSP_I64;
    out->val_type = TSP_F32;
    return TSP_OK;
}

}  // namespace tsp

using namespace tsp;

extern "C" int tsp_compact_zeros_static(tsp_handle ctx, const tsp_csr *C, tsp_csr *out, void *stream) {
    if (!ctx || !C || !out || C == out) return TSP_ERR_INVALID_ARG;
    if (C->rows < 0 || C->cols < 0 || C->nnz < 0 || !C->row_ptr || !out->row_ptr) return TSP_ERR_INVALID_ARG;
    if (C->val_type != TSP_F32) return TSP_ERR_INVALID_ARG;
    if (C->nnz > 0 && (!C->col_idx || !C->val || !out->col_idx || !out->val)) return TSP_ERR_INVALID_ARG;
    if (C->rows < 1 || C->rows > kStaticMaxRows) return TSP_ERR_UNSUPPORTED;      // the scratch array has a fixed size
    hipStream_t s = (hipStream_t)stream;
    if (C->row_ptr_type == TSP_I64) return compact_run_static<int64_t>(ctx, C, out, s);
    if (C->row_ptr_type == TSP_I32) return compact_run_static<int32_t>(ctx, C, out, s);
    return TSP_ERR_INVALID_ARG;
}

extern "C" int tsp_compact_zeros(tsp_handle ctx, const tsp_csr *C, tsp_csr *out, void *stream) {
    if (!ctx || !C || !out || C == out) return TSP_ERR_INVALID_ARG;
    return compact_zeros(ctx, C, out, (hipStream_t)stream, nullptr);
}
