// Device-wide exclusive prefix sums (the "prefix sum" of Section 4.1 / Algorithm 1, the counts-to-offsets steps
// that turns per-tile-row and per-row counts into offsets and total sizes).
#include "common.hpp"

namespace tsp {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanBlock = kScanThreads * kScanItems;   // elements per block

size_t scan_tmp_entries(int64_t n) { return (size_t)(2 * ((n + kScanBlock - 1) / kScanBlock) + 2); }

// Inclusive scan of one value per thread across the block; returns the inclusive prefix and the
// block total through `total`.
__device__ __forceinline__ int64_t block_inclusive_scan(int64_t v, int64_t *total, int64_t *lds /*[5]*/) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int64_t u = __shfl_up(v, o, 64);
        if (lane >= o) v += u;
    }
    __syncthreads();                 // lds may still be read from a previous call
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    int64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        int64_t x = lds[w];
        if (w < wave) before += x;
        all += x;
    }
    *total = all;
    return v + before;
}

__device__ __forceinline__ int64_t block_max(int64_t v, int64_t *lds /*[4]*/) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = max(v, (int64_t)__shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int64_t m = lds[0];
#pragma unroll
    for (int w = 1; w < kScanThreads / 64; ++w) m = max(m, lds[w]);
    return m;
}

// Pass 1: per-block sum, and the largest sum of an aligned group of 16 inputs.
__global__ __launch_bounds__(kScanThreads) void k_scan_reduce(const int32_t *__restrict__ in, int64_t n,
                                                              int64_t *__restrict__ sums,
                                                              int64_t *__restrict__ maxs) {
    __shared__ int64_t lds[8];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    static_assert(kScanItems == 8, "two neighbouring threads hold an aligned group of 16 inputs");
    int64_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < n) s += in[base + i];
    int64_t total;
    block_inclusive_scan(s, &total, lds);
    int64_t m = s + (int64_t)__shfl_xor(s, 1, 64);     // inputs 16k..16k+15
    m = block_max(m, lds);
    if (threadIdx.x == 0) {
        sums[blockIdx.x] = total;
        maxs[blockIdx.x] = m;
    }
}

// Pass 2 (one block): exclusive scan of the block sums in place; grand total and maximum.
__global__ __launch_bounds__(kScanThreads) void k_scan_sums(int64_t *__restrict__ sums,
                                                            const int64_t *__restrict__ maxs, int64_t nblocks,
                                                            int64_t *__restrict__ d_total,
                                                            int64_t *__restrict__ d_max) {
    __shared__ int64_t lds[8];
    int64_t carry = 0, mx = 0;
    for (int64_t base = 0; base < nblocks; base += kScanThreads) {
        int64_t i = base + threadIdx.x;
        int64_t v = i < nblocks ? sums[i] : 0;
        if (i < nblocks) mx = max(mx, maxs[i]);
        int64_t total;
        int64_t inc = block_inclusive_scan(v, &total, lds);
        if (i < nblocks) sums[i] = carry + inc - v;
        carry += total;
    }
    mx = block_max(mx, lds);
    if (threadIdx.x == 0) {
        sums[nblocks] = carry;
        if (d_total) *d_total = carry;
        if (d_max) *d_max = mx;
    }
}

// Pass 3: scan each block again, offset by the scanned block sums; the last block writes out[n].
template <typename TOut>
__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const int32_t *__restrict__ in, TOut *__restrict__ out,
                                                             int64_t n, const int64_t *__restrict__ sums) {
    __shared__ int64_t lds[8];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    int64_t x[kScanItems];
    int64_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        x[i] = base + i < n ? (int64_t)in[base + i] : 0;
        s += x[i];
    }
    int64_t total;
    int64_t run = sums[blockIdx.x] + block_inclusive_scan(s, &total, lds) - s;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < n) out[base + i] = (TOut)run;
        run += x[i];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) out[n] = (TOut)sums[gridDim.x];
}

template <typename TOut>
__global__ void k_scan_empty(TOut *out, int64_t *d_total, int64_t *d_max) {
    out[0] = 0;
    if (d_total) *d_total = 0;
    if (d_max) *d_max = 0;
}

template <typename TOut>
static int scan_impl(tsp_context *ctx, const int32_t *in, TOut *out, int64_t n, int64_t *d_total,
                     int64_t *d_max, int64_t *tmp, hipStream_t s) {
    if (n <= 0) {
        hipLaunchKernelGGL(k_scan_empty<TOut>, dim3(1), dim3(1), 0, s, out, d_total, d_max);
        TSP_HIP_CHECK(ctx, hipGetLastError());
        return TSP_OK;
    }
    const int64_t nblocks = (n + kScanBlock - 1) / kScanBlock;
    int64_t *sums = tmp, *maxs = tmp + nblocks + 1;
    hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s, in, n, sums, maxs);
    hipLaunchKernelGGL(k_scan_sums, dim3(1), dim3(kScanThreads), 0, s, sums, maxs, nblocks, d_total, d_max);
    hipLaunchKernelGGL(k_scan_apply<TOut>, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s, in, out, n, sums);
    TSP_HIP_CHECK(ctx, hipGetLastError());
    return TSP_OK;
}

int scan_exclusive_i32_to_i32(tsp_context *ctx, const int32_t *in, int32_t *out, int64_t n, int64_t *d_total,
                              int64_t *d_max, int64_t *tmp, hipStream_t s) {
    return scan_impl<int32_t>(ctx, in, out, n, d_total, d_max, tmp, s);
}
int scan_exclusive_i32_to_i64(tsp_context *ctx, const int32_t *in, int64_t *out, int64_t n, int64_t *d_total,
                              int64_t *d_max, int64_t *tmp, hipStream_t s) {
    return scan_impl<int64_t>(ctx, in, out, n, d_total, d_max, tmp, s);
}

}  // namespace tsp
