// Order of work for the kernels that walk the task list (counting pass, multiplication pass; paper
// Sections 4.2 and 4.3) on products whose tile-rows of C are long.
//
// The task list is sorted by output tile, row-major (Section 4.1), and a tile C[I,J] reads the tiles
// B[K,J] of all inner indices K of its tile-row.  Walked row-major, every tile-row of C streams the
// tile-rows of B it meets from memory again: on a power-law graph that is hundreds of gigabytes for a B
// of a few hundred megabytes.  The paper names exactly this as the limit of its multiplication kernel
// (Section 6.2: the task-list entries point to scattered tiles).  Here the output tiles are handed out
// in vertical strips instead: a strip is a range of tile columns chosen so that the tiles of B inside it
// (about kStripTiles of them) stay in the L2 cache of one XCD while all tile-rows of C pass through the
// strip.  Nothing about the task list or the result changes, only which workgroup takes which tiles:
// a descriptor per workgroup {first output tile, number of tiles (at most 16, all of one tile-row and
// one strip)}, in strip-major order.
#include "common.hpp"

#include <algorithm>
#include <new>

namespace tsp {

constexpr int kStripBinsLog2 = 13;              // histogram of B's tile columns: at most 8192 bins (64 KB of LDS)
constexpr int kStripBlockTiles = 16;            // output tiles per workgroup of the kernels that use the order
constexpr int64_t kStripTiles = 32768;          // tiles of B per strip: about 1.3 MB of headers and operand groups
constexpr int kStripMax = 1024;                 // most strips

// Tiles of B per bin of tile columns (bin = tile column >> shift).  A wave per tile-row.
__global__ __launch_bounds__(256) void k_strip_hist(int64_t tile_rows, const int32_t *__restrict__ trp,
                                                    const int32_t *__restrict__ tend,
                                                    const int32_t *__restrict__ tcol, int shift, int bins,
                                                    uint32_t *__restrict__ hist) {
    const int64_t K = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (K >= tile_rows) return;
    const int lane = threadIdx.x & 63;
    for (int t = trp[K] + lane; t < tend[K]; t += 64) {
        const uint32_t bin = (uint32_t)tcol[t] >> shift;
        if (bin < (uint32_t)bins) atomicAdd(&hist[bin], 1u);
    }
}

// Strip boundaries (in tile columns) from the histogram: strip k ends where the running number of tiles
// passes k+1 parts of the total.  One block.  bound[0..strips]: bound[0] = 0, bound[strips] = past the
// last tile column; a strip may be empty (a single bin heavier than a part).
__global__ __launch_bounds__(1024) void k_strip_bounds(const uint32_t *__restrict__ hist, int bins, int shift,
                                                       int strips, int32_t *__restrict__ bound) {
    __shared__ uint32_t s_wave[16];
    __shared__ uint32_t s_carry;
    extern __shared__ uint32_t s_prefix[];       // inclusive prefix per bin (B has fewer than 2^31 tiles)
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < bins; base += 1024) {
        const int i = base + threadIdx.x;
        const uint32_t x = i < bins ? hist[i] : 0;
        const uint32_t inc = wave_inclusive_scan(x);
        if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = inc;
        __syncthreads();
        uint32_t before = s_carry;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) before += s_wave[w];
        if (i < bins) s_prefix[i] = before + inc;
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = before + inc;
        __syncthreads();
    }
    const uint64_t total = s_carry;
    for (int k = threadIdx.x; k <= strips; k += 1024) {
        int b;
        if (k == 0) {
            b = 0;
        } else if (k == strips) {
            b = bins;
        } else {
            // first bin whose inclusive prefix reaches k parts of the total: the strip ends after it
            const uint64_t want = (total * (uint64_t)k + strips - 1) / strips;
            int lo = 0, hi = bins;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (s_prefix[mid] < want) lo = mid + 1; else hi = mid;
            }
            b = min(lo + 1, bins);
        }
        bound[k] = k == strips ? INT32_MAX : (int32_t)((int64_t)b << shift);
    }
}

// Per (strip w, tile-row I), index w*ntr + I: the stretch of the tile-row's output tiles whose tile column
// lies in the strip (the tiles of a tile-row ascend by column), and the workgroups it takes.
__global__ __launch_bounds__(256) void k_strip_count(int64_t ntr, int strips, const int32_t *__restrict__ bound,
                                                     const int32_t *__restrict__ c_tile_row_ptr,
                                                     const int32_t *__restrict__ c_tile_col,
                                                     int32_t *__restrict__ first, int32_t *__restrict__ count,
                                                     int32_t *__restrict__ blocks) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= ntr * strips) return;
    const int w = (int)(p / ntr);
    const int64_t I = p % ntr;
    const int c0 = c_tile_row_ptr[I], c1 = c_tile_row_ptr[I + 1];
    auto lower = [&](int32_t col) {              // first tile of the tile-row at or past tile column `col`
        int lo = c0, hi = c1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (c_tile_col[mid] < col) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    const int b0 = bound[w], b1 = bound[w + 1];
    const int lo = b0 <= 0 ? c0 : lower(b0), hi = b1 == INT32_MAX ? c1 : lower(b1);
    const int n = max(hi - lo, 0);
    first[p] = lo;
    count[p] = n;
    blocks[p] = (n + kStripBlockTiles - 1) / kStripBlockTiles;
}

// One descriptor per workgroup, at the places the prefix sum of `blocks` assigns; descriptors past the
// total keep a count of zero (the array is cleared before).
__global__ __launch_bounds__(256) void k_strip_desc(int64_t n, const int32_t *__restrict__ first,
                                                    const int32_t *__restrict__ count,
                                                    const int32_t *__restrict__ block_ptr, int2 *__restrict__ desc,
                                                    int64_t capacity) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n) return;
    const int lo = first[p], tiles = count[p];
    int64_t at = block_ptr[p];
    for (int k = 0; k < tiles; k += kStripBlockTiles, ++at)
        if (at < capacity) desc[at] = make_int2(lo + k, min(kStripBlockTiles, tiles - k));
}

// Builds the strip order of a plan (see the top of the file).
int strips_build(tsp_context *ctx, tsp_plan_s *P, const tsp_tiles_s *B, hipStream_t s) {
    const int64_t ntr = P->c_tile_rows;
    if (ntr <= 0 || P->c_tiles <= 0 || B->ntiles <= 0) return TSP_OK;
    int shift = 0;
    while (((B->tile_cols + ((int64_t)1 << shift) - 1) >> shift) > ((int64_t)1 << kStripBinsLog2)) ++shift;
    const int bins = (int)((B->tile_cols + ((int64_t)1 << shift) - 1) >> shift);
    const int64_t per_strip = ctx->strip_order >= 16 ? ctx->strip_order : kStripTiles;
    const int strips = (int)std::min<int64_t>(kStripMax, std::max<int64_t>(1, (B->ntiles + per_strip - 1) / per_strip));
    const int64_t n = ntr * strips;
    if (n >= INT32_MAX) return TSP_OK;                       // (no strip order: the kernels fall back to row-major)
    const int64_t capacity = (P->c_tiles + kStripBlockTiles - 1) / kStripBlockTiles + n;
    uint32_t *hist = ctx_alloc_n<uint32_t>(ctx, (size_t)bins, s);
    int32_t *bound = ctx_alloc_n<int32_t>(ctx, (size_t)strips + 1, s);
    int32_t *first = ctx_alloc_n<int32_t>(ctx, (size_t)n, s), *count = ctx_alloc_n<int32_t>(ctx, (size_t)n, s);
    int32_t *blocks = ctx_alloc_n<int32_t>(ctx, (size_t)n, s);
    int32_t *block_ptr = ctx_alloc_n<int32_t>(ctx, (size_t)n + 1, s);
    int64_t *tmp = ctx_alloc_n<int64_t>(ctx, scan_tmp_entries(n), s);
    int2 *desc = ctx_alloc_n<int2>(ctx, (size_t)capacity, s);
    auto done = [&](int code) {
        ctx_free(ctx, hist, s);
        ctx_free(ctx, bound, s);
        ctx_free(ctx, first, s);
        ctx_free(ctx, count, s);
        ctx_free(ctx, blocks, s);
        ctx_free(ctx, tmp, s);
        if (code) {
            ctx_free(ctx, block_ptr, s);
            ctx_free(ctx, desc, s);
        }
        return code;
    };
    if (!hist || !bound || !first || !count || !blocks || !block_ptr || !tmp || !desc) return done(TSP_ERR_ALLOC_FAILED);
    hipError_t e = hipMemsetAsync(hist, 0, (size_t)bins * sizeof(uint32_t), s);
    if (e == hipSuccess) e = hipMemsetAsync(desc, 0, (size_t)capacity * sizeof(int2), s);
    if (e != hipSuccess) return done(hip_fail(ctx, e));
    hipLaunchKernelGGL(k_strip_hist, dim3((unsigned)((B->tile_rows + 3) / 4)), dim3(256), 0, s, B->tile_rows,
                       B->tile_row_ptr, B->tile_row_end, B->tile_col, shift, bins, hist);
    hipLaunchKernelGGL(k_strip_bounds, dim3(1), dim3(1024), (size_t)bins * sizeof(uint32_t), s, hist, bins, shift, strips,
                       bound);
    hipLaunchKernelGGL(k_strip_count, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, ntr, strips, bound,
                       P->c_tile_row_ptr, P->c_tile_col, first, count, blocks);
    int rc = scan_exclusive_i32_to_i32(ctx, blocks, block_ptr, n, nullptr, nullptr, tmp, s);
    if (rc) return done(rc);
    hipLaunchKernelGGL(k_strip_desc, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n, first, count, block_ptr, desc,
                       capacity);
    e = hipGetLastError();
    if (e != hipSuccess) return done(hip_fail(ctx, e));
    P->strip_desc = desc;
    P->strip_capacity = capacity;
    P->strip_block_ptr = block_ptr;              // its last entry is the number of workgroups
    P->strip_entries = n;
    return done(TSP_OK);
}

}  // namespace tsp
