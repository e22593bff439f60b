// CSR -> tile ("bitmap") format, paper Section 2.1.2 with 16x16 tiles: a tile occupancy scan
// (how many non-empty tiles each tile-row has), a prefix sum, and a packing pass that writes, per
// non-empty tile, its tile column, its bitmap (16 row masks) and its elements.
//
// Work decomposition: 16 lanes own one tile-row, one lane per CSR row.  Because the columns of a
// CSR row ascend, so do its tile columns, and the distinct tile columns of the tile-row come out
// of a 16-way merge: every step takes the smallest pending tile column over the 16 lanes; the
// lanes whose row has entries in that tile consume them.  The element storage is laid out for
// the matrix-core operand registers (see tsp_tiles_view in tsp.h): 16-byte groups of 8 fp16,
// row-wise groups for a left operand, column-wise groups for a right operand, empty groups
// skipped.  A tile-row can hold at most as many groups as it has stored entries, so group
// offsets start at row_ptr[16*I] and no second prefix sum is needed.
#include "common.hpp"

#include <hip/hip_fp16.h>

#include <climits>
#include <new>

namespace tsp {

constexpr int kConvThreads = 256;                 // 16 tile-rows per block
constexpr int kGroupsPerBlock = kConvThreads / 16;

__device__ __forceinline__ uint16_t to_half_bits(uint16_t v) { return v; }
__device__ __forceinline__ uint16_t to_half_bits(float v) { return __half_as_ushort(__float2half_rn(v)); }

template <typename RP>
__global__ __launch_bounds__(kConvThreads) void k_validate_csr(const RP *__restrict__ row_ptr,
                                                               const int32_t *__restrict__ col, int64_t rows,
                                                               int64_t cols, int64_t nnz,
                                                               int64_t *__restrict__ d_scalars) {
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const int64_t p = (int64_t)row_ptr[row], e = (int64_t)row_ptr[row + 1];
    bool bad = (row == 0 && p != 0) || (row == rows - 1 && e != nnz) || p < 0 || e > nnz || p > e;
    if (!bad) {
        int64_t prev = -1;
        for (int64_t q = p; q < e; ++q) {
            const int64_t c = col[q];
            bad |= (c <= prev) | (c >= cols);
            prev = c;
        }
    }
    if (bad) d_scalars[S_INVALID] = 1;
}

template <typename RP>
__device__ __forceinline__ void row_range(const RP *row_ptr, int64_t row, int64_t rows, int64_t nnz, bool in_grid,
                                          int64_t &p, int64_t &e) {
    p = e = 0;
    if (in_grid && row < rows) {
        p = (int64_t)row_ptr[row];
        e = (int64_t)row_ptr[row + 1];
        p = min(max(p, (int64_t)0), nnz);      // never read col[] outside the array, whatever row_ptr holds
        e = min(max(e, p), nnz);
    }
}

// Occupancy scan: number of non-empty tiles per tile-row.
template <typename RP>
__global__ __launch_bounds__(kConvThreads) void k_count_tiles(const RP *__restrict__ row_ptr,
                                                              const int32_t *__restrict__ col, int64_t rows,
                                                              int64_t nnz, int64_t tile_rows,
                                                              int32_t *__restrict__ tiles_per_row) {
    const int64_t I = (int64_t)blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 4);
    const int r = threadIdx.x & 15;
    int64_t p, e;
    row_range(row_ptr, I * T + r, rows, nnz, I < tile_rows, p, e);
    int cur = p < e ? (col[p] >> 4) : INT_MAX;
    int count = 0;
    for (;;) {
        const int m = group16_min(cur);
        if (__all(m == INT_MAX)) break;
        if (m != INT_MAX) {
            ++count;
            if (cur == m) {
                do { ++p; } while (p < e && (col[p] >> 4) == m);
                cur = p < e ? (col[p] >> 4) : INT_MAX;
            }
        }
    }
    if (r == 0 && I < tile_rows) tiles_per_row[I] = count;
}

// Packing pass.
template <typename RP, typename VT>
__global__ __launch_bounds__(kConvThreads) void k_fill_tiles(
    const RP *__restrict__ row_ptr, const int32_t *__restrict__ col, const VT *__restrict__ val, int64_t rows,
    int64_t nnz, int64_t tile_rows, const int32_t *__restrict__ tile_row_ptr, int64_t tile_capacity,
    int64_t group_capacity, int forms,
    int32_t *__restrict__ tile_col, uint16_t *__restrict__ row_mask, uint32_t *__restrict__ lmask,
    uint32_t *__restrict__ rmask, uint32_t *__restrict__ loff, uint32_t *__restrict__ roff,
    uint4 *__restrict__ ldata, uint4 *__restrict__ rdata) {
    __shared__ __align__(16) uint16_t dense_all[kGroupsPerBlock][T * T];
    const int g = threadIdx.x >> 4, r = threadIdx.x & 15;
    uint16_t *dense = dense_all[g];
    const int64_t I = (int64_t)blockIdx.x * kGroupsPerBlock + g;
    int64_t p, e;
    row_range(row_ptr, I * T + r, rows, nnz, I < tile_rows, p, e);
    int64_t t = 0;
    uint32_t lrun = 0, rrun = 0;
    if (I < tile_rows) {
        t = tile_row_ptr[I];
        int64_t b = (int64_t)row_ptr[min(I * T, rows)];
        lrun = rrun = (uint32_t)min(max(b, (int64_t)0), nnz);
    }
    int cur = p < e ? (col[p] >> 4) : INT_MAX;
    const uint32_t below_lo = (1u << r) - 1u, below_hi = (1u << (16 + r)) - 1u;
    for (;;) {
        const int m = group16_min(cur);
        if (__all(m == INT_MAX)) break;
        const bool active = m != INT_MAX;
        // dense image of the tile in LDS; every lane clears and fills its own row
        uint4 *myrow = reinterpret_cast<uint4 *>(dense + r * T);
        myrow[0] = make_uint4(0, 0, 0, 0);
        myrow[1] = make_uint4(0, 0, 0, 0);
        uint32_t mask = 0;
        if (active && cur == m) {
            do {
                const int c = col[p] & 15;
                mask |= 1u << c;
                dense[r * T + c] = to_half_bits(val[p]);
                ++p;
            } while (p < e && (col[p] >> 4) == m);
            cur = p < e ? (col[p] >> 4) : INT_MAX;
        }
        wave_sync();
        // group masks: left form g = h*16 + row, right form g = h*16 + column
        const uint32_t lm = group16_ballot((mask & 0xFFu) != 0) | (group16_ballot((mask >> 8) != 0) << 16);
        const uint32_t rm = group16_or(r < 8 ? mask : (mask << 16));
        if (active && t < tile_capacity) {
            if (forms & TSP_FORM_LEFT) {
                const int64_t g0 = (int64_t)lrun + __popc(lm & below_lo), g1 = (int64_t)lrun + __popc(lm & below_hi);
                if ((mask & 0xFFu) && g0 < group_capacity) ldata[g0] = myrow[0];
                if ((mask >> 8) && g1 < group_capacity) ldata[g1] = myrow[1];
            }
            if (forms & TSP_FORM_RIGHT) {
                // lane r gathers column r of the tile
                uint32_t w[8];
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    w[k] = (uint32_t)dense[(2 * k) * T + r] | ((uint32_t)dense[(2 * k + 1) * T + r] << 16);
                const int64_t g0 = (int64_t)rrun + __popc(rm & below_lo), g1 = (int64_t)rrun + __popc(rm & below_hi);
                // (the capacity tests can only fail for a non-canonical input)
                if (((rm >> r) & 1u) && g0 < group_capacity) rdata[g0] = make_uint4(w[0], w[1], w[2], w[3]);
                if (((rm >> (16 + r)) & 1u) && g1 < group_capacity) rdata[g1] = make_uint4(w[4], w[5], w[6], w[7]);
            }
            row_mask[t * T + r] = (uint16_t)mask;
            if (r == 0) {
                tile_col[t] = m;
                lmask[t] = lm;
                rmask[t] = rm;
                if (forms & TSP_FORM_LEFT) loff[t] = lrun;
                if (forms & TSP_FORM_RIGHT) roff[t] = rrun;
            }
            lrun += __popc(lm);
            rrun += __popc(rm);
            ++t;
        }
        wave_sync();   // column reads above finish before the rows are cleared again
    }
}

template <typename RP>
static int launch_convert_rp(tsp_context *ctx, const tsp_csr *A, tsp_tiles_s *t, int32_t *counts, int64_t *tmp,
                             hipStream_t s) {
    const RP *rp = static_cast<const RP *>(A->row_ptr);
    const unsigned grid = (unsigned)((t->tile_rows + kGroupsPerBlock - 1) / kGroupsPerBlock);
    if (ctx->validate && A->rows > 0) {
        KernelTimer kt(ctx, TSP_KERNEL_VALIDATE, s);
        hipLaunchKernelGGL(k_validate_csr<RP>, dim3((unsigned)((A->rows + kConvThreads - 1) / kConvThreads)),
                           dim3(kConvThreads), 0, s, rp, A->col_idx, A->rows, A->cols, A->nnz, ctx->d_scalars);
    }
    if (grid) {
        KernelTimer kt(ctx, TSP_KERNEL_COUNT_TILES, s);
        hipLaunchKernelGGL(k_count_tiles<RP>, dim3(grid), dim3(kConvThreads), 0, s, rp, A->col_idx, A->rows, A->nnz,
                           t->tile_rows, counts);
    }
    int rc;
    {
        KernelTimer kt(ctx, TSP_KERNEL_SCAN_TILES, s);
        rc = scan_exclusive_i32_to_i32(ctx, counts, t->tile_row_ptr, t->tile_rows, ctx->d_scalars + t->scalar_slot,
                                       nullptr, tmp, s);
    }
    if (rc) return rc;
    if (grid) {
        KernelTimer kt(ctx, TSP_KERNEL_FILL_TILES, s);
        if (A->val_type == TSP_F16)
            hipLaunchKernelGGL((k_fill_tiles<RP, uint16_t>), dim3(grid), dim3(kConvThreads), 0, s, rp, A->col_idx,
                               static_cast<const uint16_t *>(A->val), A->rows, A->nnz, t->tile_rows, t->tile_row_ptr,
                               t->tile_capacity, t->group_capacity, t->forms, t->tile_col, t->row_mask, t->lmask, t->rmask, t->loff,
                               t->roff, t->ldata, t->rdata);
        else
            hipLaunchKernelGGL((k_fill_tiles<RP, float>), dim3(grid), dim3(kConvThreads), 0, s, rp, A->col_idx,
                               static_cast<const float *>(A->val), A->rows, A->nnz, t->tile_rows, t->tile_row_ptr,
                               t->tile_capacity, t->group_capacity, t->forms, t->tile_col, t->row_mask, t->lmask, t->rmask, t->loff,
                               t->roff, t->ldata, t->rdata);
    }
    TSP_HIP_CHECK(ctx, hipGetLastError());
    return TSP_OK;
}

static int check_csr_host(const tsp_csr *A) {
    if (!A) return TSP_ERR_INVALID_ARG;
    if (A->rows < 0 || A->cols < 0 || A->nnz < 0) return TSP_ERR_INVALID_ARG;
    if (A->row_ptr_type != TSP_I32 && A->row_ptr_type != TSP_I64) return TSP_ERR_INVALID_ARG;
    if (A->val_type != TSP_F16 && A->val_type != TSP_F32) return TSP_ERR_INVALID_ARG;
    if (!A->row_ptr) return TSP_ERR_INVALID_ARG;
    if (A->nnz > 0 && (!A->col_idx || !A->val)) return TSP_ERR_INVALID_ARG;
    if (A->rows >= INT32_MAX - 16 || A->cols >= INT32_MAX - 16 || A->nnz >= INT32_MAX) return TSP_ERR_INDEX_OVERFLOW;
    if ((A->rows == 0 || A->cols == 0) && A->nnz != 0) return TSP_ERR_NOT_CANONICAL;
    return TSP_OK;
}

void tiles_release(tsp_context *ctx, tsp_tiles_s *t, hipStream_t s) {
    if (!t) return;
    ctx_free(ctx, t->tile_row_ptr, s);
    ctx_free(ctx, t->tile_col, s);
    ctx_free(ctx, t->row_mask, s);
    ctx_free(ctx, t->lmask, s);
    ctx_free(ctx, t->rmask, s);
    ctx_free(ctx, t->loff, s);
    ctx_free(ctx, t->roff, s);
    ctx_free(ctx, t->ldata, s);
    ctx_free(ctx, t->rdata, s);
    delete t;
}

// Enqueues the whole conversion without synchronising: the tile arrays are sized by the bound
// ntiles <= min(nnz, tile_rows*tile_cols); the exact count is left in d_scalars[scalar_slot].
int convert_enqueue(tsp_context *ctx, const tsp_csr *A, int forms, int scalar_slot, tsp_tiles_s **out,
                    hipStream_t s) {
    *out = nullptr;
    int rc = check_csr_host(A);
    if (rc) return rc;
    if (!(forms & (TSP_FORM_LEFT | TSP_FORM_RIGHT)) || (forms & ~(TSP_FORM_LEFT | TSP_FORM_RIGHT)))
        return TSP_ERR_INVALID_ARG;
    tsp_tiles_s *t = new (std::nothrow) tsp_tiles_s();
    if (!t) return TSP_ERR_ALLOC_FAILED;
    t->rows = A->rows;
    t->cols = A->cols;
    t->nnz = A->nnz;
    t->tile_rows = (A->rows + T - 1) / T;
    t->tile_cols = (A->cols + T - 1) / T;
    t->forms = forms;
    t->scalar_slot = scalar_slot;
    const double grid_tiles = (double)t->tile_rows * (double)t->tile_cols;
    t->tile_capacity = grid_tiles < (double)A->nnz ? (int64_t)grid_tiles : A->nnz;
    t->group_capacity = A->nnz;
    const size_t cap = (size_t)t->tile_capacity;
    t->tile_row_ptr = ctx_alloc_n<int32_t>(ctx, (size_t)t->tile_rows + 1, s);
    t->tile_col = ctx_alloc_n<int32_t>(ctx, cap, s);
    t->row_mask = ctx_alloc_n<uint16_t>(ctx, cap * T, s);
    t->lmask = ctx_alloc_n<uint32_t>(ctx, cap, s);
    t->rmask = ctx_alloc_n<uint32_t>(ctx, cap, s);
    bool ok = t->tile_row_ptr && t->tile_col && t->row_mask && t->lmask && t->rmask;
    if (forms & TSP_FORM_LEFT) {
        t->loff = ctx_alloc_n<uint32_t>(ctx, cap, s);
        t->ldata = ctx_alloc_n<uint4>(ctx, (size_t)t->group_capacity, s);
        ok = ok && t->loff && t->ldata;
    }
    if (forms & TSP_FORM_RIGHT) {
        t->roff = ctx_alloc_n<uint32_t>(ctx, cap, s);
        t->rdata = ctx_alloc_n<uint4>(ctx, (size_t)t->group_capacity, s);
        ok = ok && t->roff && t->rdata;
    }
    int32_t *counts = ctx_alloc_n<int32_t>(ctx, (size_t)t->tile_rows + 1, s);
    int64_t *tmp = ctx_alloc_n<int64_t>(ctx, scan_tmp_entries(t->tile_rows), s);
    ok = ok && counts && tmp;
    rc = ok ? TSP_OK : TSP_ERR_ALLOC_FAILED;
    if (!rc)
        rc = A->row_ptr_type == TSP_I32 ? launch_convert_rp<int32_t>(ctx, A, t, counts, tmp, s)
                                        : launch_convert_rp<int64_t>(ctx, A, t, counts, tmp, s);
    ctx_free(ctx, counts, s);
    ctx_free(ctx, tmp, s);
    if (rc) {
        tiles_release(ctx, t, s);
        return rc;
    }
    *out = t;
    return TSP_OK;
}

__global__ void k_clear_scalars(int64_t *d_scalars) {
    if (threadIdx.x < kScalars) d_scalars[threadIdx.x] = 0;
}

}  // namespace tsp

using namespace tsp;

extern "C" int tsp_convert(tsp_handle ctx, const tsp_csr *A, int forms, tsp_tiles *out, void *stream) {
    if (!ctx || !out) return TSP_ERR_INVALID_ARG;
    *out = nullptr;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_clear_scalars, dim3(1), dim3(64), 0, s, ctx->d_scalars);
    phase_begin(ctx, TSP_PHASE_CONVERT, s);
    tsp_tiles_s *t = nullptr;
    int rc = convert_enqueue(ctx, A, forms, S_TILES_A, &t, s);
    phase_end(ctx, TSP_PHASE_CONVERT, s);
    if (rc) return rc;
    rc = read_scalars(ctx, s);
    if (!rc && ctx->h_scalars[S_INVALID]) rc = TSP_ERR_NOT_CANONICAL;
    if (rc) {
        tiles_release(ctx, t, s);
        return rc;
    }
    t->ntiles = ctx->h_scalars[S_TILES_A];
    ctx->stats.a_tiles = t->ntiles;
    *out = t;
    return TSP_OK;
}

extern "C" int tsp_tiles_free(tsp_handle ctx, tsp_tiles tiles, void *stream) {
    if (!ctx) return TSP_ERR_INVALID_ARG;
    tiles_release(ctx, tiles, (hipStream_t)stream);
    return TSP_OK;
}

extern "C" int tsp_tiles_get_view(tsp_tiles t, tsp_tiles_view *v) {
    if (!t || !v) return TSP_ERR_INVALID_ARG;
    v->rows = t->rows;
    v->cols = t->cols;
    v->tile_rows = t->tile_rows;
    v->tile_cols = t->tile_cols;
    v->ntiles = t->ntiles;
    v->forms = t->forms;
    v->tile_row_ptr = t->tile_row_ptr;
    v->tile_col = t->tile_col;
    v->row_mask = t->row_mask;
    v->left_group_mask = t->lmask;
    v->right_group_mask = t->rmask;
    v->left_group_off = t->loff;
    v->right_group_off = t->roff;
    v->left_elements = reinterpret_cast<const uint16_t *>(t->ldata);
    v->right_elements = reinterpret_cast<const uint16_t *>(t->rdata);
    v->left_groups_capacity = t->ldata ? t->group_capacity : 0;
    v->right_groups_capacity = t->rdata ? t->group_capacity : 0;
    return TSP_OK;
}
