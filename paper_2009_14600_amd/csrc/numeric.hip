// Multiplication pass and CSR emission (paper Sections 4.3 and 4.4, Algorithm 1 line 18).
//
// One wave owns one output tile and walks the tile's task-list segment, two pairs per step: the
// pairs of a C tile form one 16 x 16p by 16p x 16 product, so the inner (K) dimension of
// v_mfma_f32_16x16x32_f16 is filled with the inner indices of two consecutive pairs
// (lanes 0-31 feed pair p, lanes 32-63 feed pair p+1) and the four fp32 accumulator registers
// of a lane carry the tile through the whole segment: the segmented reduction happens in
// registers, in task-list order, with no atomics (the paper pairs two 8x8 output tiles on the
// diagonal of one 16x16 tensor-core fragment instead, Section 4.4).
//
// Operand registers of the instruction: lane l holds, for the left matrix, row l%16 and inner
// indices 8*(l/16)..+7; for the right matrix, column l%16 and the same inner indices.  The tile
// format stores exactly those 8-value groups (see tsp.h), so an operand is one 16-byte load, or
// zero when the group mask says the group is empty: nothing is "placed by bitmap" at run time.
// The accumulator of lane l holds column l%16, rows 4*(l/16)..+3 of the output tile.
//
// Emission: the counting pass left, per C tile, the 16 row masks of its structural pattern and
// the number of entries each CSR row has to the left of the tile; the lane that holds element
// (i,j) writes column 16J+j and the value at row_ptr[16I+i] + left(i) + popcount(mask_i below j).
#include "common.hpp"

#include <new>

namespace tsp {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

union Group {
    uint4 u;
    half8 h;
};

constexpr int kNumThreads = 256;   // 4 waves = 4 output tiles per block

__global__ __launch_bounds__(kNumThreads) void k_numeric(
    int64_t c_tiles, const int64_t *__restrict__ pair_off, const int32_t *__restrict__ pair_a,
    const int32_t *__restrict__ pair_b, const uint32_t *__restrict__ a_lmask, const uint32_t *__restrict__ a_loff,
    const uint4 *__restrict__ a_ldata, const uint32_t *__restrict__ b_rmask, const uint32_t *__restrict__ b_roff,
    const uint4 *__restrict__ b_rdata, const int32_t *__restrict__ c_tile_row, const int32_t *__restrict__ c_tile_col,
    const uint16_t *__restrict__ c_row_mask, const uint32_t *__restrict__ c_row_off,
    const int64_t *__restrict__ c_row_ptr, int32_t *__restrict__ c_col, float *__restrict__ c_val) {
    const int64_t c = (int64_t)blockIdx.x * (kNumThreads / 64) + (threadIdx.x >> 6);
    if (c >= c_tiles) return;                       // uniform per wave
    const int lane = threadIdx.x & 63;
    const int hl = lane & 31, upper = lane >> 5;
    const uint32_t bit = 1u << hl, below = bit - 1u;
    const int64_t s0 = pair_off[c], s1 = pair_off[c + 1];
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t p = s0; p < s1; p += 2) {
        const int64_t q = p + upper;
        Group av, bv;
        av.u = make_uint4(0, 0, 0, 0);
        bv.u = make_uint4(0, 0, 0, 0);
        if (q < s1) {
            const int64_t a = pair_a[q], b = pair_b[q];
            const uint32_t lm = a_lmask[a], rm = b_rmask[b];
            if (lm & bit) av.u = a_ldata[(int64_t)a_loff[a] + __popc(lm & below)];
            if (rm & bit) bv.u = b_rdata[(int64_t)b_roff[b] + __popc(rm & below)];
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av.h, bv.h, acc, 0, 0, 0);
    }
    const int64_t I = c_tile_row[c], J = c_tile_col[c];
    const int j = lane & 15, ig = lane >> 4;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int i = 4 * ig + v;
        const uint32_t cm = c_row_mask[c * T + i];
        if ((cm >> j) & 1u) {
            const int64_t pos = c_row_ptr[I * T + i] + (int64_t)c_row_off[c * T + i] + __popc(cm & ((1u << j) - 1u));
            c_col[pos] = (int32_t)(J * T + j);
            c_val[pos] = acc[v];
        }
    }
}

int numeric_enqueue(tsp_context *ctx, tsp_tiles_s *A, tsp_tiles_s *B, tsp_plan_s *P, tsp_csr *C, hipStream_t s) {
    std::memset(C, 0, sizeof(*C));
    if (!(A->forms & TSP_FORM_LEFT) || !(B->forms & TSP_FORM_RIGHT)) return TSP_ERR_INVALID_ARG;
    if (A->cols != B->rows || P->c_rows != A->rows || P->c_cols != B->cols) return TSP_ERR_SHAPE_MISMATCH;
    int64_t *row_ptr = ctx_alloc_n<int64_t>(ctx, (size_t)P->c_rows + 1, s);
    int32_t *col = ctx_alloc_n<int32_t>(ctx, (size_t)P->c_nnz, s);
    float *val = ctx_alloc_n<float>(ctx, (size_t)P->c_nnz, s);
    if (!row_ptr || !col || !val) {
        ctx_free(ctx, row_ptr, s);
        ctx_free(ctx, col, s);
        ctx_free(ctx, val, s);
        return TSP_ERR_ALLOC_FAILED;
    }
    phase_begin(ctx, TSP_PHASE_NUMERIC, s);
    hipError_t e = hipMemcpyAsync(row_ptr, P->c_row_ptr, sizeof(int64_t) * (size_t)(P->c_rows + 1),
                                  hipMemcpyDeviceToDevice, s);
    if (e == hipSuccess && P->c_tiles > 0) {
        KernelTimer kt(ctx, TSP_KERNEL_NUMERIC, s);
        const unsigned grid = (unsigned)((P->c_tiles + kNumThreads / 64 - 1) / (kNumThreads / 64));
        hipLaunchKernelGGL(k_numeric, dim3(grid), dim3(kNumThreads), 0, s, P->c_tiles, P->pair_off, P->pair_a,
                           P->pair_b, A->lmask, A->loff, A->ldata, B->rmask, B->roff, B->rdata, P->c_tile_row,
                           P->c_tile_col, P->c_row_mask, P->c_row_off, P->c_row_ptr, col, val);
        e = hipGetLastError();
    }
    phase_end(ctx, TSP_PHASE_NUMERIC, s);
    if (e != hipSuccess) {
        ctx_free(ctx, row_ptr, s);
        ctx_free(ctx, col, s);
        ctx_free(ctx, val, s);
        return hip_fail(ctx, e);
    }
    C->rows = P->c_rows;
    C->cols = P->c_cols;
    C->nnz = P->c_nnz;
    C->row_ptr = row_ptr;
    C->col_idx = col;
    C->val = val;
    C->row_ptr_type = TSP_I64;
    C->val_type = TSP_F32;
    return TSP_OK;
}

}  // namespace tsp

using namespace tsp;

extern "C" int tsp_numeric(tsp_handle ctx, tsp_tiles A, tsp_tiles B, tsp_plan plan, tsp_csr *C, void *stream) {
    if (!ctx || !A || !B || !plan || !C) return TSP_ERR_INVALID_ARG;
    return numeric_enqueue(ctx, A, B, plan, C, (hipStream_t)stream);
}
