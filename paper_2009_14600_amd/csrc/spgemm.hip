// tsp_spgemm: the whole pipeline of Algorithm 1, CSR in, CSR out.
#include "common.hpp"

#include <algorithm>

namespace tsp {
__global__ void k_clear_scalars_all(int64_t *d_scalars) {
    if (threadIdx.x < kScalars) d_scalars[threadIdx.x] = 0;
}
// Intermediate products of A*B: for every stored a_ik the number of stored entries of row k of B (the
// paper's NNZ of C-bar, Table 1).  Indices outside B are skipped (a non-canonical input is reported elsewhere).
template <typename RA, typename RB>
__global__ __launch_bounds__(256) void k_products(const int32_t *__restrict__ a_col, int64_t a_nnz,
                                                  const RB *__restrict__ b_row_ptr, int64_t b_rows, int64_t *d_scalars) {
    __shared__ unsigned long long part[4];
    unsigned long long n = 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < a_nnz; e += (int64_t)gridDim.x * 256) {
        const uint32_t k = (uint32_t)a_col[e];
        if (k < (uint64_t)b_rows) {
            const int64_t len = (int64_t)b_row_ptr[k + 1] - (int64_t)b_row_ptr[k];
            if (len > 0) n += (unsigned long long)len;
        }
    }
    for (int d = 32; d >= 1; d >>= 1) n += __shfl_xor(n, d, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long all = part[0] + part[1] + part[2] + part[3];
        if (all) atomicAdd(reinterpret_cast<unsigned long long *>(d_scalars + S_PRODUCTS), all);
    }
}
}  // namespace tsp

using namespace tsp;

static void count_products(tsp_context *ctx, const tsp_csr *A, const tsp_csr *B, hipStream_t s) {
    if (A->nnz <= 0 || B->rows <= 0) return;
    const unsigned blocks = (unsigned)std::min<int64_t>(2048, (A->nnz + 255) / 256);
    if (B->row_ptr_type == TSP_I32)
        hipLaunchKernelGGL((k_products<int32_t, int32_t>), dim3(blocks), dim3(256), 0, s, A->col_idx, A->nnz,
                           static_cast<const int32_t *>(B->row_ptr), B->rows, ctx->d_scalars);
    else
        hipLaunchKernelGGL((k_products<int32_t, int64_t>), dim3(blocks), dim3(256), 0, s, A->col_idx, A->nnz,
                           static_cast<const int64_t *>(B->row_ptr), B->rows, ctx->d_scalars);
}

static bool same_matrix(const tsp_csr *A, const tsp_csr *B) {
    return A == B || (A->rows == B->rows && A->cols == B->cols && A->nnz == B->nnz && A->row_ptr == B->row_ptr &&
                      A->col_idx == B->col_idx && A->val == B->val && A->row_ptr_type == B->row_ptr_type &&
                      A->val_type == B->val_type);
}

extern "C" int tsp_spgemm(tsp_handle ctx, const tsp_csr *A, const tsp_csr *B, tsp_csr *C, void *stream) {
    if (!ctx || !A || !B || !C) return TSP_ERR_INVALID_ARG;
    std::memset(C, 0, sizeof(*C));
    if (A->cols != B->rows) return TSP_ERR_SHAPE_MISMATCH;
    hipStream_t s = (hipStream_t)stream;
    const bool alias = same_matrix(A, B);
    tsp_tiles_s *ta = nullptr, *tb = nullptr;
    tsp_plan_s *plan = nullptr;

    total_begin(ctx, s);
    // (the multiplication kernel of the previous call has usually left the scalar block zeroed)
    if (!ctx->scalars_clean) hipLaunchKernelGGL(k_clear_scalars_all, dim3(1), dim3(64), 0, s, ctx->d_scalars);
    ctx->scalars_clean = false;
    phase_begin(ctx, TSP_PHASE_CONVERT, s);
    int rc = convert_enqueue(ctx, A, alias ? (TSP_FORM_LEFT | TSP_FORM_RIGHT) : TSP_FORM_LEFT, S_TILES_A, &ta, s);
    if (!rc && !alias) rc = convert_enqueue(ctx, B, TSP_FORM_RIGHT, S_TILES_B, &tb, s);
    phase_end(ctx, TSP_PHASE_CONVERT, s);
    // (behind the converters, whose host-side checks have seen both matrices; the count travels to the host
    // with the sizes the symbolic phase reads back)
    if (!rc && ctx->count_products) count_products(ctx, A, B, s);
    if (!rc) rc = symbolic_run(ctx, ta, alias ? ta : tb, &plan, s);
    ctx->stats.products = !rc && ctx->count_products ? ctx->h_scalars[S_PRODUCTS] : -1;
    if (!rc) rc = numeric_enqueue(ctx, ta, alias ? ta : tb, plan, C, s, /*last_of_call=*/true);   // the plan ends here
    if (!rc && ctx->compact) {                    // Algorithm 1, the compaction steps: strictly sparse result
        tsp_csr structural = *C;
        bool taken = false;                       // (no entry is zero: C keeps the arrays it has)
        rc = compact_zeros(ctx, &structural, C, s, &taken);
        if (!taken) tsp_csr_free(ctx, &structural, stream);
    }
    total_end(ctx, s);
    if (ctx->timers) {
        hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess && !rc) rc = hip_fail(ctx, e);
        collect_timers(ctx);
    }
    plan_release(ctx, plan, s);
    tiles_release(ctx, ta, s);
    tiles_release(ctx, tb, s);
    if (rc) {
        tsp_csr tmp = *C;
        if (tmp.row_ptr || tmp.col_idx || tmp.val) tsp_csr_free(ctx, &tmp, stream);
        std::memset(C, 0, sizeof(*C));
    }
    return rc;
}
