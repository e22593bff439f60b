// tsp_spgemm: the whole pipeline of Algorithm 1, CSR in, CSR out.
#include "common.hpp"

namespace tsp {
__global__ void k_clear_scalars_all(int64_t *d_scalars) {
    if (threadIdx.x < kScalars) d_scalars[threadIdx.x] = 0;
}
}  // namespace tsp

using namespace tsp;

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
    if (!rc) rc = symbolic_run(ctx, ta, alias ? ta : tb, &plan, s);
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
