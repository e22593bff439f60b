// Multiplication pass and CSR emission (paper Sections 4.3 and 4.4, Algorithm 1 line 18).
//
// One wave owns one output tile at a time and walks the tile's task-list segment: the pairs of a C
// tile form one 16 x 16p by 16p x 16 product, so the inner (K) dimension of
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
// The paper notes that this kernel is bound by the scattered tile reads behind the task list
// (Section 6.2).  The chain task-list entry -> tile header -> tile elements is three dependent
// memory accesses, so a wave takes a run of four or eight consecutive output tiles, whose task-list
// segments are contiguous, and reads 64 entries and their tile headers at once, one per lane: the
// first two accesses are paid once per run, not per tile.  The entries are handed to the two
// half-waves with cross-lane reads.  The loop over the run's tiles is fully unrolled, each tile
// requests only the operands it has entries for, and a tile is written out after the next tile's
// loads have been requested.  All gathers go through buffer descriptors whose range check returns
// zeros for masked-off lanes (no branches, no zero-filled registers).  Workgroup ids are remapped so
// that consecutive runs of output tiles execute on the same XCD and share its L2.
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

constexpr int kNumThreads = 256;       // 4 waves per block
constexpr int kMaxTilesPerWave = 8;    // consecutive output tiles one wave walks: 4 or 8
constexpr int kXcds = 8;

struct Header {          // tile headers of one task-list entry, held by the lane that read the entry
    uint32_t lm, lo, rm, ro;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Read-only array behind a buffer descriptor: a lane that passes valid = false (or an index past the
// end) gets zeros back from the hardware range check, so predicated loads need neither branches nor
// zero-initialised registers.  Offsets are 32-bit: the array must be smaller than 4 GiB.
struct BufferArray {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ BufferArray(const void *base, uint64_t bytes)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (uint32_t)bytes, 0x00020000)) {}
    __device__ __forceinline__ uint32_t u32(uint32_t index, bool valid) const {
        return __builtin_amdgcn_raw_buffer_load_b32(rsrc, valid ? index * 4u : 0xFFFFFFFFu, 0, 0);
    }
    __device__ __forceinline__ uint4 group(uint32_t index, bool valid) const {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, valid ? index * 16u : 0xFFFFFFFFu, 0, 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    }
};
// Same interface on plain pointers, for arrays of 4 GiB and more.
struct PointerArray {
    const void *base;
    __device__ __forceinline__ PointerArray(const void *b, uint64_t) : base(b) {}
    __device__ __forceinline__ uint32_t u32(uint32_t index, bool valid) const {
        return valid ? static_cast<const uint32_t *>(base)[index] : 0u;
    }
    __device__ __forceinline__ uint4 group(uint32_t index, bool valid) const {
        return valid ? static_cast<const uint4 *>(base)[index] : make_uint4(0, 0, 0, 0);
    }
};

struct NumericSizes {
    uint64_t pairs, a_tiles, b_tiles, a_groups, b_groups;   // element counts of the arrays
};

// What a lane needs to emit its four accumulator values of one output tile.
struct Emission {
    uint2 cm2;            // row masks of rows 4*ig .. 4*ig+3 (16 bits each)
    uint4 coff4;          // entries of those CSR rows to the left of the tile
    longlong2 rb01, rb23; // starts of those CSR rows
    int32_t col;          // column of this lane inside C
};

template <class Array, int kTilesPerWave>
__global__ __launch_bounds__(kNumThreads) void k_numeric(
    const int64_t c_tiles, const int tiles_per_wave, const NumericSizes z, const int64_t *__restrict__ pair_off,
    const int32_t *__restrict__ pair_a_, const int32_t *__restrict__ pair_b_, const uint32_t *__restrict__ a_lmask_,
    const uint32_t *__restrict__ a_loff_, const uint4 *__restrict__ a_ldata_, const uint32_t *__restrict__ b_rmask_,
    const uint32_t *__restrict__ b_roff_, const uint4 *__restrict__ b_rdata_, const int32_t *__restrict__ c_tile_row,
    const int32_t *__restrict__ c_tile_col, const uint16_t *__restrict__ c_row_mask,
    const uint32_t *__restrict__ c_row_off, const int64_t *__restrict__ c_row_ptr, int32_t *__restrict__ c_col,
    float *__restrict__ c_val) {
    // consecutive logical blocks on the same XCD (workgroups are dealt to the XCDs round-robin)
    const int per_xcd = gridDim.x / kXcds;
    const int logical = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    // wave-uniform values are kept in scalar registers; their loads become scalar loads
    const int64_t wave = (int64_t)logical * (kNumThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t run_begin = wave * tiles_per_wave;
    if (run_begin >= c_tiles) return;
    const int64_t run_end = min(run_begin + tiles_per_wave, c_tiles);
    const int lane = threadIdx.x & 63;
    const int hl = lane & 31, upper = lane >> 5;
    const uint32_t bit = 1u << hl, below = bit - 1u;
    const int j = lane & 15, ig = lane >> 4;
    const Array pair_a(pair_a_, z.pairs * 4), pair_b(pair_b_, z.pairs * 4);
    const Array a_lmask(a_lmask_, z.a_tiles * 4), a_loff(a_loff_, z.a_tiles * 4);
    const Array b_rmask(b_rmask_, z.b_tiles * 4), b_roff(b_roff_, z.b_tiles * 4);
    const Array a_ldata(a_ldata_, z.a_groups * 16), b_rdata(b_rdata_, z.b_groups * 16);

    auto emit = [&](const Emission &em, const float4v &acc) {
        const uint32_t cm[4] = {em.cm2.x & 0xFFFFu, em.cm2.x >> 16, em.cm2.y & 0xFFFFu, em.cm2.y >> 16};
        const uint32_t coff[4] = {em.coff4.x, em.coff4.y, em.coff4.z, em.coff4.w};
        const int64_t rbase[4] = {em.rb01.x, em.rb01.y, em.rb23.x, em.rb23.y};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if ((cm[v] >> j) & 1u) {
                const int64_t pos = rbase[v] + (int64_t)(coff[v] + __popc(cm[v] & ((1u << j) - 1u)));
                c_col[pos] = em.col;
                c_val[pos] = acc[v];
            }
        }
    };
    Emission em_prev{};
    float4v acc_prev = {0.f, 0.f, 0.f, 0.f};
    bool have_prev = false;
  // the run is walked in groups of kTilesPerWave tiles
  for (int64_t c_begin = run_begin; c_begin < run_end; c_begin += kTilesPerWave) {
    const int n_tiles = (int)min((int64_t)kTilesPerWave, run_end - c_begin);
    // segment bounds of the group's tiles, relative to the first one (one vector load, then scalars)
    const int64_t off_lane = pair_off[c_begin + min(lane, n_tiles)];
    const int64_t base = ((int64_t)__builtin_amdgcn_readlane((int)(off_lane >> 32), 0) << 32) |
                         (uint32_t)__builtin_amdgcn_readlane((int)off_lane, 0);
    const int rel_lane = (int)(off_lane - base);
    const int rel_end = __builtin_amdgcn_readlane(rel_lane, kTilesPerWave);        // lanes >= n_tiles hold the end

    // 64 consecutive task-list entries starting at relative position `start`, one per lane, with the
    // headers of their tiles; lanes past the end of the wave's entries hold all-zero headers
    auto load_headers = [&](int start) {
        const bool valid = start + lane < rel_end;
        const uint32_t e = (uint32_t)(base + start + lane);
        const uint32_t a = pair_a.u32(e, valid), b = pair_b.u32(e, valid);
        return Header{a_lmask.u32(a, valid), a_loff.u32(a, valid), b_rmask.u32(b, valid), b_roff.u32(b, valid)};
    };
    // operands of the entry held by lane `src` for this lane, or zeros when the entry is not part of
    // the current segment (valid == false) or the group is empty
    auto load_operands = [&](const Header &h, int src, bool valid, Group &av, Group &bv) {
        const uint32_t lm = (uint32_t)__shfl((int)h.lm, src, 64), lo = (uint32_t)__shfl((int)h.lo, src, 64);
        const uint32_t rm = (uint32_t)__shfl((int)h.rm, src, 64), ro = (uint32_t)__shfl((int)h.ro, src, 64);
        av.u = a_ldata.group(lo + __popc(lm & below), valid && (lm & bit) != 0);
        bv.u = b_rdata.group(ro + __popc(rm & below), valid && (rm & bit) != 0);
    };
    // multiply the `count` entries that start at lane `o` of the headers h into acc, two entries per
    // MFMA; the loads of up to four MFMAs are requested together, `between` runs once after the first
    // batch of loads has been requested
    auto multiply = [&](const Header &h, int o, int count, float4v &acc, auto between) {
        bool first = true;
        for (int it = 0; it < count; it += 8) {
            Group a0, b0, a1, b1, a2, b2, a3, b3;
            const int left = count - it;                                // > 0, uniform
            load_operands(h, (o + it + upper) & 63, upper < left, a0, b0);
            if (left > 2) load_operands(h, (o + it + 2 + upper) & 63, 2 + upper < left, a1, b1);
            if (left > 4) load_operands(h, (o + it + 4 + upper) & 63, 4 + upper < left, a2, b2);
            if (left > 6) load_operands(h, (o + it + 6 + upper) & 63, 6 + upper < left, a3, b3);
            if (first) between();
            first = false;
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, b0.h, acc, 0, 0, 0);
            if (left > 2) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, b1.h, acc, 0, 0, 0);
            if (left > 4) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2.h, b2.h, acc, 0, 0, 0);
            if (left > 6) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a3.h, b3.h, acc, 0, 0, 0);
        }
        if (first) between();
    };

    int h_start = 0;                              // relative position of the entry lane 0 of `heads` holds
    Header heads = load_headers(0);
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        if (t < n_tiles) {                        // uniform
            const int64_t c = c_begin + t;
            const int r0 = __builtin_amdgcn_readlane(rel_lane, t), r1 = __builtin_amdgcn_readlane(rel_lane, t + 1);
            const int n = r1 - r0, first_part = min(n, 64);
            // what the emission needs, requested before the multiplication: row masks (4 x 16 bit), the
            // rows' entry counts left of the tile (4 x 32 bit) and the rows' starts (4 x 64 bit; the plan
            // pads row_ptr to whole tile-rows, so rows past the matrix edge read valid memory)
            const int64_t I = c_tile_row[c], J = c_tile_col[c];
            Emission em;
            em.cm2 = *reinterpret_cast<const uint2 *>(c_row_mask + c * T + 4 * ig);
            em.coff4 = *reinterpret_cast<const uint4 *>(c_row_off + c * T + 4 * ig);
            em.rb01 = *reinterpret_cast<const longlong2 *>(c_row_ptr + I * T + 4 * ig);
            em.rb23 = *reinterpret_cast<const longlong2 *>(c_row_ptr + I * T + 4 * ig + 2);
            em.col = (int32_t)(J * T + j);
            // the 64 entries in `heads` must cover the first 64 entries of this segment
            if (r0 < h_start || r0 + first_part > h_start + 64) {
                h_start = r0;
                heads = load_headers(h_start);
            }
            float4v acc = {0.f, 0.f, 0.f, 0.f};
            // the previous tile is written out after this tile's loads are on their way, so that no
            // wait for a load ever includes the acknowledgement of a store
            multiply(heads, r0 - h_start, first_part, acc, [&]() {
                if (have_prev) emit(em_prev, acc_prev);
            });
            // segments longer than 64 entries: the rest, 64 at a time
            for (int s = r0 + 64; s < r1; s += 64) {
                const Header h = load_headers(s);
                multiply(h, 0, min(r1 - s, 64), acc, []() {});
            }
            em_prev = em;
            acc_prev = acc;
            have_prev = true;
        }
    }
  }
    if (have_prev) emit(em_prev, acc_prev);
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
        // Tiles one wave walks.  Short runs keep the tiles in flight on an XCD close together, so that
        // the B tiles they share stay in that XCD's L2; long runs amortise the header gather when the
        // segments are short (measured on the stencil and Laplacian workloads).
        const int tiles_per_wave = P->pairs > 4 * P->c_tiles ? 4 : 8;
        const int64_t tiles_per_block = (int64_t)(kNumThreads / 64) * tiles_per_wave;
        int64_t blocks = (P->c_tiles + tiles_per_block - 1) / tiles_per_block;
        blocks = (blocks + kXcds - 1) / kXcds * kXcds;             // the XCD remap needs a multiple of 8
        const NumericSizes z{(uint64_t)P->pairs, (uint64_t)A->tile_capacity, (uint64_t)B->tile_capacity,
                             (uint64_t)A->group_capacity, (uint64_t)B->group_capacity};
        const uint64_t limit = (1ull << 32) - 64;
        const bool narrow = z.pairs * 4 < limit && z.a_groups * 16 < limit && z.b_groups * 16 < limit &&
                            z.a_tiles * 4 < limit && z.b_tiles * 4 < limit && !ctx->force_wide;
        auto kernel = narrow ? (tiles_per_wave == 4 ? k_numeric<BufferArray, 4> : k_numeric<BufferArray, 8>)
                             : (tiles_per_wave == 4 ? k_numeric<PointerArray, 4> : k_numeric<PointerArray, 8>);
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kNumThreads), 0, s, P->c_tiles, tiles_per_wave, z, P->pair_off,
                           P->pair_a, P->pair_b, A->lmask, A->loff, A->ldata, B->rmask, B->roff, B->rdata,
                           P->c_tile_row, P->c_tile_col, P->c_row_mask, P->c_row_off, P->c_row_ptr, col, val);
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
