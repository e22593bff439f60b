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
constexpr int kGroupTiles = 4;         // output tiles computed together and written out row by row
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

// What a lane needs to write out its column of one output tile: lane l of a group of four tiles
// holds, after the transposition, column l%16 of all 16 rows of tile l/16.
struct Emission {
    uint4 m0, m1;             // the tile's 16 row masks, 16 bits each
    uint4 o0, o1, o2, o3;     // per row: position of the tile's first entry, from the start of the tile-row
    int64_t base;             // position of the tile-row's first entry in C
    int32_t col;              // column of this lane inside C
    bool valid;               // the lane's tile exists
};

__device__ __forceinline__ void swap_rows(float &x, float &y, bool halves) {
    // rows = groups of 16 lanes.  halves == false: rows 1, 3 of x <-> rows 0, 2 of y;
    // halves == true: rows 2, 3 of x <-> rows 0, 1 of y
    const unsigned a = __float_as_uint(x), b = __float_as_uint(y);
    const auto r = halves ? __builtin_amdgcn_permlane32_swap(a, b, false, false)
                          : __builtin_amdgcn_permlane16_swap(a, b, false, false);
    x = __uint_as_float(r[0]);
    y = __uint_as_float(r[1]);
}

template <class Array, int kTilesPerWave>
__global__ __launch_bounds__(kNumThreads) void k_numeric(
    const int64_t c_tiles, const NumericSizes z, const int64_t *__restrict__ pair_off,
    const int32_t *__restrict__ pair_a_, const int32_t *__restrict__ pair_b_, const uint32_t *__restrict__ a_lmask_,
    const uint32_t *__restrict__ a_loff_, const uint4 *__restrict__ a_ldata_, const uint32_t *__restrict__ b_rmask_,
    const uint32_t *__restrict__ b_roff_, const uint4 *__restrict__ b_rdata_, const int32_t *__restrict__ c_tile_row,
    const int32_t *__restrict__ c_tile_col, const uint16_t *__restrict__ c_row_mask,
    const uint32_t *__restrict__ c_row_off, const int64_t *__restrict__ c_row_ptr, int32_t *__restrict__ c_col,
    float *__restrict__ c_val) {
    static_assert(kTilesPerWave % kGroupTiles == 0 && kTilesPerWave <= 32, "whole groups; offsets fit one wave load");
    // consecutive logical blocks on the same XCD (workgroups are dealt to the XCDs round-robin)
    const int per_xcd = gridDim.x / kXcds;
    const int logical = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    // wave-uniform values are kept in scalar registers; their loads become scalar loads
    const int64_t wave = (int64_t)logical * (kNumThreads / 64) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t run_begin = wave * kTilesPerWave;
    if (run_begin >= c_tiles) return;
    const int run_tiles = (int)min((int64_t)kTilesPerWave, c_tiles - run_begin);
    const int lane = threadIdx.x & 63;
    const int hl = lane & 31, upper = lane >> 5;
    const uint32_t bit = 1u << hl, below = bit - 1u;
    const int j = lane & 15, tq = lane >> 4;
    const Array pair_a(pair_a_, z.pairs * 4), pair_b(pair_b_, z.pairs * 4);
    const Array a_lmask(a_lmask_, z.a_tiles * 4), a_loff(a_loff_, z.a_tiles * 4);
    const Array b_rmask(b_rmask_, z.b_tiles * 4), b_roff(b_roff_, z.b_tiles * 4);
    const Array a_ldata(a_ldata_, z.a_groups * 16), b_rdata(b_rdata_, z.b_groups * 16);

    // segment bounds of the run's tiles, relative to the first one (one vector load, then scalars)
    const int64_t off_lane = pair_off[run_begin + min(lane, run_tiles)];
    const int64_t base = ((int64_t)__builtin_amdgcn_readlane((int)(off_lane >> 32), 0) << 32) |
                         (uint32_t)__builtin_amdgcn_readlane((int)off_lane, 0);
    const int rel_lane = (int)(off_lane - base);
    const int rel_end = __builtin_amdgcn_readlane(rel_lane, kTilesPerWave);        // lanes >= run_tiles hold the end

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
    // MFMA; the loads of up to four MFMAs are requested together
    auto multiply = [&](const Header &h, int o, int count, float4v &acc) {
        for (int it = 0; it < count; it += 8) {
            Group a0, b0, a1, b1, a2, b2, a3, b3;
            const int left = count - it;                                // > 0, uniform
            load_operands(h, (o + it + upper) & 63, upper < left, a0, b0);
            if (left > 2) load_operands(h, (o + it + 2 + upper) & 63, 2 + upper < left, a1, b1);
            if (left > 4) load_operands(h, (o + it + 4 + upper) & 63, 4 + upper < left, a2, b2);
            if (left > 6) load_operands(h, (o + it + 6 + upper) & 63, 6 + upper < left, a3, b3);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, b0.h, acc, 0, 0, 0);
            if (left > 2) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, b1.h, acc, 0, 0, 0);
            if (left > 4) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2.h, b2.h, acc, 0, 0, 0);
            if (left > 6) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a3.h, b3.h, acc, 0, 0, 0);
        }
    };

    int h_start = 0;                              // relative position of the entry lane 0 of `heads` holds
    Header heads = load_headers(0);
#pragma unroll
    for (int g = 0; g < kTilesPerWave / kGroupTiles; ++g) {
        if (g * kGroupTiles < run_tiles) {        // uniform
            // Requested before the multiplications, used after them: what lane (tq, j) needs to write
            // out column j of tile tq of this group (requesting them afterwards saves 26 registers and
            // gains occupancy, but measured slower: the kernel then waits for them with nothing to do).
            Emission em;
            em.valid = g * kGroupTiles + tq < run_tiles;
            {
                const int64_t c = run_begin + (em.valid ? g * kGroupTiles + tq : 0);
                const uint4 *mp = reinterpret_cast<const uint4 *>(c_row_mask + c * T);
                const uint4 *op = reinterpret_cast<const uint4 *>(c_row_off + c * T);
                em.m0 = mp[0]; em.m1 = mp[1];
                em.o0 = op[0]; em.o1 = op[1]; em.o2 = op[2]; em.o3 = op[3];
                em.base = c_row_ptr[(int64_t)c_tile_row[c] * T];
                em.col = c_tile_col[c] * T + j;
            }
            float4v acc[kGroupTiles];
#pragma unroll
            for (int t = 0; t < kGroupTiles; ++t) {
                acc[t] = float4v{0.f, 0.f, 0.f, 0.f};
                const int tile = g * kGroupTiles + t;
                if (tile < run_tiles) {           // uniform
                    const int r0 = __builtin_amdgcn_readlane(rel_lane, tile);
                    const int r1 = __builtin_amdgcn_readlane(rel_lane, tile + 1);
                    const int n = r1 - r0, first_part = min(n, 64);
                    // the 64 entries in `heads` must cover the first 64 entries of this segment
                    if (r0 < h_start || r0 + first_part > h_start + 64) {
                        h_start = r0;
                        heads = load_headers(h_start);
                    }
                    multiply(heads, r0 - h_start, first_part, acc[t]);
                    // segments longer than 64 entries: the rest, 64 at a time
                    for (int s = r0 + 64; s < r1; s += 64) {
                        const Header h = load_headers(s);
                        multiply(h, 0, min(r1 - s, 64), acc[t]);
                    }
                }
            }
            // Transposition between tile index and row block: register v of tile t holds rows 4q+v in
            // lanes 16q..16q+15; afterwards rows[v][q] holds row 4q+v of tile tq in lanes 16tq..16tq+15,
            // so that one store instruction writes one CSR row across the four tiles, which are
            // neighbours in that row: one contiguous run per instruction instead of four.
            float rows[4][kGroupTiles];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
#pragma unroll
                for (int t = 0; t < kGroupTiles; ++t) rows[v][t] = acc[t][v];
                swap_rows(rows[v][0], rows[v][1], false);
                swap_rows(rows[v][2], rows[v][3], false);
                swap_rows(rows[v][0], rows[v][2], true);
                swap_rows(rows[v][1], rows[v][3], true);
            }
            const uint32_t mw[8] = {em.m0.x, em.m0.y, em.m0.z, em.m0.w, em.m1.x, em.m1.y, em.m1.z, em.m1.w};
            const uint32_t ow[16] = {em.o0.x, em.o0.y, em.o0.z, em.o0.w, em.o1.x, em.o1.y, em.o1.z, em.o1.w,
                                     em.o2.x, em.o2.y, em.o2.z, em.o2.w, em.o3.x, em.o3.y, em.o3.z, em.o3.w};
#pragma unroll
            for (int r = 0; r < T; ++r) {
                const uint32_t m = (r & 1) ? mw[r >> 1] >> 16 : mw[r >> 1] & 0xFFFFu;
                if (em.valid && ((m >> j) & 1u)) {
                    const int64_t pos = em.base + (int64_t)ow[r] + __popc(m & ((1u << j) - 1u));
                    c_col[pos] = em.col;
                    c_val[pos] = rows[r & 3][r >> 2];
                }
            }
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
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kNumThreads), 0, s, P->c_tiles, z, P->pair_off,
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
