// Multiplication pass and CSR emission (paper Sections 4.3 and 4.4; the multiplication kernel of Algorithm 1).
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
// zero when the group mask says the group is empty: nothing is expanded through the bitmap at run time.
// The accumulator of lane l holds column l%16, rows 4*(l/16)..+3 of the output tile.
//
// The paper notes that this kernel is bound by the scattered tile reads behind the task list
// (Section 6.2).  The chain task-list entry -> tile header -> tile elements is three dependent
// memory accesses, so a wave takes a group of four consecutive output tiles, whose task-list
// segments are contiguous, and gathers 64 entries and their tile headers at once, one per lane,
// into LDS: the first two accesses are paid once per group, and every multiplication step reads its
// two headers back with one LDS load.  The loop over the group's tiles is fully unrolled and each
// tile requests the operands of up to four MFMAs together.  In the kernels for arrays below 4 GiB
// all accesses go through buffer descriptors with 32-bit byte offsets whose range check returns
// zeros for masked-off lanes (no branches, no zero-filled registers).  Workgroup ids are remapped
// so that consecutive groups of output tiles execute on the same XCD and share its L2.
//
// Emission: the counting pass left, per C tile, the 16 row masks of its structural pattern and
// per row the position of the tile's first entry, counted from the start of the tile-row.  The four
// accumulators of the group are transposed across the lanes so that lane (t, j) holds column j of
// all 16 rows of tile t; row r is then written by one store instruction for all four tiles, which
// are neighbours in CSR row 16I+r: the lane writes column 16J+j and its value at
// start(tile-row) + position(tile, r) + popcount(mask_r below j).  Masks and positions are fetched
// one word per lane and handed round the 16 lanes of a tile when a row is written.
// Where every tile-row of C is short and sparse a wave takes a whole tile-row instead and assembles
// its output in LDS (see kWholeRows below).
//
// Measured on gfx950: on products with tens of entries per output tile and more the kernel is bound
// by the vector-memory path of the CU (operand loads of 1 KB per instruction, stores that cost by the
// cache lines they touch, header gathers that cost by the lane), and shortening waits or instruction
// counts alone does not change its duration; on very sparse tiles it is bound by instruction issue.
#include "common.hpp"

#include <algorithm>
#include <new>
#include <utility>

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
constexpr int kBlockEntries = 64;      // task-list entries staged at a time: one per lane
constexpr int kRowTilesUnrolled = 16;  // ... up to which its loop over the groups of four tiles is unrolled (2 % faster)
constexpr int kRowTiles = 60;          // whole-tile-row kernel: most output tiles a tile-row may have (one lane each)
constexpr int kRowEntries = 448;       // ... and most structural entries (its output is assembled in LDS)
constexpr int64_t kSparseTileEntries = 3;   // kHalves is used for operands with at most this many entries per tile on average

struct Header {          // tile headers of one task-list entry, as the lanes of the wave read them from LDS
    uint32_t lm, lo, rm, ro;   // group masks and BYTE offsets of the first group: left form of A, right form of B
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSkip = 0xFFFFFFFFu;   // byte offset that the range check of a buffer descriptor rejects

// Array behind a buffer descriptor: a byte offset of kSkip (or any offset past the end) reads zeros
// and writes nothing, so predicated accesses need neither branches nor zero-initialised registers.
// Offsets are 32-bit: the array must be smaller than 4 GiB.
struct BufferArray {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ BufferArray(const void *base, uint64_t bytes)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (uint32_t)bytes, 0x00020000)) {}
    __device__ __forceinline__ uint32_t u32(uint32_t byte_off) const {
        return __builtin_amdgcn_raw_buffer_load_b32(rsrc, byte_off, 0, 0);
    }
    __device__ __forceinline__ uint2 u64(uint32_t byte_off) const {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_off, 0, 0);
        return make_uint2(v.x, v.y);
    }
    template <int kPlus>
    __device__ __forceinline__ uint4 u128(uint32_t byte_off) const {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, kPlus, 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    __device__ __forceinline__ void put(uint32_t byte_off, uint32_t value) const {
        __builtin_amdgcn_raw_buffer_store_b32(value, rsrc, byte_off, 0, 0);
    }
};
struct NumericSizes {
    uint64_t pairs, a_tiles, b_tiles, a_groups, b_groups;   // element counts of the arrays
};

// What a lane needs to write out its column of one output tile: lane l of a group of four tiles
// holds, after the transposition, column l%16 of all 16 rows of tile l/16.
struct Emission {
    uint32_t masks;           // row masks 2(j%8) (low half) and 2(j%8)+1 (high half) of the tile (zero: no such tile)
    uint32_t first;           // row j: position of the tile's first entry, from the start of the tile-row
    int64_t base;             // position of the tile-row's first entry in C
    int32_t col;              // column of this lane inside C
};

// Value that lane kFrom of every row of 16 lanes holds, in all lanes of that row.  All lanes of the
// row must be active.
template <int kFrom>
__device__ __forceinline__ uint32_t row_broadcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x150 + kFrom, 0xF, 0xF, false);   // row_newbcast
}

template <typename F, int... kR>
__device__ __forceinline__ void for_each_row(F &&f, std::integer_sequence<int, kR...>) {
    (f(std::integral_constant<int, kR>{}), ...);
}

__device__ __forceinline__ void swap_rows(float &x, float &y, bool halves) {
    // rows = groups of 16 lanes.  halves == false: rows 1, 3 of x <-> rows 0, 2 of y;
    // halves == true: rows 2, 3 of x <-> rows 0, 1 of y
    const unsigned a = __float_as_uint(x), b = __float_as_uint(y);
    const auto r = halves ? __builtin_amdgcn_permlane32_swap(a, b, false, false)
                          : __builtin_amdgcn_permlane16_swap(a, b, false, false);
    x = __uint_as_float(r[0]);
    y = __uint_as_float(r[1]);
}

// kNarrow: every array is smaller than 4 GiB and is addressed through a buffer descriptor with
// 32-bit byte offsets; otherwise 64-bit pointers and branches.
// kMatrixCores == false: the block products run on the vector ALUs, every lane looping over the
// inner index for its four output elements (the paper's comparison build without tensor cores,
// Section 5, Algorithm 2); everything around the product is shared.
//
// kWholeRows: a wave takes one whole tile-row of C (at most kRowTiles tiles and kRowEntries entries,
// which the host has checked) instead of kTilesPerWave consecutive tiles.  The entries of a tile-row
// are one contiguous stretch of col_idx and val, so the wave puts them together in LDS, at the
// positions the counting pass assigned, and writes the stretch with full-width stores.  Written
// tile by tile, a row of a sparse tile is a run of a few entries, and a store costs by the
// 64-byte lines it touches, not by the bytes it carries.
//
// kHalves: for operands whose tiles hold a few entries (a power-law graph: two per tile).  The inner dimension
// of the instruction is four slots of eight inner indices, and a pair of tiles fills two of them, one per half
// of its 16 inner indices.  Where the A tile has nothing in a half of its columns, or the B tile nothing in
// that half of its rows, the slot multiplies zeros: on such a graph a pair has 1.17 halves that meet, not 2.
// Here the halves that meet are listed when the entries are staged (entry and half, in task-list order), and a
// step takes four of them, of up to four different pairs: 0.29 steps and operand loads per pair instead of 0.5.
template <bool kNarrow, int kTilesPerWave, bool kMatrixCores, bool kWholeRows = false, bool kHalves = false>
__global__ __launch_bounds__(kNumThreads) void k_numeric(
    const int64_t c_tiles, const int64_t c_nnz, const NumericSizes z, const int64_t c_rows, const int32_t c_tile_rows,
    const int32_t *__restrict__ c_tile_row_ptr, const int64_t *__restrict__ pair_off,
    const int2 *__restrict__ pair_ab_, const uint2 *__restrict__ a_lhead_,
    const uint4 *__restrict__ a_ldata_, const uint2 *__restrict__ b_rhead_, const uint4 *__restrict__ b_rdata_, const int32_t *__restrict__ c_tile_row,
    const int32_t *__restrict__ c_tile_col, const uint16_t *__restrict__ c_row_mask,
    const uint32_t *__restrict__ c_row_off, const int64_t *__restrict__ c_row_ptr, int32_t *__restrict__ c_col,
    float *__restrict__ c_val, int64_t *__restrict__ scalars_to_clear, const int2 *__restrict__ strip_desc,
    const int32_t *__restrict__ strip_total, const int xcd_chunk) {
    if (scalars_to_clear && blockIdx.x == 0 && threadIdx.x < kScalars) scalars_to_clear[threadIdx.x] = 0;
    static_assert(kTilesPerWave % kGroupTiles == 0 && kTilesPerWave < 64, "whole groups; offsets fit one wave load");
    // headers of the 64 task-list entries a wave is working on, one 16-byte record per entry; one
    // spare record per wave: the second half-wave may address the entry after the last one
    __shared__ uint4 lds_heads[kNumThreads / 64][kBlockEntries + 16];
    // operand groups of one step, as the lanes loaded them (vector-ALU build only)
    __shared__ uint4 lds_operands[kMatrixCores ? 1 : kNumThreads / 64][2][64];
    // column and value of every entry of the wave's tile-row, in CSR order (whole-tile-row kernel only)
    __shared__ uint32_t lds_entries[kWholeRows ? kNumThreads / 64 : 1][2][kWholeRows ? kRowEntries : 1];
    // kHalves: the halves of the staged entries that meet, 2 * entry + half, in task-list order
    static_assert(!kHalves || (kMatrixCores && !kWholeRows), "the list of halves feeds the MFMA steps of the tile-group kernel");
    __shared__ uint8_t lds_halves[kHalves ? kNumThreads / 64 : 1][kHalves ? 2 * kBlockEntries + 4 : 4];
    // consecutive logical blocks on the same XCD (workgroups are dealt to the XCDs round-robin)
    const int64_t logical = xcd_chunked_index(blockIdx.x, xcd_chunk);
    // wave-uniform values are kept in scalar registers; their loads become scalar loads
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t wave = (int64_t)logical * (kNumThreads / 64) + wave_in_block;
    int64_t run_begin;
    int run_tiles;
    if constexpr (kWholeRows) {
        static_assert(kTilesPerWave == kRowTilesUnrolled || kTilesPerWave == kRowTiles, "the groups cover a whole tile-row");
        if (wave >= c_tile_rows) return;
        run_begin = c_tile_row_ptr[wave];                                       // wave = tile-row of C
        run_tiles = min(c_tile_row_ptr[wave + 1] - (int)run_begin, kTilesPerWave);
        if (run_tiles <= 0 || run_begin + run_tiles > c_tiles) return;
    } else if (strip_desc) {
        // order in vertical strips: the block's tiles are the ones its descriptor names
        if (logical >= *strip_total) return;
        const int2 d = strip_desc[logical];
        run_begin = (int64_t)d.x + wave_in_block * kTilesPerWave;
        run_tiles = min(kTilesPerWave, d.y - wave_in_block * kTilesPerWave);
        if (run_tiles <= 0 || run_begin + run_tiles > c_tiles) return;
    } else {
        run_begin = wave * kTilesPerWave;
        if (run_begin >= c_tiles) return;
        run_tiles = (int)min((int64_t)kTilesPerWave, c_tiles - run_begin);
    }
    const int lane = threadIdx.x & 63;
    const int hl = lane & 31, upper = lane >> 5;
    const uint32_t bit = 1u << hl, below = bit - 1u;
    const int j = lane & 15, tq = lane >> 4;
    // descriptors (used by the narrow kernels only)
    const BufferArray pair_ab(pair_ab_, z.pairs * 8);
    const BufferArray a_lhead(a_lhead_, z.a_tiles * 8), b_rhead(b_rhead_, z.b_tiles * 8);
    const BufferArray a_ldata(a_ldata_, z.a_groups * 16), b_rdata(b_rdata_, z.b_groups * 16);
    uint4 *const my_heads = lds_heads[wave_in_block];
    const uint4 *const my_half = my_heads + upper;    // lanes 32-63 read the entry after the one lanes 0-31 read
    uint8_t *const my_halves = lds_halves[kHalves ? wave_in_block : 0];
    uint32_t halves_before = 0;                       // kHalves: listed halves of the staged entries before this lane's
    int halves_total = 0;                             // ... and of all 64 (uniform)

    // segment bounds of the run's tiles, relative to the first one (one vector load, then scalars)
    const int64_t off_lane = pair_off[run_begin + min(lane, run_tiles)];
    // coordinates of the output tile this lane will write (first group), requested together with the
    // segment bounds: the start of its tile-row in C depends on them and is requested one step later
    const int64_t c_first = run_begin + (tq < run_tiles ? tq : 0);
    const int32_t I_first = kWholeRows ? (int32_t)wave : c_tile_row[c_first], J_first = c_tile_col[c_first];
    const int64_t base = ((int64_t)__builtin_amdgcn_readlane((int)(off_lane >> 32), 0) << 32) |
                         (uint32_t)__builtin_amdgcn_readlane((int)off_lane, 0);
    const int rel_lane = (int)(off_lane - base);
    const int rel_end = __builtin_amdgcn_readlane(rel_lane, kWholeRows ? run_tiles : kTilesPerWave);   // lanes >= run_tiles hold the end

    // 64 consecutive task-list entries starting at relative position `start`, one per lane: the
    // headers of their tiles go to LDS, where any lane can read any entry's record with one load
    // (entries past the end of the wave's run leave all-zero records: empty tiles)
    auto stage_headers = [&](int start) {
        const bool valid = start + lane < rel_end;
        uint4 record = make_uint4(0, 0, 0, 0);
        if constexpr (kNarrow) {
            // lanes without an entry are switched off, not sent out of range: a gather costs by the
            // lanes that take part in it
            if (valid) {
                const uint2 ab = pair_ab.u64((uint32_t)(base + start + lane) * 8u);
                const uint2 la = a_lhead.u64(ab.x * 8u), rb = b_rhead.u64(ab.y * 8u);
                // group offsets become byte offsets: the descriptors address bytes
                record = make_uint4(la.x, la.y << 4, rb.x, rb.y << 4);
            }
        } else if (valid) {
            const int64_t e = base + start + lane;
            const int2 ab = pair_ab_[e];
            const int64_t a = ab.x, b = ab.y;
            const uint2 la = a_lhead_[a], rb = b_rhead_[b];
            record = make_uint4(la.x, la.y, rb.x, rb.y);
        }
        wave_sync();                               // earlier reads of the records are done
        my_heads[lane] = record;
        if constexpr (kHalves) {
            // a half meets when the A tile has a group in that half of its columns and the B tile one in that
            // half of its rows (entries past the end have all-zero records and list nothing)
            const uint32_t h0 = ((record.x & 0xFFFFu) && (record.z & 0xFFFFu)) ? 1u : 0u;
            const uint32_t h1 = ((record.x >> 16) && (record.z >> 16)) ? 1u : 0u;
            const uint32_t inc = wave_inclusive_scan(h0 + h1);
            halves_before = inc - h0 - h1;
            halves_total = __builtin_amdgcn_readlane((int)inc, 63);
            if (h0) my_halves[halves_before] = (uint8_t)(2 * lane);
            if (h1) my_halves[halves_before + h0] = (uint8_t)(2 * lane + 1);
        }
        wave_sync();
    };
    // operands of a step (entry `src` of the block for lanes 0-31, entry src+1 for lanes 32-63, the
    // latter only if two == true): the lane's 16-byte group of the A tile and of the B tile, zeros
    // when the group is empty
    auto load_operands = [&](int src, bool two, Group &av, Group &bv) {
        const uint4 h = my_half[src];
        const uint32_t mine = (two || !upper) ? bit : 0u;
        if constexpr (kNarrow) {
            const uint32_t ao = ((uint32_t)__popc(h.x & below) << 4) + h.y;
            const uint32_t bo = ((uint32_t)__popc(h.z & below) << 4) + h.w;
            av.u = a_ldata.template u128<0>((h.x & mine) ? ao : kSkip);
            bv.u = b_rdata.template u128<0>((h.z & mine) ? bo : kSkip);
        } else {
            av.u = (h.x & mine) ? a_ldata_[(uint64_t)h.y + __popc(h.x & below)] : make_uint4(0, 0, 0, 0);
            bv.u = (h.z & mine) ? b_rdata_[(uint64_t)h.w + __popc(h.z & below)] : make_uint4(0, 0, 0, 0);
        }
    };
    // kHalves: the operands of four listed halves, `first`.. of the staged block (those at or past `end` are
    // zeros): lanes 16q..16q+15 take the half first+q, of whichever entry it belongs to
    auto load_halves = [&](int first, int end, Group &av, Group &bv) {
        const int mine = first + tq;
        const bool live = mine < end;
        const uint32_t item = live ? my_halves[mine] : 0u;
        const uint4 h = my_heads[item >> 1];
        const uint32_t slot = 1u << (j + 16 * (item & 1u)), under = slot - 1u;
        if constexpr (kNarrow) {
            const uint32_t ao = ((uint32_t)__popc(h.x & under) << 4) + h.y;
            const uint32_t bo = ((uint32_t)__popc(h.z & under) << 4) + h.w;
            av.u = a_ldata.template u128<0>((live && (h.x & slot)) ? ao : kSkip);
            bv.u = b_rdata.template u128<0>((live && (h.z & slot)) ? bo : kSkip);
        } else {
            av.u = (live && (h.x & slot)) ? a_ldata_[(uint64_t)h.y + __popc(h.x & under)] : make_uint4(0, 0, 0, 0);
            bv.u = (live && (h.z & slot)) ? b_rdata_[(uint64_t)h.w + __popc(h.z & under)] : make_uint4(0, 0, 0, 0);
        }
    };
    // multiply the `count` entries that start at entry `o` of the staged block into acc, two entries
    // per MFMA; the loads of up to four MFMAs are requested together
    auto multiply = [&](int o, int count, float4v &acc) {
        if constexpr (kHalves) {
            // the listed halves of those entries, four per MFMA
            const int i0 = __builtin_amdgcn_readlane((int)halves_before, o);
            const int i1 = o + count < 64 ? __builtin_amdgcn_readlane((int)halves_before, o + count) : halves_total;
            for (int it = i0; it < i1; it += 16) {
                Group a0, b0, a1, b1, a2, b2, a3, b3;
                const int left = i1 - it;                                  // > 0, uniform
                load_halves(it, i1, a0, b0);
                if (left > 4) load_halves(it + 4, i1, a1, b1);
                if (left > 8) load_halves(it + 8, i1, a2, b2);
                if (left > 12) load_halves(it + 12, i1, a3, b3);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, b0.h, acc, 0, 0, 0);
                if (left > 4) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, b1.h, acc, 0, 0, 0);
                if (left > 8) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2.h, b2.h, acc, 0, 0, 0);
                if (left > 12) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a3.h, b3.h, acc, 0, 0, 0);
            }
            return;
        }
        if constexpr (kMatrixCores) {
            // entries in flight: short sparse tile-rows have segments of one to four entries, and the
            // registers of the deeper batch would cost their kernel a wave per SIMD
            constexpr int kDepth = kWholeRows ? 4 : 8;
            for (int it = 0; it < count; it += kDepth) {
                Group a0, b0, a1, b1, a2, b2, a3, b3;
                const int left = count - it;                                // > 0, uniform
                load_operands(o + it, left > 1, a0, b0);
                if (left > 2) load_operands(o + it + 2, left > 3, a1, b1);
                if constexpr (kDepth > 4) {
                    if (left > 4) load_operands(o + it + 4, left > 5, a2, b2);
                    if (left > 6) load_operands(o + it + 6, left > 7, a3, b3);
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0.h, b0.h, acc, 0, 0, 0);
                if (left > 2) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1.h, b1.h, acc, 0, 0, 0);
                if constexpr (kDepth > 4) {
                    if (left > 4) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a2.h, b2.h, acc, 0, 0, 0);
                    if (left > 6) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a3.h, b3.h, acc, 0, 0, 0);
                }
            }
        } else {
            // Two entries per step, loaded exactly as for the MFMA: lane 32e + 16h + x holds, of entry
            // e, inner indices 8h..8h+7 of row x of the A tile and of column x of the B tile.  The
            // groups go through LDS; lane (tq, j) then owns c[4tq+v][j], v = 0..3, and adds
            // a[4tq+v][k] * b[k][j] over the 16 inner indices of both entries, in fp32.
            uint4(*const ops)[64] = lds_operands[wave_in_block];
            for (int it = 0; it < count; it += 2) {
                Group a, b;
                load_operands(o + it, count - it > 1, a, b);
                wave_sync();                       // the previous step's reads are done
                ops[0][lane] = a.u;
                ops[1][lane] = b.u;
                wave_sync();
#pragma unroll
                for (int eh = 0; eh < 4; ++eh) {   // entry e = eh / 2, half h = eh % 2
                    Group col;
                    col.u = ops[1][16 * eh + j];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        Group row;
                        row.u = ops[0][16 * eh + 4 * tq + v];
#pragma unroll
                        for (int x = 0; x < 8; ++x) acc[v] = fmaf((float)row.h[x], (float)col.h[x], acc[v]);
                    }
                }
            }
        }
    };

    int h_start = 0;                              // relative position of the first staged entry
    stage_headers(0);
    Group next_a, next_b;                         // whole-tile-row kernel: operands of the next tile's first step
    next_a.u = next_b.u = make_uint4(0, 0, 0, 0);
    if constexpr (kWholeRows && kMatrixCores)
        load_operands(0, __builtin_amdgcn_readlane(rel_lane, 1) > 1, next_a, next_b);
    const int64_t base_first = c_row_ptr[(int64_t)I_first * T];
    uint32_t(*const my_entries)[kWholeRows ? kRowEntries : 1] = lds_entries[kWholeRows ? wave_in_block : 0];
    int row_entries = 0;                          // whole-tile-row kernel: entries of the tile-row
    if constexpr (kWholeRows)
        row_entries = (int)min(c_row_ptr[min((int64_t)(I_first + 1) * T, c_rows)] - base_first, (int64_t)kRowEntries);
    // (unrolled, but for whole tile-rows of more than 16 tiles, whose groups are a loop)
    constexpr int kGroupUnroll = kTilesPerWave > kRowTilesUnrolled ? 1 : kTilesPerWave / kGroupTiles;
#pragma unroll kGroupUnroll
    for (int g = 0; g < kTilesPerWave / kGroupTiles; ++g) {
        if (g * kGroupTiles < run_tiles) {        // uniform
            // The row masks and row positions of the group's four tiles, requested before the
            // multiplications and used after them: one word of each per lane, handed round inside a
            // row of 16 lanes when the entries are written.
            //   Tile by tile (lane (tq, j) writes column j of tile tq after the transposition): lane j of
            //   the tile's 16 lanes takes the position of row j and the masks of rows 2(j%8), 2(j%8)+1.
            //   Whole tile-rows (lane (q, j) writes column j of rows 4q..4q+3 of every tile, as the
            //   accumulators hold them): lane 4t+v of the 16 takes the position of row 4q+v of tile t
            //   and the masks of rows 4q+(v&2), +1.
            Emission em;
            const int tile_l = kWholeRows ? j >> 2 : tq;                 // tile whose words this lane fetches
            const int row_l = kWholeRows ? 4 * tq + (j & 3) : j;        // row whose position
            const int pair_l = kWholeRows ? 2 * tq + ((j & 3) >> 1) : (j & 7);   // pair of rows whose masks
            const bool mine_exists = g * kGroupTiles + tile_l < run_tiles;
            const int64_t c_mine = run_begin + (mine_exists ? g * kGroupTiles + tile_l : 0);
            int32_t col_of[kGroupTiles];                                // whole tile-rows: this lane's column in tile t
            if constexpr (kWholeRows) {
                em.base = base_first;
                em.col = 0;
#pragma unroll
                for (int t = 0; t < kGroupTiles; ++t)
                    col_of[t] = __builtin_amdgcn_readfirstlane(c_tile_col[run_begin + min(g * kGroupTiles + t, run_tiles - 1)]) * T;
            } else if (g == 0) {
                em.base = base_first;
                em.col = J_first * T + j;
            } else {
                em.base = c_row_ptr[(int64_t)c_tile_row[c_mine] * T];
                em.col = c_tile_col[c_mine] * T + j;
            }
            if constexpr (kNarrow) {
                const BufferArray masks(c_row_mask, (uint64_t)c_tiles * T * 2), offs(c_row_off, (uint64_t)c_tiles * T * 4);
                em.masks = masks.u32(mine_exists ? (uint32_t)c_mine * (T * 2) + (uint32_t)pair_l * 4u : kSkip);
                em.first = offs.u32(mine_exists ? (uint32_t)c_mine * (T * 4) + (uint32_t)row_l * 4u : kSkip);
                // narrow arrays: positions in C fit 32 bits, the start of the tile-row is added once here
                if constexpr (!kWholeRows) em.first += (uint32_t)em.base;
            } else {
                em.masks = mine_exists ? reinterpret_cast<const uint32_t *>(c_row_mask + c_mine * T)[pair_l] : 0u;
                em.first = c_row_off[c_mine * T + row_l];
            }
            float4v acc[kGroupTiles];
            if constexpr (kWholeRows && kMatrixCores) {
                // Every task-list entry of the tile-row is staged (at most 64: the host has checked), so a
                // tile's operands do not wait for anything but the tile before it: the first step of the next
                // tile is requested before the current tile is multiplied, and a wave goes through one memory
                // round trip per two tiles instead of one per tile (the tiles of such a tile-row have one
                // or two steps each, and the round trips were 60 % of a wave's life).
#pragma unroll
                for (int t = 0; t < kGroupTiles; ++t) {
                    acc[t] = float4v{0.f, 0.f, 0.f, 0.f};
                    const int tile = g * kGroupTiles + t;
                    if (tile < run_tiles) {       // uniform
                        const int r0 = __builtin_amdgcn_readlane(rel_lane, tile);
                        const int r1 = __builtin_amdgcn_readlane(rel_lane, tile + 1);
                        const Group a_now = next_a, b_now = next_b;
                        if (tile + 1 < run_tiles)
                            load_operands(r1, __builtin_amdgcn_readlane(rel_lane, tile + 2) - r1 > 1, next_a, next_b);
                        if (r1 > r0) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_now.h, b_now.h, acc[t], 0, 0, 0);
                        if (r1 - r0 > 2) multiply(r0 + 2, r1 - r0 - 2, acc[t]);
                    }
                }
            } else
#pragma unroll
            for (int t = 0; t < kGroupTiles; ++t) {
                acc[t] = float4v{0.f, 0.f, 0.f, 0.f};
                const int tile = g * kGroupTiles + t;
                if (tile < run_tiles) {           // uniform
                    const int r0 = __builtin_amdgcn_readlane(rel_lane, tile);
                    const int r1 = __builtin_amdgcn_readlane(rel_lane, tile + 1);
                    const int n = r1 - r0, first_part = min(n, kBlockEntries);
                    // the staged block must cover the first 64 entries of this segment
                    if (r0 < h_start || r0 + first_part > h_start + kBlockEntries) {
                        h_start = r0;
                        stage_headers(h_start);
                    }
                    multiply(r0 - h_start, first_part, acc[t]);
                    // segments longer than 64 entries: the rest, 64 at a time
                    for (int s = r0 + kBlockEntries; s < r1; s += kBlockEntries) {
                        h_start = s;
                        stage_headers(s);
                        multiply(0, min(r1 - s, kBlockEntries), acc[t]);
                    }
                }
            }
            const uint32_t my_bit[2] = {1u << j, 1u << (j + 16)};
            const uint32_t my_below[2] = {(1u << j) - 1u, ((1u << j) - 1u) << 16};
            if constexpr (kWholeRows) {
                // Straight from the accumulators into the tile-row's stretch in LDS: register v of tile t
                // is row 4q+v; its mask is the low (even v) or high (odd v) half of the word that lane
                // 4t+(v&2) of this row of lanes fetched, its position is what lane 4t+v fetched.  The
                // entry of column j exists if its bit is set and sits after the set bits below it.
                uint32_t pair = 0;
                for_each_row(
                    [&](auto index) {
                        constexpr int t = decltype(index)::value / 4, v = decltype(index)::value % 4;
                        if (g * kGroupTiles + t >= run_tiles) return;          // uniform
                        if constexpr (v % 2 == 0) pair = row_broadcast<4 * t + v>(em.masks);
                        const uint32_t first = row_broadcast<4 * t + v>(em.first);
                        if (pair & my_bit[v & 1]) {
                            const uint32_t rank = (uint32_t)__popc(pair & my_below[v & 1]) + first;
                            my_entries[0][rank] = (uint32_t)(col_of[t] + j);
                            my_entries[1][rank] = __float_as_uint(acc[t][v]);
                        }
                    },
                    std::make_integer_sequence<int, T>{});
            } else {
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
                // Row r of the tile: its mask is the low (even r) or high (odd r) half of the word that
                // lane r/2 of the tile's 16 lanes fetched, its position is what lane r fetched; the entry
                // of column j exists if its bit is set and sits after the set bits below it.
                // Every load of this wave has returned by now (the last tile's operands were requested
                // after everything else and have been used).  Saying so explicitly keeps the compiler from
                // putting load waits between the stores below, where they would also wait for the stores
                // before them.
                __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0)
                const BufferArray out_col(c_col, (uint64_t)c_nnz * 4), out_val(c_val, (uint64_t)c_nnz * 4);
                uint32_t pair = 0;
                for_each_row(
                    [&](auto row) {
                        constexpr int r = decltype(row)::value;
                        if constexpr (r % 2 == 0) pair = row_broadcast<r / 2>(em.masks);
                        const uint32_t first = row_broadcast<r>(em.first);
                        // lanes without an entry are switched off rather than sent out of range: a store
                        // costs by the lanes that take part in it
                        if (pair & my_bit[r & 1]) {
                            const uint32_t rank = (uint32_t)__popc(pair & my_below[r & 1]) + first;
                            if constexpr (kNarrow) {
                                out_col.put(rank << 2, (uint32_t)em.col);
                                out_val.put(rank << 2, __float_as_uint(rows[r & 3][r >> 2]));
                            } else {
                                const int64_t pos = em.base + (int64_t)rank;
                                c_col[pos] = em.col;
                                c_val[pos] = rows[r & 3][r >> 2];
                            }
                        }
                    },
                    std::make_integer_sequence<int, T>{});
            }
        }
    }
    if constexpr (kWholeRows) {
        // the tile-row's entries, 64 consecutive ones per store instruction
        wave_sync();
        for (int at = lane; at < row_entries; at += 64) {
            const uint32_t col = my_entries[0][at], val = my_entries[1][at];
            if constexpr (kNarrow) {
                const BufferArray out_col(c_col, (uint64_t)c_nnz * 4), out_val(c_val, (uint64_t)c_nnz * 4);
                const uint32_t byte = (uint32_t)(base_first + at) << 2;
                out_col.put(byte, col);
                out_val.put(byte, val);
            } else {
                c_col[base_first + at] = (int32_t)col;
                c_val[base_first + at] = __uint_as_float(val);
            }
        }
    }
}

int numeric_enqueue(tsp_context *ctx, tsp_tiles_s *A, tsp_tiles_s *B, tsp_plan_s *P, tsp_csr *C, hipStream_t s,
                    bool last_of_call) {
    std::memset(C, 0, sizeof(*C));
    if (!(A->forms & TSP_FORM_LEFT) || !(B->forms & TSP_FORM_RIGHT)) return TSP_ERR_INVALID_ARG;
    if (A->cols != B->rows || P->c_rows != A->rows || P->c_cols != B->cols) return TSP_ERR_SHAPE_MISMATCH;
    if (!P->c_row_ptr) return TSP_ERR_INVALID_ARG;                       // a plan whose row_ptr has been handed over
    int64_t *row_ptr = last_of_call ? P->c_row_ptr : ctx_alloc_n<int64_t>(ctx, (size_t)P->c_rows + 1, s);
    int32_t *col = ctx_alloc_n<int32_t>(ctx, (size_t)P->c_nnz, s);
    float *val = ctx_alloc_n<float>(ctx, (size_t)P->c_nnz, s);
    if (!row_ptr || !col || !val) {
        if (!last_of_call) ctx_free(ctx, row_ptr, s);
        ctx_free(ctx, col, s);
        ctx_free(ctx, val, s);
        return TSP_ERR_ALLOC_FAILED;
    }
    phase_begin(ctx, TSP_PHASE_NUMERIC, s);
    hipError_t e = hipSuccess;
    if (!last_of_call)
        e = hipMemcpyAsync(row_ptr, P->c_row_ptr, sizeof(int64_t) * (size_t)(P->c_rows + 1), hipMemcpyDeviceToDevice, s);
    if (e == hipSuccess && P->c_tiles > 0) {
        KernelTimer kt(ctx, TSP_KERNEL_NUMERIC, s);
        // Tiles one wave walks: one group of four measured fastest on all workloads (more waves in
        // flight); two groups per wave remain available through TSP_OPT_NUMERIC_RUN.
        int tiles_per_wave = kGroupTiles;
        if (ctx->numeric_run_len == 4 || ctx->numeric_run_len == 8) tiles_per_wave = ctx->numeric_run_len;
        if (!ctx->matrix_cores) tiles_per_wave = kGroupTiles;
        // Short, sparse tile-rows (meshes in two dimensions, for one): a wave per tile-row, output through LDS
        const bool whole_rows = ctx->matrix_cores && ctx->numeric_run_len == 0 && P->max_row_c_tiles <= kRowTiles &&
                                P->max_row_pairs <= kBlockEntries && P->max_row_entries <= kRowEntries;
        const int64_t tiles_per_block = (int64_t)(kNumThreads / 64) * tiles_per_wave;
        int64_t blocks = whole_rows ? (P->c_tile_rows + kNumThreads / 64 - 1) / (kNumThreads / 64)
                                    : (P->c_tiles + tiles_per_block - 1) / tiles_per_block;
        const bool strips = P->strip_desc && !whole_rows && tiles_per_wave == kGroupTiles;
        static_assert(kGroupTiles * (kNumThreads / 64) == 16, "a strip descriptor names the 16 tiles of one block");
        if (strips) blocks = P->strip_capacity;
        // Consecutive blocks share tiles of B, so they should share an L2 cache: on even products every XCD
        // takes one contiguous eighth of the blocks; where a few tile-rows are far heavier than the rest
        // (hubs of a power-law graph sit at the low indices) short runs of blocks are dealt to the XCDs in turn
        const bool skewed = P->max_row_pairs > 8 * (P->pairs / std::max<int64_t>(P->c_tile_rows, 1) + 1);
        const int xcd_chunk = skewed || strips ? 8 : (int)std::max<int64_t>((blocks + kXcds - 1) / kXcds, 1);
        blocks = xcd_chunked_grid(blocks, xcd_chunk);
        const NumericSizes z{(uint64_t)P->pairs, (uint64_t)A->tile_capacity, (uint64_t)B->tile_capacity,
                             (uint64_t)A->group_capacity, (uint64_t)B->group_capacity};
        const uint64_t limit = (1ull << 32) - 64;
        const bool narrow = z.pairs * 8 < limit && z.a_groups * 16 < limit && z.b_groups * 16 < limit &&
                            z.a_tiles * 8 < limit && z.b_tiles * 8 < limit && (uint64_t)P->c_tiles * T * 4 < limit &&
                            (uint64_t)P->c_nnz * 4 < limit && !ctx->force_wide;
        auto kernel = narrow ? (tiles_per_wave == 4 ? k_numeric<true, 4, true> : k_numeric<true, 8, true>)
                             : (tiles_per_wave == 4 ? k_numeric<false, 4, true> : k_numeric<false, 8, true>);
        // operands whose tiles hold a handful of entries: a step takes the halves that meet (see kHalves)
        const bool sparse_tiles = ctx->matrix_cores && tiles_per_wave == kGroupTiles && A->ntiles > 0 && B->ntiles > 0 &&
                                  A->nnz <= kSparseTileEntries * A->ntiles && B->nnz <= kSparseTileEntries * B->ntiles;
        if (sparse_tiles) kernel = narrow ? k_numeric<true, 4, true, false, true> : k_numeric<false, 4, true, false, true>;
        if (!ctx->matrix_cores) kernel = narrow ? k_numeric<true, 4, false> : k_numeric<false, 4, false>;
        if (whole_rows && P->max_row_c_tiles <= kRowTilesUnrolled)
            kernel = narrow ? k_numeric<true, kRowTilesUnrolled, true, true> : k_numeric<false, kRowTilesUnrolled, true, true>;
        else if (whole_rows)
            kernel = narrow ? k_numeric<true, kRowTiles, true, true> : k_numeric<false, kRowTiles, true, true>;
        hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kNumThreads), 0, s, P->c_tiles, P->c_nnz, z, P->c_rows,
                           (int32_t)P->c_tile_rows, P->c_tile_row_ptr, P->pair_off,
                           P->pair_ab, A->lhead, A->ldata, B->rhead, B->rdata,
                           P->c_tile_row, P->c_tile_col, P->c_row_mask, P->c_row_off, P->c_row_ptr, col, val,
                           last_of_call && !ctx->compact ? ctx->d_scalars : nullptr,
                           strips ? P->strip_desc : nullptr, strips ? P->strip_block_ptr + P->strip_entries : nullptr,
                           xcd_chunk);
        if (last_of_call && !ctx->compact && hipPeekAtLastError() == hipSuccess) ctx->scalars_clean = true;
        e = hipGetLastError();
    }
    phase_end(ctx, TSP_PHASE_NUMERIC, s);
    if (e != hipSuccess) {
        if (!last_of_call) ctx_free(ctx, row_ptr, s);
        ctx_free(ctx, col, s);
        ctx_free(ctx, val, s);
        return hip_fail(ctx, e);
    }
    if (last_of_call) P->c_row_ptr = nullptr;
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
