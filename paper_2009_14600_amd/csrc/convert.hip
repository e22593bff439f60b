// CSR -> tile ("bitmap") format, paper Section 2.1.2 with 16x16 tiles, in one pass over the matrix:
// per non-empty tile its tile column, its bitmap (16 row masks) and its elements.
//
// Where things go needs no counting pass and no prefix sum: tile-row I (16 CSR rows, whose entries
// are the stretch [e0, e1) of the CSR arrays) keeps its tiles in the tile slots e0, e0+1, ... and its
// element groups in the group slots e0, e0+1, ... of each form.  A tile-row has at most e1-e0 tiles
// and at most e1-e0 groups per form, so the stretches of different tile-rows cannot meet; the slots
// in between stay unused (the arrays are sized by nnz and never touched there).
//
// A group of G threads (one wave, or one block for long tile-rows) owns one tile-row and visits its
// entries in parallel:
//   1. every entry marks its tile column in an LDS bitmap that spans the tile-row's first to last
//      tile column; the popcount is the number of tiles and the rank of a bit is the tile's
//      position inside the tile-row, so the tiles come out sorted by column without a sort;
//   2. every entry ORs its bit into its tile's row masks (LDS); from the 16 row masks of a tile
//      follow the two group masks (which 8-element row pieces / column pieces are non-empty) and,
//      by a prefix sum inside the tile-row, the group offsets;
//   3. the groups are zeroed and every entry stores its value into its slot of the left-form and
//      of the right-form group of its tile: in LDS, from where the groups are written out whole, when
//      a block owns the tile-row and the groups of a window of tiles fit the staging area; in memory
//      otherwise.
// The element storage is laid out for the matrix-core operand registers (see tsp_tiles_view in
// tsp.h).  Tile-rows whose tile columns span more than the LDS bitmap take a second path: 16 lanes
// merge the 16 sorted rows, one tile per step (any span, one tile at a time).
// The same pass checks that the input is canonical (it reads every index anyway).
#include "common.hpp"

#include <hip/hip_fp16.h>

#include <algorithm>
#include <climits>
#include <new>

namespace tsp {

constexpr int kConvThreads = 256;
enum : int32_t { ROW_FAST = 0, ROW_MERGE = 1 };

template <int G> struct ConvCfg;
template <int G> constexpr int conv_block_threads() { return G == 64 ? 256 : G; }
template <> struct ConvCfg<64> {                  // one wave per tile-row, four tile-rows per block
    static constexpr int kWords = 512;            // bitmap words: tile columns may span 16384
    static constexpr int kWindow = 32;            // tiles handled per pass over the entries
    static constexpr int kStage = 0;              // element groups a window may assemble in LDS (0: none; this
                                                  // kernel lives on blocks per CU, and LDS decides how many)
};
template <> struct ConvCfg<128> {                 // one 128-thread block per tile-row
    static constexpr int kWords = 1024;
    static constexpr int kWindow = 64;
    static constexpr int kStage = 512;
};
template <> struct ConvCfg<256> {                 // one 256-thread block per tile-row
    static constexpr int kWords = 1024;           // span of 32768 tile columns
    static constexpr int kWindow = 128;
    static constexpr int kStage = 1024;
};

__device__ __forceinline__ uint16_t to_half_bits(uint16_t v) { return v; }
__device__ __forceinline__ uint16_t to_half_bits(float v) { return __half_as_ushort(__float2half_rn(v)); }

template <typename RP, typename VT>
struct ConvArgs {
    const RP *row_ptr;
    const int32_t *col;
    const VT *val;
    int64_t rows, cols, nnz, tile_rows, tile_capacity, group_capacity;
    int forms, validate;
    int32_t *row_class;                 // per tile-row: which path takes it
    int32_t *tile_row_ptr, *tile_row_end;  // per tile-row: first tile slot, one past the last
    // tile arrays
    int32_t *tile_col;
    uint16_t *row_mask;
    uint32_t *lmask, *rmask;
    uint2 *lhead, *rhead;
    uint4 *ldata, *rdata;
    int64_t *d_scalars;
};

template <int G>
__device__ __forceinline__ void group_sync() {
    if (G == 64) wave_sync(); else __syncthreads();
}

// Reductions over the G threads of a group.  red: LDS scratch of 8 words per group (G = 256 only).
template <int G>
__device__ __forceinline__ int group_max(int v, int *red) {
    v = wave_max(v);
    if (G > 64) {
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        v = red[0];
#pragma unroll
        for (int w = 1; w < G / 64; ++w) v = max(v, red[w]);
    }
    return v;
}
template <int G>
__device__ __forceinline__ uint32_t group_sum(uint32_t v, int *red) {
    v = wave_sum(v);
    if (G > 64) {
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = (int)v;
        __syncthreads();
        v = 0;
#pragma unroll
        for (int w = 0; w < G / 64; ++w) v += (uint32_t)red[w];
    }
    return v;
}
// In-place exclusive scan of arr[0..n) by the group; returns the total.
template <int G>
__device__ __forceinline__ uint32_t group_exclusive_scan(uint32_t *arr, int n, int *red) {
    const int gt = threadIdx.x % G, wave = (threadIdx.x % G) >> 6;
    uint32_t carry = 0;
    for (int base = 0; base < n; base += G) {
        const int i = base + gt;
        const uint32_t x = i < n ? arr[i] : 0;
        const uint32_t v = wave_inclusive_scan(x);
        uint32_t before = 0, all = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
        if (G > 64) {
            __syncthreads();
            if ((threadIdx.x & 63) == 63) red[wave] = (int)v;
            __syncthreads();
            all = 0;
#pragma unroll
            for (int w = 0; w < G / 64; ++w) {
                const uint32_t y = (uint32_t)red[w];
                if (w < wave) before += y;
                all += y;
            }
        }
        if (i < n) arr[i] = carry + before + v - x;
        carry += all;
    }
    group_sync<G>();
    return carry;
}

// ------------------------------------------------------------------------------------------------
// Fast path: LDS bitmap over the tile-row's span of tile columns.
// ------------------------------------------------------------------------------------------------
// kConvCache: entries per thread kept in registers between the passes (tile-rows with more entries
// than G*kConvCache read the CSR arrays again in every pass)
template <int G, int kConvCache, typename RP, typename VT>
__device__ __forceinline__ void convert_rows(const ConvArgs<RP, VT> &a) {
    constexpr int kWords = ConvCfg<G>::kWords, kWindow = ConvCfg<G>::kWindow, kGroups = conv_block_threads<G>() / G;
    constexpr int kStage = ConvCfg<G>::kStage;
    static_assert(kStage == 0 || kGroups == 1, "the staging area belongs to one tile-row");
    __shared__ uint4 s_stage[kStage > 0 ? kStage : 1];
    __shared__ int s_rp_all[kGroups][20];
    __shared__ uint32_t s_bm_all[kGroups][kWords], s_pre_all[kGroups][kWords];
    __shared__ uint32_t s_mask_all[kGroups][kWindow * 8];
    __shared__ uint32_t s_lm_all[kGroups][kWindow], s_rm_all[kGroups][kWindow];
    __shared__ uint32_t s_lo_all[kGroups][kWindow], s_ro_all[kGroups][kWindow];
    __shared__ int s_red_all[kGroups][8];
    const int gi = threadIdx.x / G, gt = threadIdx.x % G;
    int *s_rp = s_rp_all[gi];
    uint32_t *s_bm = s_bm_all[gi], *s_pre = s_pre_all[gi], *s_mask = s_mask_all[gi];
    uint32_t *s_lm = s_lm_all[gi], *s_rm = s_rm_all[gi], *s_lo = s_lo_all[gi], *s_ro = s_ro_all[gi];
    int *s_red = s_red_all[gi];
    const int64_t I = (int64_t)blockIdx.x * kGroups + gi;
    if (I >= a.tile_rows) return;                 // whole group (G > 64: whole block)
    bool bad = false;

    // The 17 row pointers of the tile-row, one per lane, clamped into [0, nnz] and made non-decreasing
    // (a running maximum) so that whatever they hold the entry ranges are disjoint stretches inside the
    // arrays; nnz < 2^31, so the clamped values fit 32 bits.
    if (gt < 64) {
        const int64_t row = min(I * T + min(gt, 16), a.rows);
        const int64_t raw = (int64_t)a.row_ptr[row];
        int v = (int)min(max(raw, (int64_t)0), a.nnz);
        // inclusive running maximum over the lanes
        v = max(v, TSP_DPP(v, v, 0x111, 0xf, false));
        v = max(v, TSP_DPP(v, v, 0x112, 0xf, false));
        v = max(v, TSP_DPP(v, v, 0x114, 0xf, false));
        v = max(v, TSP_DPP(v, v, 0x118, 0xf, false));
        v = max(v, TSP_DPP(v, v, 0x142, 0xa, false));
        if (gt <= 16) {
            s_rp[gt] = v;
            bad = raw != (int64_t)v || (row == 0 && raw != 0) || (row == a.rows && raw != a.nnz);
        }
    }
    group_sync<G>();
    const int64_t e0 = s_rp[0], e1 = s_rp[16];
    // the tile-row's slots: tiles and groups both start at slot e0 (see the top of the file)
    const int64_t t0 = e0;
    uint32_t lrun = (uint32_t)e0, rrun = (uint32_t)e0;
    auto finish = [&](int ntiles, int row_class) {
        const bool any_bad = group_max<G>(bad ? 1 : 0, s_red) != 0;
        if (gt == 0) {
            a.tile_row_ptr[I] = (int32_t)t0;
            a.tile_row_end[I] = (int32_t)(t0 + ntiles);
            a.row_class[I] = row_class;
            if (any_bad && a.validate) a.d_scalars[S_INVALID] = 1;
        }
    };
    if (e0 == e1) {
        finish(0, ROW_FAST);
        return;
    }
    auto row_of = [&](int64_t e) {
        const int x = (int)e;
        int r = x >= s_rp[8] ? 8 : 0;
        r += x >= s_rp[r + 4] ? 4 : 0;
        r += x >= s_rp[r + 2] ? 2 : 0;
        r += x >= s_rp[r + 1] ? 1 : 0;
        return r;
    };

    // Tile-rows of up to G*kConvCache entries keep their column indices and values in registers: all
    // loads are requested at once and the later passes do not touch the CSR arrays again.
    const bool cached = e1 - e0 <= (int64_t)G * kConvCache;
    int c_reg[kConvCache], p_reg[kConvCache];
    VT v_reg[kConvCache];
    int jmin = INT_MAX, jmax = -1;
    if (cached) {
#pragma unroll
        for (int k = 0; k < kConvCache; ++k) {
            const int64_t e = e0 + gt + (int64_t)k * G;
            c_reg[k] = e < e1 ? a.col[e] : 0;
            v_reg[k] = e < e1 ? a.val[e] : VT(0);
            p_reg[k] = a.validate && e < e1 && e > e0 ? a.col[e - 1] : -1;   // left neighbour, for the order check
        }
#pragma unroll
        for (int k = 0; k < kConvCache; ++k) {
            const int64_t e = e0 + gt + (int64_t)k * G;
            if (e < e1) {
                jmin = min(jmin, c_reg[k] >> 4);
                jmax = max(jmax, c_reg[k] >> 4);
            }
        }
    } else if (gt < 16) {                         // first and last entry of every non-empty row
        const int64_t p = s_rp[gt], e = s_rp[gt + 1];
        if (p < e) {
            jmin = a.col[p] >> 4;
            jmax = a.col[e - 1] >> 4;
        }
    }
    jmin = -group_max<G>(-jmin, s_red);
    jmax = group_max<G>(jmax, s_red);
    const int64_t span = (int64_t)jmax - jmin + 1;
    const int words = (int)((span + 31) >> 5);
    if (jmin < 0 || span <= 0 || words > kWords) {
        // the merge path takes this tile-row (and validates it); a span that cannot occur in a matrix
        // of this width means the indices are out of range
        bad |= jmin < 0 || jmax >= (a.cols + T - 1) / T;
        const bool any_bad = group_max<G>(bad ? 1 : 0, s_red) != 0;
        if (gt == 0) {
            // an empty range until the merge kernel writes the real one: where that kernel does not run
            // (a matrix too narrow for an over-wide span, so only bad indices lead here) the later kernels
            // must still find bounds they can walk
            a.tile_row_ptr[I] = (int32_t)t0;
            a.tile_row_end[I] = (int32_t)t0;
            a.row_class[I] = ROW_MERGE;
            if (any_bad && a.validate) a.d_scalars[S_INVALID] = 1;
        }
        return;
    }
    // f(e, column, value, column of the entry before e) for every entry this thread owns
    auto for_each_entry = [&](auto f) {
        if (cached) {
#pragma unroll
            for (int k = 0; k < kConvCache; ++k) {
                const int64_t e = e0 + gt + (int64_t)k * G;
                if (e < e1) f(e, c_reg[k], v_reg[k], p_reg[k]);
            }
        } else {
            for (int64_t e = e0 + gt; e < e1; e += G)
                f(e, a.col[e], a.val[e], a.validate && e > e0 ? a.col[e - 1] : -1);
        }
    };

    // 1. tile columns -> bitmap
    for (int w = gt; w < words; w += G) s_bm[w] = 0;
    group_sync<G>();
    for_each_entry([&](int64_t e, int c, VT, int before) {
        const uint32_t j = (uint32_t)((c >> 4) - jmin);
        if (j < (uint32_t)span) atomicOr(&s_bm[j >> 5], 1u << (j & 31));
        if (a.validate) {
            bad |= c < 0 || c >= a.cols || j >= (uint32_t)span;
            if (e > s_rp[row_of(e)]) bad |= c <= before;
        }
    });
    group_sync<G>();
    for (int w = gt; w < words; w += G) s_pre[w] = __popc(s_bm[w]);
    group_sync<G>();
    const int ntiles = (int)group_exclusive_scan<G>(s_pre, words, s_red);
    auto tile_rank = [&](int c) -> int {          // position of the entry's tile inside the tile-row, or -1
        const uint32_t j = (uint32_t)((c >> 4) - jmin);
        if (j >= (uint32_t)span) return -1;
        return (int)s_pre[j >> 5] + __popc(s_bm[j >> 5] & ((1u << (j & 31)) - 1u));
    };

    uint16_t *const l16 = reinterpret_cast<uint16_t *>(a.ldata), *const r16 = reinterpret_cast<uint16_t *>(a.rdata);
    // tile columns, ascending
    for (int w = gt; w < words; w += G) {
        uint32_t bits = s_bm[w];
        int64_t t = t0 + s_pre[w];
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            if (t < a.tile_capacity) a.tile_col[t] = jmin + w * 32 + b;
            ++t;
        }
    }
    // Entries held in registers: from here on only the tile, the row and the column inside the tile of an
    // entry are needed, so the column register takes those three (tile << 8 | row << 4 | column % 16) and
    // the later passes look nothing up again.  (A tile-row in registers has at most G*kConvCache <= 2^23 tiles.)
    // Not in the one-wave kernels: there the lookups are cheaper than the registers the packing costs.
    constexpr bool kPlaced = G > 64;
    if (kPlaced && cached) {
#pragma unroll
        for (int k = 0; k < kConvCache; ++k) {
            const int64_t e = e0 + gt + (int64_t)k * G;
            if (e < e1) c_reg[k] = (tile_rank(c_reg[k]) << 8) | (row_of(e) << 4) | (c_reg[k] & 15);
        }
    }
    // f(tile of the entry, row inside the tile, column inside the tile, value) for every entry of this thread
    auto for_each_placed_entry = [&](auto f) {
        if (cached) {
#pragma unroll
            for (int k = 0; k < kConvCache; ++k) {
                const int64_t e = e0 + gt + (int64_t)k * G;
                if (e >= e1) continue;
                if (kPlaced) f(c_reg[k] >> 8, (c_reg[k] >> 4) & 15, c_reg[k] & 15, v_reg[k]);
                else f(tile_rank(c_reg[k]), row_of(e), c_reg[k] & 15, v_reg[k]);
            }
        } else {
            for (int64_t e = e0 + gt; e < e1; e += G) {
                const int c = a.col[e];
                f(tile_rank(c), row_of(e), c & 15, a.val[e]);
            }
        }
    };
    // A tile-row with more tiles than a window holds, and too many entries for the registers, would
    // read all its entries again for every window.  Its CSR rows are sorted by column, so the entries of
    // a window of tiles are one stretch of every row: each window walks the 16 rows from where the
    // previous one ended (s_cur), and the tile-row is read once per pass.
    const bool long_row = !cached && ntiles > kWindow;              // uniform over the group
    // (where each row's walk stands: lane r of every wave keeps row r's place)
    int cur = long_row ? s_rp[min((int)(threadIdx.x & 63), T)] : 0;
    // f(r, c, value or 0, tile inside the window) for the window's entries; `advance`: the last pass of the window
    auto for_each_window_entry = [&](int win0, int nw, bool with_values, bool advance, auto f) {
        for (int r = 0; r < T; ++r) {
            const int end = s_rp[r + 1];
            int stop = end;                                           // first entry of this lane's stride past the window
            for (int e = __builtin_amdgcn_readlane(cur, r) + gt; e < end; e += G) {
                const int c = a.col[e];
                const int t = tile_rank(c) - win0;
                if (t >= nw) {
                    stop = e;
                    break;
                }
                if (t >= 0) f(r, c, with_values ? a.val[e] : VT(0), t);
            }
            if (advance) {
                stop = -group_max<G>(-stop, s_red);
                if ((int)(threadIdx.x & 63) == r) cur = stop;
            }
        }
    };
    if (__builtin_expect(long_row, 0)) {          // (its own copy of the loop: the common path below stays as it is)
        for (int win0 = 0; win0 < ntiles; win0 += kWindow) {
            const int nw = min(kWindow, ntiles - win0);
            // 2. row masks of the tiles of this window
            for (int k = gt; k < nw * 8; k += G) s_mask[k] = 0;
            group_sync<G>();
            for_each_window_entry(win0, nw, false, false, [&](int r, int c, VT, int t) {
                atomicOr(&s_mask[t * 8 + (r >> 1)], 1u << ((r & 1) * 16 + (c & 15)));
            });
            group_sync<G>();
            for (int t = gt; t < nw; t += G) {
                uint32_t lm = 0, rm = 0;
    #pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t m2 = s_mask[t * 8 + k];              // rows 2k (low half) and 2k+1 (high half)
                    lm |= ((m2 & 0x000000FFu) ? 1u << (2 * k) : 0u) | ((m2 & 0x0000FF00u) ? 1u << (16 + 2 * k) : 0u) |
                          ((m2 & 0x00FF0000u) ? 1u << (2 * k + 1) : 0u) | ((m2 & 0xFF000000u) ? 1u << (17 + 2 * k) : 0u);
                    const uint32_t cols = (m2 | (m2 >> 16)) & 0xFFFFu;  // columns present in rows 2k, 2k+1
                    rm |= k < 4 ? cols : cols << 16;
                }
                s_lm[t] = lm;
                s_rm[t] = rm;
                s_lo[t] = __popc(lm);
                s_ro[t] = __popc(rm);
            }
            group_sync<G>();
            const uint32_t ltot = group_exclusive_scan<G>(s_lo, nw, s_red);
            const uint32_t rtot = group_exclusive_scan<G>(s_ro, nw, s_red);
            // the window's groups are zeroed; the entries drop their values into their slots below
            const uint4 zero = make_uint4(0, 0, 0, 0);
            if (a.forms & TSP_FORM_LEFT)
                for (int64_t g = (int64_t)lrun + gt, end = min((int64_t)lrun + ltot, a.group_capacity); g < end; g += G)
                    a.ldata[g] = zero;
            if (a.forms & TSP_FORM_RIGHT)
                for (int64_t g = (int64_t)rrun + gt, end = min((int64_t)rrun + rtot, a.group_capacity); g < end; g += G)
                    a.rdata[g] = zero;
            // tile headers and bitmaps
            for (int t = gt; t < nw; t += G) {
                const int64_t tg = t0 + win0 + t;
                if (tg < a.tile_capacity) {
                    uint4 *dst = reinterpret_cast<uint4 *>(a.row_mask + tg * T);
                    dst[0] = make_uint4(s_mask[t * 8 + 0], s_mask[t * 8 + 1], s_mask[t * 8 + 2], s_mask[t * 8 + 3]);
                    dst[1] = make_uint4(s_mask[t * 8 + 4], s_mask[t * 8 + 5], s_mask[t * 8 + 6], s_mask[t * 8 + 7]);
                    a.lmask[tg] = s_lm[t];
                    a.rmask[tg] = s_rm[t];
                    if (a.forms & TSP_FORM_LEFT) a.lhead[tg] = make_uint2(s_lm[t], lrun + s_lo[t]);
                    if (a.forms & TSP_FORM_RIGHT) a.rhead[tg] = make_uint2(s_rm[t], rrun + s_ro[t]);
                }
            }
            // the zeros must be in L2 before any value is stored over them: every wave waits for its own
            // stores, then the group meets
            __builtin_amdgcn_s_waitcnt(0x0F70);
            group_sync<G>();
            // 3. values
            for_each_window_entry(win0, nw, true, true, [&](int r, int c, VT value, int t) {
                const int cc = c & 15;
                const uint16_t v = to_half_bits(value);
                if (a.forms & TSP_FORM_LEFT) {
                    const int g = (cc >> 3) * 16 + r;
                    const int64_t idx = (int64_t)lrun + s_lo[t] + __popc(s_lm[t] & ((1u << g) - 1u));
                    if (idx < a.group_capacity) l16[idx * 8 + (cc & 7)] = v;
                }
                if (a.forms & TSP_FORM_RIGHT) {
                    const int g = (r >> 3) * 16 + cc;
                    const int64_t idx = (int64_t)rrun + s_ro[t] + __popc(s_rm[t] & ((1u << g) - 1u));
                    if (idx < a.group_capacity) r16[idx * 8 + (r & 7)] = v;
                }
            });
            lrun += ltot;
            rrun += rtot;
            group_sync<G>();
        }
        finish(ntiles, ROW_FAST);
        return;
    }
    for (int win0 = 0; win0 < ntiles; win0 += kWindow) {
        const int nw = min(kWindow, ntiles - win0);
        // 2. row masks of the tiles of this window
        for (int k = gt; k < nw * 8; k += G) s_mask[k] = 0;
        group_sync<G>();
        for_each_placed_entry([&](int tile, int r, int cc, VT) {
            const int t = tile - win0;
            if (t >= 0 && t < nw) atomicOr(&s_mask[t * 8 + (r >> 1)], 1u << ((r & 1) * 16 + cc));
        });
        group_sync<G>();
        for (int t = gt; t < nw; t += G) {
            uint32_t lm = 0, rm = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t m2 = s_mask[t * 8 + k];              // rows 2k (low half) and 2k+1 (high half)
                lm |= ((m2 & 0x000000FFu) ? 1u << (2 * k) : 0u) | ((m2 & 0x0000FF00u) ? 1u << (16 + 2 * k) : 0u) |
                      ((m2 & 0x00FF0000u) ? 1u << (2 * k + 1) : 0u) | ((m2 & 0xFF000000u) ? 1u << (17 + 2 * k) : 0u);
                const uint32_t cols = (m2 | (m2 >> 16)) & 0xFFFFu;  // columns present in rows 2k, 2k+1
                rm |= k < 4 ? cols : cols << 16;
            }
            s_lm[t] = lm;
            s_rm[t] = rm;
            s_lo[t] = __popc(lm);
            s_ro[t] = __popc(rm);
        }
        group_sync<G>();
        const uint32_t ltot = group_exclusive_scan<G>(s_lo, nw, s_red);
        const uint32_t rtot = group_exclusive_scan<G>(s_ro, nw, s_red);
        // Where the window's groups fit the staging area they are put together in LDS and written out whole
        // (no wait for zeros to reach L2, no two-byte stores to memory).
        const uint32_t lstage = (a.forms & TSP_FORM_LEFT) ? ltot : 0u, rstage = (a.forms & TSP_FORM_RIGHT) ? rtot : 0u;
        const bool staged = kStage > 0 && lstage + rstage <= (uint32_t)kStage;      // uniform over the group
        // otherwise the groups are zeroed in memory and the entries drop their values into their slots below
        const uint4 zero = make_uint4(0, 0, 0, 0);
        if (staged) {
            for (uint32_t g = gt; g < lstage + rstage; g += G) s_stage[g] = zero;
        } else {
        if (a.forms & TSP_FORM_LEFT)
            for (int64_t g = (int64_t)lrun + gt, end = min((int64_t)lrun + ltot, a.group_capacity); g < end; g += G)
                a.ldata[g] = zero;
        if (a.forms & TSP_FORM_RIGHT)
            for (int64_t g = (int64_t)rrun + gt, end = min((int64_t)rrun + rtot, a.group_capacity); g < end; g += G)
                a.rdata[g] = zero;
        }
        // tile headers and bitmaps
        for (int t = gt; t < nw; t += G) {
            const int64_t tg = t0 + win0 + t;
            if (tg < a.tile_capacity) {
                uint4 *dst = reinterpret_cast<uint4 *>(a.row_mask + tg * T);
                dst[0] = make_uint4(s_mask[t * 8 + 0], s_mask[t * 8 + 1], s_mask[t * 8 + 2], s_mask[t * 8 + 3]);
                dst[1] = make_uint4(s_mask[t * 8 + 4], s_mask[t * 8 + 5], s_mask[t * 8 + 6], s_mask[t * 8 + 7]);
                a.lmask[tg] = s_lm[t];
                a.rmask[tg] = s_rm[t];
                if (a.forms & TSP_FORM_LEFT) a.lhead[tg] = make_uint2(s_lm[t], lrun + s_lo[t]);
                if (a.forms & TSP_FORM_RIGHT) a.rhead[tg] = make_uint2(s_rm[t], rrun + s_ro[t]);
            }
        }
        if (staged) {
            group_sync<G>();
            uint16_t *const stage16 = reinterpret_cast<uint16_t *>(s_stage);
            for_each_placed_entry([&](int tile, int r, int cc, VT value) {
                const int t = tile - win0;
                if (t >= 0 && t < nw) {
                    const uint16_t v = to_half_bits(value);
                    if (a.forms & TSP_FORM_LEFT) {
                        const int g = (cc >> 3) * 16 + r;
                        stage16[(s_lo[t] + __popc(s_lm[t] & ((1u << g) - 1u))) * 8 + (cc & 7)] = v;
                    }
                    if (a.forms & TSP_FORM_RIGHT) {
                        const int g = (r >> 3) * 16 + cc;
                        stage16[(lstage + s_ro[t] + __popc(s_rm[t] & ((1u << g) - 1u))) * 8 + (r & 7)] = v;
                    }
                }
            });
            group_sync<G>();
            for (uint32_t g = gt; g < lstage; g += G)
                if ((int64_t)lrun + g < a.group_capacity) a.ldata[(int64_t)lrun + g] = s_stage[g];
            for (uint32_t g = gt; g < rstage; g += G)
                if ((int64_t)rrun + g < a.group_capacity) a.rdata[(int64_t)rrun + g] = s_stage[lstage + g];
            lrun += ltot;
            rrun += rtot;
            group_sync<G>();
            continue;
        }
        // the zeros must be in L2 before any value is stored over them: every wave waits for its own
        // stores, then the group meets
        __builtin_amdgcn_s_waitcnt(0x0F70);
        group_sync<G>();
        // 3. values
        for_each_placed_entry([&](int tile, int r, int cc, VT value) {
            const int t = tile - win0;
            if (t >= 0 && t < nw) {
                const uint16_t v = to_half_bits(value);
                if (a.forms & TSP_FORM_LEFT) {
                    const int g = (cc >> 3) * 16 + r;
                    const int64_t idx = (int64_t)lrun + s_lo[t] + __popc(s_lm[t] & ((1u << g) - 1u));
                    if (idx < a.group_capacity) l16[idx * 8 + (cc & 7)] = v;
                }
                if (a.forms & TSP_FORM_RIGHT) {
                    const int g = (r >> 3) * 16 + cc;
                    const int64_t idx = (int64_t)rrun + s_ro[t] + __popc(s_rm[t] & ((1u << g) - 1u));
                    if (idx < a.group_capacity) r16[idx * 8 + (r & 7)] = v;
                }
            }
        });
        lrun += ltot;
        rrun += rtot;
        group_sync<G>();
    }
    finish(ntiles, ROW_FAST);
}

template <int G, int kConvCache, typename RP, typename VT>
__global__ __launch_bounds__(conv_block_threads<G>()) void k_convert_rows(const ConvArgs<RP, VT> a) {
    convert_rows<G, kConvCache, RP, VT>(a);
}
// The same for short tile-rows (few entries per thread in registers): asking for seven waves per SIMD
// (as many as the LDS of seven blocks per CU allows) makes the compiler fit 72 registers with three
// spilled words, and this kernel lives on waves in flight.
template <int G, int kConvCache, typename RP, typename VT>
__global__ __launch_bounds__(conv_block_threads<G>()) __attribute__((amdgpu_waves_per_eu(7, 8))) void k_convert_rows_light(
    const ConvArgs<RP, VT> a) {
    convert_rows<G, kConvCache, RP, VT>(a);
}

// ... and for six entries per thread: four waves per SIMD cost the compiler seven registers.
template <int G, int kConvCache, typename RP, typename VT>
__global__ __launch_bounds__(conv_block_threads<G>()) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_convert_rows_mid(
    const ConvArgs<RP, VT> a) {
    convert_rows<G, kConvCache, RP, VT>(a);
}

// ------------------------------------------------------------------------------------------------
// Merge path for tile-rows whose span does not fit the bitmap: 16 lanes own one tile-row, one lane
// per CSR row.  The columns of a CSR row ascend, so do its tile columns, and the distinct tile
// columns of the tile-row come out of a 16-way merge: every step takes the smallest pending tile
// column over the 16 lanes; the lanes whose row has entries in that tile consume them.
// ------------------------------------------------------------------------------------------------
constexpr int kMergeGroupsPerBlock = kConvThreads / 16;

template <typename RP, typename VT>
__global__ __launch_bounds__(kConvThreads) void k_convert_merge(const ConvArgs<RP, VT> a) {
    __shared__ __align__(16) uint16_t dense_all[kMergeGroupsPerBlock][T * T];
    const int g = threadIdx.x >> 4, r = threadIdx.x & 15;
    uint16_t *dense = dense_all[g];
    const int64_t I = (int64_t)blockIdx.x * kMergeGroupsPerBlock + g;
    const bool mine = I < a.tile_rows && a.row_class[I] == ROW_MERGE;
    bool bad = false;
    int64_t p = 0, e = 0;
    if (mine && I * T + r < a.rows) {
        const int64_t row = I * T + r;
        p = (int64_t)a.row_ptr[row];
        e = (int64_t)a.row_ptr[row + 1];
        bad |= p < 0 || e > a.nnz || p > e || (row == 0 && p != 0) || (row == a.rows - 1 && e != a.nnz);
        p = min(max(p, (int64_t)0), a.nnz);      // never read outside the arrays, whatever row_ptr holds
        e = min(max(e, p), a.nnz);
    }
    // the tile-row's slots start at the first entry of its first row (lane 0 of the group)
    const int64_t first = __shfl(p, 0, 16);
    int64_t t = first;
    uint32_t lrun = (uint32_t)first, rrun = (uint32_t)first;
    int ntiles = 0;
    int cur = p < e ? (a.col[p] >> 4) : INT_MAX;
    int prev_col = -1;
    const uint32_t below_lo = (1u << r) - 1u, below_hi = (1u << (16 + r)) - 1u;
    for (;;) {
        const int m = group16_min(cur);
        if (__all(m == INT_MAX)) break;
        const bool active = m != INT_MAX;
        uint4 *myrow = reinterpret_cast<uint4 *>(dense + r * T);
        myrow[0] = make_uint4(0, 0, 0, 0);        // dense image of the tile in LDS; every lane fills its own row
        myrow[1] = make_uint4(0, 0, 0, 0);
        uint32_t mask = 0;
        if (active && cur == m) {
            do {
                const int c = a.col[p];
                bad |= c <= prev_col || c >= a.cols;
                prev_col = c;
                mask |= 1u << (c & 15);
                dense[r * T + (c & 15)] = to_half_bits(a.val[p]);
                ++p;
            } while (p < e && (a.col[p] >> 4) == m);
            cur = p < e ? (a.col[p] >> 4) : INT_MAX;
        }
        wave_sync();
        // group masks: left form g = h*16 + row, right form g = h*16 + column
        const uint32_t lm = group16_ballot((mask & 0xFFu) != 0) | (group16_ballot((mask >> 8) != 0) << 16);
        const uint32_t rm = group16_or(r < 8 ? mask : (mask << 16));
        if (active) {
            ++ntiles;
            if (t < a.tile_capacity) {
                if (a.forms & TSP_FORM_LEFT) {
                    const int64_t g0 = (int64_t)lrun + __popc(lm & below_lo), g1 = (int64_t)lrun + __popc(lm & below_hi);
                    if ((mask & 0xFFu) && g0 < a.group_capacity) a.ldata[g0] = myrow[0];
                    if ((mask >> 8) && g1 < a.group_capacity) a.ldata[g1] = myrow[1];
                }
                if (a.forms & TSP_FORM_RIGHT) {
                    uint32_t w[8];                 // lane r gathers column r of the tile
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        w[k] = (uint32_t)dense[(2 * k) * T + r] | ((uint32_t)dense[(2 * k + 1) * T + r] << 16);
                    const int64_t g0 = (int64_t)rrun + __popc(rm & below_lo), g1 = (int64_t)rrun + __popc(rm & below_hi);
                    if (((rm >> r) & 1u) && g0 < a.group_capacity) a.rdata[g0] = make_uint4(w[0], w[1], w[2], w[3]);
                    if (((rm >> (16 + r)) & 1u) && g1 < a.group_capacity) a.rdata[g1] = make_uint4(w[4], w[5], w[6], w[7]);
                }
                a.row_mask[t * T + r] = (uint16_t)mask;
                if (r == 0) {
                    a.tile_col[t] = m;
                    a.lmask[t] = lm;
                    a.rmask[t] = rm;
                    if (a.forms & TSP_FORM_LEFT) a.lhead[t] = make_uint2(lm, lrun);
                    if (a.forms & TSP_FORM_RIGHT) a.rhead[t] = make_uint2(rm, rrun);
                }
            }
            lrun += __popc(lm);
            rrun += __popc(rm);
            ++t;
        }
        wave_sync();   // column reads above finish before the rows are cleared again
    }
    const bool any_bad = group16_or(bad ? 1u : 0u) != 0;
    if (mine && r == 0) {
        a.tile_row_ptr[I] = (int32_t)first;
        a.tile_row_end[I] = (int32_t)(first + ntiles);
        if (any_bad && a.validate) a.d_scalars[S_INVALID] = 1;
    }
}

template <typename RP, typename VT>
static int launch_convert(tsp_context *ctx, const tsp_csr *A, tsp_tiles_s *t, int32_t *row_class, hipStream_t s) {
    const int64_t ntr = t->tile_rows;
    ConvArgs<RP, VT> a{};
    a.row_ptr = static_cast<const RP *>(A->row_ptr);
    a.col = A->col_idx;
    a.val = static_cast<const VT *>(A->val);
    a.rows = A->rows;
    a.cols = A->cols;
    a.nnz = A->nnz;
    a.tile_rows = ntr;
    a.tile_capacity = t->tile_capacity;
    a.group_capacity = t->group_capacity;
    a.forms = t->forms;
    a.validate = ctx->validate;
    a.row_class = row_class;
    a.tile_row_ptr = t->tile_row_ptr;
    a.tile_row_end = t->tile_row_end;
    a.tile_col = t->tile_col;
    a.row_mask = t->row_mask;
    a.lmask = t->lmask;
    a.rmask = t->rmask;
    a.lhead = t->lhead;
    a.rhead = t->rhead;
    a.ldata = t->ldata;
    a.rdata = t->rdata;
    a.d_scalars = ctx->d_scalars;
    // threads per tile-row from the mean number of entries per tile-row (the kernel is bound by
    // dependent steps, so small groups, many in flight, win as long as the entries fit their registers);
    // the merge path only when a tile-row could span more tile columns than the chosen bitmap holds
    // Registers per thread for the entries: the mean tile-row plus 15 %, so that most tile-rows stay in
    // registers without the kernel paying (in occupancy) for registers it does not use.
    const int64_t per_row = ntr > 0 ? A->nnz / ntr : 0, need = per_row + (3 * per_row + 19) / 20;
    const int G = need <= 64 * 8 ? 64 : need <= 128 * 8 ? 128 : 256;
    const int64_t want = (need + G - 1) / G;
    const int cache = G == 64 ? (want <= 2 ? 2 : want <= 4 ? 4 : 8) : (want <= 6 ? 6 : 8);
    const int64_t bitmap_span =
        32ll * (G == 64 ? ConvCfg<64>::kWords : G == 128 ? ConvCfg<128>::kWords : ConvCfg<256>::kWords);
    // (tile-rows of a narrow matrix cannot exceed the bitmap, and then the merge kernel is not launched)
    const bool may_merge = t->tile_cols > bitmap_span;
    const unsigned grid_fast = (unsigned)(G == 64 ? (ntr + 3) / 4 : ntr);
    const unsigned grid_merge = (unsigned)((ntr + kMergeGroupsPerBlock - 1) / kMergeGroupsPerBlock);
    if (ntr > 0) {
        KernelTimer kt(ctx, TSP_KERNEL_CONVERT, s);
#define TSP_LAUNCH_ROWS(g, c, threads) \
    hipLaunchKernelGGL((k_convert_rows<g, c, RP, VT>), dim3(grid_fast), dim3(threads), 0, s, a)
        if (G == 64 && cache == 2)
            hipLaunchKernelGGL((k_convert_rows_light<64, 2, RP, VT>), dim3(grid_fast), dim3(256), 0, s, a);
        else if (G == 64 && cache == 4)
            hipLaunchKernelGGL((k_convert_rows_light<64, 4, RP, VT>), dim3(grid_fast), dim3(256), 0, s, a);
        else if (G == 64) TSP_LAUNCH_ROWS(64, 8, 256);
        else if (G == 128 && cache == 6)
            hipLaunchKernelGGL((k_convert_rows_mid<128, 6, RP, VT>), dim3(grid_fast), dim3(128), 0, s, a);
        else if (G == 128) TSP_LAUNCH_ROWS(128, 8, 128);
        else if (cache == 6)
            hipLaunchKernelGGL((k_convert_rows_mid<256, 6, RP, VT>), dim3(grid_fast), dim3(256), 0, s, a);
        else TSP_LAUNCH_ROWS(256, 8, 256);
#undef TSP_LAUNCH_ROWS
        if (may_merge)
            hipLaunchKernelGGL((k_convert_merge<RP, VT>), dim3(grid_merge), dim3(kConvThreads), 0, s, a);
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
    ctx_free(ctx, t->tile_row_end, s);
    ctx_free(ctx, t->tile_col, s);
    ctx_free(ctx, t->row_mask, s);
    ctx_free(ctx, t->lmask, s);
    ctx_free(ctx, t->rmask, s);
    ctx_free(ctx, t->lhead, s);
    ctx_free(ctx, t->rhead, s);
    ctx_free(ctx, t->ldata, s);
    ctx_free(ctx, t->rdata, s);
    delete t;
}

// Enqueues the whole conversion without synchronising: the tile arrays have one slot per stored entry
// (see the top of the file); the number of tiles is the sum of tile_row_end - tile_row_ptr, which the
// symbolic phase (or tsp_convert) adds up.
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
    t->tile_capacity = A->nnz;
    t->group_capacity = A->nnz;
    const size_t cap = (size_t)t->tile_capacity;
    t->tile_row_ptr = ctx_alloc_n<int32_t>(ctx, (size_t)t->tile_rows + 1, s);
    t->tile_row_end = ctx_alloc_n<int32_t>(ctx, (size_t)t->tile_rows + 1, s);
    t->tile_col = ctx_alloc_n<int32_t>(ctx, cap, s);
    t->row_mask = ctx_alloc_n<uint16_t>(ctx, cap * T, s);
    t->lmask = ctx_alloc_n<uint32_t>(ctx, cap, s);
    t->rmask = ctx_alloc_n<uint32_t>(ctx, cap, s);
    bool ok = t->tile_row_ptr && t->tile_row_end && t->tile_col && t->row_mask && t->lmask && t->rmask;
    if (forms & TSP_FORM_LEFT) {
        t->lhead = ctx_alloc_n<uint2>(ctx, cap, s);
        t->ldata = ctx_alloc_n<uint4>(ctx, (size_t)t->group_capacity, s);
        ok = ok && t->lhead && t->ldata;
    }
    if (forms & TSP_FORM_RIGHT) {
        t->rhead = ctx_alloc_n<uint2>(ctx, cap, s);
        t->rdata = ctx_alloc_n<uint4>(ctx, (size_t)t->group_capacity, s);
        ok = ok && t->rhead && t->rdata;
    }
    int32_t *scratch = ctx_alloc_n<int32_t>(ctx, (size_t)t->tile_rows + 1, s);   // path of every tile-row
    ok = ok && scratch;
    rc = ok ? TSP_OK : TSP_ERR_ALLOC_FAILED;
    if (!rc) {
        const bool i32 = A->row_ptr_type == TSP_I32, f16 = A->val_type == TSP_F16;
        rc = i32 ? (f16 ? launch_convert<int32_t, uint16_t>(ctx, A, t, scratch, s)
                        : launch_convert<int32_t, float>(ctx, A, t, scratch, s))
                 : (f16 ? launch_convert<int64_t, uint16_t>(ctx, A, t, scratch, s)
                        : launch_convert<int64_t, float>(ctx, A, t, scratch, s));
    }
    ctx_free(ctx, scratch, s);
    if (rc) {
        tiles_release(ctx, t, s);
        return rc;
    }
    *out = t;
    return TSP_OK;
}

// Number of tiles of a tile matrix (tsp_convert only; tsp_spgemm lets the symbolic phase add them up).
__global__ __launch_bounds__(256) void k_tiles_total(int64_t tile_rows, const int32_t *__restrict__ trp,
                                                    const int32_t *__restrict__ tend, int64_t *d_scalars, int slot) {
    __shared__ uint32_t part[4];
    uint32_t n = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < tile_rows; i += (int64_t)gridDim.x * 256)
        n += (uint32_t)(tend[i] - trp[i]);
    n = wave_sum(n);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long all = (unsigned long long)part[0] + part[1] + part[2] + part[3];
        if (all) atomicAdd(reinterpret_cast<unsigned long long *>(d_scalars + slot), all);
    }
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
    ctx->scalars_clean = false;
    phase_begin(ctx, TSP_PHASE_CONVERT, s);
    tsp_tiles_s *t = nullptr;
    int rc = convert_enqueue(ctx, A, forms, S_TILES_A, &t, s);
    phase_end(ctx, TSP_PHASE_CONVERT, s);
    if (rc) return rc;
    if (t->tile_rows > 0) {
        const unsigned blocks = (unsigned)std::min<int64_t>(64, (t->tile_rows + 255) / 256);
        hipLaunchKernelGGL(k_tiles_total, dim3(blocks), dim3(256), 0, s, t->tile_rows, t->tile_row_ptr, t->tile_row_end,
                           ctx->d_scalars, (int)S_TILES_A);
    }
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
    v->tile_slots = t->tile_capacity;
    v->tile_row_ptr = t->tile_row_ptr;
    v->tile_row_end = t->tile_row_end;
    v->tile_col = t->tile_col;
    v->row_mask = t->row_mask;
    v->left_group_mask = t->lmask;
    v->right_group_mask = t->rmask;
    v->left_head = reinterpret_cast<const uint32_t *>(t->lhead);
    v->right_head = reinterpret_cast<const uint32_t *>(t->rhead);
    v->left_elements = reinterpret_cast<const uint16_t *>(t->ldata);
    v->right_elements = reinterpret_cast<const uint16_t *>(t->rdata);
    v->left_groups_capacity = t->ldata ? t->group_capacity : 0;
    v->right_groups_capacity = t->rdata ? t->group_capacity : 0;
    return TSP_OK;
}
