// Tile-level symbolic phase and counting pass (paper Sections 4.1 and 4.2; Algorithm 1 up to the counting kernel).
//
// The paper expands every (A tile, B tile) correspondence into a global list, culls it, sorts it
// twice and reduces it by key.  Here one workgroup owns one tile-row I of C and never leaves LDS:
//   1. candidates: for each tile A[I,K], each tile B[K,J] (tile correspondence);
//   2. cull: the pair survives iff some inner index k has a non-empty column k in the A tile and a
//      non-empty row k in the B tile (the boolean test on the occupancy words; a surviving pair
//      contributes at least one structural entry, so no listed C tile is empty);
//   3. the surviving J of the tile-row are marked in an LDS bitmap over tile columns; its popcount
//      is the number of C tiles of the row and the rank of a bit is the C tile's position, which
//      sorts the row by J without a sort;
//   4. per C tile a word records which A tiles (by position in the tile-row, 32 at a time)
//      contribute: bitwise OR is order independent, so the pair count (popcount) and each pair's
//      position inside its segment (popcount of the lower bits = ascending inner index K) are
//      deterministic although the candidates are visited in parallel.
// Prefix sums over the tile-rows give the C tile offsets and the task-list offsets.
// The counting pass then forms, per C tile, the boolean product of the bitmaps of its pairs
// (Section 4.2 runs the multiplication on 0/1 tiles for this; here integer bit operations on
// the 16-bit row masks, which gives the same pattern), and the per-row counts give row_ptr of C.
//
// Kernels: k_sym_count (steps 1-3, sizes per tile-row; k_sym_count_half gives short tile-rows half a wave
// each, k_sym_count_segmented does so against a very wide B), k_sym_row_scan (their prefix sums, one chained launch), then either k_sym_emit_listed (tile-rows
// with few pairs: survivors enumerated once into an LDS list; with enough tile-rows it also runs the
// counting pass and the row offsets; a block or half a wave per tile-row) or k_sym_emit (any tile-row; more
// C tiles than the LDS window holds are worked off window by window; on skewed products the heaviest
// tile-rows first, in the order k_work_hist and k_work_order set up), k_count_masks and k_row_offsets
// (k_row_offsets_wide for tile-rows with many tiles) where the list kernel has not done their work, and
// k_row_ptr.
#include "common.hpp"
#include "chain.hpp"

#include <algorithm>
#include <climits>
#include <new>

namespace tsp {

constexpr int kSymThreads = 256;
constexpr int kSymThreadsLong = 512;   // block of the counting and task-list kernels on tile-rows with very many candidates
constexpr int64_t kLongRowCandidates = 8192;    // ... that many per tile-row on average
constexpr int kMaxWords = 4096;        // LDS bitmap words per tile-row: span of 131072 tile columns
constexpr int kDirectWords = 1024;     // counting kernel: widest tile grid of B whose bitmap is indexed by the column itself
constexpr int kWindow = 4096;          // C tiles of one tile-row handled per LDS window
constexpr int kRowLeftOver = -1;       // row_words of a tile-row that the segmented counting kernel leaves to the full one
constexpr int kSurvivorUnroll = 4;     // B tiles one lane requests per trip of the candidate loop: long tile-rows of B
constexpr int kSurvivorUnrollShort = 2;   // ... and short ones

struct TileRefs {
    const int32_t *trp;      // first tile of every tile-row
    const int32_t *tend;     // one past the last
    const int32_t *tcol;     // tile_col
    const uint32_t *lmask;   // left group mask  -> row occupancy
    const uint32_t *rmask;   // right group mask -> column occupancy
    int32_t tile_rows;
};

__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t *lds /*[>=16]*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t s = 0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += lds[w];
    return s;
}

// In-place exclusive scan of arr[0..n) by the whole block; returns the total.
__device__ __forceinline__ uint32_t block_exclusive_scan_lds(uint32_t *arr, int n, uint32_t *lds /*[>=17]*/) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    uint32_t carry = 0;
    for (int base = 0; base < n; base += blockDim.x) {
        const int i = base + threadIdx.x;
        const uint32_t x = i < n ? arr[i] : 0;
        const uint32_t v = wave_inclusive_scan(x);
        __syncthreads();
        if (lane == 63) lds[wave] = v;
        __syncthreads();
        uint32_t before = 0, all = 0;
        for (int w = 0; w < nw; ++w) {
            uint32_t y = lds[w];
            if (w < wave) before += y;
            all += y;
        }
        if (i < n) arr[i] = carry + before + v - x;
        carry += all;
    }
    __syncthreads();
    return carry;
}

// Visits every surviving candidate pair of tile-row I whose A tile index lies in [a_begin,a_end).
// `lanes_per_a` lanes share one A tile and stride over the tiles of B's tile-row K.
// f(a, b, J) is called once per survivor; *candidates counts all candidates visited by this thread.
// kLongRows: built for operands whose B tile-rows are long (more tiles than lanes share an A tile).
// kBatched: every trip requests several B tiles, those past the end of the tile-row switched off, so a
// short tile-row of B takes one round trip; otherwise only full trips are batched and the rest goes tile by
// tile (better where f is heavy: the list kernel with a block per tile-row, whose f appends to an LDS list,
// loses 3 % with batching; the other kernels gain up to 30 % of their time).
// tid, nthreads: this thread's place among the threads that share the tile-row (a block, or part of a wave).
template <bool kLongRows, bool kBatched, class F>
__device__ __forceinline__ void for_each_survivor(const TileRefs &A, const TileRefs &B, int a_begin, int a_end,
                                                  int lanes_per_a, uint32_t *candidates, int tid, int nthreads, F f) {
    const int sub = tid / lanes_per_a, l = tid % lanes_per_a;
    const int nsub = nthreads / lanes_per_a;
    for (int a = a_begin + sub; a < a_end; a += nsub) {
        const uint32_t K = (uint32_t)A.tcol[a];
        if (K >= (uint32_t)B.tile_rows) continue;            // only possible for a non-canonical input
        const uint32_t col_occ = fold16(A.rmask[a]);
        const int b0 = B.trp[K], b1 = B.tend[K];
        if constexpr (kBatched) {
            constexpr int kPerTrip = kLongRows ? kSurvivorUnroll : kSurvivorUnrollShort;
            for (int b = b0 + l; b < b1; b += kPerTrip * lanes_per_a) {
                uint32_t occ[kPerTrip];
                int col[kPerTrip];
#pragma unroll
                for (int u = 0; u < kPerTrip; ++u) {
                    const int bu = b + u * lanes_per_a;
                    occ[u] = bu < b1 ? B.lmask[bu] : 0u;
                    col[u] = bu < b1 ? B.tcol[bu] : 0;
                }
#pragma unroll
                for (int u = 0; u < kPerTrip; ++u) {
                    const int bu = b + u * lanes_per_a;
                    if (bu < b1) {
                        ++*candidates;
                        if (col_occ & fold16(occ[u])) f(a, bu, col[u]);
                    }
                }
            }
        } else {
            int b = b0 + l;
            if constexpr (kLongRows)
            for (; b + (kSurvivorUnroll - 1) * lanes_per_a < b1; b += kSurvivorUnroll * lanes_per_a) {
                uint32_t occ[kSurvivorUnroll];
                int col[kSurvivorUnroll];
#pragma unroll
                for (int u = 0; u < kSurvivorUnroll; ++u) {
                    occ[u] = B.lmask[b + u * lanes_per_a];
                    col[u] = B.tcol[b + u * lanes_per_a];
                }
                *candidates += kSurvivorUnroll;
#pragma unroll
                for (int u = 0; u < kSurvivorUnroll; ++u)
                    if (col_occ & fold16(occ[u])) f(a, b + u * lanes_per_a, col[u]);
            }
            for (; b < b1; b += lanes_per_a) {
                ++*candidates;
                if (col_occ & fold16(B.lmask[b])) f(a, b, B.tcol[b]);
            }
        }
    }
}

template <bool kLongRows, bool kBatched, class F>
__device__ __forceinline__ void for_each_survivor(const TileRefs &A, const TileRefs &B, int a_begin, int a_end,
                                                  int lanes_per_a, uint32_t *candidates, F f) {
    for_each_survivor<kLongRows, kBatched>(A, B, a_begin, a_end, lanes_per_a, candidates, (int)threadIdx.x,
                                           (int)blockDim.x, f);
}

// The same walk, restricted to the B tiles whose tile column is below j_end, for tile-rows of C that are
// worked off in several windows of tile columns: the tiles of a tile-row of B are sorted by column, so a
// window's candidates are a stretch of it.  Where a window ended in B's tile-row K for A tile `a` is kept
// in cursor[a] (read when from_cursor, written when keep_cursor; one word per tile of A).
template <bool kLongRows, class F>
__device__ __forceinline__ void for_each_survivor_below(const TileRefs &A, const TileRefs &B, int a_begin, int a_end,
                                                        int lanes_per_a, int j_end, int32_t *cursor, bool from_cursor,
                                                        bool keep_cursor, int *lds_next_col, F f) {
    const int sub = threadIdx.x / lanes_per_a, l = threadIdx.x % lanes_per_a;
    const int nsub = blockDim.x / lanes_per_a;
    // all lanes of a group of lanes_per_a lanes run the same trip count of the outer loop (the reduction
    // at its end needs them all)
    for (int a0 = a_begin; a0 < a_end; a0 += nsub) {
        const int a = a0 + sub;
        int stop = INT_MAX;                                   // first tile of this lane's stride at or past j_end
        int stop_col = INT_MAX;                               // ... and its tile column
        if (a < a_end) {
            const uint32_t K = (uint32_t)A.tcol[a];
            if (K < (uint32_t)B.tile_rows) {
                const uint32_t col_occ = fold16(A.rmask[a]);
                const int b1 = B.tend[K];
                const int b0 = from_cursor ? __hip_atomic_load(&cursor[a], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                           : B.trp[K];
                int b = b0 + l;
                stop = b1;
                bool open = true;
                if constexpr (kLongRows)
                    for (; open && b + (kSurvivorUnroll - 1) * lanes_per_a < b1; b += kSurvivorUnroll * lanes_per_a) {
                        uint32_t occ[kSurvivorUnroll];
                        int col[kSurvivorUnroll];
#pragma unroll
                        for (int u = 0; u < kSurvivorUnroll; ++u) {
                            occ[u] = B.lmask[b + u * lanes_per_a];
                            col[u] = B.tcol[b + u * lanes_per_a];
                        }
#pragma unroll
                        for (int u = 0; u < kSurvivorUnroll; ++u) {
                            if (open && col[u] >= j_end) {
                                open = false;
                                stop = b + u * lanes_per_a;
                                stop_col = col[u];
                            }
                            if (open && (col_occ & fold16(occ[u]))) f(a, b + u * lanes_per_a, col[u]);
                        }
                    }
                for (; open && b < b1; b += lanes_per_a) {
                    const int col = B.tcol[b];
                    if (col >= j_end) {
                        open = false;
                        stop = b;
                        stop_col = col;
                    } else if (col_occ & fold16(B.lmask[b])) {
                        f(a, b, col);
                    }
                }
                stop = min(stop, b1);
            }
        }
        if (keep_cursor) {                                    // uniform
            for (int d = lanes_per_a >> 1; d >= 1; d >>= 1) {
                stop = min(stop, __shfl_xor(stop, d, 64));
                stop_col = min(stop_col, __shfl_xor(stop_col, d, 64));   // (sorted: the earliest stop has the lowest column)
            }
            if (l == 0 && a < a_end && stop != INT_MAX) {
                __hip_atomic_store(&cursor[a], stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (stop_col != INT_MAX) atomicMin(lds_next_col, stop_col);
            }
        }
    }
}

// Pass 1 per tile-row: span of candidate tile columns, number of C tiles, of surviving pairs, of
// candidates.  Dynamic LDS: max_words words.
template <bool kLongRows>
__global__ __launch_bounds__(kSymThreadsLong) void k_sym_count(TileRefs A, TileRefs B, int lanes_per_a, int max_words,
                                                           int direct_words, int only_marked,
                                                           int32_t *__restrict__ row_jmin,
                                                           int32_t *__restrict__ row_c_tiles,
                                                           int32_t *__restrict__ row_pairs,
                                                           int32_t *__restrict__ row_words,
                                                           int32_t *__restrict__ row_cand,
                                                           int64_t *__restrict__ d_scalars,
                                                           uint32_t *__restrict__ save_bitmap,
                                                           uint32_t *__restrict__ save_cnt,
                                                           const int32_t *__restrict__ order) {
    extern __shared__ uint32_t lds_dyn[];
    __shared__ uint32_t red[32];
    __shared__ int s_jmin, s_jmax;
    uint32_t *bm = lds_dyn;
    // block b takes tile-row b, or the tile-row the kept order of work puts in place b
    const int I = order ? min(max(order[blockIdx.x], 0), (int)gridDim.x - 1) : (int)blockIdx.x;
    // second launch after k_sym_count_segmented: only the tile-rows that kernel has left to this one
    if (only_marked && row_words[I] != kRowLeftOver) return;
    const int a0 = A.trp[I], a1 = A.tend[I];
    if (threadIdx.x == 0) {
        s_jmin = INT_MAX;
        s_jmax = -1;
    }
    __syncthreads();
    int jmin = INT_MAX, jmax = -1;
    uint32_t cand = 0, surv = 0;
    if (direct_words > 0) {
        // B's whole tile grid fits the bitmap: mark tile columns as they are, and read the extent of the
        // tile-row off the bitmap afterwards (no pass over the tile-rows of B for it: three dependent
        // gathers less)
        // With save_bitmap the pass also keeps what the task-list kernel would otherwise find out again by
        // walking the candidates twice more: the tile-row's bitmap, and the number of surviving pairs per tile
        // column (16-bit counters, two per word, behind the bitmap: a tile-row of A has fewer than 65535 tiles,
        // or the task-list kernel ignores them).
        uint32_t *cnt16 = bm + direct_words;
        for (int w = threadIdx.x; w < direct_words; w += blockDim.x) bm[w] = 0;
        if (save_bitmap)
            for (int w = threadIdx.x; w < direct_words * 16; w += blockDim.x) cnt16[w] = 0;
        __syncthreads();
        if (save_bitmap)
            for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &cand, [&](int, int, int J) {
                if ((uint32_t)J < (uint32_t)direct_words * 32u) {
                    atomicOr(&bm[J >> 5], 1u << (J & 31));
                    atomicAdd(&cnt16[J >> 1], 1u << ((J & 1) * 16));
                    ++surv;
                }
            });
        else
        for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &cand, [&](int, int, int J) {
            if ((uint32_t)J < (uint32_t)direct_words * 32u) {
                atomicOr(&bm[J >> 5], 1u << (J & 31));
                ++surv;
            }
        });
        __syncthreads();
        if (save_bitmap) {
            for (int w = threadIdx.x; w < direct_words; w += blockDim.x) save_bitmap[(int64_t)I * direct_words + w] = bm[w];
            for (int w = threadIdx.x; w < direct_words * 16; w += blockDim.x)
                save_cnt[(int64_t)I * direct_words * 16 + w] = cnt16[w];
        }
        uint32_t tiles = 0;
        for (int w = threadIdx.x; w < direct_words; w += blockDim.x) {
            const uint32_t bits = bm[w];
            if (bits) {
                tiles += __popc(bits);
                jmin = min(jmin, w * 32);              // word-aligned: the later passes only need J - jmin >= 0
                jmax = max(jmax, w * 32 + 31);
            }
        }
        if (jmax >= 0) {
            atomicMin(&s_jmin, jmin);
            atomicMax(&s_jmax, jmax);
        }
        tiles = block_sum_u32(tiles, red);             // (its barriers also order the two atomics above)
        surv = block_sum_u32(surv, red);
        cand = block_sum_u32(cand, red);
        if (threadIdx.x == 0) {
            const bool any = s_jmax >= 0;
            row_jmin[I] = any ? s_jmin : 0;
            row_c_tiles[I] = (int32_t)tiles;
            row_pairs[I] = (int32_t)surv;
            row_words[I] = any ? (s_jmax - s_jmin + 1) >> 5 : 0;
            row_cand[I] = (int32_t)cand;
        }
        return;
    }
    for (int a = a0 + threadIdx.x; a < a1; a += blockDim.x) {
        const uint32_t K = (uint32_t)A.tcol[a];
        if (K >= (uint32_t)B.tile_rows) continue;
        const int b0 = B.trp[K], b1 = B.tend[K];
        if (b0 < b1) {
            jmin = min(jmin, B.tcol[b0]);
            jmax = max(jmax, B.tcol[b1 - 1]);
        }
    }
    if (jmax >= 0) {
        atomicMin(&s_jmin, jmin);
        atomicMax(&s_jmax, jmax);
    }
    __syncthreads();
    jmin = s_jmin;
    jmax = s_jmax;
    if (jmax < 0 || jmin < 0) {       // no candidates in this tile-row
        if (threadIdx.x == 0) {
            row_jmin[I] = 0;
            row_c_tiles[I] = 0;
            row_pairs[I] = 0;
            row_words[I] = 0;
            row_cand[I] = 0;
        }
        return;
    }
    const int64_t span = (int64_t)jmax - jmin + 1;
    const int words = (int)((span + 31) >> 5);
    if (words > max_words) {
        if (threadIdx.x == 0) {
            d_scalars[S_UNSUPPORTED] = 1;
            row_jmin[I] = 0;
            row_c_tiles[I] = 0;
            row_pairs[I] = 0;
            row_words[I] = 0;
            row_cand[I] = 0;
        }
        return;
    }
    for (int w = threadIdx.x; w < words; w += blockDim.x) bm[w] = 0;
    __syncthreads();
    for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &cand, [&](int, int, int J) {
        const uint32_t j = (uint32_t)(J - jmin);
        if (j < (uint32_t)span) {
            atomicOr(&bm[j >> 5], 1u << (j & 31));
            ++surv;
        }
    });
    __syncthreads();
    uint32_t cnt = 0;
    for (int w = threadIdx.x; w < words; w += blockDim.x) cnt += __popc(bm[w]);
    cnt = block_sum_u32(cnt, red);
    surv = block_sum_u32(surv, red);
    cand = block_sum_u32(cand, red);
    if (threadIdx.x == 0) {
        row_jmin[I] = jmin;
        row_c_tiles[I] = (int32_t)cnt;
        row_pairs[I] = (int32_t)surv;
        row_words[I] = words;
        row_cand[I] = (int32_t)cand;
    }
}

// The same pass with two tile-rows per wave (32 lanes each), for operands with short tile-rows: the pass
// is a chain of dependent gathers, its duration is the number of waves over the waves the chip holds
// times the length of that chain, and tile-rows with a few dozen candidates leave most lanes of a wave
// idle anyway.  The two halves of a wave never wait for each other (no block barriers: LDS traffic
// inside a wave is ordered by wave_sync).  Dynamic LDS: 2*max_words words.
template <bool kLongRows>
__global__ __launch_bounds__(64) void k_sym_count_half(TileRefs A, TileRefs B, int lanes_per_a, int max_words,
                                                       int32_t *__restrict__ row_jmin,
                                                       int32_t *__restrict__ row_c_tiles,
                                                       int32_t *__restrict__ row_pairs,
                                                       int32_t *__restrict__ row_words,
                                                       int32_t *__restrict__ row_cand,
                                                       int64_t *__restrict__ d_scalars) {
    extern __shared__ uint32_t lds_dyn[];
    __shared__ int s_ext[2][2];                    // first and last candidate tile column of the tile-row
    __shared__ uint32_t s_cnt[2][3];               // C tiles, surviving pairs, candidates
    constexpr int kLanes = 32;
    const int half = threadIdx.x / kLanes, tid = threadIdx.x % kLanes;
    const int I = (int)blockIdx.x * 2 + half;
    uint32_t *bm = lds_dyn + half * max_words;
    if (tid == 0) {
        s_ext[half][0] = INT_MAX;
        s_ext[half][1] = -1;
        s_cnt[half][0] = s_cnt[half][1] = s_cnt[half][2] = 0;
    }
    wave_sync();
    const bool live = I < A.tile_rows;             // (an odd number of tile-rows: the last half idles)
    const int a0 = live ? A.trp[I] : 0, a1 = live ? A.tend[I] : 0;
    int jmin = INT_MAX, jmax = -1;
    for (int a = a0 + tid; a < a1; a += kLanes) {
        const uint32_t K = (uint32_t)A.tcol[a];
        if (K >= (uint32_t)B.tile_rows) continue;
        const int b0 = B.trp[K], b1 = B.tend[K];
        if (b0 < b1) {
            jmin = min(jmin, B.tcol[b0]);
            jmax = max(jmax, B.tcol[b1 - 1]);
        }
    }
    if (jmax >= 0) {
        atomicMin(&s_ext[half][0], jmin);
        atomicMax(&s_ext[half][1], jmax);
    }
    wave_sync();
    jmin = s_ext[half][0];
    jmax = s_ext[half][1];
    const int64_t span = (int64_t)jmax - jmin + 1;
    const int words = (int)((span + 31) >> 5);
    const bool any = live && jmax >= 0 && jmin >= 0;
    const bool fits = words <= max_words;
    if (any && !fits && tid == 0) d_scalars[S_UNSUPPORTED] = 1;
    const bool walk = any && fits;                 // uniform over the half
    if (walk)
        for (int w = tid; w < words; w += kLanes) bm[w] = 0;
    wave_sync();
    uint32_t cand = 0, surv = 0;
    if (walk)
        for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &cand, tid, kLanes, [&](int, int, int J) {
            const uint32_t j = (uint32_t)(J - jmin);
            if (j < (uint32_t)span) {
                atomicOr(&bm[j >> 5], 1u << (j & 31));
                ++surv;
            }
        });
    wave_sync();
    uint32_t tiles = 0;
    if (walk)
        for (int w = tid; w < words; w += kLanes) tiles += __popc(bm[w]);
    if (tiles) atomicAdd(&s_cnt[half][0], tiles);
    if (surv) atomicAdd(&s_cnt[half][1], surv);
    if (cand) atomicAdd(&s_cnt[half][2], cand);
    wave_sync();
    if (live && tid == 0) {
        row_jmin[I] = walk ? jmin : 0;
        row_c_tiles[I] = (int32_t)s_cnt[half][0];
        row_pairs[I] = (int32_t)s_cnt[half][1];
        row_words[I] = walk ? words : 0;
        row_cand[I] = (int32_t)s_cnt[half][2];
    }
}

// The same for a B with a wide tile grid, where a bitmap over the span of a tile-row's candidates would be
// sized for the widest span possible (up to 16 KB a tile-row, which leaves a CU a handful of waves) while
// the candidates of a short tile-row sit in a few clusters: the bitmap is kept in segments of 1024 tile
// columns, handed out on demand from kSegSlots slots per tile-row.  A tile-row that needs more is marked
// kRowLeftOver in row_words and done by a second launch of k_sym_count with the full bitmap.  The extent of
// the tile-row is read off the segments (no pass over B's tile-rows for it).
constexpr int kSegSlots = 16, kSegWords = 32;      // 32 words = 1024 tile columns per segment
template <bool kLongRows>
__global__ __launch_bounds__(64) void k_sym_count_segmented(TileRefs A, TileRefs B, int lanes_per_a, int max_words,
                                                            int32_t *__restrict__ row_jmin,
                                                            int32_t *__restrict__ row_c_tiles,
                                                            int32_t *__restrict__ row_pairs,
                                                            int32_t *__restrict__ row_words,
                                                            int32_t *__restrict__ row_cand,
                                                            int64_t *__restrict__ d_scalars) {
    __shared__ int s_seg[2][kSegSlots];                          // which segment a slot holds, -1: free
    __shared__ uint32_t s_bits[2][kSegSlots][kSegWords];
    __shared__ int s_ext[2][2];
    __shared__ uint32_t s_cnt[2][4];                             // C tiles, surviving pairs, candidates, slots ran out
    constexpr int kLanes = 32;
    const int half = threadIdx.x / kLanes, tid = threadIdx.x % kLanes;
    const int I = (int)blockIdx.x * 2 + half;
    if (tid < kSegSlots) s_seg[half][tid] = -1;
    for (int w = tid; w < kSegSlots * kSegWords; w += kLanes) s_bits[half][w / kSegWords][w % kSegWords] = 0;
    if (tid == 0) {
        s_ext[half][0] = INT_MAX;
        s_ext[half][1] = -1;
        s_cnt[half][0] = s_cnt[half][1] = s_cnt[half][2] = s_cnt[half][3] = 0;
    }
    wave_sync();
    const bool live = I < A.tile_rows;
    const int a0 = live ? A.trp[I] : 0, a1 = live ? A.tend[I] : 0;
    uint32_t cand = 0, surv = 0;
    bool out_of_slots = false;
    for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &cand, tid, kLanes, [&](int, int, int J) {
        if (J < 0) return;                         // (tile columns come from the converter and are not negative)
        const int seg = J >> 10;
        int slot = -1;
        for (int k = 0; k < kSegSlots && slot < 0; ++k) {
            int held = s_seg[half][k];
            if (held == -1) held = atomicCAS(&s_seg[half][k], -1, seg);   // free: claim it (or see who did)
            if (held == -1 || held == seg) slot = k;
        }
        if (slot < 0) {
            out_of_slots = true;
            return;
        }
        atomicOr(&s_bits[half][slot][(J >> 5) & (kSegWords - 1)], 1u << (J & 31));
        ++surv;
    });
    if (out_of_slots) s_cnt[half][3] = 1;
    wave_sync();
    uint32_t tiles = 0;
    int jmin = INT_MAX, jmax = -1;
    for (int w = tid; w < kSegSlots * kSegWords; w += kLanes) {
        const uint32_t bits = s_bits[half][w / kSegWords][w % kSegWords];
        if (bits) {
            const int first = s_seg[half][w / kSegWords] * 1024 + (w % kSegWords) * 32;   // word-aligned extent
            tiles += __popc(bits);
            jmin = min(jmin, first);
            jmax = max(jmax, first + 31);
        }
    }
    if (jmax >= 0) {
        atomicMin(&s_ext[half][0], jmin);
        atomicMax(&s_ext[half][1], jmax);
    }
    if (tiles) atomicAdd(&s_cnt[half][0], tiles);
    if (surv) atomicAdd(&s_cnt[half][1], surv);
    if (cand) atomicAdd(&s_cnt[half][2], cand);
    wave_sync();
    if (live && tid == 0) {
        const bool any = s_ext[half][1] >= 0;
        const int words = any ? (s_ext[half][1] - s_ext[half][0] + 1) >> 5 : 0;
        if (s_cnt[half][3]) {                      // left to the kernel with the full bitmap
            row_words[I] = kRowLeftOver;
        } else if (words > max_words) {            // span beyond what the later passes hold
            d_scalars[S_UNSUPPORTED] = 1;
            row_jmin[I] = 0;
            row_c_tiles[I] = 0;
            row_pairs[I] = 0;
            row_words[I] = 0;
            row_cand[I] = 0;
        } else {
            row_jmin[I] = any ? s_ext[half][0] : 0;
            row_c_tiles[I] = (int32_t)s_cnt[half][0];
            row_pairs[I] = (int32_t)s_cnt[half][1];
            row_words[I] = words;
            row_cand[I] = (int32_t)s_cnt[half][2];
        }
    }
}

// Prefix sums over the tile-rows (Algorithm 1: counts -> offsets and total sizes) in one
// launch: C tiles per row -> c_tile_row_ptr, pairs per row -> row_pair_ptr, plus the totals and maxima
// the host needs to size the task list.  A block scans 1024 tile-rows; the blocks are chained.
// k_row_ptr turns row lengths into row_ptr in one launch, 2048 rows (128 tile-rows) per block, from the
// number of entries of every tile-row, which the counting pass leaves in an array (one plain store per
// tile-row: thousands of atomics on a few addresses cost tens of microseconds).  Every block adds up the
// tile-rows before it, so the launch is for up to kMaxChunks blocks; beyond, the three-kernel scan.
constexpr int kChunkTileRows = 128, kChunkRows = kChunkTileRows * T;
constexpr int64_t kMaxChunks = 256;

constexpr int kRowScanThreads = 256, kRowScanItems = 4, kRowScanBlock = kRowScanThreads * kRowScanItems;
struct TileCount {           // an operand whose number of tiles is still to be summed (slot < 0: nothing to do)
    const int32_t *trp, *tend;
    int64_t tile_rows;
    int slot;
};
__global__ __launch_bounds__(kRowScanThreads) void k_sym_row_scan(
    int64_t ntr, const int32_t *__restrict__ row_c_tiles, const int32_t *__restrict__ row_pairs,
    const int32_t *__restrict__ row_words, const int32_t *__restrict__ row_cand,
    int32_t *__restrict__ c_tile_row_ptr, int64_t *__restrict__ row_pair_ptr, ChainSlot *slots, unsigned epoch,
    int64_t *__restrict__ d_scalars, TileCount count_a, TileCount count_b, int64_t *h_scalars_dev,
    int64_t publish_tag) {
    __shared__ uint64_t lds[kRowScanThreads / 64 + kChainValues];
    __shared__ int lds_m[3][kRowScanThreads / 64];
    __shared__ uint32_t lds_t[2][kRowScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * kRowScanBlock + (int64_t)threadIdx.x * kRowScanItems;
    int32_t xc[kRowScanItems], xp[kRowScanItems];
    uint64_t sc = 0, sp = 0, cand = 0;
    int max_c = 0, max_w = 0, max_p = 0;
#pragma unroll
    for (int k = 0; k < kRowScanItems; ++k) {
        const bool in = i0 + k < ntr;
        xc[k] = in ? row_c_tiles[i0 + k] : 0;
        xp[k] = in ? row_pairs[i0 + k] : 0;
        sc += (uint32_t)xc[k];
        sp += (uint32_t)xp[k];
        max_c = max(max_c, xc[k]);
        max_p = max(max_p, xp[k]);
        max_w = max(max_w, in ? row_words[i0 + k] : 0);
        cand += in ? (uint32_t)row_cand[i0 + k] : 0u;
    }
    // tiles of the operands whose converter has not been waited for: summed here, one atomic per block
    uint32_t tiles_a = 0, tiles_b = 0;
#pragma unroll
    for (int k = 0; k < kRowScanItems; ++k) {
        if (count_a.slot >= 0 && i0 + k < count_a.tile_rows) tiles_a += (uint32_t)(count_a.tend[i0 + k] - count_a.trp[i0 + k]);
        if (count_b.slot >= 0 && i0 + k < count_b.tile_rows) tiles_b += (uint32_t)(count_b.tend[i0 + k] - count_b.trp[i0 + k]);
    }
    tiles_a = wave_sum(tiles_a);
    tiles_b = wave_sum(tiles_b);
    if (lane == 0) {
        lds_t[0][wave] = tiles_a;
        lds_t[1][wave] = tiles_b;
    }
    // maxima and tile counts: one atomic per block (a few dozen blocks at most per million rows), issued
    // before the block's sums go into the chain, so that whoever has taken those sums in sees them too
    max_c = wave_max(max_c);
    max_w = wave_max(max_w);
    max_p = wave_max(max_p);
    __syncthreads();
    if (lane == 0) {
        lds_m[0][wave] = max_c;
        lds_m[1][wave] = max_w;
        lds_m[2][wave] = max_p;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int mc = 0, mw = 0, mp = 0;
        for (int w = 0; w < kRowScanThreads / 64; ++w) {
            mc = max(mc, lds_m[0][w]);
            mw = max(mw, lds_m[1][w]);
            mp = max(mp, lds_m[2][w]);
        }
        atomicMax((unsigned long long *)&d_scalars[S_MAX_ROW_PAIRS], (unsigned long long)mp);
        atomicMax((unsigned long long *)&d_scalars[S_MAX_ROW_C_TILES], (unsigned long long)mc);
        atomicMax((unsigned long long *)&d_scalars[S_MAX_ROW_WORDS], (unsigned long long)mw);
        unsigned long long ta = 0, tb = 0;
        for (int w = 0; w < kRowScanThreads / 64; ++w) {
            ta += lds_t[0][w];
            tb += lds_t[1][w];
        }
        if (ta) atomicAdd((unsigned long long *)&d_scalars[count_a.slot], ta);
        if (tb) atomicAdd((unsigned long long *)&d_scalars[count_b.slot], tb);
    }
    unsigned long long agg[kChainValues], prefix[kChainValues];
    uint64_t total, unused;
    const uint64_t local_c = block_exclusive_scan64<kRowScanThreads>(sc, &total, lds);
    agg[0] = total;
    const uint64_t local_p = block_exclusive_scan64<kRowScanThreads>(sp, &total, lds);
    agg[1] = total;
    (void)block_exclusive_scan64<kRowScanThreads>(cand, &total, lds);
    agg[2] = total;
    (void)unused;
    chain_exclusive_prefix(slots, epoch, agg, prefix, lds + kRowScanThreads / 64, d_scalars + S_INTERNAL);
    uint64_t run_c = prefix[0] + local_c, run_p = prefix[1] + local_p;
#pragma unroll
    for (int k = 0; k < kRowScanItems; ++k) {
        if (i0 + k < ntr) {
            c_tile_row_ptr[i0 + k] = (int32_t)run_c;
            row_pair_ptr[i0 + k] = (int64_t)run_p;
        }
        run_c += (uint32_t)xc[k];
        run_p += (uint32_t)xp[k];
    }
    // The last block of the chain has taken in, directly or through the blocks before it, the sums of all
    // others, each released after its block's atomics: it writes the totals and hands the scalar block
    // to the host.
    if (blockIdx.x == gridDim.x - 1) {
        if (threadIdx.x == 0) {
            c_tile_row_ptr[ntr] = (int32_t)(prefix[0] + agg[0]);
            row_pair_ptr[ntr] = (int64_t)(prefix[1] + agg[1]);
            d_scalars[S_C_TILES] = (int64_t)(prefix[0] + agg[0]);
            d_scalars[S_PAIRS] = (int64_t)(prefix[1] + agg[1]);
            d_scalars[S_CANDIDATES] = (int64_t)(prefix[2] + agg[2]);
        }
        publish_scalars(d_scalars, h_scalars_dev, publish_tag);
    }
}

// Tile-rows in descending order of work, for products with a few very heavy tile-rows (hubs of a power-law
// graph): a block per tile-row in index order starts a heavy tile-row in the middle of the range when most
// of the launch is over, and the launch then waits for that one block.  A counting sort by the power of two
// of the work (32 buckets, heaviest first; the order inside a bucket is left to the atomics and has no
// influence on any result: every tile-row writes to places of its own).
constexpr int kOrderThreads = 256, kOrderItems = 4, kOrderBuckets = 32;
__device__ __forceinline__ int work_bucket(int32_t work) { return work <= 0 ? 0 : 32 - __clz(work); }   // 0..31

__global__ __launch_bounds__(kOrderThreads) void k_work_hist(int64_t ntr, const int32_t *__restrict__ work,
                                                             uint32_t *__restrict__ hist) {
    __shared__ uint32_t lds_hist[kOrderBuckets];
    if (threadIdx.x < kOrderBuckets) lds_hist[threadIdx.x] = 0;
    __syncthreads();
    const int64_t i0 = ((int64_t)blockIdx.x * kOrderThreads + threadIdx.x) * kOrderItems;
#pragma unroll
    for (int k = 0; k < kOrderItems; ++k)
        if (i0 + k < ntr) atomicAdd(&lds_hist[work_bucket(work[i0 + k])], 1u);
    __syncthreads();
    if (threadIdx.x < kOrderBuckets && lds_hist[threadIdx.x]) atomicAdd(&hist[threadIdx.x], lds_hist[threadIdx.x]);
}

// hist: the finished histogram; taken: 32 zeroed counters (places handed out per bucket so far)
__global__ __launch_bounds__(kOrderThreads) void k_work_order(int64_t ntr, const int32_t *__restrict__ work,
                                                              const uint32_t *__restrict__ hist,
                                                              uint32_t *__restrict__ taken, int32_t *__restrict__ order) {
    __shared__ uint32_t lds_count[kOrderBuckets], lds_base[kOrderBuckets];
    if (threadIdx.x < kOrderBuckets) lds_count[threadIdx.x] = 0;
    __syncthreads();
    const int64_t i0 = ((int64_t)blockIdx.x * kOrderThreads + threadIdx.x) * kOrderItems;
    int bucket[kOrderItems];
    uint32_t rank[kOrderItems];
#pragma unroll
    for (int k = 0; k < kOrderItems; ++k) {
        bucket[k] = i0 + k < ntr ? work_bucket(work[i0 + k]) : -1;
        rank[k] = bucket[k] >= 0 ? atomicAdd(&lds_count[bucket[k]], 1u) : 0u;
    }
    __syncthreads();
    if (threadIdx.x < kOrderBuckets) {
        // first place of the bucket: after all heavier buckets; then this block's share of it
        uint32_t heavier = 0;
        for (int b = (int)threadIdx.x + 1; b < kOrderBuckets; ++b) heavier += hist[b];
        const uint32_t mine = lds_count[threadIdx.x];
        lds_base[threadIdx.x] = heavier + (mine ? atomicAdd(&taken[threadIdx.x], mine) : 0u);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kOrderItems; ++k)
        if (bucket[k] >= 0) {
            const uint32_t at = lds_base[bucket[k]] + rank[k];
            if (at < (uint32_t)ntr) order[at] = (int32_t)(i0 + k);     // (always, unless `work` changed between the two launches)
        }
}

// Pass 2 per tile-row: C tile coordinates, task-list offsets, task list.
// Dynamic LDS: 2*words_cap + 2*window words.  Tile-rows with more C tiles than the window holds take
// several windows; `cursor` (one word per tile of A, nullptr when no tile-row needs it) carries their
// places in B's tile-rows from window to window.
template <bool kLongRows>
__global__ __launch_bounds__(kSymThreadsLong) void k_sym_emit(
    TileRefs A, TileRefs B, int lanes_per_a, int words_cap, int window,
    const int32_t *__restrict__ row_jmin, const int32_t *__restrict__ row_words,
    const int32_t *__restrict__ c_tile_row_ptr, const int64_t *__restrict__ row_pair_ptr,
    int32_t *__restrict__ c_tile_row, int32_t *__restrict__ c_tile_col, int64_t *__restrict__ pair_off,
    int2 *__restrict__ pair_ab, int32_t *cursor, int64_t A_capacity,
    const int32_t *__restrict__ order, const uint32_t *__restrict__ saved_bitmap,
    const uint32_t *__restrict__ saved_cnt, int saved_words, int64_t pairs) {
    extern __shared__ uint32_t lds_dyn[];
    __shared__ uint32_t red[32];
    uint32_t *bm = lds_dyn;
    uint32_t *wpre = bm + words_cap;
    uint32_t *contrib = wpre + words_cap;
    uint32_t *cnt = contrib + window;
    // block b takes tile-row b, or the tile-row the host's order of work puts in place b
    const int I = order ? min(max(order[blockIdx.x], 0), (int)gridDim.x - 1) : (int)blockIdx.x;
    const int c0 = c_tile_row_ptr[I], nC = c_tile_row_ptr[I + 1] - c0;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) pair_off[c_tile_row_ptr[gridDim.x]] = row_pair_ptr[gridDim.x];
    if (nC <= 0 || (nC > window && !cursor)) return;      // (the host provides the cursors whenever a tile-row needs them)
    const int a0 = A.trp[I], a1 = A.tend[I];
    const int jmin = row_jmin[I];
    // the bitmap extent the first pass found for this tile-row (rows over the limit have nC = 0)
    const int words = min(row_words[I], words_cap);
    const int64_t span = (int64_t)words * 32;
    uint32_t dummy = 0;
    // what the counting kernel has kept for this tile-row: its bitmap and the pairs per tile column
    const bool saved = saved_bitmap && a1 - a0 < 65535 && (jmin & 31) == 0 && (jmin >> 5) + words <= saved_words;
    if (saved) {
        for (int w = threadIdx.x; w < words; w += blockDim.x) bm[w] = saved_bitmap[(int64_t)I * saved_words + (jmin >> 5) + w];
    } else {
        for (int w = threadIdx.x; w < words; w += blockDim.x) bm[w] = 0;
        __syncthreads();
        for_each_survivor<kLongRows, true>(A, B, a0, a1, lanes_per_a, &dummy, [&](int, int, int J) {
            const uint32_t j = (uint32_t)(J - jmin);
            if (j < (uint32_t)span) atomicOr(&bm[j >> 5], 1u << (j & 31));
        });
    }
    __syncthreads();
    for (int w = threadIdx.x; w < words; w += blockDim.x) wpre[w] = __popc(bm[w]);
    __syncthreads();
    block_exclusive_scan_lds(wpre, words, red);
    // C tile coordinates, ascending J
    for (int w = threadIdx.x; w < words; w += blockDim.x) {
        uint32_t bits = bm[w];
        int c = c0 + (int)wpre[w];
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            c_tile_row[c] = I;
            c_tile_col[c] = jmin + w * 32 + bit;
            ++c;
        }
    }
    const int64_t row_base = row_pair_ptr[I];
    // (a tile-row of at most 32 A tiles: the count pass leaves the contributor words of its only chunk
    // behind for the emit pass; not so when the counts come from the counting kernel and no count pass runs)
    const bool one_chunk = (a1 - a0) <= 32 && !saved;
    // A tile-row with more C tiles than the LDS window holds is worked off window by window, and every
    // window only walks its own stretch of B's tile-rows (for_each_survivor_below): the stretches are
    // shorter than the tile-rows, so fewer lanes share an A tile and more A tiles are in flight.
    const bool multi = nC > window;
    int lanes_w = lanes_per_a;
    if (multi) {
        int windows = (nC + window - 1) / window, f = 1;
        while (f < windows) f <<= 1;
        lanes_w = max(4, min(lanes_per_a, 2 * lanes_per_a / f));   // (measured on hub tile-rows of an R-MAT graph)
    }
    __shared__ int s_j_end, s_next_col;
    // per chunk of 32 A tiles (at the index of its first tile, behind the cursors): the lowest tile column
    // its tiles of A still have ahead in B's tile-rows; a window below that column skips the chunk
    int32_t *const chunk_next_col = cursor ? cursor + A_capacity : nullptr;
    uint32_t win_base = 0;
    for (int win0 = 0; win0 < nC; win0 += window) {
        const int nw = min(window, nC - win0);
        int j_end = INT_MAX;                       // tile column of the first C tile after the window
        const bool more = win0 + nw < nC;
        if (multi) {
            if (more) {
                const int k = win0 + nw;
                for (int w = threadIdx.x; w < words; w += blockDim.x) {
                    const uint32_t bits = bm[w];
                    const int before = (int)wpre[w];
                    if (before <= k && k < before + __popc(bits)) {       // the k-th C tile is bit (k - before) of this word
                        uint32_t x = bits;
                        for (int i = before; i < k; ++i) x &= x - 1;
                        s_j_end = jmin + w * 32 + (__ffs(x) - 1);
                    }
                }
            }
            __syncthreads();
            if (more) j_end = s_j_end;
        }
        // every surviving pair of A tiles [ch, ch_end) whose C tile lies in this window
        auto skip_chunk = [&](int ch) {             // uniform: nothing of this chunk lies in the window
            return multi && win0 > 0 &&
                   __hip_atomic_load(&chunk_next_col[ch], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= j_end;
        };
        auto walk = [&](int ch, int ch_end, bool keep, auto f) {
            if (multi)
                for_each_survivor_below<kLongRows>(A, B, ch, ch_end, lanes_w, j_end, cursor, win0 > 0, keep && more,
                                                   &s_next_col, f);
            else
                for_each_survivor<kLongRows, true>(A, B, ch, ch_end, lanes_per_a, &dummy, f);
        };
        auto rank_in_window = [&](int J) -> int {
            const uint32_t j = (uint32_t)(J - jmin);
            if (j >= (uint32_t)span) return -1;
            const uint32_t word = bm[j >> 5];
            const int c = (int)wpre[j >> 5] + __popc(word & ((1u << (j & 31)) - 1u)) - win0;
            return (c >= 0 && c < nw) ? c : -1;
        };
        for (int c = threadIdx.x; c < nw; c += blockDim.x) cnt[c] = 0;
        if (saved) {
            __syncthreads();
            // pairs per C tile of the window, as the counting kernel left them per tile column
            const uint16_t *per_col = reinterpret_cast<const uint16_t *>(saved_cnt) + (int64_t)I * saved_words * 32;
            for (int w = threadIdx.x; w < words; w += blockDim.x) {
                uint32_t bits = bm[w];
                int c = (int)wpre[w] - win0;       // position in the window of the word's first C tile
                while (bits) {
                    const int bit = __ffs(bits) - 1;
                    bits &= bits - 1;
                    if (c >= 0 && c < nw) cnt[c] = per_col[jmin + w * 32 + bit];
                    ++c;
                }
            }
            __syncthreads();
        }
        // count pass: 32 A tiles at a time
        for (int ch = a0; ch < a1 && !saved; ch += 32) {
            if (skip_chunk(ch)) continue;
            for (int c = threadIdx.x; c < nw; c += blockDim.x) contrib[c] = 0;
            __syncthreads();
            walk(ch, min(ch + 32, a1), false, [&](int a, int, int J) {
                const int c = rank_in_window(J);
                if (c >= 0) atomicOr(&contrib[c], 1u << (a - ch));
            });
            __syncthreads();
            for (int c = threadIdx.x; c < nw; c += blockDim.x) cnt[c] += __popc(contrib[c]);
            __syncthreads();
        }
        const uint32_t win_total = block_exclusive_scan_lds(cnt, nw, red);
        for (int c = threadIdx.x; c < nw; c += blockDim.x)
            pair_off[c0 + win0 + c] = row_base + (int64_t)win_base + (int64_t)cnt[c];
        // emit pass
        for (int ch = a0; ch < a1; ch += 32) {
            if (skip_chunk(ch)) continue;
            if (multi && more) {                     // (uniform) the chunk's next column is collected by the last walk
                if (threadIdx.x == 0) s_next_col = INT_MAX;
                __syncthreads();
            }
            if (!one_chunk) {
                for (int c = threadIdx.x; c < nw; c += blockDim.x) contrib[c] = 0;
                __syncthreads();
                walk(ch, min(ch + 32, a1), false, [&](int a, int, int J) {
                    const int c = rank_in_window(J);
                    if (c >= 0) atomicOr(&contrib[c], 1u << (a - ch));
                });
                __syncthreads();
            }
            walk(ch, min(ch + 32, a1), true, [&](int a, int b, int J) {
                const int c = rank_in_window(J);
                if (c >= 0) {
                    const int64_t pos = row_base + (int64_t)win_base + (int64_t)cnt[c] +
                                        __popc(contrib[c] & ((1u << (a - ch)) - 1u));
                    if ((uint64_t)pos < (uint64_t)pairs) {     // (always: the counts and the walks see the same survivors)
                        pair_ab[pos] = make_int2(a, b);
                    }
                }
            });
            __syncthreads();
            if (multi && more && threadIdx.x == 0)
                __hip_atomic_store(&chunk_next_col[ch], s_next_col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!one_chunk) {
                for (int c = threadIdx.x; c < nw; c += blockDim.x) cnt[c] += __popc(contrib[c]);
                __syncthreads();
            }
        }
        win_base += win_total;
        __syncthreads();
    }
}

// The threads that work on one tile-row together: a whole block (kTeamLanes == 0), or a part of a wave
// (kTeamLanes lanes), whose LDS traffic needs no block barrier.
template <int kTeamLanes>
struct Team {
    __device__ static __forceinline__ int tid() { return kTeamLanes ? (int)threadIdx.x % kTeamLanes : (int)threadIdx.x; }
    __device__ static __forceinline__ int size() { return kTeamLanes ? kTeamLanes : (int)blockDim.x; }
    __device__ static __forceinline__ int index() { return kTeamLanes ? (int)threadIdx.x / kTeamLanes : 0; }
    __device__ static __forceinline__ void sync() {
        if (kTeamLanes) wave_sync();
        else __syncthreads();
    }
};

// In-place exclusive scan of arr[0..n) by the team; returns the total.
template <int kTeamLanes>
__device__ __forceinline__ uint32_t team_exclusive_scan_lds(uint32_t *arr, int n, uint32_t *lds /*[>=17], block only*/) {
    if constexpr (kTeamLanes == 0) {
        return block_exclusive_scan_lds(arr, n, lds);
    } else {
        const int tid = Team<kTeamLanes>::tid();
        uint32_t carry = 0;
        for (int base = 0; base < n; base += kTeamLanes) {
            const int i = base + tid;
            const uint32_t x = i < n ? arr[i] : 0;
            uint32_t v = x;
#pragma unroll
            for (int o = 1; o < kTeamLanes; o <<= 1) {
                const uint32_t up = __shfl_up(v, o, kTeamLanes);
                if (tid >= o) v += up;
            }
            if (i < n) arr[i] = carry + v - x;
            carry += __shfl(v, kTeamLanes - 1, kTeamLanes);
        }
        wave_sync();
        return carry;
    }
}

// OR over the set bits k of `am` of row mask k of the B tile; x, y hold the 16 row masks, two per
// 32-bit word (row 2i in the low half).  Four bits of `am` select among four rows, i.e. two words: the
// two AND masks (all ones in the half whose row is selected) come from a 16-entry table in LDS, so a
// word costs one and-or, and a nibble two instructions for its table address.  Entries of the table
// are 8 bytes: 16 of them cover every LDS bank once, and lanes with the same nibble read the same address.
struct RowSelectTable {
    uint2 entry[16];
    __device__ __forceinline__ void fill() {       // by the first 16 threads of the block; a barrier follows
        if (threadIdx.x < 16) {
            const uint32_t v = threadIdx.x;
            entry[v] = make_uint2(((v & 1u) ? 0x0000FFFFu : 0u) | ((v & 2u) ? 0xFFFF0000u : 0u),
                                  ((v & 4u) ? 0x0000FFFFu : 0u) | ((v & 8u) ? 0xFFFF0000u : 0u));
        }
    }
};
__device__ __forceinline__ uint32_t boolean_row_product(uint32_t am, const uint4 &x, const uint4 &y,
                                                        const RowSelectTable &table) {
    const uint2 m0 = table.entry[am & 15u], m1 = table.entry[(am >> 4) & 15u];
    const uint2 m2 = table.entry[(am >> 8) & 15u], m3 = table.entry[(am >> 12) & 15u];
    uint32_t acc = x.x & m0.x;
    acc |= x.y & m0.y;
    acc |= x.z & m1.x;
    acc |= x.w & m1.y;
    acc |= y.x & m2.x;
    acc |= y.y & m2.y;
    acc |= y.z & m3.x;
    acc |= y.w & m3.y;
    return acc;
}

// The same pass for products all of whose tile-rows have few task-list entries (at most kListCap) and
// fit one LDS window: the surviving pairs are enumerated once and kept in an LDS list; counting them
// per C tile and placing them then works on the list (the general kernel enumerates the candidates
// three times, and the enumeration, a chain of dependent gathers, is what it spends its time on).
// It also runs the counting pass for its C tiles.
// Dynamic LDS: 2*words_cap + 10*window + 3*list_cap words (list_cap: most entries any tile-row has).
constexpr int kPairsPerTrip = 2;       // pairs a lane group of the fused counting pass takes per trip
constexpr int kListCap = 1024;
constexpr int kListTeamLanes = 32;     // lanes that share a tile-row where tile-rows have few candidates (16: slower)
constexpr int kListTiles = 512;        // and at most this many C tiles per tile-row (their bitmaps sit in LDS)
// kFuseMasks: also run the counting pass (worth it when there are enough tile-rows to fill the chip;
// with few, long tile-rows the separate kernel, one lane group per C tile, has more parallelism).
template <bool kLongRows, bool kFuseMasks, int kTeamLanes>
__global__ __launch_bounds__(kTeamLanes ? 64 : kSymThreads) void k_sym_emit_listed(
    TileRefs A, TileRefs B, int lanes_per_a, int words_cap, int window, int list_cap, int team_words,
    const int32_t *__restrict__ row_jmin, const int32_t *__restrict__ row_words,
    const int32_t *__restrict__ c_tile_row_ptr, const int64_t *__restrict__ row_pair_ptr,
    int32_t *__restrict__ c_tile_row, int32_t *__restrict__ c_tile_col, int64_t *__restrict__ pair_off,
    int2 *__restrict__ pair_ab, const uint16_t *__restrict__ a_row_mask,
    const uint16_t *__restrict__ b_row_mask, uint16_t *__restrict__ c_row_mask, uint32_t *__restrict__ c_row_off,
    int32_t *__restrict__ row_nnz, int64_t c_rows, int64_t *d_scalars, uint32_t *__restrict__ tile_row_entries) {
    extern __shared__ uint32_t lds_dyn[];
    using team = Team<kTeamLanes>;
    constexpr int kTeams = kTeamLanes ? 64 / kTeamLanes : 1;
    __shared__ uint32_t red[32];
    __shared__ int s_n_all[kTeams];
    __shared__ RowSelectTable row_select;
    __shared__ uint32_t s_part_all[kTeams][(kTeamLanes ? kTeamLanes : kSymThreads) / 16][T];
    if (kFuseMasks) {
        row_select.fill();                           // (barriers before its first use; in a wave of two teams
        if (kTeamLanes) wave_sync();                 // the other team may have left by then)
    }
    const int tid = team::tid(), team_index = team::index();
    int &s_n = s_n_all[team_index];
    uint32_t(*const s_part)[T] = s_part_all[team_index];
    uint32_t *bm = lds_dyn + (size_t)team_index * team_words;
    uint32_t *wpre = bm + words_cap;
    uint32_t *contrib = wpre + words_cap;
    uint32_t *cnt = contrib + window;
    int *list_a = reinterpret_cast<int *>(cnt + window), *list_b = list_a + list_cap;
    int *list_c = list_b + list_cap;                 // tile column, later the C tile's position in the row
    uint32_t *cmask = reinterpret_cast<uint32_t *>(list_c + list_cap);   // 8 words (16 row masks) per C tile
    const int I = (int)blockIdx.x * kTeams + team_index, nthreads = team::size();
    if (I >= A.tile_rows) return;                    // (an odd number of tile-rows: the last team idles)
    const int c0 = c_tile_row_ptr[I], nC = c_tile_row_ptr[I + 1] - c0;
    if (I == A.tile_rows - 1 && tid == 0) pair_off[c_tile_row_ptr[A.tile_rows]] = row_pair_ptr[A.tile_rows];
    if (nC <= 0) {                                   // an empty tile-row of C: its 16 rows are empty
        if (kFuseMasks && tid < T && (int64_t)I * T + tid < c_rows) row_nnz[(int64_t)I * T + tid] = 0;
        if (kFuseMasks && tid == 0) tile_row_entries[I] = 0;
        return;
    }
    const int a0 = A.trp[I], a1 = A.tend[I];
    const int jmin = row_jmin[I];
    const int64_t row_base = row_pair_ptr[I];
    if (tid == 0) s_n = 0;
    // the bitmap extent the first pass found for this tile-row
    const int words = min(row_words[I], words_cap);
    const int64_t span = (int64_t)words * 32;
    for (int w = tid; w < words; w += nthreads) bm[w] = 0;
    team::sync();
    uint32_t dummy = 0;
    for_each_survivor<kLongRows, (kTeamLanes != 0)>(A, B, a0, a1, lanes_per_a, &dummy, tid, nthreads, [&](int a, int b, int J) {
        const uint32_t j = (uint32_t)(J - jmin);
        if (j < (uint32_t)span) {
            atomicOr(&bm[j >> 5], 1u << (j & 31));
            const int k = atomicAdd(&s_n, 1);      // any order: positions come from the bit words below
            if (k < list_cap) {
                list_a[k] = a;
                list_b[k] = b;
                list_c[k] = (int)j;
            }
        }
    });
    team::sync();
    const int n = min(s_n, list_cap);
    for (int w = tid; w < words; w += nthreads) wpre[w] = __popc(bm[w]);
    team::sync();
    team_exclusive_scan_lds<kTeamLanes>(wpre, words, red);
    for (int w = tid; w < words; w += nthreads) {     // C tile coordinates, ascending J
        uint32_t bits = bm[w];
        int c = c0 + (int)wpre[w];
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            c_tile_row[c] = I;
            c_tile_col[c] = jmin + w * 32 + bit;
            ++c;
        }
    }
    for (int k = tid; k < n; k += nthreads) {          // tile column -> position of the C tile in the row
        const uint32_t j = (uint32_t)list_c[k];
        list_c[k] = (int)wpre[j >> 5] + __popc(bm[j >> 5] & ((1u << (j & 31)) - 1u));
    }
    for (int c = tid; c < nC; c += nthreads) cnt[c] = 0;
    const bool one_chunk = (a1 - a0) <= 32;
    // count pass: which of 32 A tiles at a time contribute to each C tile
    for (int ch = a0; ch < a1; ch += 32) {
        for (int c = tid; c < nC; c += nthreads) contrib[c] = 0;
        team::sync();
        for (int k = tid; k < n; k += nthreads) {
            const uint32_t rel = (uint32_t)(list_a[k] - ch);
            if (rel < 32u) atomicOr(&contrib[list_c[k]], 1u << rel);
        }
        team::sync();
        for (int c = tid; c < nC; c += nthreads) cnt[c] += __popc(contrib[c]);
        team::sync();
    }
    team_exclusive_scan_lds<kTeamLanes>(cnt, nC, red);
    for (int c = tid; c < nC; c += nthreads) pair_off[c0 + c] = row_base + (int64_t)cnt[c];
    // emit pass: a pair sits after the pairs of its C tile with a lower A tile
    for (int ch = a0; ch < a1; ch += 32) {
        if (!one_chunk) {
            for (int c = tid; c < nC; c += nthreads) contrib[c] = 0;
            team::sync();
            for (int k = tid; k < n; k += nthreads) {
                const uint32_t rel = (uint32_t)(list_a[k] - ch);
                if (rel < 32u) atomicOr(&contrib[list_c[k]], 1u << rel);
            }
            team::sync();
        }
        for (int k = tid; k < n; k += nthreads) {
            const uint32_t rel = (uint32_t)(list_a[k] - ch);
            if (rel < 32u) {
                const int c = list_c[k];
                const int64_t pos = row_base + (int64_t)cnt[c] + __popc(contrib[c] & ((1u << rel) - 1u));
                pair_ab[pos] = make_int2(list_a[k], list_b[k]);
            }
        }
        if (!one_chunk) {
            team::sync();
            for (int c = tid; c < nC; c += nthreads) cnt[c] += __popc(contrib[c]);
            team::sync();
        }
    }
    if constexpr (!kFuseMasks) return;
    // Counting pass (Section 4.2) for the tile-row's C tiles, from the same list: 16 lanes per pair, lane
    // r forms row r of the boolean product of the two bitmaps and ORs it into the C tile's bitmap in LDS.
    // kPairsPerTrip pairs per trip, their bitmaps requested together (four or two per trip take the same
    // time, eight cost registers).
    for (int w = tid; w < nC * 8; w += nthreads) cmask[w] = 0;
    team::sync();
    {
        const int g = tid >> 4, r = tid & 15, groups = nthreads >> 4;
        // The bitmaps of the next trip are requested before the products of the current one are formed: a trip
        // is a memory round trip for a few dozen instructions of work.  (A trip past the end of the list reads
        // the last entry again and selects nothing of it: no branches and no zero-filled registers around
        // the loads.)
        uint32_t am[kPairsPerTrip];
        uint4 x[kPairsPerTrip], y[kPairsPerTrip];
        int c_of[kPairsPerTrip];
        auto request = [&](int k0) {
#pragma unroll
            for (int u = 0; u < kPairsPerTrip; ++u) {
                const int k = min(k0 + u, n - 1);
                am[u] = a_row_mask[(int64_t)list_a[k] * T + r];
                const uint4 *bp = reinterpret_cast<const uint4 *>(b_row_mask + (int64_t)list_b[k] * T);
                x[u] = bp[0];
                y[u] = bp[1];
                c_of[u] = list_c[k];
            }
        };
        const int stride = groups * kPairsPerTrip;
        if constexpr (kTeamLanes != 0) {
            // (half a wave per tile-row: the second set of registers would cost the kernel its eighth wave per
            // SIMD, and with it the single round in which all tile-rows of a large product are resident)
            for (int k0 = g * kPairsPerTrip; k0 < n; k0 += stride) {
                request(k0);
#pragma unroll
                for (int u = 0; u < kPairsPerTrip; ++u) {
                    const uint32_t m = boolean_row_product(k0 + u < n ? am[u] : 0u, x[u], y[u], row_select);
                    const uint32_t m16 = (m | (m >> 16)) & 0xFFFFu;
                    if (m16) atomicOr(&cmask[c_of[u] * 8 + (r >> 1)], m16 << ((r & 1) * 16));
                }
            }
        } else {
        if (g * kPairsPerTrip < n) request(g * kPairsPerTrip);
        for (int k0 = g * kPairsPerTrip; k0 < n; k0 += stride) {
            uint32_t am_now[kPairsPerTrip];
            uint4 x_now[kPairsPerTrip], y_now[kPairsPerTrip];
            int c_now[kPairsPerTrip];
#pragma unroll
            for (int u = 0; u < kPairsPerTrip; ++u) {
                am_now[u] = k0 + u < n ? am[u] : 0u;
                x_now[u] = x[u];
                y_now[u] = y[u];
                c_now[u] = c_of[u];
            }
            if (k0 + stride < n) request(k0 + stride);
#pragma unroll
            for (int u = 0; u < kPairsPerTrip; ++u) {
                const uint32_t m = boolean_row_product(am_now[u], x_now[u], y_now[u], row_select);
                const uint32_t m16 = (m | (m >> 16)) & 0xFFFFu;
                if (m16) atomicOr(&cmask[c_now[u] * 8 + (r >> 1)], m16 << ((r & 1) * 16));
            }
        }
        }
    }
    team::sync();
    uint32_t *out_words = reinterpret_cast<uint32_t *>(c_row_mask) + (int64_t)c0 * 8;
    for (int w = tid; w < nC * 8; w += nthreads) out_words[w] = cmask[w];
    // ... and what k_row_offsets does for this tile-row: lane r of every 16-lane group takes CSR row
    // 16I+r for a stretch of the C tiles, the groups' sums are exchanged through LDS.
    {
        const int g = tid >> 4, r = tid & 15, groups = nthreads >> 4;
        const int word = r >> 1, shift = (r & 1) * 16;
        const int stretch = (nC + groups - 1) / groups;
        const int cb = min(nC, g * stretch), ce = min(nC, cb + stretch);
        uint32_t part = 0;
        for (int c = cb; c < ce; ++c) part += __popc((cmask[c * 8 + word] >> shift) & 0xFFFFu);
        s_part[g][r] = part;
        team::sync();
        uint32_t total = 0, earlier = 0;           // entries of row r in the tile-row, and in the stretches before this one
        for (int h = 0; h < groups; ++h) {
            const uint32_t v = s_part[h][r];
            total += v;
            earlier += h < g ? v : 0u;
        }
        uint64_t before = total;                   // inclusive prefix over the 16 rows
#pragma unroll
        for (int d = 1; d < T; d <<= 1) {
            const uint64_t up = __shfl_up(before, d, T);
            if (r >= d) before += up;
        }
        if (g == 0) {
            const int64_t row = (int64_t)I * T + r;
            if (row < c_rows) row_nnz[row] = (int32_t)total;
            if (r == T - 1) {
                if (before > 0xFFFFFFFFull) d_scalars[S_UNSUPPORTED] = 1;
                tile_row_entries[I] = (uint32_t)before;
            }
        }
        uint32_t run = (uint32_t)(before - total) + earlier;
        for (int c = cb; c < ce; ++c) {
            c_row_off[(int64_t)(c0 + c) * T + r] = run;
            run += __popc((cmask[c * 8 + word] >> shift) & 0xFFFFu);
        }
    }
}

// Counting pass (Section 4.2) as a kernel of its own: a block takes 16 consecutive C tiles, whose task-list
// segments are one contiguous stretch, and every lane takes one entry of the stretch at a time: it fetches
// the 16 row masks of the A tile and of the B tile (32 bytes each), forms all 16 rows of the boolean
// product (row r: OR over the set bits k of the A tile's row mask r of the B tile's row mask k) and ORs
// them into the bitmap of the entry's C tile, which the block keeps in LDS.  With a lane per entry no
// lane idles on a short segment or on an empty row of a sparse A tile: 16 lanes per C tile, each owning
// one row, issued three times as many instructions per entry on tiles with two or three elements.
constexpr int kMaskTilesStrips = 16;   // C tiles per block with the order in strips (a descriptor names 16 tiles)
template <int kMaskTiles>
__global__ __launch_bounds__(256) void k_count_masks(int64_t c_tiles, const int64_t *__restrict__ pair_off,
                                                     const int2 *__restrict__ pair_ab,
                                                     const uint16_t *__restrict__ a_row_mask,
                                                     const uint16_t *__restrict__ b_row_mask,
                                                     uint16_t *__restrict__ c_row_mask,
                                                     const int2 *__restrict__ strip_desc,
                                                     const int32_t *__restrict__ strip_total, const int xcd_chunk) {
    __shared__ uint32_t cmask[kMaskTiles][8];      // row masks 2i (low half) and 2i+1 of every tile
    __shared__ uint32_t seg[kMaskTiles + 1];       // first entry of every tile's segment, from the block's first
    __shared__ RowSelectTable row_select;
    row_select.fill();
    const int64_t logical = xcd_chunked_index(blockIdx.x, xcd_chunk);
    // the block's output tiles: consecutive ones, or the ones its descriptor names (order in strips)
    int64_t c_first = logical * kMaskTiles;
    int tiles = (int)max((int64_t)0, min((int64_t)kMaskTiles, c_tiles - c_first));
    if (strip_desc) {
        int2 d = make_int2(0, 0);
        if (logical < *strip_total) d = strip_desc[logical];
        c_first = d.x;
        tiles = c_first + d.y <= c_tiles ? d.y : 0;
    }
    if (tiles <= 0) return;                        // whole block
    const int64_t base = pair_off[c_first];
    if (threadIdx.x <= kMaskTiles) {
        const int64_t off = pair_off[c_first + min((int)threadIdx.x, tiles)] - base;
        seg[threadIdx.x] = (uint32_t)min(max(off, (int64_t)0), (int64_t)0x7FFFFFFF);
    }
    for (int w = threadIdx.x; w < kMaskTiles * 8; w += 256) cmask[w >> 3][w & 7] = 0;
    __syncthreads();
    const uint32_t total = seg[kMaskTiles];
    for (uint32_t e = threadIdx.x; e < total; e += 256) {
        int t = 0;                                 // the C tile of entry e: the last tile whose segment starts at or before it
#pragma unroll
        for (int step = kMaskTiles / 2; step >= 1; step >>= 1)
            if (seg[t + step] <= e) t += step;
        const int2 ab = pair_ab[base + e];
        const int64_t a = ab.x, b = ab.y;
        const uint4 *ap = reinterpret_cast<const uint4 *>(a_row_mask + a * T);
        const uint4 *bp = reinterpret_cast<const uint4 *>(b_row_mask + b * T);
        const uint4 a0 = ap[0], a1 = ap[1], x = bp[0], y = bp[1];
        const uint32_t aw[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t w = 0;
            if (aw[i]) {                           // (both rows of the word empty: the usual case on sparse tiles)
                const uint32_t lo = boolean_row_product(aw[i] & 0xFFFFu, x, y, row_select);
                const uint32_t hi = boolean_row_product(aw[i] >> 16, x, y, row_select);
                w = ((lo | (lo >> 16)) & 0xFFFFu) | ((hi | (hi << 16)) & 0xFFFF0000u);
            }
            if (w) atomicOr(&cmask[t][i], w);
        }
    }
    __syncthreads();
    const int r = threadIdx.x & 15;
    for (int t = threadIdx.x >> 4; t < tiles; t += 16)
        c_row_mask[(c_first + t) * T + r] = (uint16_t)((cmask[t][r >> 1] >> ((r & 1) * 16)) & 0xFFFFu);
}

// row_ptr of C from the row lengths: block b takes rows [2048 b, 2048 b + 2048), starts from the
// entries of the tile-rows before them and scans its own rows.  The last block has read every
// tile-row and also leaves nnz(C) and the largest tile-row.
__global__ __launch_bounds__(256) void k_row_ptr(const int32_t *__restrict__ row_nnz, int64_t c_rows,
                                                 const uint32_t *__restrict__ tile_row_entries, int64_t c_tile_rows,
                                                 int64_t *__restrict__ c_row_ptr, int64_t *d_scalars,
                                                 int64_t *h_scalars_dev, int64_t publish_tag) {
    __shared__ uint64_t lds[256 / 64];
    constexpr int kItems = kChunkRows / 256;
    const bool last = blockIdx.x == gridDim.x - 1;
    const int64_t tile_rows_before = (int64_t)blockIdx.x * kChunkTileRows;
    // the block's own row lengths, requested first: they travel while the tile-rows before are added up
    const int64_t base = (int64_t)blockIdx.x * kChunkRows + (int64_t)threadIdx.x * kItems;
    int32_t x[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) x[i] = base + i < c_rows ? row_nnz[base + i] : 0;
    uint64_t before = 0;
    uint32_t largest = 0;
    // four tile-rows per load, four loads in flight (the array is padded to a multiple of four)
    const uint4 *entries4 = reinterpret_cast<const uint4 *>(tile_row_entries);
    const int64_t quads = ((last ? c_tile_rows : tile_rows_before) + 3) / 4;
    for (int64_t q0 = threadIdx.x; q0 < quads; q0 += 4 * 256) {
        uint4 e[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) e[u] = q0 + u * 256 < quads ? entries4[q0 + u * 256] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t I = (q0 + u * 256) * 4;
            const uint32_t v[4] = {e[u].x, e[u].y, e[u].z, e[u].w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (I + k < c_tile_rows) {
                    if (I + k < tile_rows_before) before += v[k];
                    largest = max(largest, v[k]);
                }
        }
    }
    uint64_t entries_before;
    (void)block_exclusive_scan64<256>(before, &entries_before, lds);
    uint64_t mine = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) mine += (uint32_t)x[i];
    uint64_t total;
    uint64_t run = entries_before + block_exclusive_scan64<256>(mine, &total, lds);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (base + i < c_rows) c_row_ptr[base + i] = (int64_t)run;
        run += (uint32_t)x[i];
    }
    if (last) {
        largest = (uint32_t)wave_max((int)min(largest, 0x7FFFFFFFu));
        __syncthreads();
        if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = largest;
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < 256 / 64; ++w) largest = max(largest, (uint32_t)lds[w]);
            c_row_ptr[c_rows] = (int64_t)(entries_before + total);
            d_scalars[S_C_NNZ] = (int64_t)(entries_before + total);
            d_scalars[S_MAX_ROW_ENTRIES] = (int64_t)largest;
        }
        // no other block of this launch writes a scalar, and the kernels before it have finished
        publish_scalars(d_scalars, h_scalars_dev, publish_tag);
    }
}

// Per tile-row of C (16 lanes, lane r = row r): the length of CSR row 16I+r, and for every tile of
// the tile-row the position of its first entry in that row, counted from the first entry of the
// tile-row (entries of rows 16I..16I+r-1 plus the row's entries in the tiles to the left).  The
// multiplication pass adds the start of the tile-row and the rank inside the tile.  Offsets are
// 32-bit: a tile-row of C with 2^32 entries or more raises the "unsupported" flag.
__global__ __launch_bounds__(256) void k_row_offsets(int64_t c_tile_rows, int64_t c_rows,
                                                     const int32_t *__restrict__ c_tile_row_ptr,
                                                     const uint16_t *__restrict__ c_row_mask,
                                                     uint32_t *__restrict__ c_row_off,
                                                     int32_t *__restrict__ row_nnz, int64_t *d_scalars,
                                                     uint32_t *__restrict__ tile_row_entries) {
    const int64_t I = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4;
    const int r = threadIdx.x & 15;
    if (I >= c_tile_rows) return;                  // whole 16-lane groups leave together
    const int64_t c0 = c_tile_row_ptr[I], c1 = c_tile_row_ptr[I + 1];
    uint32_t total = 0;                            // <= 16 * tiles of the tile-row: fits
    for (int64_t c = c0; c < c1; ++c) total += __popc(c_row_mask[c * T + r]);
    const int64_t row = I * T + r;
    if (row < c_rows) row_nnz[row] = (int32_t)total;
    uint64_t before = total;                       // inclusive prefix over the 16 rows
#pragma unroll
    for (int d = 1; d < T; d <<= 1) {
        const uint64_t up = __shfl_up(before, d, T);
        if (r >= d) before += up;
    }
    if (r == T - 1) {
        if (before > 0xFFFFFFFFull) d_scalars[S_UNSUPPORTED] = 1;
        tile_row_entries[I] = (uint32_t)before;
    }
    uint32_t run = (uint32_t)(before - total);
    for (int64_t c = c0; c < c1; ++c) {
        c_row_off[c * T + r] = run;
        run += __popc(c_row_mask[c * T + r]);
    }
}

// The same for tile-rows with many tiles: a block per tile-row, its 16 lane groups each take a stretch of
// the tiles and exchange their sums through LDS (a hub tile-row of a power-law graph has tens of
// thousands of tiles, which one lane group would walk twice on its own).
__global__ __launch_bounds__(256) void k_row_offsets_wide(int64_t c_rows, const int32_t *__restrict__ c_tile_row_ptr,
                                                          const uint16_t *__restrict__ c_row_mask,
                                                          uint32_t *__restrict__ c_row_off,
                                                          int32_t *__restrict__ row_nnz, int64_t *d_scalars,
                                                          uint32_t *__restrict__ tile_row_entries) {
    __shared__ uint32_t s_part[256 / 16][T];
    const int64_t I = blockIdx.x;
    const int g = threadIdx.x >> 4, r = threadIdx.x & 15;
    constexpr int kGroups = 256 / 16;
    const int64_t c0 = c_tile_row_ptr[I], c1 = c_tile_row_ptr[I + 1];
    const int64_t stretch = (c1 - c0 + kGroups - 1) / kGroups;
    const int64_t cb = min(c1, c0 + g * stretch), ce = min(c1, cb + stretch);
    uint32_t part = 0;
#pragma unroll 8
    for (int64_t c = cb; c < ce; ++c) part += __popc(c_row_mask[c * T + r]);
    s_part[g][r] = part;
    __syncthreads();
    uint32_t total = 0, earlier = 0;
#pragma unroll
    for (int h = 0; h < kGroups; ++h) {
        const uint32_t v = s_part[h][r];
        total += v;
        earlier += h < g ? v : 0u;
    }
    uint64_t before = total;                       // inclusive prefix over the 16 rows
#pragma unroll
    for (int d = 1; d < T; d <<= 1) {
        const uint64_t up = __shfl_up(before, d, T);
        if (r >= d) before += up;
    }
    if (g == 0) {
        const int64_t row = I * T + r;
        if (row < c_rows) row_nnz[row] = (int32_t)total;
        if (r == T - 1) {
            if (before > 0xFFFFFFFFull) d_scalars[S_UNSUPPORTED] = 1;
            tile_row_entries[I] = (uint32_t)before;
        }
    }
    uint32_t run = (uint32_t)(before - total) + earlier;
    // (eight masks requested together: the loop is a chain of loads otherwise)
    int64_t c = cb;
    for (; c + 8 <= ce; c += 8) {
        uint32_t m[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) m[u] = c_row_mask[(c + u) * T + r];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            c_row_off[(c + u) * T + r] = run;
            run += __popc(m[u]);
        }
    }
    for (; c < ce; ++c) {
        c_row_off[c * T + r] = run;
        run += __popc(c_row_mask[c * T + r]);
    }
}

bool row_ptr_in_one_launch(tsp_context *ctx, const int32_t *row_len, int64_t rows, const uint32_t *group_len,
                           int64_t *row_ptr, hipStream_t s) {
    const int64_t groups = (rows + T - 1) / T, chunks = (groups + kChunkTileRows - 1) / kChunkTileRows;
    if (chunks < 1 || chunks > kMaxChunks) return false;
    hipLaunchKernelGGL(k_row_ptr, dim3((unsigned)chunks), dim3(256), 0, s, row_len, rows, group_len, groups, row_ptr,
                       ctx->d_scalars, ctx->h_scalars_dev, ++ctx->publish_tag);
    return true;
}

void plan_release(tsp_context *ctx, tsp_plan_s *p, hipStream_t s) {
    if (!p) return;
    ctx_free(ctx, p->c_tile_row_ptr, s);
    ctx_free(ctx, p->c_tile_row, s);
    ctx_free(ctx, p->c_tile_col, s);
    ctx_free(ctx, p->pair_off, s);
    ctx_free(ctx, p->pair_ab, s);
    ctx_free(ctx, p->c_row_mask, s);
    ctx_free(ctx, p->c_row_off, s);
    ctx_free(ctx, p->c_row_ptr, s);
    ctx_free(ctx, p->strip_desc, s);
    ctx_free(ctx, p->strip_block_ptr, s);
    delete p;
}

// Strip order (strips.hip) for the kernels that walk the task list: only on request (TSP_OPT_STRIP_ORDER).
// Measured on a power-law graph (262,144 rows, 2.5e9 task-list entries): the strips cut the traffic behind
// the L2 caches to a quarter (multiplication kernel 540 -> 133 GB, counting kernel 222 -> 52 GB), and both
// kernels took 3-5 % longer: on such tiles they are bound by the instructions issued per task-list entry,
// not by memory.
static bool strips_wanted(const tsp_context *ctx, const tsp_plan_s *, const tsp_tiles_s *) {
    return ctx->strip_order == 1 || ctx->strip_order >= 16;
}

static int lanes_per_a_tile(const tsp_tiles_s *B) {
    // lanes that share one A tile stride over the tiles of one tile-row of B: match its mean length
    const double mean = B->tile_rows > 0 && B->ntiles > 0 ? (double)B->ntiles / (double)B->tile_rows : 1.0;
    // (with the unrolled candidate loop a lane takes kSurvivorUnroll tiles per trip, so a quarter of
    // the lanes do: more A tiles are then in flight per block)
    int l = 4;
    while (l < 64 && l * (mean > 8.0 ? kSurvivorUnroll : 1) < mean) l <<= 1;
    return l;
}

int symbolic_run(tsp_context *ctx, tsp_tiles_s *A, tsp_tiles_s *B, tsp_plan_s **out, hipStream_t s) {
    *out = nullptr;
    if (A->cols != B->rows) return TSP_ERR_SHAPE_MISMATCH;
    tsp_plan_s *P = new (std::nothrow) tsp_plan_s();
    if (!P) return TSP_ERR_ALLOC_FAILED;
    P->c_rows = A->rows;
    P->c_cols = B->cols;
    P->c_tile_rows = A->tile_rows;
    const int64_t ntr = A->tile_rows;
    int rc = TSP_OK;
    int32_t *row_jmin = nullptr, *row_c_tiles = nullptr, *row_pairs = nullptr, *row_nnz = nullptr;
    uint32_t *tile_row_entries = nullptr;
    int32_t *row_words = nullptr, *row_cand = nullptr;
    int32_t *cursor = nullptr, *order = nullptr;
    uint32_t *order_hist = nullptr;
    uint32_t *saved_bitmap = nullptr, *saved_cnt = nullptr;   // kept by the counting kernel for the task-list kernel
    int saved_words = 0;
    int64_t *row_pair_ptr = nullptr, *tmp = nullptr;
    auto cleanup = [&](int code) {
        ctx_free(ctx, row_jmin, s);
        ctx_free(ctx, row_c_tiles, s);
        ctx_free(ctx, row_pairs, s);
        ctx_free(ctx, row_words, s);
        ctx_free(ctx, row_cand, s);
        ctx_free(ctx, cursor, s);
        if (order != ctx->hint_order) ctx_free(ctx, order, s);
        ctx_free(ctx, order_hist, s);
        ctx_free(ctx, row_nnz, s);
        ctx_free(ctx, tile_row_entries, s);
        ctx_free(ctx, row_pair_ptr, s);
        ctx_free(ctx, tmp, s);
        ctx_free(ctx, saved_bitmap, s);
        ctx_free(ctx, saved_cnt, s);
        if (code) plan_release(ctx, P, s);
        return code;
    };

    // a failed HIP call leaves through cleanup(), which releases the scratch arrays and the plan
#define SYM_CHECK(expr)                                              \
    do {                                                             \
        hipError_t e_ = (expr);                                      \
        if (e_ != hipSuccess) return cleanup(hip_fail(ctx, e_));     \
    } while (0)
    phase_begin(ctx, TSP_PHASE_SYMBOLIC, s);
    row_jmin = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    row_c_tiles = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    row_pairs = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    row_words = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    row_cand = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    row_pair_ptr = ctx_alloc_n<int64_t>(ctx, (size_t)ntr + 1, s);
    P->c_tile_row_ptr = ctx_alloc_n<int32_t>(ctx, (size_t)ntr + 1, s);
    const int64_t scan_n = ntr > P->c_rows ? ntr : P->c_rows;
    tmp = ctx_alloc_n<int64_t>(ctx, scan_tmp_entries(scan_n), s);
    if (!row_jmin || !row_c_tiles || !row_pairs || !row_words || !row_cand || !row_pair_ptr || !P->c_tile_row_ptr || !tmp)
        return cleanup(TSP_ERR_ALLOC_FAILED);

    const int64_t n_chunks = (ntr + kChunkTileRows - 1) / kChunkTileRows;     // blocks of k_row_ptr
    TileRefs ra{A->tile_row_ptr, A->tile_row_end, A->tile_col, A->lmask, A->rmask, (int32_t)A->tile_rows};
    TileRefs rb{B->tile_row_ptr, B->tile_row_end, B->tile_col, B->lmask, B->rmask, (int32_t)B->tile_rows};
    // tiles-per-tile-row of B is not known on the host before the first read-back: estimate the
    // sharing width from the bound nnz/tile_rows (an upper bound on the mean), capped
    int lanes = 4;
    bool long_rows = false;                // B tile-rows long enough for the unrolled candidate loop
    bool listed = false;                   // task list built by k_sym_emit_listed
    bool fused_masks = false;              // ... which has also run the counting pass
    {
        const double mean_bound = B->tile_rows > 0 ? (double)B->nnz / (double)B->tile_rows : 1.0;
        while (lanes < 8 && lanes * 4 < mean_bound) lanes <<= 1;
        long_rows = mean_bound > 128.0;
        if (B->ntiles >= 0) {
            lanes = lanes_per_a_tile(B);
            long_rows = (double)B->ntiles > 8.0 * (double)B->tile_rows;
        }
    }
    if (ntr > 0) {
        KernelTimer kt(ctx, TSP_KERNEL_SYM_COUNT, s);
        // the bitmap cannot be wider than B's tile grid; short tile-rows get one wave each, so that
        // many more of them are in flight (the kernels are bound by dependent loads, not by work)
        const int max_words = (int)std::min<int64_t>(kMaxWords, (B->tile_cols + 31) / 32 + 1);
        const int64_t per_row = A->nnz / ntr;
        int threads = per_row <= 256 ? 64 : per_row <= 4096 ? 128 : kSymThreads;
        // where B's tile grid is narrow the bitmap simply covers all of it (worth it while the two sweeps
        // over the whole bitmap cost a block less than the three dependent gathers they replace:
        // measured, up to about six words per thread)
        const int64_t grid_words = (B->tile_cols + 31) / 32;
        const int direct_words = grid_words <= std::min<int64_t>(kDirectWords, 6 * threads) ? (int)grid_words : 0;
        // short tile-rows of A: two per wave (with more of them than the chip holds waves, half the time);
        // against a wide B with the bitmap in segments, and a second launch for the tile-rows it leaves over
        const bool halves = threads == 64 && direct_words == 0 && per_row <= 128;
        // A product that takes the general task-list kernel, against a B whose tile grid fits the bitmap (hubs of
        // a graph meet most of B): the pass keeps the bitmaps and the pairs per tile column for that kernel, which
        // then walks the candidates twice instead of four times.  The counters cost the pass LDS and time (on
        // such a graph 26 -> 42 ms, for 133 -> 100 ms in the task-list kernel), and where the list kernel runs
        // they are wasted; which kernel will run is known only after this pass, so the handle goes by what the
        // previous call with operands of the same sizes did.  The result is the same either way.
        size_t count_lds = (size_t)max_words * sizeof(uint32_t);
        const bool general_expected = ctx->hint_general && ctx->hint_sizes[0] == A->rows && ctx->hint_sizes[1] == A->nnz &&
                                      ctx->hint_sizes[2] == B->rows && ctx->hint_sizes[3] == B->nnz;
        if (direct_words > 0 && general_expected && (int64_t)ntr * direct_words * 17 * 4 <= ((int64_t)1 << 30) &&
            (size_t)direct_words * 17 * sizeof(uint32_t) <= 60 * 1024) {
            saved_words = direct_words;
            saved_bitmap = ctx_alloc_n<uint32_t>(ctx, (size_t)ntr * direct_words, s);
            saved_cnt = ctx_alloc_n<uint32_t>(ctx, (size_t)ntr * direct_words * 16, s);
            if (!saved_bitmap || !saved_cnt) return cleanup(TSP_ERR_ALLOC_FAILED);
            count_lds = std::max(count_lds, (size_t)direct_words * 17 * sizeof(uint32_t));
            // (the counters take LDS, LDS decides how many blocks a CU holds, and the pass lives on waves in
            // flight: larger blocks keep as many; the heaviest tile-rows, one block each, decide when the launch
            // ends: 128, 256, 512, 1024 threads: 76, 42, 29, 32 ms on an R-MAT graph of scale 18)
            if (count_lds > 8 * 1024) threads = kSymThreadsLong;
        }
        if (halves && max_words > 1024) {
            hipLaunchKernelGGL(long_rows ? k_sym_count_segmented<true> : k_sym_count_segmented<false>,
                               dim3((unsigned)((ntr + 1) / 2)), dim3(64), 0, s, ra, rb, std::min(lanes, 8), max_words,
                               row_jmin, row_c_tiles, row_pairs, row_words, row_cand, ctx->d_scalars);
            hipLaunchKernelGGL(long_rows ? k_sym_count<true> : k_sym_count<false>, dim3((unsigned)ntr), dim3(threads),
                               max_words * sizeof(uint32_t), s, ra, rb, lanes, max_words, 0, /*only_marked=*/1,
                               row_jmin, row_c_tiles, row_pairs, row_words, row_cand, ctx->d_scalars, nullptr, nullptr,
                               nullptr);
        } else if (halves)
            hipLaunchKernelGGL(long_rows ? k_sym_count_half<true> : k_sym_count_half<false>,
                               dim3((unsigned)((ntr + 1) / 2)), dim3(64), 2 * max_words * sizeof(uint32_t), s, ra, rb,
                               std::min(lanes, 8), max_words, row_jmin, row_c_tiles, row_pairs, row_words, row_cand,
                               ctx->d_scalars);
        else
            hipLaunchKernelGGL(long_rows ? k_sym_count<true> : k_sym_count<false>, dim3((unsigned)ntr), dim3(threads),
                               count_lds, s, ra, rb, lanes, max_words, direct_words,
                               /*only_marked=*/0, row_jmin, row_c_tiles, row_pairs, row_words, row_cand, ctx->d_scalars,
                               saved_bitmap, saved_cnt,
                               general_expected && ctx->hint_order_rows == ntr ? ctx->hint_order : nullptr);
        SYM_CHECK(hipGetLastError());
    }
    {
        KernelTimer kt(ctx, TSP_KERNEL_SCAN_SYM, s);
        // the same launch sums the tiles of operands that come straight from the converter
        const TileCount ca{A->tile_row_ptr, A->tile_row_end, A->tile_rows, A->ntiles < 0 ? A->scalar_slot : -1};
        const TileCount cb{B->tile_row_ptr, B->tile_row_end, B->tile_rows, B->ntiles < 0 && B != A ? B->scalar_slot : -1};
        int64_t rows_covered = ntr;
        if (ca.slot >= 0) rows_covered = std::max(rows_covered, ca.tile_rows);
        if (cb.slot >= 0) rows_covered = std::max(rows_covered, cb.tile_rows);
        const int64_t blocks = rows_covered > 0 ? (rows_covered + kRowScanBlock - 1) / kRowScanBlock : 1;
        unsigned epoch = 0;
        ChainSlot *slots = static_cast<ChainSlot *>(chain_prepare(ctx, blocks, &epoch, s));
        if (!slots) return cleanup(TSP_ERR_ALLOC_FAILED);
        hipLaunchKernelGGL(k_sym_row_scan, dim3((unsigned)blocks), dim3(kRowScanThreads), 0, s, ntr, row_c_tiles,
                           row_pairs, row_words, row_cand, P->c_tile_row_ptr, row_pair_ptr, slots, epoch,
                           ctx->d_scalars, ca, cb, ctx->h_scalars_dev, ++ctx->publish_tag);
        SYM_CHECK(hipGetLastError());
    }
    if (!rc) rc = wait_published_scalars(ctx, ctx->publish_tag, s);        // ---- sync 1: sizes of the task list
    if (rc) return cleanup(rc);
    const int64_t *h = ctx->h_scalars;
    if (h[S_INVALID]) return cleanup(TSP_ERR_NOT_CANONICAL);
    if (h[S_UNSUPPORTED]) return cleanup(TSP_ERR_UNSUPPORTED);
    if (h[S_INTERNAL]) return cleanup(TSP_ERR_HIP);
    if (A->ntiles < 0) A->ntiles = h[A->scalar_slot];
    if (B->ntiles < 0) B->ntiles = h[B->scalar_slot];
    P->c_tiles = h[S_C_TILES];
    P->pairs = h[S_PAIRS];
    P->candidates = h[S_CANDIDATES];
    P->max_row_c_tiles = h[S_MAX_ROW_C_TILES];
    P->max_row_pairs = h[S_MAX_ROW_PAIRS];
    if (P->c_tiles >= INT32_MAX) return cleanup(TSP_ERR_INDEX_OVERFLOW);

    P->c_tile_row = ctx_alloc_n<int32_t>(ctx, (size_t)P->c_tiles, s);
    P->c_tile_col = ctx_alloc_n<int32_t>(ctx, (size_t)P->c_tiles, s);
    P->pair_off = ctx_alloc_n<int64_t>(ctx, (size_t)P->c_tiles + 1, s);
    P->pair_ab = ctx_alloc_n<int2>(ctx, (size_t)P->pairs, s);
    P->c_row_mask = ctx_alloc_n<uint16_t>(ctx, (size_t)P->c_tiles * T, s);
    P->c_row_off = ctx_alloc_n<uint32_t>(ctx, (size_t)P->c_tiles * T, s);
    // padded to whole tile-rows: the numeric pass reads the 16 row starts of a tile-row unconditionally
    P->c_row_ptr = ctx_alloc_n<int64_t>(ctx, (size_t)P->c_tile_rows * T + T + 1, s);
    row_nnz = ctx_alloc_n<int32_t>(ctx, (size_t)P->c_rows + 1, s);
    tile_row_entries = ctx_alloc_n<uint32_t>(ctx, (size_t)ntr + 4, s);     // read four at a time
    if (!P->c_tile_row || !P->c_tile_col || !P->pair_off || !P->pair_ab || !P->c_row_mask ||
        !P->c_row_off || !P->c_row_ptr || !row_nnz || !tile_row_entries)
        return cleanup(TSP_ERR_ALLOC_FAILED);

    if (ntr > 0) {
        const int words_cap = (int)(h[S_MAX_ROW_WORDS] > 0 ? h[S_MAX_ROW_WORDS] : 1);
        int window = (int)(h[S_MAX_ROW_C_TILES] < kWindow ? h[S_MAX_ROW_C_TILES] : kWindow);
        if (window < 1) window = 1;
        const size_t lds = (size_t)(2 * words_cap + 2 * window) * sizeof(uint32_t);
        lanes = lanes_per_a_tile(B);
        long_rows = (double)B->ntiles > 48.0 * (double)B->tile_rows;
        // tile-rows with more C tiles than the LDS window holds are worked off in several windows and keep,
        // in one word per tile of A, where the previous window ended in B's tile-row
        if (h[S_MAX_ROW_C_TILES] > window) {
            cursor = ctx_alloc_n<int32_t>(ctx, 2 * (size_t)A->tile_capacity, s);    // and one per chunk of 32 of them
            if (!cursor) return cleanup(TSP_ERR_ALLOC_FAILED);
        }
        KernelTimer kt(ctx, TSP_KERNEL_SYM_EMIT, s);
        const int64_t per_row = P->candidates / ntr;
        // (the fused counting pass of the list kernel wants more lanes than the enumeration does)
        const int threads = per_row <= 256 ? 64 : per_row <= 512 ? 128 : kSymThreads;
        listed = h[S_MAX_ROW_PAIRS] <= kListCap && h[S_MAX_ROW_C_TILES] <= kListTiles;
        // LDS of the list kernel per tile-row: bitmap and its prefix, per-tile words of the window, the list, and
        // the row masks of the window when it also runs the counting pass.  A launch may ask for 64 KB: a product
        // against a very wide B (a bitmap of thousands of words) takes one tile-row per block instead of two
        // per wave, and the general kernel when even that does not fit.
        constexpr size_t kLdsLimit = 64 * 1024;
        constexpr int kTeamsPerWave = 64 / kListTeamLanes;
        const int list_cap = (int)std::max<int64_t>(h[S_MAX_ROW_PAIRS], 1);
        int team_words = 0;
        bool halves = false;
        if (listed) {
            fused_masks = ntr >= 1024;
            team_words = 2 * words_cap + 2 * window + 3 * list_cap + (fused_masks ? 8 * window : 0);
            // tile-rows with few candidates: two per wave (see k_sym_count_half)
            halves = fused_masks && threads == 64 && (size_t)team_words * kTeamsPerWave * sizeof(uint32_t) <= kLdsLimit;
            if ((size_t)team_words * sizeof(uint32_t) > kLdsLimit) {
                listed = false;
                fused_masks = false;
            }
        }
        ctx->hint_general = !listed;
        // (the order of the previous product goes; the general branch below may keep a new one)
        ctx_free(ctx, ctx->hint_order, s);
        ctx->hint_order = nullptr;
        ctx->hint_order_rows = 0;
        ctx->hint_sizes[0] = A->rows;
        ctx->hint_sizes[1] = A->nnz;
        ctx->hint_sizes[2] = B->rows;
        ctx->hint_sizes[3] = B->nnz;
        if (listed) {
            auto kernel = !fused_masks ? (long_rows ? k_sym_emit_listed<true, false, 0> : k_sym_emit_listed<false, false, 0>)
                          : halves     ? (long_rows ? k_sym_emit_listed<true, true, kListTeamLanes> : k_sym_emit_listed<false, true, kListTeamLanes>)
                                       : (long_rows ? k_sym_emit_listed<true, true, 0> : k_sym_emit_listed<false, true, 0>);
            hipLaunchKernelGGL(kernel, dim3((unsigned)(halves ? (ntr + kTeamsPerWave - 1) / kTeamsPerWave : ntr)),
                               dim3(halves ? 64 : fused_masks ? std::max(threads, 128) : threads),
                               (size_t)team_words * (halves ? kTeamsPerWave : 1) * sizeof(uint32_t), s, ra, rb,
                               halves ? std::min(lanes, 8) : lanes, words_cap, window, list_cap, team_words, row_jmin,
                               row_words, P->c_tile_row_ptr,
                               row_pair_ptr, P->c_tile_row, P->c_tile_col, P->pair_off, P->pair_ab,
                               A->row_mask, B->row_mask, P->c_row_mask, P->c_row_off, row_nnz, P->c_rows,
                               ctx->d_scalars, tile_row_entries);
        } else {
            // a few tile-rows far heavier than the rest (and enough work for two small launches to pay):
            // the heaviest go first
            const bool skewed =
                ntr >= 1024 && P->candidates >= (int64_t)1 << 22 && h[S_MAX_ROW_PAIRS] > 8 * (P->pairs / ntr + 1);
            if (ctx->work_order == 1 || (ctx->work_order == 0 && skewed)) {
                order = ctx_alloc_n<int32_t>(ctx, (size_t)ntr, s);
                order_hist = ctx_alloc_n<uint32_t>(ctx, 2 * kOrderBuckets, s);
                if (!order || !order_hist) return cleanup(TSP_ERR_ALLOC_FAILED);
                SYM_CHECK(hipMemsetAsync(order_hist, 0, 2 * kOrderBuckets * sizeof(uint32_t), s));
                const unsigned grid = (unsigned)((ntr + kOrderThreads * kOrderItems - 1) / (kOrderThreads * kOrderItems));
                hipLaunchKernelGGL(k_work_hist, dim3(grid), dim3(kOrderThreads), 0, s, ntr, row_cand, order_hist);
                hipLaunchKernelGGL(k_work_order, dim3(grid), dim3(kOrderThreads), 0, s, ntr, row_cand, order_hist,
                                   order_hist + kOrderBuckets, order);
                // the handle keeps the order: the counting kernel of the next call of this product starts with
                // the heaviest tile-rows too
                ctx->hint_order = order;
                ctx->hint_order_rows = ntr;
            }
            // tile-rows with very many candidates: larger blocks (each tile-row is one block's work, and the
            // longest ones end the launch; 256, 512, 768, 1024 threads: 69, 51, 54, 67 ms on the same graph)
            const int ethreads = per_row >= kLongRowCandidates ? kSymThreadsLong : threads;
            hipLaunchKernelGGL(long_rows ? k_sym_emit<true> : k_sym_emit<false>, dim3((unsigned)ntr), dim3(ethreads),
                               lds, s, ra, rb, lanes, words_cap, window, row_jmin, row_words,
                               P->c_tile_row_ptr,
                               row_pair_ptr, P->c_tile_row, P->c_tile_col, P->pair_off, P->pair_ab, cursor,
                               A->tile_capacity, order, saved_bitmap, saved_cnt, saved_words, P->pairs);
        }
        SYM_CHECK(hipGetLastError());
    } else {
        SYM_CHECK(hipMemsetAsync(P->pair_off, 0, sizeof(int64_t), s));
    }
    phase_end(ctx, TSP_PHASE_SYMBOLIC, s);

    phase_begin(ctx, TSP_PHASE_COUNT, s);
    // Long tile-rows of C (every one of them meets most tile-rows of B again): the kernels that walk the task
    // list take the output tiles in vertical strips, so that the part of B a strip needs stays in the L2 cache
    if (P->c_tiles > 0 && strips_wanted(ctx, P, B)) {
        rc = strips_build(ctx, P, B, s);
        if (rc) return cleanup(rc);
    }
    if (P->c_tiles > 0 && !fused_masks) {       // (otherwise the list kernel has done the counting pass already)
        // output tiles per workgroup: 64 where that still gives every CU dozens of workgroups (16, 32, 64 tiles:
        // 37.9, 35.2, 34.9 ms on an R-MAT graph of scale 18: fewer segment bounds and bitmaps to set up per entry)
        const int mask_tiles = P->strip_desc ? kMaskTilesStrips : P->c_tiles >= 64 * 8192 ? 64 : 16;
        int64_t blocks = (P->c_tiles + mask_tiles - 1) / mask_tiles;
        if (P->strip_desc) blocks = P->strip_capacity;                             // (an upper bound of the workgroups)
        // (short runs of blocks dealt to the XCDs in turn where the work is skewed: see numeric_enqueue)
        const bool skewed = P->max_row_pairs > 8 * (P->pairs / std::max<int64_t>(ntr, 1) + 1);
        const int xcd_chunk = skewed || P->strip_desc ? 8 : (int)std::max<int64_t>((blocks + 7) / 8, 1);
        const unsigned grid = (unsigned)xcd_chunked_grid(blocks, xcd_chunk);
        KernelTimer kt(ctx, TSP_KERNEL_COUNT_MASKS, s);
        hipLaunchKernelGGL(mask_tiles == 64 ? k_count_masks<64> : k_count_masks<16>,
                           dim3(grid), dim3(256), 0, s, P->c_tiles, P->pair_off, P->pair_ab,
                           A->row_mask, B->row_mask, P->c_row_mask, P->strip_desc,
                           P->strip_desc ? P->strip_block_ptr + P->strip_entries : nullptr, xcd_chunk);
    }
    if (ntr > 0 && !fused_masks) {             // (otherwise done by the list kernel as well)
        KernelTimer kt(ctx, TSP_KERNEL_ROW_OFFSETS, s);
        if (P->c_tiles >= 32 * ntr)                // tile-rows of 32 tiles and more on average: a block each
            hipLaunchKernelGGL(k_row_offsets_wide, dim3((unsigned)ntr), dim3(256), 0, s, P->c_rows, P->c_tile_row_ptr,
                               P->c_row_mask, P->c_row_off, row_nnz, ctx->d_scalars, tile_row_entries);
        else
            hipLaunchKernelGGL(k_row_offsets, dim3((unsigned)((ntr * 16 + 255) / 256)), dim3(256), 0, s, ntr, P->c_rows,
                               P->c_tile_row_ptr, P->c_row_mask, P->c_row_off, row_nnz, ctx->d_scalars,
                               tile_row_entries);
    }
    SYM_CHECK(hipGetLastError());
    bool published = false;                        // k_row_ptr puts the scalar block into the host's mirror
    {
        KernelTimer kt(ctx, TSP_KERNEL_SCAN_ROWS, s);
        if (n_chunks > 0 && n_chunks <= kMaxChunks) {
            hipLaunchKernelGGL(k_row_ptr, dim3((unsigned)n_chunks), dim3(256), 0, s, row_nnz, P->c_rows, tile_row_entries,
                               ntr, P->c_row_ptr, ctx->d_scalars, ctx->h_scalars_dev, ++ctx->publish_tag);
            SYM_CHECK(hipGetLastError());
            published = true;
        } else {
            rc = scan_exclusive_i32_to_i64(ctx, row_nnz, P->c_row_ptr, P->c_rows, ctx->d_scalars + S_C_NNZ,
                                           ctx->d_scalars + S_MAX_ROW_ENTRIES, tmp, s);
        }
    }
    phase_end(ctx, TSP_PHASE_COUNT, s);
    if (!rc) rc = published ? wait_published_scalars(ctx, ctx->publish_tag, s) : read_scalars(ctx, s);   // ---- sync 2: nnz(C)
    if (rc) return cleanup(rc);
    if (ctx->h_scalars[S_UNSUPPORTED]) return cleanup(TSP_ERR_UNSUPPORTED);
    if (ctx->h_scalars[S_INTERNAL]) return cleanup(TSP_ERR_HIP);
    P->c_nnz = ctx->h_scalars[S_C_NNZ];
    P->max_row_entries = ctx->h_scalars[S_MAX_ROW_ENTRIES];
    ctx->stats.a_tiles = A->ntiles;
    ctx->stats.b_tiles = B->ntiles;
    ctx->stats.candidate_pairs = P->candidates;
    ctx->stats.pairs = P->pairs;
    ctx->stats.c_tiles = P->c_tiles;
    ctx->stats.c_nnz = P->c_nnz;
    // the paper's selection criteria (Section 6.1) for the left operand
    ctx->stats.a_mean_row = A->rows > 0 ? (float)((double)A->nnz / (double)A->rows) : 0.f;
    ctx->stats.a_tile_fill = A->ntiles > 0 ? (float)((double)A->nnz / (double)A->ntiles) : 0.f;
    ctx->stats.in_paper_regime = A->nnz > 300000 && ctx->stats.a_mean_row > 42.f;
    ctx->stats.well_filled_tiles = ctx->stats.a_tile_fill >= 20.f;
    *out = P;
    return cleanup(TSP_OK);
}
#undef SYM_CHECK

}  // namespace tsp

using namespace tsp;

namespace tsp {
__global__ void k_clear_scalars_sym(int64_t *d_scalars) {
    if (threadIdx.x < kScalars) d_scalars[threadIdx.x] = 0;
}
}  // namespace tsp

extern "C" int tsp_symbolic(tsp_handle ctx, tsp_tiles A, tsp_tiles B, tsp_plan *out, void *stream) {
    if (!ctx || !A || !B || !out) return TSP_ERR_INVALID_ARG;
    if (A->ntiles < 0 || B->ntiles < 0) return TSP_ERR_INVALID_ARG;   // tiles must come from tsp_convert
    hipLaunchKernelGGL(k_clear_scalars_sym, dim3(1), dim3(64), 0, (hipStream_t)stream, ctx->d_scalars);
    ctx->scalars_clean = false;
    return symbolic_run(ctx, A, B, out, (hipStream_t)stream);
}

extern "C" int tsp_plan_free(tsp_handle ctx, tsp_plan plan, void *stream) {
    if (!ctx) return TSP_ERR_INVALID_ARG;
    plan_release(ctx, plan, (hipStream_t)stream);
    return TSP_OK;
}

extern "C" int tsp_plan_get_view(tsp_plan p, tsp_plan_view *v) {
    if (!p || !v) return TSP_ERR_INVALID_ARG;
    v->c_rows = p->c_rows;
    v->c_cols = p->c_cols;
    v->c_tile_rows = p->c_tile_rows;
    v->c_tiles = p->c_tiles;
    v->pairs = p->pairs;
    v->c_nnz = p->c_nnz;
    v->candidate_pairs = p->candidates;
    v->c_tile_row_ptr = p->c_tile_row_ptr;
    v->c_tile_row = p->c_tile_row;
    v->c_tile_col = p->c_tile_col;
    v->pair_off = p->pair_off;
    v->pair_ab = reinterpret_cast<const int32_t *>(p->pair_ab);
    v->c_row_mask = p->c_row_mask;
    v->c_row_off = p->c_row_off;
    v->c_row_ptr = p->c_row_ptr;
    return TSP_OK;
}
