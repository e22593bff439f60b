// The pipeline as the paper lays it out, at a tile edge T of 8, 16 or 32, kept beside the library's own
// path (convert.hip, symbolic.hip, numeric.hip) for two purposes: to show on the GPU that the result does
// not depend on the tile edge (the paper's tiles are 8x8, Section 2.1.2; this library's are 16x16), and to
// measure the paper's design choices against the ones made here on the same machine.
//
//   Section 2.1.2  tiles in the packed bitmap format: the non-empty T x T tiles in row-major order of the
//                  tile grid, per tile T row masks, the elements 2 bytes each in row-major order inside the
//                  tile, a pointer to the tile's first element.
//   Section 4.1 /  task list by expansion and sorting: every tile A[I,K] is paired with every tile B[K,J]
//   Algorithm 1    (expansion, sized by a prefix sum), pairs whose boolean tile product is empty are culled,
//                  a stable sort by (I,J) groups the pairs of an output tile and keeps K ascending inside a
//                  group, a run-length pass over the sorted keys gives the output tiles and the segment
//                  offsets.  The paper sorts with a library (Thrust); so does this file (rocPRIM's radix
//                  sort, a stable LSD sort).
//   Section 4.2    counting pass: boolean product of the bitmaps per output tile, entries per row, prefix sum.
//   Section 4.3    multiplication pass: one wave per output tile; for every pair the packed elements are
//                  placed by the bitmap into dense tiles in LDS, which are multiplied on the matrix cores
//                  (v_mfma_f32_16x16x16_f16; a 32x32 tile is 2x2 blocks of it, an 8x8 tile sits in the corner
//                  of one block), fp16 inputs, fp32 accumulation; the output tile is written to CSR by the
//                  ranks of its bitmap.
//
// Nothing here is tuned: a thread per element, per tile or per row, binary searches where the library's path
// keeps offsets, three to four host synchronisations per phase.  Every index a kernel forms comes from arrays
// the validation kernel or an earlier kernel of this file has bounded.
#include "common.hpp"

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include <algorithm>
#include <vector>

namespace tsp {
namespace paper {

constexpr int kThreads = 256;
inline unsigned grid_for(int64_t n) { return (unsigned)std::max<int64_t>(1, (n + kThreads - 1) / kThreads); }

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

struct Csr {                 // an operand as the kernels read it
    int64_t rows, cols, nnz;
    const int64_t *row_ptr;  // [rows + 1]
    const int32_t *col;      // [nnz]
    const uint16_t *val;     // [nnz] binary16 bit patterns
};

struct Tiles {               // Section 2.1.2 at tile edge T
    int64_t ntr = 0, ntc = 0, ntiles = 0;
    uint64_t *key = nullptr;        // [ntiles] tile row * ntc + tile column, ascending
    int32_t *elem_ptr = nullptr;    // [ntiles + 1] first packed element of a tile
    uint32_t *mask = nullptr;       // [ntiles * T] row masks
    uint32_t *row_occ = nullptr;    // [ntiles] bit r: row r of the tile holds an entry
    uint32_t *col_occ = nullptr;    // [ntiles] bit c: column c does
    uint16_t *elem = nullptr;       // [nnz] packed elements
    int32_t *tile_row_ptr = nullptr;   // [ntr + 1]
};

// ---- input -----------------------------------------------------------------------------------------------
template <typename R>
__global__ __launch_bounds__(kThreads) void k_rows64(const R *__restrict__ in, int64_t n, int64_t *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) out[i] = (int64_t)in[i];
}

__global__ __launch_bounds__(kThreads) void k_round_to_half(const float *__restrict__ in, int64_t n,
                                                            uint16_t *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) {
        const _Float16 h = (_Float16)in[i];          // round to nearest even (Section 2.6)
        out[i] = __builtin_bit_cast(uint16_t, h);
    }
}

// Canonical form (see the conventions of tsp.h); *bad is set to 1 otherwise.  A thread per row; the entry
// loop of a row runs only when the row's bounds lie inside [0, nnz].
__global__ __launch_bounds__(kThreads) void k_validate(Csr M, int64_t *bad) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= M.rows) return;
    const int64_t b = M.row_ptr[i], e = M.row_ptr[i + 1];
    bool ok = b >= 0 && e >= b && e <= M.nnz && (i != 0 || b == 0) && (i != M.rows - 1 || e == M.nnz);
    if (ok) {
        int64_t prev = -1;
        for (int64_t p = b; p < e; ++p) {
            const int64_t c = M.col[p];
            ok = ok && c > prev && c < M.cols;
            prev = c;
        }
    }
    if (!ok) *bad = 1;
}

// ---- Section 2.1.2: CSR -> tiles -----------------------------------------------------------------------------
// The row of entry e: the last row that starts at or before e (rows may be empty).
__device__ __forceinline__ int64_t last_at_or_before(const int64_t *__restrict__ ptr, int64_t n, int64_t e) {
    int64_t lo = 0, hi = n - 1;               // answer in [0, n-1], ptr[0] = 0 <= e
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (ptr[mid] <= e) lo = mid; else hi = mid - 1;
    }
    return lo;
}

template <int T>
__global__ __launch_bounds__(kThreads) void k_tile_keys(Csr M, int64_t ntc, uint64_t *__restrict__ key,
                                                        uint32_t *__restrict__ id, uint16_t *__restrict__ place) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= M.nnz) return;
    const int64_t row = last_at_or_before(M.row_ptr, M.rows, e);
    const int64_t col = M.col[e];
    key[e] = (uint64_t)(row / T) * (uint64_t)ntc + (uint64_t)(col / T);
    id[e] = (uint32_t)e;
    place[e] = (uint16_t)(((row % T) << 8) | (col % T));        // position inside the tile
}

// head[j] = 1 where a new key starts in the sorted keys (keys equal to `skip` start nothing)
__global__ __launch_bounds__(kThreads) void k_heads(const uint64_t *__restrict__ key, int64_t n, uint64_t skip,
                                                    int32_t *__restrict__ head) {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j < n) head[j] = key[j] != skip && (j == 0 || key[j] != key[j - 1]);
}

// Sorted entries -> tiles.  before[j] = heads before j, so entry j lies in tile before[j] + head[j] - 1.
template <int T>
__global__ __launch_bounds__(kThreads) void k_fill_tiles(int64_t n, int64_t ntiles, const uint64_t *__restrict__ skey,
                                                         const int32_t *__restrict__ head,
                                                         const int32_t *__restrict__ before,
                                                         const uint32_t *__restrict__ perm,
                                                         const uint16_t *__restrict__ place,
                                                         const uint16_t *__restrict__ val, Tiles t) {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j == 0) t.elem_ptr[ntiles] = (int32_t)n;
    if (j >= n) return;
    const int64_t tile = (int64_t)before[j] + head[j] - 1;
    if (tile < 0 || tile >= ntiles) return;                     // (never)
    if (head[j]) {
        t.key[tile] = skey[j];
        t.elem_ptr[tile] = (int32_t)j;
    }
    const uint32_t e = perm[j];
    if (e >= (uint64_t)n) return;                               // (never)
    const uint32_t p = place[e];
    atomicOr(&t.mask[tile * T + (p >> 8)], 1u << (p & 255u));
    t.elem[j] = val[e];            // the sort is stable: inside a tile the entries keep their CSR order, row-major
}

template <int T>
__global__ __launch_bounds__(kThreads) void k_occupancy(Tiles t) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= t.ntiles) return;
    uint32_t rows = 0, cols = 0;
    for (int r = 0; r < T; ++r) {
        const uint32_t m = t.mask[i * T + r];
        cols |= m;
        rows |= (m != 0u) << r;
    }
    t.row_occ[i] = rows;
    t.col_occ[i] = cols;
}

// ptr[I] = first sorted key at or past I * ntc, I = 0..ntr (ptr[ntr] = n)
__global__ __launch_bounds__(kThreads) void k_row_starts(const uint64_t *__restrict__ key, int64_t n, int64_t ntc,
                                                         int64_t ntr, int32_t *__restrict__ ptr) {
    const int64_t I = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (I > ntr) return;
    const uint64_t want = (uint64_t)I * (uint64_t)ntc;
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (key[mid] < want) lo = mid + 1; else hi = mid;
    }
    ptr[I] = (int32_t)lo;
}

// ---- Section 4.1, Algorithm 1: task list -------------------------------------------------------------------
// Tiles of B every tile of A meets: the length of B's tile-row K.
__global__ __launch_bounds__(kThreads) void k_expansion_sizes(Tiles A, Tiles B, int32_t *__restrict__ count) {
    const int64_t a = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (a >= A.ntiles) return;
    const int64_t K = (int64_t)(A.key[a] % (uint64_t)A.ntc);
    count[a] = K < B.ntr ? B.tile_row_ptr[K + 1] - B.tile_row_ptr[K] : 0;
}

// Candidate i: the pair (a, b) it stands for, its output tile as sort key, or `culled` when the boolean
// product of the two tiles is empty (no column of the A tile with an entry meets a row of the B tile with one).
__global__ __launch_bounds__(kThreads) void k_expand(int64_t n, const int64_t *__restrict__ first, Tiles A, Tiles B,
                                                     uint64_t culled, uint64_t *__restrict__ key,
                                                     uint64_t *__restrict__ pair) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int64_t a = last_at_or_before(first, A.ntiles, i);           // first[a] <= i < first[a + 1]
    const uint64_t ka = A.key[a];
    const int64_t I = (int64_t)(ka / (uint64_t)A.ntc), K = (int64_t)(ka % (uint64_t)A.ntc);
    uint64_t k = culled, ab = 0;
    if (K < B.ntr) {
        const int64_t b = (int64_t)B.tile_row_ptr[K] + (i - first[a]);
        if (b < B.tile_row_ptr[K + 1]) {
            const int64_t J = (int64_t)(B.key[b] % (uint64_t)B.ntc);
            if (A.col_occ[a] & B.row_occ[b]) k = (uint64_t)I * (uint64_t)B.ntc + (uint64_t)J;
            ab = ((uint64_t)a << 32) | (uint64_t)b;
        }
    }
    key[i] = k;
    pair[i] = ab;
}

// number of sorted keys below `culled` (they sort to the end)
__global__ void k_count_kept(const uint64_t *__restrict__ key, int64_t n, uint64_t culled, int64_t *out) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (key[mid] < culled) lo = mid + 1; else hi = mid;
    }
    *out = lo;
}

__global__ __launch_bounds__(kThreads) void k_output_tiles(int64_t kept, int64_t c_tiles, const uint64_t *__restrict__ key,
                                                           const int32_t *__restrict__ head,
                                                           const int32_t *__restrict__ before,
                                                           uint64_t *__restrict__ c_key, int64_t *__restrict__ pair_off) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i == 0) pair_off[c_tiles] = kept;
    if (i >= kept || !head[i]) return;
    const int64_t c = before[i];
    if (c >= c_tiles) return;                                   // (never)
    c_key[c] = key[i];
    pair_off[c] = i;
}

// ---- Section 4.2: counting pass ------------------------------------------------------------------------------
// Row r of output tile c: OR over the tile's pairs of the rows of the B tile that row r of the A tile selects.
template <int T>
__global__ __launch_bounds__(kThreads) void k_count_rows(int64_t c_tiles, const int64_t *__restrict__ pair_off,
                                                         const uint64_t *__restrict__ pair, Tiles A, Tiles B,
                                                         uint32_t *__restrict__ c_mask) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= c_tiles * T) return;
    const int64_t c = i / T;
    const int r = (int)(i % T);
    uint32_t out = 0;
    for (int64_t p = pair_off[c]; p < pair_off[c + 1]; ++p) {
        const uint64_t ab = pair[p];
        const int64_t a = (int64_t)(ab >> 32), b = (int64_t)(ab & 0xFFFFFFFFu);
        if (a >= A.ntiles || b >= B.ntiles) continue;           // (never)
        uint32_t sel = A.mask[a * T + r];
        while (sel) {
            const int k = __ffs(sel) - 1;
            sel &= sel - 1;
            out |= B.mask[b * T + k];
        }
    }
    c_mask[i] = out;
}

// Entries of every row of C, and per (output tile, row) the number of entries of that row in the tiles before it.
template <int T>
__global__ __launch_bounds__(kThreads) void k_row_lengths(int64_t padded_rows, const int32_t *__restrict__ c_row_start,
                                                          const uint32_t *__restrict__ c_mask,
                                                          uint32_t *__restrict__ c_off, int32_t *__restrict__ row_len) {
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (g >= padded_rows) return;
    const int64_t I = g / T;
    const int r = (int)(g % T);
    uint32_t run = 0;
    for (int64_t c = c_row_start[I]; c < c_row_start[I + 1]; ++c) {
        c_off[c * T + r] = run;
        run += __popc(c_mask[c * T + r]);
    }
    row_len[g] = (int32_t)run;
}

// ---- Section 4.3: multiplication pass, and the output tile to CSR ---------------------------------------------
template <int T>
__global__ __launch_bounds__(kThreads) void k_multiply(int64_t c_tiles, const uint64_t *__restrict__ c_key, int64_t c_ntc,
                                                       const int64_t *__restrict__ pair_off,
                                                       const uint64_t *__restrict__ pair, Tiles A, Tiles B,
                                                       const uint32_t *__restrict__ c_mask,
                                                       const uint32_t *__restrict__ c_off,
                                                       const int64_t *__restrict__ c_row_ptr, int64_t c_rows, int64_t c_nnz,
                                                       int32_t *__restrict__ c_col, float *__restrict__ c_val) {
    constexpr int TP = T < 16 ? 16 : T;       // edge of the dense tiles in LDS: whole 16x16 blocks
    constexpr int NB = TP / 16;
    __shared__ __align__(16) uint16_t lds_a[kThreads / 64][TP * TP], lds_b[kThreads / 64][TP * TP];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t c = (int64_t)blockIdx.x * (kThreads / 64) + wave;
    if (c >= c_tiles) return;                 // (the whole wave; the kernel has no block barrier)
    uint16_t *Ad = lds_a[wave], *Bd = lds_b[wave];
    float4_t acc[NB][NB];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) acc[bi][bj] = float4_t{0.f, 0.f, 0.f, 0.f};
    const int i16 = lane & 15, q = lane >> 4;
    for (int64_t p = pair_off[c]; p < pair_off[c + 1]; ++p) {
        const uint64_t ab = pair[p];
        const int64_t a = (int64_t)(ab >> 32), b = (int64_t)(ab & 0xFFFFFFFFu);
        if (a >= A.ntiles || b >= B.ntiles) continue;           // (never; uniform)
        wave_sync();                                            // the reads of the previous pair are done
        for (int i = lane; i < TP * TP / 8; i += 64) {
            reinterpret_cast<uint4 *>(Ad)[i] = make_uint4(0, 0, 0, 0);
            reinterpret_cast<uint4 *>(Bd)[i] = make_uint4(0, 0, 0, 0);
        }
        wave_sync();
        // lane r places row r of both tiles: its elements follow those of the rows before it
        uint32_t ma = lane < T ? A.mask[a * T + lane] : 0u, mb = lane < T ? B.mask[b * T + lane] : 0u;
        const uint32_t na = __popc(ma), nb = __popc(mb);
        int64_t ea = (int64_t)A.elem_ptr[a] + (wave_inclusive_scan(na) - na);
        int64_t eb = (int64_t)B.elem_ptr[b] + (wave_inclusive_scan(nb) - nb);
        const int64_t ea_end = A.elem_ptr[a + 1], eb_end = B.elem_ptr[b + 1];
        while (ma) {
            const int col = __ffs(ma) - 1;
            ma &= ma - 1;
            if (ea < ea_end) Ad[lane * TP + col] = A.elem[ea];
            ++ea;
        }
        while (mb) {
            const int col = __ffs(mb) - 1;
            mb &= mb - 1;
            if (eb < eb_end) Bd[lane * TP + col] = B.elem[eb];
            ++eb;
        }
        wave_sync();
#pragma unroll
        for (int kb = 0; kb < NB; ++kb) {
#pragma unroll
            for (int bi = 0; bi < NB; ++bi) {
                // A operand of a 16x16x16 step: lane holds row i16, inner indices 4q..4q+3
                const uint2 raw = *reinterpret_cast<const uint2 *>(&Ad[(bi * 16 + i16) * TP + kb * 16 + 4 * q]);
                const half4_t av = __builtin_bit_cast(half4_t, raw);
#pragma unroll
                for (int bj = 0; bj < NB; ++bj) {
                    // B operand: lane holds column i16, the same inner indices
                    uint16_t bits[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) bits[v] = Bd[(kb * 16 + 4 * q + v) * TP + bj * 16 + i16];
                    const uint2 packed = make_uint2((uint32_t)bits[0] | ((uint32_t)bits[1] << 16),
                                                    (uint32_t)bits[2] | ((uint32_t)bits[3] << 16));
                    const half4_t bv = __builtin_bit_cast(half4_t, packed);
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_16x16x16f16(av, bv, acc[bi][bj], 0, 0, 0);
                }
            }
        }
    }
    // the accumulator of a 16x16 block: lane holds rows 4q..4q+3 of column i16
    const uint64_t ck = c_key[c];
    const int64_t I = (int64_t)(ck / (uint64_t)c_ntc), J = (int64_t)(ck % (uint64_t)c_ntc);
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = bi * 16 + 4 * q + v, col = bj * 16 + i16;
                if (row >= T || col >= T) continue;
                const uint32_t m = c_mask[c * T + row];
                if (!((m >> col) & 1u)) continue;
                const int64_t g = I * T + row;
                if (g >= c_rows) continue;                      // (never: the bit comes from a stored entry)
                const int64_t pos = c_row_ptr[g] + (int64_t)c_off[c * T + row] + __popc(m & ((1u << col) - 1u));
                if (pos < c_nnz) {
                    c_col[pos] = (int32_t)(J * T + col);
                    c_val[pos] = acc[bi][bj][v];
                }
            }
}

// ---- host ----------------------------------------------------------------------------------------------------
struct Scope {               // device blocks of one call, returned to the handle's cache at the end
    tsp_context *ctx;
    hipStream_t s;
    std::vector<void *> owned;
    bool failed = false;
    template <typename Tp>
    Tp *get(int64_t n) {
        void *p = ctx_alloc(ctx, (size_t)std::max<int64_t>(n, 1) * sizeof(Tp), s);
        if (!p) failed = true; else owned.push_back(p);
        return static_cast<Tp *>(p);
    }
    void keep(void *p) { owned.erase(std::remove(owned.begin(), owned.end(), p), owned.end()); }
    ~Scope() { for (void *p : owned) ctx_free(ctx, p, s); }
};

#define PAPER_HIP(expr)                                            \
    do {                                                           \
        hipError_t e_ = (expr);                                    \
        if (e_ != hipSuccess) return hip_fail(ctx, e_);            \
    } while (0)
#define PAPER_ALLOC(scope) do { if ((scope).failed) return TSP_ERR_ALLOC_FAILED; } while (0)

static int read_back(tsp_context *ctx, const int64_t *d, int64_t *h, int n, hipStream_t s) {
    PAPER_HIP(hipMemcpyAsync(h, d, sizeof(int64_t) * n, hipMemcpyDeviceToHost, s));
    PAPER_HIP(hipStreamSynchronize(s));
    return TSP_OK;
}

static int bits_for(uint64_t largest_key) {
    int b = 1;
    while (b < 64 && (largest_key >> b)) ++b;
    return b;
}

template <typename V>
static int sort_pairs(tsp_context *ctx, Scope &sc, const uint64_t *key_in, uint64_t *key_out, const V *val_in, V *val_out,
                      int64_t n, int bits, hipStream_t s) {
    size_t bytes = 0;
    PAPER_HIP(rocprim::radix_sort_pairs(nullptr, bytes, key_in, key_out, val_in, val_out, (size_t)n, 0u, (unsigned)bits, s));
    void *tmp = sc.get<char>((int64_t)bytes);
    PAPER_ALLOC(sc);
    PAPER_HIP(rocprim::radix_sort_pairs(tmp, bytes, key_in, key_out, val_in, val_out, (size_t)n, 0u, (unsigned)bits, s));
    return TSP_OK;
}

// The operand in the form the kernels read, checked.
static int load_operand(tsp_context *ctx, Scope &sc, const tsp_csr *M, Csr *out, int64_t *d_flag, hipStream_t s) {
    if (M->rows < 0 || M->cols < 0 || M->nnz < 0) return TSP_ERR_INVALID_ARG;
    if (M->rows >= INT32_MAX - 16 || M->cols >= INT32_MAX - 16 || M->nnz >= INT32_MAX) return TSP_ERR_INDEX_OVERFLOW;
    if (!M->row_ptr || (M->nnz > 0 && (!M->col_idx || !M->val))) return TSP_ERR_INVALID_ARG;
    if (M->nnz > 0 && (M->rows == 0 || M->cols == 0)) return TSP_ERR_NOT_CANONICAL;
    if (M->row_ptr_type != TSP_I32 && M->row_ptr_type != TSP_I64) return TSP_ERR_INVALID_ARG;
    if (M->val_type != TSP_F16 && M->val_type != TSP_F32) return TSP_ERR_INVALID_ARG;
    int64_t *rows64 = sc.get<int64_t>(M->rows + 1);
    uint16_t *half = M->val_type == TSP_F32 ? sc.get<uint16_t>(M->nnz) : nullptr;
    PAPER_ALLOC(sc);
    if (M->row_ptr_type == TSP_I32)
        hipLaunchKernelGGL(k_rows64<int32_t>, dim3(grid_for(M->rows + 1)), dim3(kThreads), 0, s,
                           static_cast<const int32_t *>(M->row_ptr), M->rows + 1, rows64);
    else
        hipLaunchKernelGGL(k_rows64<int64_t>, dim3(grid_for(M->rows + 1)), dim3(kThreads), 0, s,
                           static_cast<const int64_t *>(M->row_ptr), M->rows + 1, rows64);
    if (half && M->nnz > 0)
        hipLaunchKernelGGL(k_round_to_half, dim3(grid_for(M->nnz)), dim3(kThreads), 0, s,
                           static_cast<const float *>(M->val), M->nnz, half);
    *out = Csr{M->rows, M->cols, M->nnz, rows64, M->col_idx, half ? half : static_cast<const uint16_t *>(M->val)};
    if (M->rows > 0) hipLaunchKernelGGL(k_validate, dim3(grid_for(M->rows)), dim3(kThreads), 0, s, *out, d_flag);
    PAPER_HIP(hipGetLastError());
    return TSP_OK;
}

template <int T>
static int make_tiles(tsp_context *ctx, Scope &sc, const Csr &M, Tiles *out, int64_t *d_scalar, hipStream_t s) {
    Tiles t;
    t.ntr = (M.rows + T - 1) / T;
    t.ntc = (M.cols + T - 1) / T;
    const int64_t n = M.nnz;
    t.tile_row_ptr = sc.get<int32_t>(t.ntr + 1);
    PAPER_ALLOC(sc);
    if (n == 0) {
        PAPER_HIP(hipMemsetAsync(t.tile_row_ptr, 0, sizeof(int32_t) * (size_t)(t.ntr + 1), s));
        t.key = sc.get<uint64_t>(1);
        t.elem_ptr = sc.get<int32_t>(1);
        t.mask = sc.get<uint32_t>(1);
        t.row_occ = sc.get<uint32_t>(1);
        t.col_occ = sc.get<uint32_t>(1);
        t.elem = sc.get<uint16_t>(1);
        PAPER_ALLOC(sc);
        PAPER_HIP(hipMemsetAsync(t.elem_ptr, 0, sizeof(int32_t), s));
        *out = t;
        return TSP_OK;
    }
    uint64_t *key = sc.get<uint64_t>(n), *skey = sc.get<uint64_t>(n);
    uint32_t *id = sc.get<uint32_t>(n), *perm = sc.get<uint32_t>(n);
    uint16_t *place = sc.get<uint16_t>(n);
    int32_t *head = sc.get<int32_t>(n), *before = sc.get<int32_t>(n + 1);
    int64_t *tmp = sc.get<int64_t>((int64_t)scan_tmp_entries(n));
    PAPER_ALLOC(sc);
    hipLaunchKernelGGL(k_tile_keys<T>, dim3(grid_for(n)), dim3(kThreads), 0, s, M, t.ntc, key, id, place);
    PAPER_HIP(hipGetLastError());
    int rc = sort_pairs<uint32_t>(ctx, sc, key, skey, id, perm, n, bits_for((uint64_t)t.ntr * (uint64_t)t.ntc), s);
    if (rc) return rc;
    hipLaunchKernelGGL(k_heads, dim3(grid_for(n)), dim3(kThreads), 0, s, skey, n, ~0ull, head);
    rc = scan_exclusive_i32_to_i32(ctx, head, before, n, d_scalar, nullptr, tmp, s);
    if (rc) return rc;
    int64_t ntiles = 0;
    rc = read_back(ctx, d_scalar, &ntiles, 1, s);
    if (rc) return rc;
    if (ntiles <= 0 || ntiles > n) return TSP_ERR_HIP;          // (never)
    t.ntiles = ntiles;
    t.key = sc.get<uint64_t>(ntiles);
    t.elem_ptr = sc.get<int32_t>(ntiles + 1);
    t.mask = sc.get<uint32_t>(ntiles * T);
    t.row_occ = sc.get<uint32_t>(ntiles);
    t.col_occ = sc.get<uint32_t>(ntiles);
    t.elem = sc.get<uint16_t>(n);
    PAPER_ALLOC(sc);
    PAPER_HIP(hipMemsetAsync(t.mask, 0, sizeof(uint32_t) * (size_t)ntiles * T, s));
    hipLaunchKernelGGL(k_fill_tiles<T>, dim3(grid_for(n)), dim3(kThreads), 0, s, n, ntiles, skey, head, before, perm,
                       place, M.val, t);
    hipLaunchKernelGGL(k_occupancy<T>, dim3(grid_for(ntiles)), dim3(kThreads), 0, s, t);
    hipLaunchKernelGGL(k_row_starts, dim3(grid_for(t.ntr + 1)), dim3(kThreads), 0, s, t.key, ntiles, t.ntc, t.ntr,
                       t.tile_row_ptr);
    PAPER_HIP(hipGetLastError());
    *out = t;
    return TSP_OK;
}

template <int T>
static int run(tsp_context *ctx, const tsp_csr *A_in, const tsp_csr *B_in, tsp_csr *C, hipStream_t s) {
    Scope sc{ctx, s};
    int64_t *d_scalars = sc.get<int64_t>(8);
    PAPER_ALLOC(sc);
    PAPER_HIP(hipMemsetAsync(d_scalars, 0, sizeof(int64_t) * 8, s));
    total_begin(ctx, s);
    phase_begin(ctx, TSP_PHASE_CONVERT, s);
    Csr A, B;
    int rc = load_operand(ctx, sc, A_in, &A, d_scalars + 7, s);
    if (!rc) rc = load_operand(ctx, sc, B_in, &B, d_scalars + 7, s);
    if (rc) return rc;
    int64_t bad = 0;
    rc = read_back(ctx, d_scalars + 7, &bad, 1, s);
    if (rc) return rc;
    if (bad) return TSP_ERR_NOT_CANONICAL;
    Tiles ta, tb;
    rc = make_tiles<T>(ctx, sc, A, &ta, d_scalars + 0, s);
    if (!rc) rc = make_tiles<T>(ctx, sc, B, &tb, d_scalars + 1, s);
    if (rc) return rc;
    phase_end(ctx, TSP_PHASE_CONVERT, s);

    // ---- task list
    phase_begin(ctx, TSP_PHASE_SYMBOLIC, s);
    const int64_t c_ntr = ta.ntr, c_ntc = tb.ntc;
    int64_t candidates = 0, kept = 0, c_tiles = 0;
    uint64_t *c_key = nullptr, *pair = nullptr;
    int64_t *pair_off = nullptr;
    int32_t *c_row_start = sc.get<int32_t>(c_ntr + 1);
    PAPER_ALLOC(sc);
    if (ta.ntiles > 0 && tb.ntiles > 0) {
        int32_t *count = sc.get<int32_t>(ta.ntiles);
        int64_t *first = sc.get<int64_t>(ta.ntiles + 1);
        int64_t *tmp = sc.get<int64_t>((int64_t)scan_tmp_entries(ta.ntiles));
        PAPER_ALLOC(sc);
        hipLaunchKernelGGL(k_expansion_sizes, dim3(grid_for(ta.ntiles)), dim3(kThreads), 0, s, ta, tb, count);
        rc = scan_exclusive_i32_to_i64(ctx, count, first, ta.ntiles, d_scalars + 2, nullptr, tmp, s);
        if (rc) return rc;
        rc = read_back(ctx, d_scalars + 2, &candidates, 1, s);
        if (rc) return rc;
        if (candidates >= INT32_MAX) return TSP_ERR_UNSUPPORTED;         // the sorted arrays are indexed with 32 bits
        if (candidates > 0) {
            const int64_t n = candidates;
            const uint64_t culled = (uint64_t)c_ntr * (uint64_t)c_ntc;   // one past the largest key
            uint64_t *key = sc.get<uint64_t>(n), *skey = sc.get<uint64_t>(n), *pr = sc.get<uint64_t>(n);
            pair = sc.get<uint64_t>(n);
            int32_t *head = sc.get<int32_t>(n), *before = sc.get<int32_t>(n + 1);
            int64_t *tmp2 = sc.get<int64_t>((int64_t)scan_tmp_entries(n));
            PAPER_ALLOC(sc);
            hipLaunchKernelGGL(k_expand, dim3(grid_for(n)), dim3(kThreads), 0, s, n, first, ta, tb, culled, key, pr);
            PAPER_HIP(hipGetLastError());
            rc = sort_pairs<uint64_t>(ctx, sc, key, skey, pr, pair, n, bits_for(culled), s);
            if (rc) return rc;
            hipLaunchKernelGGL(k_count_kept, dim3(1), dim3(1), 0, s, skey, n, culled, d_scalars + 3);
            hipLaunchKernelGGL(k_heads, dim3(grid_for(n)), dim3(kThreads), 0, s, skey, n, culled, head);
            rc = scan_exclusive_i32_to_i32(ctx, head, before, n, d_scalars + 4, nullptr, tmp2, s);
            if (rc) return rc;
            int64_t h[2] = {0, 0};
            rc = read_back(ctx, d_scalars + 3, h, 2, s);
            if (rc) return rc;
            kept = h[0];
            c_tiles = h[1];
            if (kept < 0 || kept > n || c_tiles < 0 || c_tiles > kept) return TSP_ERR_HIP;   // (never)
            c_key = sc.get<uint64_t>(c_tiles);
            pair_off = sc.get<int64_t>(c_tiles + 1);
            PAPER_ALLOC(sc);
            hipLaunchKernelGGL(k_output_tiles, dim3(grid_for(kept)), dim3(kThreads), 0, s, kept, c_tiles, skey, head,
                               before, c_key, pair_off);
            PAPER_HIP(hipGetLastError());
        }
    }
    if (c_tiles > 0)
        hipLaunchKernelGGL(k_row_starts, dim3(grid_for(c_ntr + 1)), dim3(kThreads), 0, s, c_key, c_tiles, c_ntc, c_ntr,
                           c_row_start);
    else
        PAPER_HIP(hipMemsetAsync(c_row_start, 0, sizeof(int32_t) * (size_t)(c_ntr + 1), s));
    phase_end(ctx, TSP_PHASE_SYMBOLIC, s);

    // ---- counting pass
    phase_begin(ctx, TSP_PHASE_COUNT, s);
    const int64_t padded_rows = c_ntr * T;
    uint32_t *c_mask = sc.get<uint32_t>(c_tiles * T), *c_off = sc.get<uint32_t>(c_tiles * T);
    int32_t *row_len = sc.get<int32_t>(padded_rows);
    int64_t *c_row_ptr = sc.get<int64_t>(A.rows + 1);
    int64_t *tmp3 = sc.get<int64_t>((int64_t)scan_tmp_entries(A.rows));
    PAPER_ALLOC(sc);
    if (c_tiles > 0)
        hipLaunchKernelGGL(k_count_rows<T>, dim3(grid_for(c_tiles * T)), dim3(kThreads), 0, s, c_tiles, pair_off, pair, ta,
                           tb, c_mask);
    if (padded_rows > 0)
        hipLaunchKernelGGL(k_row_lengths<T>, dim3(grid_for(padded_rows)), dim3(kThreads), 0, s, padded_rows, c_row_start,
                           c_mask, c_off, row_len);
    PAPER_HIP(hipGetLastError());
    rc = scan_exclusive_i32_to_i64(ctx, row_len, c_row_ptr, A.rows, d_scalars + 5, nullptr, tmp3, s);
    if (rc) return rc;
    int64_t c_nnz = 0;
    rc = read_back(ctx, d_scalars + 5, &c_nnz, 1, s);
    if (rc) return rc;
    phase_end(ctx, TSP_PHASE_COUNT, s);

    // ---- multiplication pass
    phase_begin(ctx, TSP_PHASE_NUMERIC, s);
    int32_t *c_col = sc.get<int32_t>(c_nnz);
    float *c_val = sc.get<float>(c_nnz);
    PAPER_ALLOC(sc);
    if (c_tiles > 0) {
        const int64_t blocks = (c_tiles + kThreads / 64 - 1) / (kThreads / 64);
        hipLaunchKernelGGL(k_multiply<T>, dim3((unsigned)blocks), dim3(kThreads), 0, s, c_tiles, c_key, c_ntc, pair_off,
                           pair, ta, tb, c_mask, c_off, c_row_ptr, A.rows, c_nnz, c_col, c_val);
        PAPER_HIP(hipGetLastError());
    }
    phase_end(ctx, TSP_PHASE_NUMERIC, s);
    total_end(ctx, s);
    if (ctx->timers) {
        PAPER_HIP(hipStreamSynchronize(s));
        collect_timers(ctx);
    }
    sc.keep(c_row_ptr);
    sc.keep(c_col);
    sc.keep(c_val);
    C->rows = A.rows;
    C->cols = B.cols;
    C->nnz = c_nnz;
    C->row_ptr = c_row_ptr;
    C->col_idx = c_col;
    C->val = c_val;
    C->row_ptr_type = TSP_I64;
    C->val_type = TSP_F32;
    ctx->stats.a_tiles = ta.ntiles;
    ctx->stats.b_tiles = tb.ntiles;
    ctx->stats.candidate_pairs = candidates;
    ctx->stats.pairs = kept;
    ctx->stats.c_tiles = c_tiles;
    ctx->stats.c_nnz = c_nnz;
    ctx->stats.products = -1;
    return TSP_OK;
}

}  // namespace paper
}  // namespace tsp

extern "C" int tsp_spgemm_paper(tsp_handle ctx, int tile_edge, const tsp_csr *A, const tsp_csr *B, tsp_csr *C,
                                void *stream) {
    if (!ctx || !A || !B || !C) return TSP_ERR_INVALID_ARG;
    std::memset(C, 0, sizeof(*C));
    if (tile_edge != 8 && tile_edge != 16 && tile_edge != 32) return TSP_ERR_INVALID_ARG;
    if (A->cols != B->rows) return TSP_ERR_SHAPE_MISMATCH;
    hipStream_t s = (hipStream_t)stream;
    switch (tile_edge) {
        case 8: return tsp::paper::run<8>(ctx, A, B, C, s);
        case 16: return tsp::paper::run<16>(ctx, A, B, C, s);
        default: return tsp::paper::run<32>(ctx, A, B, C, s);
    }
}
