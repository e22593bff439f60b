// Internal declarations shared by the translation units of libtsp.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "tsp.h"

namespace tsp {

constexpr int T = 16;               // tile edge: one output tile = one 16x16 MFMA accumulator
constexpr int kScalars = 32;        // device/host scalar slots of a handle

// Slots of the handle's device scalar block (int64 each).
enum Scalar {
    S_INVALID = 0,       // != 0: an input CSR is not canonical
    S_UNSUPPORTED = 1,   // != 0: a documented limit was exceeded on the device
    S_TILES_A = 2,
    S_TILES_B = 3,
    S_C_TILES = 4,
    S_PAIRS = 5,
    S_CANDIDATES = 6,
    S_MAX_ROW_C_TILES = 7,   // max over C tile-rows of the number of C tiles
    S_MAX_ROW_WORDS = 8,     // max over C tile-rows of bitmap words needed
    S_C_NNZ = 9,
    S_MAX_ROW_A_TILES = 10,
    S_INTERNAL = 11,         // != 0: a bounded device-side wait ran out (should never happen)
    S_MAX_ROW_PAIRS = 12,    // max over C tile-rows of the number of task-list entries
    S_MAX_ROW_ENTRIES = 13,  // max over C tile-rows of the number of structural entries
    S_PRODUCTS = 14,         // intermediate products (TSP_OPT_COUNT_PRODUCTS)
    S_PUBLISHED = 31,        // host mirror only: a slot without a value (publish_scalars tags every slot)
};

struct Block {
    void *ptr;
    size_t bytes;
};
struct LiveBlock {           // a block handed out: with canaries the caller's part starts one guard zone into it
    void *base;
    size_t bytes;            // of the whole block
    size_t user_bytes;       // of the caller's part (a multiple of 256)
    bool guarded;
};

}  // namespace tsp

struct tsp_context {
    tsp_allocator allocator{};
    bool user_allocator = false;
    int device = 0;
    std::vector<tsp::Block> cache;                 // free blocks, reusable
    std::unordered_map<void *, tsp::LiveBlock> live;   // blocks handed out, by the pointer the caller got
    int canaries = 0;                              // TSP_OPT_WORKSPACE_CANARIES
    bool canaries_used = false;                    // ... has been on at some time: the counter is worth reading
    int64_t held_bytes = 0, peak_bytes = 0;
    int validate = 1;
    int timers = 0;
    int force_wide = 0;                            // use the 64-bit-pointer kernels whatever the sizes
    int work_order = 0;                            // TSP_OPT_WORK_ORDER
    int strip_order = 0;                           // TSP_OPT_STRIP_ORDER
    int count_products = 0;                        // TSP_OPT_COUNT_PRODUCTS
    int numeric_run_len = 0;                       // tiles per wave of the multiplication kernel, 0: automatic
    int matrix_cores = 1;                          // 0: block products on the vector ALUs
    int compact = 0;                               // 1: tsp_spgemm removes zero-valued entries from C
    bool hint_general = false;                     // the last product took the general task-list kernel ...
    int64_t hint_sizes[4] = {-1, -1, -1, -1};      // ... with these rows and nnz of A and of B
    int32_t *hint_order = nullptr;                 // ... and took its tile-rows in this order (heaviest first), or null
    int64_t hint_order_rows = 0;
    int last_hip = 0;
    tsp_stats stats{};
    void *chain_slots = nullptr;                   // device, for the chained scans (chain.hpp)
    int64_t chain_capacity = 0;                    // slots allocated
    unsigned chain_epoch = 0;                      // tag of the last chained scan
    int64_t *d_scalars = nullptr;                  // device, kScalars entries
    bool scalars_clean = false;                    // all zero: the previous tsp_spgemm left them so
    int64_t *h_scalars = nullptr;                  // pinned host mirror
    int64_t *h_scalars_dev = nullptr;              // the mirror's address on the device
    int64_t publish_tag = 0;                       // tag of the last publication asked for
    hipEvent_t ev[2 * TSP_PHASE_COUNT_ + 2]{};     // begin/end per phase, + total begin/end
    bool ev_created = false;
    bool ev_recorded[2 * TSP_PHASE_COUNT_ + 2]{};
    hipEvent_t kev[2 * TSP_KERNEL_COUNT_]{};       // begin/end per kernel
    bool kev_recorded[TSP_KERNEL_COUNT_]{};
};

struct tsp_tiles_s {
    int64_t rows = 0, cols = 0, nnz = 0;
    int64_t tile_rows = 0, tile_cols = 0;
    int64_t ntiles = -1;                 // -1 until read back from the device
    int64_t tile_capacity = 0;
    int forms = 0;
    int scalar_slot = 0;                 // S_TILES_A or S_TILES_B: where the device leaves ntiles
    int32_t *tile_row_ptr = nullptr;               // first tile slot of every tile-row
    int32_t *tile_row_end = nullptr;               // one past its last tile
    int32_t *tile_col = nullptr;
    uint16_t *row_mask = nullptr;
    uint32_t *lmask = nullptr, *rmask = nullptr;
    uint2 *lhead = nullptr, *rhead = nullptr;      // per form: {group mask, index of the tile's first group}
    uint4 *ldata = nullptr, *rdata = nullptr;
    int64_t group_capacity = 0;
};

struct tsp_plan_s {
    int64_t c_rows = 0, c_cols = 0, c_tile_rows = 0;
    int64_t c_tiles = 0, pairs = 0, c_nnz = 0, candidates = 0;
    int64_t max_row_c_tiles = 0, max_row_pairs = 0, max_row_entries = 0;   // largest tile-row of C
    int32_t *c_tile_row_ptr = nullptr;
    int32_t *c_tile_row = nullptr, *c_tile_col = nullptr;
    int64_t *pair_off = nullptr;
    int2 *pair_ab = nullptr;                 // task list: {tile of A, tile of B} per entry
    uint16_t *c_row_mask = nullptr;
    uint32_t *c_row_off = nullptr;
    int64_t *c_row_ptr = nullptr;
    // order of work in vertical strips (strips.hip), absent for short tile-rows of C
    int2 *strip_desc = nullptr;              // per workgroup {first output tile, tiles (0: none)}
    int64_t strip_capacity = 0;              // descriptors allocated: an upper bound of the workgroups
    int32_t *strip_block_ptr = nullptr;      // [strip_entries + 1]; the last entry is the number of workgroups
    int64_t strip_entries = 0;
};

namespace tsp {

// ---- host helpers (context.hip) -------------------------------------------------------
void *ctx_alloc(tsp_context *ctx, size_t bytes, hipStream_t s);          // NULL on failure
void ctx_free(tsp_context *ctx, void *p, hipStream_t s);                 // back into the cache
int hip_fail(tsp_context *ctx, hipError_t e);                            // records e, returns TSP_ERR_HIP
int read_scalars(tsp_context *ctx, hipStream_t s);                       // d_scalars -> h_scalars, syncs
// row_ptr[0..rows] = exclusive prefix of row_len[0..rows) in one launch, the total into S_C_NNZ of the
// scalar block, which the launch also hands to the host (wait_published_scalars with ctx->publish_tag).
// group_len[g] = sum of row_len over rows 16g..16g+15, padded with zeros to a multiple of four entries.
// Returns false, without launching anything, for more rows than one launch covers.
bool row_ptr_in_one_launch(tsp_context *ctx, const int32_t *row_len, int64_t rows, const uint32_t *group_len,
                           int64_t *row_ptr, hipStream_t s);
// Waits until the kernel that was given `tag` has put the scalar block into h_scalars (publish_scalars).
int wait_published_scalars(tsp_context *ctx, int64_t tag, hipStream_t s);
// Slots for a chained scan over `blocks` blocks and a fresh epoch tag; nullptr on failure.
void *chain_prepare(tsp_context *ctx, int64_t blocks, unsigned *epoch, hipStream_t s);
void phase_begin(tsp_context *ctx, int phase, hipStream_t s);
void phase_end(tsp_context *ctx, int phase, hipStream_t s);
void total_begin(tsp_context *ctx, hipStream_t s);
void total_end(tsp_context *ctx, hipStream_t s);
void collect_timers(tsp_context *ctx);                                   // after a sync

// Brackets the kernel launches inside its scope with events when the handle's timers are on.
struct KernelTimer {
    tsp_context *ctx;
    int id;
    hipStream_t s;
    KernelTimer(tsp_context *c, int kernel_id, hipStream_t stream);
    ~KernelTimer();
};

template <typename Tp>
inline Tp *ctx_alloc_n(tsp_context *ctx, size_t n, hipStream_t s) {
    return static_cast<Tp *>(ctx_alloc(ctx, (n ? n : 1) * sizeof(Tp), s));
}

#define TSP_HIP_CHECK(ctx, expr)                                   \
    do {                                                           \
        hipError_t e_ = (expr);                                    \
        if (e_ != hipSuccess) return ::tsp::hip_fail((ctx), e_);   \
    } while (0)

// ---- scans (scan.hip) -----------------------------------------------------------------
// out[i] = sum of in[0..i), i = 0..n (n+1 entries).  If d_total != nullptr, *d_total = out[n]
// as int64; if d_max != nullptr, *d_max = the largest sum of 16 consecutive inputs in[16k..16k+16)
// (the entries of a tile-row, when the inputs are row lengths), 0 for n = 0.
// tmp: workspace of scan_tmp_entries(n) int64.
size_t scan_tmp_entries(int64_t n);
int scan_exclusive_i32_to_i32(tsp_context *ctx, const int32_t *in, int32_t *out, int64_t n,
                              int64_t *d_total, int64_t *d_max, int64_t *tmp, hipStream_t s);
int scan_exclusive_i32_to_i64(tsp_context *ctx, const int32_t *in, int64_t *out, int64_t n,
                              int64_t *d_total, int64_t *d_max, int64_t *tmp, hipStream_t s);

// ---- phases (internal forms; the C ABI wraps them) -------------------------------------
int convert_enqueue(tsp_context *ctx, const tsp_csr *A, int forms, int scalar_slot, tsp_tiles_s **out,
                    hipStream_t s);
void tiles_release(tsp_context *ctx, tsp_tiles_s *t, hipStream_t s);
int symbolic_run(tsp_context *ctx, tsp_tiles_s *A, tsp_tiles_s *B, tsp_plan_s **out, hipStream_t s);
void plan_release(tsp_context *ctx, tsp_plan_s *p, hipStream_t s);
// Order of work in vertical strips for the kernels that walk the task list of a plan with long tile-rows.
int strips_build(tsp_context *ctx, tsp_plan_s *P, const tsp_tiles_s *B, hipStream_t s);
// last_of_call (tsp_spgemm): C gets the plan's row_ptr array itself instead of a copy, so the plan cannot
// be used again, and the kernel zeroes the handle's scalar block, which nothing reads any more, for the
// next call (one launch less per call).
int numeric_enqueue(tsp_context *ctx, tsp_tiles_s *A, tsp_tiles_s *B, tsp_plan_s *plan, tsp_csr *C,
                    hipStream_t s, bool last_of_call = false);
// taken (may be null): the caller owns C and gives it up; when no entry is zero *out takes C's arrays as they
// are (no copy) and *taken is set, so that the caller does not free them.
int compact_zeros(tsp_context *ctx, const tsp_csr *C, tsp_csr *out, hipStream_t s, bool *taken);
// Looks up, once per device, the address of the fixed scratch array behind tsp_compact_zeros_static on the
// current device (tsp_create calls it, so that the entry point itself finds the pointer ready).
int static_scratch_setup(tsp_context *ctx, unsigned char **ptr);

#ifdef __HIPCC__
// ---- device helpers -------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Orders LDS traffic between the lanes of one wave (no block barrier needed).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup b of a launch runs on XCD b % 8, each XCD with an L2 cache of its own.  Logical block index
// for workgroup b such that `chunk` consecutive logical blocks run on one XCD (and share its L2) and the
// chunks are dealt to the XCDs in turn (so that a part of the index range that is heavier than the rest
// does not fall to one XCD).  chunk = ceil(blocks / 8) gives every XCD one contiguous eighth.  The launch
// must cover ceil(blocks / (8 chunk)) * 8 chunk workgroups; indices past `blocks` have nothing to do.
__device__ __forceinline__ int64_t xcd_chunked_index(unsigned b, int chunk) {
    const unsigned q = b >> 3, x = b & 7u;
    return ((int64_t)(q / (unsigned)chunk) * 8 + x) * chunk + q % (unsigned)chunk;
}
inline int64_t xcd_chunked_grid(int64_t blocks, int chunk) {
    const int64_t span = 8 * (int64_t)chunk;
    return (blocks + span - 1) / span * span;
}

// The scalar block copied into the host's pinned mirror by the block of a kernel that knows every other
// writer of the block has finished (all threads of that block call this, at least kScalars of them).  The
// host polls the mirror: it has the sizes it waits for as soon as they exist, without a copy (a launch of
// its own) and without waiting for the queue to drain.  Every 8-byte slot carries the publication's tag in
// its top 16 bits (the scalars are counts below 2^48), so the host knows a slot is new by the slot itself:
// no store has to be ordered behind another across the bus, and the kernel does not wait for a fence.
constexpr int kPublishTagShift = 48;
__host__ __device__ inline uint64_t publish_tag16(int64_t tag) { return (uint64_t)(tag % 65535) + 1u; }   // never 0
__device__ __forceinline__ void publish_scalars(int64_t *d_scalars, int64_t *h_scalars_dev, int64_t tag) {
    __threadfence();                               // this block's own plain stores to the scalar block
    __syncthreads();
    if (threadIdx.x < kScalars) {
        const uint64_t v = threadIdx.x == S_PUBLISHED
                               ? 0u
                               : (uint64_t)__hip_atomic_load(&d_scalars[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t slot = (publish_tag16(tag) << kPublishTagShift) | (v & ((1ull << kPublishTagShift) - 1u));
        __hip_atomic_store(&h_scalars_dev[threadIdx.x], (int64_t)slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Cross-lane operations on the data-parallel-primitive path (VALU speed, no LDS round trips).
// A "row" is 16 consecutive lanes; row_ror rotates inside a row, row_shr shifts inside a row,
// row_bcast:15 / row_bcast:31 carry a row's (half-wave's) last lane into the following rows.
#define TSP_DPP(old, src, ctrl, row_mask, bound) \
    __builtin_amdgcn_update_dpp((old), (src), (ctrl), (row_mask), 0xf, (bound))

__device__ __forceinline__ int group16_min(int v) {          // all 16 lanes of the row get the minimum
    v = min(v, TSP_DPP(v, v, 0x128, 0xf, false));
    v = min(v, TSP_DPP(v, v, 0x124, 0xf, false));
    v = min(v, TSP_DPP(v, v, 0x122, 0xf, false));
    v = min(v, TSP_DPP(v, v, 0x121, 0xf, false));
    return v;
}
__device__ __forceinline__ uint32_t group16_or(uint32_t v) {
    v |= (uint32_t)TSP_DPP((int)v, (int)v, 0x128, 0xf, false);
    v |= (uint32_t)TSP_DPP((int)v, (int)v, 0x124, 0xf, false);
    v |= (uint32_t)TSP_DPP((int)v, (int)v, 0x122, 0xf, false);
    v |= (uint32_t)TSP_DPP((int)v, (int)v, 0x121, 0xf, false);
    return v;
}
// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    int v = (int)x;
    v += TSP_DPP(0, v, 0x111, 0xf, true);     // row_shr:1
    v += TSP_DPP(0, v, 0x112, 0xf, true);     // row_shr:2
    v += TSP_DPP(0, v, 0x114, 0xf, true);     // row_shr:4
    v += TSP_DPP(0, v, 0x118, 0xf, true);     // row_shr:8
    v += TSP_DPP(0, v, 0x142, 0xa, false);    // row_bcast:15 into rows 1 and 3
    v += TSP_DPP(0, v, 0x143, 0xc, false);    // row_bcast:31 into rows 2 and 3
    return (uint32_t)v;
}
// The same for 64-bit values below 2^46: the low 20 bits and the rest are scanned separately
// (sums of 64 such parts fit 32 bits) and recombined; addition is linear, so this is exact.
__device__ __forceinline__ uint64_t wave_inclusive_scan64(uint64_t x) {
    const uint32_t lo = wave_inclusive_scan((uint32_t)x & 0xFFFFFu), hi = wave_inclusive_scan((uint32_t)(x >> 20));
    return ((uint64_t)hi << 20) + lo;
}
// Exclusive prefix of one 64-bit value per thread over a block of kThreads threads (every thread
// of the block calls it); *total receives the block total.  lds: kThreads/64 words of scratch.
template <int kThreads>
__device__ __forceinline__ uint64_t block_exclusive_scan64(uint64_t x, uint64_t *total, uint64_t *lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t inc = wave_inclusive_scan64(x);
    __syncthreads();                       // lds may still be in use by a previous call
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const uint64_t y = lds[w];
        if (w < wave) before += y;
        all += y;
    }
    *total = all;
    return before + inc - x;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {   // total in every lane
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(x), 63);
}
__device__ __forceinline__ int wave_max(int v) {             // maximum in every lane
    v = max(v, TSP_DPP(v, v, 0x111, 0xf, false));
    v = max(v, TSP_DPP(v, v, 0x112, 0xf, false));
    v = max(v, TSP_DPP(v, v, 0x114, 0xf, false));
    v = max(v, TSP_DPP(v, v, 0x118, 0xf, false));
    v = max(v, TSP_DPP(v, v, 0x142, 0xa, false));
    v = max(v, TSP_DPP(v, v, 0x143, 0xc, false));
    return __builtin_amdgcn_readlane(v, 63);
}
// 16-bit slice of a wave ballot that belongs to this lane's 16-lane group.
__device__ __forceinline__ uint32_t group16_ballot(bool pred) {
    unsigned long long b = __ballot(pred);
    return (uint32_t)(b >> (lane_id() & 48)) & 0xFFFFu;
}
__device__ __forceinline__ uint32_t fold16(uint32_t m) { return (m | (m >> 16)) & 0xFFFFu; }
#endif

}  // namespace tsp
