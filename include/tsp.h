/*
 * tsp - tiled mixed-precision sparse matrix-matrix multiply C = A*B for AMD MI355X (gfx950).
 *
 * C ABI of libtsp.so.  The library follows the tSparse pipeline (paper Sections 3 and 4,
 * Algorithm 1): CSR inputs are cut into 16x16 tiles of which only the non-empty ones are
 * kept, with an occupancy bitmap each (Section 2.1.2); a task list of contributing
 * (A tile, B tile) pairs is built per output tile, sorted by output tile (Section 4.1); a
 * counting pass sizes the output from the bitmaps alone (Section 4.2); the multiplication
 * pass multiplies every pair as a small dense block, fp16 inputs with fp32 accumulation
 * (Sections 2.6 and 4.3), on the matrix cores; the result is written back as CSR.
 *
 * Conventions
 *  - Every function returns TSP_OK (0) or a negative tsp_status.  No exceptions, no aborts.
 *  - All matrix arrays are DEVICE pointers.  Structs and out-parameters are HOST memory.
 *  - `stream` arguments are a hipStream_t passed as void* (NULL = the default stream).  All
 *    device work of a call is enqueued on that stream.  Calls that have to size an allocation
 *    synchronise the stream; each function says how often.
 *  - A handle may be used by one host thread and one stream at a time.
 *  - CSR inputs must be canonical: row_ptr[0] = 0, row_ptr non-decreasing, row_ptr[rows] = nnz,
 *    column indices inside [0, cols) and strictly ascending within a row.  With validation on
 *    (the default) a violation returns TSP_ERR_NOT_CANONICAL; with it off the behaviour is
 *    undefined.  A stored entry is structural whatever its value (an explicit 0.0 counts).
 *  - The output pattern is structural: position (i,j) is present when some k has a_ik and
 *    b_kj stored, also when the terms cancel (the counting pass of Section 4.2 defines the
 *    size).  The numeric-zero compaction of Section 4.4 is a separate call,
 *    tsp_compact_zeros, or the option TSP_OPT_COMPACT_ZEROS.
 */
#ifndef TSP_H
#define TSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TSP_OK = 0,
    TSP_ERR_INVALID_ARG = -1,     /* NULL pointer, negative size, unknown enum value                  */
    TSP_ERR_SHAPE_MISMATCH = -2,  /* A.cols != B.rows                                                 */
    TSP_ERR_NOT_CANONICAL = -3,   /* input CSR violates the conventions above (validation on)         */
    TSP_ERR_ALLOC_FAILED = -4,    /* the device allocator returned NULL                               */
    TSP_ERR_INDEX_OVERFLOW = -5,  /* a size exceeds the index width of the format (see tsp_csr)       */
    TSP_ERR_HIP = -6,             /* a HIP runtime call failed; tsp_last_hip_error() has the code     */
    TSP_ERR_UNSUPPORTED = -7      /* a documented limit of this build is exceeded                     */
} tsp_status;

enum { TSP_I32 = 0, TSP_I64 = 1 };   /* row_ptr element type   */
enum { TSP_F16 = 0, TSP_F32 = 1 };   /* value element type     */

/*
 * CSR matrix, device arrays.  Inputs: row_ptr is int32[rows+1] (TSP_I32) or int64[rows+1]
 * (TSP_I64); col_idx is int32[nnz]; val is IEEE binary16 bit patterns uint16[nnz] (TSP_F16) or
 * float[nnz] (TSP_F32, rounded to nearest-even fp16 on the device before use, the input
 * conversion the paper includes in its timing, Section 6.3).  Limits: rows, cols < 2^31 - 16,
 * nnz < 2^31.  Outputs of this library: row_ptr int64[rows+1], col_idx int32[nnz], val
 * float[nnz].
 */
typedef struct {
    int64_t rows, cols, nnz;
    void *row_ptr;
    int32_t *col_idx;
    void *val;
    int32_t row_ptr_type;   /* TSP_I32 | TSP_I64 */
    int32_t val_type;       /* TSP_F16 | TSP_F32 */
} tsp_csr;

/*
 * Device allocator used for every workspace and output array.  alloc returns a device pointer
 * aligned to at least 256 bytes, or NULL; free releases a pointer alloc returned.  Both are
 * called from the host thread that calls the library; `stream` is the stream of that call.
 * The handle keeps freed blocks in a cache of its own and reuses them, so in the steady state
 * (same problem sizes call after call) the callbacks are not invoked.
 */
typedef struct {
    void *(*alloc)(void *user, size_t bytes, void *stream);
    void (*free)(void *user, void *ptr, void *stream);
    void *user;
} tsp_allocator;

typedef struct tsp_context *tsp_handle;
typedef struct tsp_tiles_s *tsp_tiles;   /* a matrix in tile (bitmap) format, device resident */
typedef struct tsp_plan_s *tsp_plan;     /* task list + output pattern of one product          */

/* Option keys for tsp_set_option. */
enum {
    TSP_OPT_VALIDATE = 1,      /* 1 (default): check that CSR inputs are canonical                 */
    TSP_OPT_PHASE_TIMERS = 2,  /* 1: bracket every phase with HIP events on the call's stream and   */
                               /*    report the durations in tsp_stats; 0 (default): no events      */
    TSP_OPT_WIDE_INDEX = 3,    /* 1: always use the kernels that address arrays of 4 GiB and more   */
                               /*    through 64-bit pointers; 0 (default): chosen from the sizes    */
    TSP_OPT_NUMERIC_RUN = 4,   /* output tiles one wave of the multiplication kernel walks: 4 or 8; */
                               /*    0 (default): 4, or a whole tile-row of C where every tile-row  */
                               /*    has at most 60 tiles, 64 task-list entries and 448 entries     */
    TSP_OPT_MATRIX_CORES = 5,  /* 1 (default): block products on the MFMA units (Section 4.3);      */
                               /*    0: on the vector ALUs, one fp32 FMA per inner index and output */
                               /*    element (the paper's comparison build, Section 5, Algorithm 2) */
    TSP_OPT_COMPACT_ZEROS = 6, /* 1: tsp_spgemm finishes with tsp_compact_zeros (the compaction     */
                               /*    steps that end Algorithm 1); 0 (default): C keeps every        */
                               /*    structural position                                            */
    TSP_OPT_WORK_ORDER = 7,    /* order in which the general task-list kernel takes the tile-rows   */
                               /*    of C: 1: heaviest first (by candidate pairs, Section 4.1),     */
                               /*    2: by index, 0 (default): heaviest first where a few tile-rows */
                               /*    are far heavier than the rest.  The result does not depend on  */
                               /*    it                                                             */
    TSP_OPT_COUNT_PRODUCTS = 10, /* 1: tsp_spgemm also counts the intermediate products (one small    */
                               /*    kernel over the entries of A) and reports them in tsp_stats;    */
                               /*    0 (default): tsp_stats.products = -1                            */
    TSP_OPT_WORKSPACE_CANARIES = 11, /* 1: every block the handle takes from the allocator from now on (workspace */
                               /*    and outputs) carries a guard zone of 256 bytes in front of and behind the */
                               /*    part in use, filled with a pattern when the block is handed out and       */
                               /*    compared when it is released; tsp_stats.workspace_violations counts the   */
                               /*    words found changed: a kernel wrote outside its array.  A debugging aid:  */
                               /*    two small launches per block.  0 (default): none                          */
    TSP_OPT_STRIP_ORDER = 8    /* order in which the counting and the multiplication kernel (4.2,   */
                               /*    4.3) take the output tiles: 1: in vertical strips of tile      */
                               /*    columns sized so that the tiles of B a strip meets stay in the  */
                               /*    L2 cache; 0 (default) and 2: row-major as the task list is      */
                               /*    sorted (faster wherever measured: the strips cut the memory     */
                               /*    traffic, which does not bind these kernels); a value of 16 or   */
                               /*    more: strips of about that many tiles of B.  The result does    */
                               /*    not depend on it                                                */
};

/* Phases reported in tsp_stats.phase_us, in pipeline order. */
enum {
    TSP_PHASE_CONVERT = 0,     /* CSR -> tiles, one pass (Section 2.1.2)                            */
    TSP_PHASE_SYMBOLIC = 1,    /* tile correspondence, zero-product cull, sizing, task list (4.1)   */
    TSP_PHASE_COUNT = 2,       /* counting pass on bitmaps, row_ptr of C (Section 4.2)              */
    TSP_PHASE_NUMERIC = 3,     /* multiplication pass + CSR emission (Sections 4.3, 4.4)            */
    TSP_PHASE_COUNT_ = 4
};

/* Kernels reported in tsp_stats.kernel_us (a prefix sum of three small launches is timed as one).
 * When every tile-row of C is short, the task-list kernel also runs the counting pass and the row
 * offsets; their two entries then read 0. */
enum {
    TSP_KERNEL_CONVERT = 0,      /* CSR -> tiles, one pass (when B is not A: B's conversion)        */
    TSP_KERNEL_SYM_COUNT = 1,    /* C tiles and task-list entries per tile-row                      */
    TSP_KERNEL_SCAN_SYM = 2,     /* their prefix sums                                               */
    TSP_KERNEL_SYM_EMIT = 3,     /* C tile coordinates and task list                                */
    TSP_KERNEL_COUNT_MASKS = 4,  /* counting pass: boolean products of the bitmaps                  */
    TSP_KERNEL_ROW_OFFSETS = 5,  /* entries per CSR row, write offsets per (C tile, row)            */
    TSP_KERNEL_SCAN_ROWS = 6,    /* row_ptr of C                                                    */
    TSP_KERNEL_NUMERIC = 7,      /* multiplication pass + CSR emission                              */
    TSP_KERNEL_COUNT_ = 8
};

/* Counters and timings of the most recent tsp_spgemm / phase calls on a handle. */
typedef struct {
    int64_t a_tiles, b_tiles;        /* non-empty tiles of the operands                              */
    int64_t candidate_pairs;         /* (A tile, B tile) pairs with matching inner tile index         */
    int64_t pairs;                   /* pairs left after the zero-product cull = task list length     */
    int64_t c_tiles;                 /* output tiles (all structurally non-empty)                     */
    int64_t c_nnz;                   /* structural nonzeros of C                                      */
    int64_t workspace_bytes;         /* bytes currently held by the handle (cache + live objects)     */
    int64_t workspace_peak_bytes;    /* high-water mark of the above                                  */
    float phase_us[TSP_PHASE_COUNT_];/* device time per phase of the last call, if timers are on      */
    float total_us;                  /* first event to last event of the last tsp_spgemm, if timers on */
    float kernel_us[TSP_KERNEL_COUNT_]; /* device time per kernel of the last tsp_spgemm, if timers on  */
                                     /* (when B is not A, the conversion entries describe B's)        */
    int64_t products;                /* intermediate products of the last tsp_spgemm (the paper's      */
                                     /* NNZ of C-bar, Table 1; 2 * products = the FLOP of the product), */
                                     /* counted when TSP_OPT_COUNT_PRODUCTS is on, else -1              */
    /* The paper's selection criteria for the last product's left operand (Section 6.1): the tiled method */
    /* pays off for NNZ(A) > 300000 with more than 42 entries per row on average, and for well-filled     */
    /* tiles (5 of 64 slots of an 8x8 tile and more, i.e. 20 entries per 16x16 tile).  Reported, not acted */
    /* on: this library has no non-tiled path to fall back to.                                            */
    float a_mean_row;                /* NNZ(A) / rows                                                  */
    float a_tile_fill;               /* NNZ(A) / tiles(A): entries per 16x16 tile                      */
    int32_t in_paper_regime;         /* 1: NNZ(A) > 300000 and a_mean_row > 42                         */
    int32_t well_filled_tiles;       /* 1: a_tile_fill >= 20                                           */
    int64_t workspace_violations;    /* words of guard zones found changed since tsp_create             */
                                     /* (TSP_OPT_WORKSPACE_CANARIES; blocks still in use are not yet     */
                                     /* compared: free the outputs first)                                */
} tsp_stats;

/* Create a handle on the current HIP device.  allocator == NULL selects hipMalloc/hipFree. */
int tsp_create(tsp_handle *handle, const tsp_allocator *allocator);

/* Free every block the handle still holds (cache and live objects) and the handle itself. */
int tsp_destroy(tsp_handle handle);

int tsp_set_option(tsp_handle handle, int key, int64_t value);

/* Return every cached (not live) block to the allocator. */
int tsp_trim(tsp_handle handle, void *stream);

/*
 * C = A*B (paper Section 2.2, Algorithm 1), CSR in, CSR out, everything on `stream`.
 * A and B are borrowed and never modified; they may be the same object (A*A converts once).
 * On success *C is filled: rows = A.rows, cols = B.cols, nnz, row_ptr (TSP_I64), col_idx,
 * val (TSP_F32), the three arrays freshly taken from the handle's allocator and owned by the
 * caller, who releases them with tsp_csr_free.  Columns ascend strictly within each row.
 * On failure *C is zeroed and nothing is leaked.  The calling thread waits twice for results of
 * the device (the sizes of the task list and of C, which size the allocations: the steps Algorithm 1
 * calls AllocateMemGPU; it polls pinned memory for them for up to half a millisecond, then blocks);
 * the multiplication pass that fills col_idx and val is enqueued after the second wait and is NOT
 * waited for: C.nnz and the pointers are final when the call returns, the
 * contents once the stream has reached that point (hipStreamSynchronize, or further work on the
 * same stream).  With TSP_OPT_PHASE_TIMERS the call waits for the end.
 * Errors: INVALID_ARG, SHAPE_MISMATCH, NOT_CANONICAL, ALLOC_FAILED, INDEX_OVERFLOW, HIP,
 * UNSUPPORTED (a tile-row of C spans more than 131072 tile columns between its first and its
 * last candidate tile, i.e. 2097152 columns; or a tile-row of C holds 2^32 entries or more).
 */
int tsp_spgemm(tsp_handle handle, const tsp_csr *A, const tsp_csr *B, tsp_csr *C, void *stream);

/* Release the arrays of a matrix returned by this library and zero the struct. */
int tsp_csr_free(tsp_handle handle, tsp_csr *C, void *stream);

/*
 * Compaction of zeros (paper Section 4.4; the two compaction steps that end Algorithm 1): *out = C without the entries
 * whose value compares equal to zero (+0.0 and -0.0; NaN stays), order kept, so that a product
 * whose terms cancelled, or that only met stored zeros, leaves no entry behind.  C: device CSR with
 * float values (TSP_F32) and a 32- or 64-bit row_ptr, borrowed, not modified; row ranges are
 * clamped to [0, C.nnz], so a malformed row_ptr cannot cause an out-of-bounds access.  *out:
 * row_ptr (TSP_I64), col_idx, val (TSP_F32) from the handle's allocator, owned by the caller
 * (tsp_csr_free); zeroed on failure.  Synchronises the stream once (the new nnz sizes the
 * allocation).  C and out must be different objects.
 * Errors: INVALID_ARG, ALLOC_FAILED, INDEX_OVERFLOW, HIP.
 */
int tsp_compact_zeros(tsp_handle handle, const tsp_csr *C, tsp_csr *out, void *stream);

/*
 * tsp_compact_zeros for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same result as tsp_compact_zeros, but the call
 * allocates nothing, on the device or through the handle's allocator: the caller brings the output
 * arrays, and the pass's scratch (survivor counts per row and per 16 rows) lives in a fixed device array
 * inside the library (about 2.2 MB per GPU the library runs on, held until the process ends).
 * In: C as for tsp_compact_zeros.  In/out: *out with row_ptr -> int64[C.rows + 1], col_idx ->
 * int32[capacity], val -> float[capacity], capacity >= C.nnz, device arrays owned by the caller, not
 * overlapping C's; on success rows, cols, nnz and the two type fields are filled in and the arrays hold
 * the compacted matrix (entries past nnz are not written).  Do not pass *out to tsp_csr_free.
 * Limits: 1 <= C.rows <= TSP_COMPACT_STATIC_MAX_ROWS, else TSP_ERR_UNSUPPORTED and nothing is enqueued.
 * Synchronises the stream once (the new nnz).  All calls on one GPU share the one scratch array, which
 * keeps the previous call's contents (every call overwrites what it reads): calls that overlap on the
 * same GPU, from any handle or stream, race.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
#define TSP_COMPACT_STATIC_MAX_ROWS 524288
int tsp_compact_zeros_static(tsp_handle handle, const tsp_csr *C, tsp_csr *out, void *stream);

/* ----- the pipeline phase by phase (tsp_spgemm is exactly these calls in order) ----------- */

enum {
    TSP_FORM_LEFT = 1,    /* element storage for use as the left operand  (row-wise groups)    */
    TSP_FORM_RIGHT = 2    /* element storage for use as the right operand (column-wise groups) */
};

/*
 * CSR -> tile format (Section 2.1.2 with 16x16 tiles), one pass over the matrix.  `forms` is a
 * bit set of TSP_FORM_*.  Synchronises the stream once (tile count, validation result).
 * The result is owned by the caller (tsp_tiles_free).  The tile arrays have one slot per stored
 * entry of A (52 bytes each) although only the slots of actual tiles are written: that is
 * what lets the conversion run without a counting pass (see tsp_tiles_view).
 */
int tsp_convert(tsp_handle handle, const tsp_csr *A, int forms, tsp_tiles *out, void *stream);
int tsp_tiles_free(tsp_handle handle, tsp_tiles tiles, void *stream);

/*
 * Read-only view of a tile matrix, for inspection and tests.  Device pointers unless noted.
 * The tiles of tile-row I are the tile indices tile_row_ptr[I] .. tile_row_end[I]-1, ascending
 * tile column among them.  tile_row_ptr[I] is the position of the tile-row's first entry in the
 * CSR arrays, so tile indices ("slots") run up to tile_slots = nnz and the indices between two
 * tile-rows are unused: their array elements are never written and must not be read.  A tile
 * index is what the task list of a plan holds.
 * row_mask[t*16 + r] has bit c set when slot (r,c) of tile t is occupied.
 * Element storage is in 16-byte groups of 8 fp16 values, zero filled where a slot is empty,
 * and only non-empty groups are stored.  Left form: group id g = h*16 + r holds slots
 * (r, 8h..8h+7); right form: group id g = h*16 + c holds slots (8h..8h+7, c).  Bit g of the
 * group mask says whether group g is stored; the stored groups of a tile are consecutive, in
 * ascending g, starting at the group index *_head[2t + 1] of the form's element array.
 */
typedef struct {
    int64_t rows, cols;              /* of the matrix (host values)                                 */
    int64_t tile_rows, tile_cols;    /* ceil(rows/16), ceil(cols/16)                                */
    int64_t ntiles;                  /* number of tiles                                             */
    int64_t tile_slots;              /* length of the per-tile arrays (= nnz of the matrix)          */
    int32_t forms;
    const int32_t *tile_row_ptr;     /* int32[tile_rows] first tile index of every tile-row          */
    const int32_t *tile_row_end;     /* int32[tile_rows] one past its last tile index                */
    const int32_t *tile_col;         /* int32[tile_slots]                                            */
    const uint16_t *row_mask;        /* uint16[tile_slots * 16]                                      */
    const uint32_t *left_group_mask, *right_group_mask;   /* uint32[tile_slots] (always present)     */
    const uint32_t *left_head, *right_head;   /* uint32[tile_slots * 2] per tile {group mask, index of   */
                                              /* its first group} of the form (NULL if form absent)     */
    const uint16_t *left_elements, *right_elements;       /* fp16 bits, 8 per group (NULL if absent) */
    int64_t left_groups_capacity, right_groups_capacity;  /* groups the element arrays can hold     */
} tsp_tiles_view;
int tsp_tiles_get_view(tsp_tiles tiles, tsp_tiles_view *view);

/*
 * Symbolic phase + counting pass for C = A*B on tile matrices (Sections 4.1 and 4.2; Algorithm 1
 * up to the counting kernel): tile correspondence, zero-product cull on the occupancy words, sizing scans, task
 * list grouped by output tile (output tiles row-major, pairs of a tile in ascending inner
 * index), boolean product of the bitmaps per output tile, row_ptr of C.  A needs no particular
 * form, nor does B.  Synchronises the stream twice (task-list size; nnz of C).
 */
int tsp_symbolic(tsp_handle handle, tsp_tiles A, tsp_tiles B, tsp_plan *out, void *stream);
int tsp_plan_free(tsp_handle handle, tsp_plan plan, void *stream);

/* Read-only view of a plan.  Device pointers unless noted. */
typedef struct {
    int64_t c_rows, c_cols;          /* host values                                                 */
    int64_t c_tile_rows;
    int64_t c_tiles, pairs, c_nnz, candidate_pairs;
    const int32_t *c_tile_row_ptr;   /* int32[c_tile_rows + 1]                                      */
    const int32_t *c_tile_row;       /* int32[c_tiles]                                              */
    const int32_t *c_tile_col;       /* int32[c_tiles], ascending inside a tile-row                 */
    const int64_t *pair_off;         /* int64[c_tiles + 1] segment offsets into the task list       */
    const int32_t *pair_ab;          /* int32[2 * pairs]: entry e = {tile in A, tile in B}          */
    const uint16_t *c_row_mask;      /* uint16[c_tiles * 16] structural pattern of each output tile */
    const uint32_t *c_row_off;       /* uint32[c_tiles * 16] position of the tile's first entry in  */
                                     /* CSR row 16I+r, counted from the first entry of tile-row I   */
    const int64_t *c_row_ptr;        /* int64[c_rows + 1]                                           */
} tsp_plan_view;
int tsp_plan_get_view(tsp_plan plan, tsp_plan_view *view);

/*
 * Multiplication pass + CSR emission (Sections 4.3, 4.4): every task-list pair is multiplied
 * as a 16x16x16 block product on the matrix cores, fp16 inputs, fp32 accumulation, the pairs of
 * one output tile accumulated in registers in task-list order; the tile's structural entries
 * are written straight to their CSR positions.  A must hold TSP_FORM_LEFT, B TSP_FORM_RIGHT,
 * and the plan must come from tsp_symbolic on the same pair of tile matrices.  Allocates C
 * (see tsp_spgemm for ownership).  Does not synchronise.
 */
int tsp_numeric(tsp_handle handle, tsp_tiles A, tsp_tiles B, tsp_plan plan, tsp_csr *C, void *stream);

/*
 * C = A*B by the pipeline as the paper lays it out, at a tile edge of 8 (the paper's, Section 2.1.2),
 * 16 or 32: tiles in the packed bitmap format (2 bytes per element, row masks, an element pointer per
 * tile); the task list by expansion of all tile pairs with a matching inner tile index, cull of the
 * pairs whose boolean tile product is empty, a stable library sort by output tile and a run-length
 * pass (Section 4.1, Algorithm 1); the counting pass on the bitmaps (Section 4.2); the multiplication
 * pass with the packed elements of every pair placed by the bitmap into dense tiles in LDS and
 * multiplied on the matrix cores, one wave per output tile (Section 4.3); the output tiles written
 * to CSR.  Same inputs, conventions, output format and ownership as tsp_spgemm, and the same result:
 * the structural pattern exactly, the values up to the order of the fp32 additions.  It exists to show
 * that the result does not depend on the tile edge and to measure the paper's design against this
 * library's; it is not tuned, validates its inputs always, and synchronises the stream about ten
 * times.  tile_edge other than 8, 16, 32: TSP_ERR_INVALID_ARG; more than 2^31 - 2 candidate tile pairs:
 * TSP_ERR_UNSUPPORTED.  tsp_stats reports the tile and pair counts at that tile edge and, with the
 * timers on, the four phases.
 */
int tsp_spgemm_paper(tsp_handle handle, int tile_edge, const tsp_csr *A, const tsp_csr *B, tsp_csr *C, void *stream);

int tsp_get_stats(tsp_handle handle, tsp_stats *out);
const char *tsp_strerror(int status);
int tsp_last_hip_error(tsp_handle handle);   /* hipError_t of the last TSP_ERR_HIP on this handle */

#ifdef __cplusplus
}
#endif
#endif /* TSP_H */
