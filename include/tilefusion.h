/*
 * tilefusion.h -- C ABI of the tile-fusion library for the matrix chain  D = A (B C)  on gfx950.
 *
 * The operation (paper Section 1, Eq. 1): A is an n x n CSR sparse matrix, B is n x bCol and
 * either dense or CSR sparse, C is a dense bCol x cCol matrix.  Unfused, the chain is
 * D1 = B C followed by D = A D1.  Tile fusion (Section 3) inspects the sparsity pattern of A
 * once, builds a schedule of two wavefronts -- fused tiles that produce a block of D1 rows and
 * at once consume them for the rows of D that depend on nothing else, then the leftover rows
 * of D -- and reuses that schedule for every later execution (Section 3, first paragraph).
 *
 * Conventions for every call
 *   - Dense matrices are row-major and contiguous; B is n x bCol, C is bCol x cCol, D is n x cCol.
 *   - Dense operands and every pointer handed to an execution call are DEVICE pointers, aligned
 *     to 16 bytes.  The element type of B, C, D is the element type of A.
 *   - CSR matrices use int32 row pointers (n_rows + 1 entries, rowptr[0] = 0) and int32 column
 *     indices.  Explicit zeros, duplicate and unsorted column indices are legal; entries are
 *     summed in an unspecified order.
 *   - D is overwritten (the listings of Section 3.2 accumulate into zeroed outputs).
 *   - The caller owns A, B, C and D.  The plan owns a device copy of A (pattern and values), the
 *     schedule and a workspace with one slot for every D1 row that crosses tiles (no other D1
 *     row ever reaches device memory: Section 3.1, one synchronisation between two wavefronts).
 *   - Errors are reported by return code; tf_last_error() gives a message for the calling
 *     thread's most recent failure.  No call throws or aborts.
 */
#ifndef TILEFUSION_H
#define TILEFUSION_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TF_OK = 0,
    TF_EINVAL = 1,        /* null pointer, non-positive size, bad alignment, bad parameter   */
    TF_EBADCSR = 2,       /* malformed CSR: rowptr not monotone, rowptr[n] != nnz, col range  */
    TF_ENOMEM = 3,        /* host or device allocation failed                                 */
    TF_EHIP = 4,          /* a HIP runtime call failed                                        */
    TF_EUNSUPPORTED = 5,  /* shape outside what the kernels cover (see tf_plan_create)        */
    TF_EMISMATCH = 6      /* plan and call disagree (dtype, kind of B, shape of B)            */
} tf_status;

typedef enum { TF_F32 = 0, TF_F64 = 1 } tf_dtype;

/* A CSR matrix.  Caller-owned, read-only.  on_device tells where the three arrays live
 * (all three in the same place). */
typedef struct tf_csr {
    int64_t n_rows;
    int64_t n_cols;
    int64_t nnz;
    const int32_t *rowptr;
    const int32_t *colidx;
    const void *vals;
    int32_t dtype;      /* tf_dtype */
    int32_t on_device;  /* 0 = host pointers, 1 = device pointers */
} tf_csr;

/* Inputs of the scheduler (Algorithm 1) besides the pattern.  Zero selects the default.
 * With ct_size = 0 and p = 0 and neither TF_FLAG_REORDER nor TF_FLAG_NO_SPLIT (in particular with
 * tp = NULL) the tiling is left to the library: ctSize 2048, p = a quarter of the compute units,
 * half of the LDS per tile where two workgroups per compute unit pay (dense B, small bCol x cCol);
 * tiles of consecutive rows as in Algorithm 1 unless they fuse under half of the entries of a
 * matrix whose rows stay near the diagonal and graph-grown tiles spill fewer D1 rows; and where
 * the fused rows that read the fast memory hold under 2 % of the entries (graphs) they are left
 * to the second wavefront, so that the first wavefront needs no tile in fast memory at all.
 * With ct_size or p given, step 1 is Algorithm 1 to the letter. */
typedef struct tf_tile_params {
    int32_t ct_size;         /* coarse tile size ctSize (Section 3.1.1); default 2048           */
    int32_t p;               /* wanted number of tiles per wavefront ("cores"); default 32 when
                                ct_size is given, else a quarter of the compute units            */
    int64_t fast_mem_bytes;  /* fast memory of one tile: the LDS a workgroup may use;
                                default = the device's LDS per workgroup (160 KiB on gfx950)    */
    int32_t col_slice;       /* columns of C/D handled by one workgroup; default = cCol, capped
                                at what the kernels cover; a last narrower slice is allowed     */
    uint32_t flags;          /* TF_FLAG_* */
    int32_t gather_slices;   /* column slices of the D1 workspace, each gathered by its own XCDs
                                in the second wavefront: 1, 2, 4 or 8, slices of a power of two
                                of columns, at least 16 and at least 64 bytes.  Default: 1 for
                                matrices whose rows stay near the diagonal, more for matrices
                                whose rows reach far (graphs), see tf_schedule_view.d1_slices   */
    int32_t reserved0;
} tf_tile_params;

/* Skip step 2 (tile splitting): tiles that do not fit the fast memory make plan creation fail. */
#define TF_FLAG_NO_SPLIT 1u
/* Build the schedule only: no device is touched and no device memory is allocated, A must be in
 * host memory, fast_mem_bytes is taken as given (default 160 KiB).  The plan serves
 * tf_plan_schedule; execution calls on it fail with TF_EINVAL. */
#define TF_FLAG_SCHEDULE_ONLY 2u
/* Tiles are grown along the dependence graph (breadth first over the column indices of A,
 * starting from the lowest row not yet in a tile) instead of being ranges of consecutive rows, each
 * as large as the fast memory allows and at most t rows.  The paper forms tiles from consecutive
 * iterations (Section 3.1.1) because that is cheap and keeps spatial locality; on matrices whose
 * rows depend on far-away rows (stencils in natural ordering) consecutive tiles small enough
 * for LDS fuse nothing, while graph-grown tiles do. */
#define TF_FLAG_REORDER 4u
/* The chain with the transpose of C (Section 3.2 notes that the fused code also covers it):
 * D = A (B C^T).  The dense-B calls on such a plan take C as a cCol x bCol row-major array, so
 * that element (k, c) of the multiplier is C[c * bCol + k]; everything else is unchanged.  Only
 * plans for a dense B accept the flag (a sparse B gathers whole rows of C; plan creation fails
 * with TF_EUNSUPPORTED). */
#define TF_FLAG_C_TRANSPOSED 8u
/* Rows of D1 = B C that no row of A reads (columns of A without a stored entry) are not computed
 * by the fused calls: they leave the tiles' first lists.  The paper's schedule runs every
 * iteration of both operations exactly once (Section 3.1); this flag gives that up for the first
 * operation, D is unchanged.  The unfused calls still compute all of D1, and after a fused call
 * the workspace rows of skipped D1 rows are not written.  (A plan for a CSR B whose first
 * wavefront streams leaves the rows out one by one instead; the schedule view is the same.) */
#define TF_FLAG_SKIP_UNREAD 16u
/* The plan serves the fused calls only: the packed copy of all rows of A that the unfused
 * baseline runs on is not built (saves its time and device memory); tf_unfused_* then fail with
 * TF_EINVAL. */
#define TF_FLAG_NO_BASELINE 32u

typedef struct tf_plan tf_plan; /* opaque, library-owned */

/* Host-readable view of a plan's schedule.  All pointers are HOST memory owned by the plan and
 * stay valid until tf_plan_destroy.  A tile v of the first wavefront produces the D1 rows
 *   first_rows[tile_first_ptr[v] .. tile_first_ptr[v+1])      (the tile's "first" list;
 *                                         n_first_rows entries in all: n unless rows are skipped)
 * and then computes the rows of D
 *   second_rows[tile_second_ptr[v] .. tile_second_ptr[v+1])   (the tile's "second" list);
 * unit u of the second wavefront computes the rows wf1_rows[wf1_unit_ptr[u] .. wf1_unit_ptr[u+1]).
 * spill[i] != 0 marks D1 rows that are also stored to device memory because a row of the
 * second wavefront reads them. */
typedef struct tf_schedule_view {
    int64_t n;
    int64_t nnz;
    int32_t t;                  /* uniform tile size chosen by step 1                          */
    int32_t col_slice;
    int32_t n_slices;
    int32_t dtype;
    int32_t b_is_sparse;
    int32_t reserved0;
    int64_t n_coarse_tiles;     /* tiles after step 1                                          */
    int64_t n_tiles;            /* tiles after step 2                                          */
    const int32_t *tile_first_ptr;
    const int32_t *first_rows;
    const int32_t *tile_second_ptr;
    const int32_t *second_rows;
    int64_t n_wf1_units;
    const int32_t *wf1_unit_ptr;
    const int32_t *wf1_rows;
    const uint8_t *spill;
    int64_t n_fused_rows;
    int64_t n_wf1_rows;
    int64_t n_spill_rows;
    int64_t fused_nnz;          /* stored entries of A that belong to fused rows               */
    double fused_ratio_eq3;     /* Eq. 3 literally: fused rows / (|I| + |J|) = / 2n            */
    double fused_ratio_rows;    /* fused rows / n                                              */
    double fused_ratio_nnz;     /* share of the second operation's work done in wavefront 0    */
    int64_t fast_mem_bytes;     /* the budget the tiles were fitted to                         */
    int64_t lds_fixed_bytes;    /* LDS a fused workgroup uses besides its D1 tile              */
    int64_t lds_bytes_per_row;  /* LDS per D1 row of a tile (the row, its id twice, an estimate of
                                   its packed entries); footprint = fixed + rows_pad * this    */
    int32_t lds_row_granule;    /* rows_pad = rows rounded up to a multiple of this            */
    int32_t second_block_in_lds; /* 1: the packed entries of a tile's fused rows are staged in LDS;
                                   0: they did not fit beside the largest tile and are read in place */
    double eq2_cost_max;        /* largest Eq. 2 data-movement cost over the tiles (elements)  */
    double plan_seconds;        /* host time spent building the schedule (without the packed
                                   copy of A that only the unfused baseline uses)              */
    int64_t alg_bytes;          /* algorithmic HBM bytes of one fused execution: A, B, C and D once,
                                   every spilled D1 row written once and read once.  A CSR B is
                                   not known to the plan and is NOT included: the caller adds
                                   4 (n + 1) + nnz(B) (4 + element size)                         */
    int64_t alg_bytes_unfused;  /* the same for the unfused two-kernel execution (all of D1
                                   written once and read once)                                   */
    int64_t second_block_bytes; /* largest per-tile block of packed entries (fused rows)       */
    int64_t lds_launch_bytes;   /* LDS one fused workgroup is launched with (0: schedule only) */
    int64_t n_first_rows;       /* D1 rows the first wavefront produces (length of first_rows) */
    const int32_t *spill_slot;  /* n entries: slot of the D1 row in the workspace, -1 = not spilled */
    int64_t n_direct_rows;      /* fused rows of D that are their own D1 row times a single diagonal
                                   entry, or empty: stored from the registers that hold the D1 row
                                   (they are listed in second_rows like every fused row)         */
    int32_t d1_slices;          /* workspace layout: d1_slices column slices of d1_slice_cols     */
    int32_t d1_slice_cols;      /* columns, slice after slice, each d1_rows x d1_slice_cols       */
    int64_t d1_rows;            /* row-major: element (slot, c) is at (c / d1_slice_cols) d1_rows
                                   d1_slice_cols + slot d1_slice_cols + c mod d1_slice_cols       */
    int32_t first_wavefront_streams; /* 1: no fused row reads the LDS tile (all are direct rows), so
                                   the first wavefront runs without tiles in LDS, streaming through
                                   the rows like the plain first operation                        */
    int32_t grown_tiles;        /* 1: tiles were grown along the dependence graph (TF_FLAG_REORDER,
                                   or the library's own choice), 0: ranges of consecutive rows   */
    int64_t n_demoted_rows;     /* rows that their tile could have fused but that the library left
                                   to the second wavefront (only when the tiling was left to the
                                   library, see tf_plan_create); 0 = step 1 is maximal            */
    int32_t far_rows;           /* 1: the rows of A reach far from the diagonal (a graph)         */
    int32_t automatic;          /* 1: the tiling was left to the library                          */
} tf_schedule_view;

/* Inspector: builds the fused schedule for the pattern of A (Algorithm 1: step 1, coarse tile
 * fusion; step 2, tile splitting against the fast-memory size) plus the spill set and the
 * balanced units of the second wavefront.  bCol and cCol are the column counts of B and C;
 * for a sparse B, bCol is the number of columns of B (= rows of C).  b_is_sparse selects which
 * execution call the plan serves.  tp may be NULL for defaults.
 * Validates: A square, 0 <= nnz < 2^31, rowptr monotone with rowptr[0] = 0 and rowptr[n] = nnz,
 * 0 <= col < n, bCol > 0, cCol > 0, one D1 row fits the fast memory.
 * Synchronous; allocates host and device memory owned by the plan.  On failure *out is NULL.
 * Matrices of 2^18 entries or more are inspected by several host threads (as many as the
 * machine reports, at most 16; the environment variable TF_HOST_THREADS=k lowers that to k);
 * the schedule does not depend on their number. */
tf_status tf_plan_create(const tf_csr *A, int64_t bCol, int64_t cCol, int32_t b_is_sparse,
                         const tf_tile_params *tp, tf_plan **out);

/* Frees everything the plan owns.  NULL is accepted. */
tf_status tf_plan_destroy(tf_plan *plan);

/* Fills *out with the plan's schedule (host pointers, see tf_schedule_view). */
tf_status tf_plan_schedule(const tf_plan *plan, tf_schedule_view *out);

/* Fused execution of D = A (B C) with dense B (Section 3.2, fused GeMM-SpMM listing): first
 * wavefront = one launch over the fused tiles, second wavefront = one launch over the leftover
 * rows; stream order is the single barrier between them.  B, C, D are device pointers.
 * Asynchronous on `hip_stream` (a hipStream_t, NULL = the default stream); allocates nothing,
 * never synchronises.  Two executions of one plan must not overlap (they share the plan's
 * workspace). */
tf_status tf_gemm_spmm(const tf_plan *plan, const void *B, const void *C, void *D,
                       void *hip_stream);

/* tf_gemm_spmm for callers that cannot allocate device memory and do not want a plan-owned
 * workspace to be touched: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments and result as tf_gemm_spmm, but the D1 rows that cross tiles
 * go to a fixed array of 64 MiB that is part of the library's code object (one copy per GPU,
 * held until the process ends) instead of the plan's workspace.  The call allocates nothing.
 * A plan whose workspace (tf_schedule_view: d1_slices x d1_rows x d1_slice_cols elements) exceeds
 * 64 MiB is rejected with TF_EUNSUPPORTED.  All calls on one GPU share that GPU's array, whatever
 * the plan: calls that overlap in time on one GPU race (serialise them on one stream).  The array
 * keeps the last call's contents; nothing in it needs clearing between calls, since every row is
 * written by the first wavefront before the second one reads it. */
tf_status tf_gemm_spmm_static(const tf_plan *plan, const void *B, const void *C, void *D,
                              void *hip_stream);

/* Fused execution with CSR B (Section 3.2, fused SpMM-SpMM listing).  B must be on the device,
 * n x bCol with the plan's bCol and dtype; C is bCol x cCol.  B may alias A's arrays.
 * B's arrays live on the device and are NOT validated by the execution calls (only its shape
 * and element type are): a well-formed CSR (monotone rowptr with rowptr[0] = 0, 0 <= column <
 * bCol) is the caller's precondition; tf_csr_validate checks it where that is in doubt. */
tf_status tf_spmm_spmm(const tf_plan *plan, const tf_csr *B, const void *C, void *D,
                       void *hip_stream);

/* The unfused two-kernel baseline on the same plan (Section 4.1: an unfused parallel
 * implementation with the same optimisations): D1 = B C for all rows into a workspace of n rows,
 * then D = A D1 for all rows.  Same argument rules as the fused calls, except that the first
 * unfused call on a plan allocates that workspace (call tf_plan_prepare_unfused beforehand where
 * the call itself must not allocate, e.g. under stream capture). */
tf_status tf_unfused_gemm_spmm(const tf_plan *plan, const void *B, const void *C, void *D,
                               void *hip_stream);
tf_status tf_unfused_spmm_spmm(const tf_plan *plan, const tf_csr *B, const void *C, void *D,
                               void *hip_stream);

/* One wavefront of the fused execution on its own (wavefront 0 = fused tiles, 1 = leftover
 * rows), for per-kernel timing and tests.  Pass the dense B in B_dense or the CSR B in B_csr
 * according to the plan (the other NULL; both may be NULL for wavefront 1, which reads only the
 * plan's workspace).  Wavefront 1 is only meaningful after wavefront 0 of the same inputs. */
tf_status tf_run_wavefront(const tf_plan *plan, int32_t wavefront, const void *B_dense,
                           const tf_csr *B_csr, const void *C, void *D, void *hip_stream);

/* Allocates the workspace of the unfused baseline (all n rows of D1) if it does not exist yet. */
tf_status tf_plan_prepare_unfused(const tf_plan *plan);

/* Device pointer of the plan's D1 workspace: after a fused execution slot spill_slot[i] holds D1
 * row i, in the layout that tf_schedule_view describes (d1_slices, d1_slice_cols, d1_rows).
 * tf_plan_workspace_unfused: the baseline's workspace, same layout with n rows and slot = row
 * (NULL before the first unfused call or tf_plan_prepare_unfused).  For tests. */
tf_status tf_plan_workspace(const tf_plan *plan, void **d1_device);
tf_status tf_plan_workspace_unfused(const tf_plan *plan, void **d1_device);

/* Checks a CSR matrix given with host or device arrays (device arrays are copied to the host):
 * rowptr[0] = 0, rowptr monotone, rowptr[n_rows] = nnz, 0 <= column < n_cols.  TF_OK or
 * TF_EBADCSR.  Synchronous; meant for a CSR B before it is handed to tf_spmm_spmm. */
tf_status tf_csr_validate(const tf_csr *M);

/* Message for the most recent failure on the calling thread ("" if none). */
const char *tf_last_error(void);

/* Library version, "major.minor". */
const char *tf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TILEFUSION_H */
