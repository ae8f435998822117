/*
 * hcspmm -- hybrid-core SpMM for graph adjacency matrices on AMD MI355X (gfx950).
 *
 * C ABI of the library.  The method follows "HC-SpMM" (arxiv 2412.08902):
 *   - the sparse matrix A (CSR) is cut into row windows of 16 rows, the minimum
 *     hybrid unit                                       (Section IV-A);
 *   - inside a window the non-zero columns are moved to the front ("condensed")
 *                                                        (Section IV-A);
 *   - a three-parameter linear model on (number of non-zero columns, sparsity)
 *     decides per window whether the matrix cores or the scalar cores compute
 *     it; the decision is taken once, in preprocessing, and stored as one flag
 *     per window (0 = scalar path, 1 = matrix path)      (Section IV-C);
 *   - Z = A X is then computed window by window on the chosen path, windows
 *     own disjoint output rows so nothing is merged      (Alg. 1-4, Eq. 1);
 *   - the GNN layer couples the aggregation with the dense update X W
 *                                                        (Section V-A, Eq. 1-2).
 *   - the layer's backward pass aggregates the incoming gradient first and
 *     then applies both products of the update          (Section V-A, Eq. 3-4);
 *   - an offline vertex reordering raises the windows' computing intensity
 *                                                        (Section V-B, Alg. 5/6).
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device pointers owned by the caller; "host"
 *     pointers are ordinary host memory.  The library never frees caller
 *     memory.  Dense matrices are row-major with a leading dimension given in
 *     ELEMENTS.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     hcspmm_spmm / hcspmm_gcn_layer only enqueue work on it and return;
 *     hcspmm_prepare and hcspmm_plan_export synchronise with it.
 *   - No entry point throws, aborts or prints.  Every failure is a status
 *     code; hcspmm_last_error() returns a thread-local description of the most
 *     recent failure on the calling thread.
 *   - All index arithmetic on row*ld and nnz*d is done in 64 bits; CSR indices
 *     are int32, so nnz < 2^31.
 *   - Device memory the library holds beyond its plans: one 16 MiB static array
 *     per GPU (scratch of hcspmm_spmm_noalloc) and, per GPU, up to 64 MiB of
 *     blocks of at most 16 MiB each that preparations and destroyed plans leave
 *     behind for the next preparation (an allocation costs more than the
 *     kernels of a small matrix's preparation); both live until the process ends.
 */
#ifndef HCSPMM_H
#define HCSPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hcspmm_plan hcspmm_plan;   /* opaque, library-owned */

typedef enum {
    HCSPMM_OK = 0,
    HCSPMM_EINVAL = 1,        /* NULL pointer, negative size, bad enum, bad leading dimension */
    HCSPMM_EBADCSR = 2,       /* rowptr not monotone / rowptr[0] != 0 / rowptr[n] != nnz / column out of range */
    HCSPMM_EALLOC = 3,        /* device or host allocation failed */
    HCSPMM_EHIP = 4,          /* a HIP runtime call failed */
    HCSPMM_EUNSUPPORTED = 5   /* valid request outside the implemented envelope (see each call) */
} hcspmm_status;

typedef enum { HCSPMM_F32 = 0, HCSPMM_BF16 = 1, HCSPMM_F16 = 2 } hcspmm_dtype;

/* How windows are routed.  PER_WINDOW is the selector of Section IV-C as it stands: one decision
 * per window, nothing else.  HYBRID (the default) takes the same decisions and then applies a
 * launch guard, because here the two paths are separate kernel launches: when both paths got
 * work and the smaller side holds fewer than 2^18 non-zeros and less than 1/8 of all non-zeros,
 * its windows join the other path (the scalar side is checked for the matrix side's windows
 * first) -- a launch that cannot repay its fixed cost is not made.  The two ALL_* modes force one
 * path for every non-empty window (used to measure the selector against the pure paths).
 * Empty windows always take the scalar path.
 * ALL_CSR is also the plan for a matrix whose structure keeps changing: the scalar path reads
 * plain CSR (the paper's scalar path has no preprocessing either), so hcspmm_prepare skips the
 * condensing step and only validates the arrays and builds the row-length launch tables; the
 * window features (ncols, wptr, total_ncols) of such a plan are computed on the first
 * hcspmm_plan_info / hcspmm_plan_export call instead. */
typedef enum {
    HCSPMM_ROUTE_HYBRID = 0, HCSPMM_ROUTE_ALL_CSR = 1, HCSPMM_ROUTE_ALL_MFMA = 2, HCSPMM_ROUTE_PER_WINDOW = 3
} hcspmm_route_mode;

/* Update stage of the aggregate-then-update layer and of the backward pass: AUTO lets the library pick the faster
 * route for the shape, FUSED takes the fused kernels whenever the shape allows them, SPLIT never does. */
typedef enum { HCSPMM_UPDATE_AUTO = 0, HCSPMM_UPDATE_FUSED = 1, HCSPMM_UPDATE_SPLIT = 2 } hcspmm_update_fusion;

/* Kernels of the matrix path.  PER_WINDOW (what AUTO selects): one wave, or for wide windows one workgroup, per
 * window; windows that share columns meet in L2 through the launch order.  RUNS: runs of four neighbouring
 * matrix-path windows, one workgroup each, share their gathered X rows through LDS (Section IV-B: loading X is
 * the larger part of the matrix path) -- used when the plan and the call allow it (rows with ascending columns,
 * n_cols <= 2^22, X rows readable in 16-byte pieces, no fused update), else PER_WINDOW.  RUNS is kept as an option
 * because it measured slower on every benchmark graph: the rows it saves are the ones L2 already served. */
typedef enum { HCSPMM_MATRIX_AUTO = 0, HCSPMM_MATRIX_PER_WINDOW = 1, HCSPMM_MATRIX_RUNS = 2 } hcspmm_matrix_kernels;

/*
 * Options of hcspmm_prepare.  Fill with hcspmm_default_options() first.
 *
 * Selector (Section IV-C).  The paper's model is  z = w1*ncols + w2*sparsity + b
 * with sparsity = 1 - nnzw/(H*ncols); training label 1 means "scalar cores are
 * faster".  It is evaluated exactly in 64-bit integers after multiplying by
 * H*ncols > 0:
 *     z' = sel_coef[0]*H*ncols^2 + sel_coef[1]*(H*ncols - nnzw) + sel_coef[2]*H*ncols
 *     route = 1 (matrix path)  iff  z' < 0
 * so sel_coef = (w1, w2, b) scaled by one common positive factor.  The paper
 * does not print its coefficients (they are fitted per GPU model and
 * precision); the defaults shipped here were fitted on MI355X for each
 * (mfma_dtype, d_hint, nnz) bucket and are returned by hcspmm_default_selector().
 */
typedef struct {
    int32_t struct_size;          /* sizeof(hcspmm_options), for ABI growth */
    int32_t window_rows;          /* H; only 16 is implemented */
    int32_t route_mode;           /* hcspmm_route_mode */
    int32_t mfma_dtype;           /* hcspmm_dtype the matrix path will multiply in (selects default coefficients) */
    int32_t d_hint;               /* dense width the plan will mostly be used with (selects default coefficients); 0 = 64 */
    int32_t use_custom_selector;  /* 0: shipped coefficients for (mfma_dtype, d_hint); 1: sel_coef below */
    int64_t sel_coef[3];
    int32_t update_fusion;        /* hcspmm_update_fusion: how hcspmm_aggregate_update / hcspmm_layer_backward on this plan
                                     choose between the fused update stage and SpMM + GEMM (for tests and measurements) */
    int32_t matrix_kernels;       /* hcspmm_matrix_kernels: which kernels serve the matrix path (for tests and measurements) */
} hcspmm_options;

void hcspmm_default_options(hcspmm_options* opt /* host, out */);

/* Shipped selector coefficients for a precision, dense width and matrix size (the table has one
 * row per precision, width bucket and non-zero-count bucket).  coef: host, out, 3 entries. */
hcspmm_status hcspmm_default_selector(int32_t mfma_dtype, int32_t d_hint, int64_t nnz, int64_t* coef);

/*
 * Preprocessing (Section IV-A windows + condensing, Section IV-C selection;
 * the paper's Appendix F "preprocessing").  Runs entirely on the GPU.
 *
 *   n_rows, n_cols   shape of A (n_rows >= 0, 1 <= n_cols < 2^27)
 *   nnz              number of stored entries (0 <= nnz < 2^31)
 *   d_rowptr         device, int32[n_rows+1]
 *   d_colind         device, int32[nnz]; rows need not be sorted; duplicate (row, col) entries are summed
 *   d_vals           device, float[nnz]
 *   opt              host, NULL = defaults
 *   out_plan         host, receives the plan
 *
 * The plan BORROWS d_rowptr / d_colind / d_vals: they must stay valid until
 * hcspmm_plan_destroy, and d_rowptr / d_colind unchanged.  The plan depends on the
 * structure only (windows, condensed columns, selector features are functions of the indices),
 * and every kernel reads the values through d_vals at call time: the CALLER MAY OVERWRITE
 * d_vals IN PLACE between calls (edge weights that change per layer or per epoch) without
 * preparing again.  A structural change needs a new plan (a prepare costs about two SpMM calls on
 * the large configurations).  Everything the plan allocates it owns.
 * Validates the CSR on the device (HCSPMM_EBADCSR).  Synchronises with `stream`.
 */
hcspmm_status hcspmm_prepare(int32_t n_rows, int32_t n_cols, int64_t nnz,
                             const int32_t* d_rowptr, const int32_t* d_colind, const float* d_vals,
                             const hcspmm_options* opt, void* stream, hcspmm_plan** out_plan);

/*
 * Preprocessing again after the matrix's STRUCTURE changed (edges inserted or deleted; the paper's
 * Appendix F counts preprocessing as the price of a changing graph).  The caller hands over the new
 * CSR arrays (same n_rows and n_cols; nnz and all three arrays may differ, the plan borrows the new
 * ones from now on) and the list of rows whose set of entries changed.  Windows without a changed
 * row keep their distinct-column counts, so the passes over the column indices -- validation and
 * counting, the part of hcspmm_prepare proportional to the non-zeros -- run over the touched windows
 * only; routes (selector and launch guard), the window lists and the launch tables are then rebuilt
 * for the whole matrix, which costs time proportional to the rows, not to the non-zeros.  The
 * condensed structure (column lists, condensed columns) of untouched windows that were and remain on
 * the matrix path is copied to its new offsets, that of the others is built.  The result is the plan
 * hcspmm_prepare would build for the new arrays, bit for bit.
 *
 *   nnz, d_rowptr, d_colind, d_vals   the new matrix, as for hcspmm_prepare
 *   h_changed_rows   host, int32[n_changed]: every row whose column indices (their values or their
 *                    number) differ from the old matrix, in any order, repeats allowed.  A row that
 *                    changed but is not listed leaves the plan inconsistent with the matrix.
 * Falls back to a preparation from scratch when an eighth of the windows or more are touched, or when the
 * plan's window features were never computed (HCSPMM_ROUTE_ALL_CSR plans, whose preparation has no
 * pass over the column indices to save).  Synchronises with `stream`; no call may be using the plan.
 * On an error the plan is unchanged and still valid for the old arrays.
 * A plan that has been updated keeps the device blocks of its last updates (scratch and the arrays of
 * the plan it replaced, about as much again as the plan's own arrays) for the next update instead of
 * returning them to the runtime; hcspmm_plan_destroy releases them.  hcspmm_plan_info's device_bytes
 * does not count them.
 */
hcspmm_status hcspmm_plan_update(hcspmm_plan* plan, int64_t nnz, const int32_t* d_rowptr, const int32_t* d_colind,
                                 const float* d_vals, const int32_t* h_changed_rows /* host */, int32_t n_changed,
                                 void* stream);

/* Sizes of a plan's arrays (host struct, filled by hcspmm_plan_info). */
typedef struct {
    int32_t window_rows;      /* H */
    int32_t n_rows, n_cols;
    int64_t nnz;
    int32_t n_windows;        /* W = ceil(n_rows / H) */
    int64_t total_ncols;      /* sum over windows of ncols = length of wcols */
    int32_t n_mfma_windows;   /* windows with route 1 */
    int32_t n_csr_windows;    /* windows with route 0 */
    int64_t nnz_mfma;         /* non-zeros inside route-1 windows */
    int32_t route_mode;
    int32_t mfma_dtype;
    int32_t d_hint;
    int64_t sel_coef[3];      /* coefficients the routes were computed with */
    int64_t device_bytes;     /* device memory owned by the plan */
    /* how the scalar path's rows are scheduled (launch tables, not part of the canonical plan) */
    int32_t n_short_rows;     /* rows walked by lane groups, several consecutive rows per group */
    int32_t n_mid_rows;       /* rows handled one wave per row */
    int32_t n_long_rows;      /* rows cut into segments, one workgroup per segment */
    int32_t n_segments;
    int64_t nnz_long;         /* non-zeros inside mid and long rows */
    int32_t n_mfma_small;     /* route-1 windows handled one wave per window */
    int32_t n_mfma_big;       /* route-1 windows handled one workgroup per window */
    /* runs of neighbouring route-1 windows with merged column lists (0 when the plan has no run tables) */
    int32_t n_runs;
    int32_t n_run_slices;     /* workgroups of the run kernel */
    int64_t run_union_cols;   /* sum over runs of the merged list's length (total_ncols of the same windows counts shared columns per window) */
} hcspmm_plan_info_t;

/* Synchronises with the device the first time it is called on an HCSPMM_ROUTE_ALL_CSR plan (it then
 * computes the window features that prepare skipped); otherwise host-only. */
hcspmm_status hcspmm_plan_info(const hcspmm_plan* plan, hcspmm_plan_info_t* info /* host, out */);

/*
 * Copies the canonical plan arrays to host memory (each pointer may be NULL to
 * skip that array; sizes from hcspmm_plan_info):
 *   ncols  int32[W]    distinct columns per window                    (Section IV-A / V-B)
 *   nnzw   int32[W]    non-zeros per window
 *   route  uint8[W]    0 = scalar path, 1 = matrix path                (Section IV-C)
 *   wptr   int64[W+1]  offsets into wcols
 *   wcols  int32[total_ncols]  per window: its distinct column ids, ascending
 *   ecol   int32[nnz]  per non-zero (CSR order): position of its column in its window's wcols
 *          (hcspmm_prepare builds wcols / ecol for matrix-path windows only, no kernel reads the
 *          others; asking for either array here computes the rest first)
 *   mfma_windows int32[n_mfma_windows], csr_windows int32[n_csr_windows]: ascending window ids per route
 * Synchronises with the device.
 */
hcspmm_status hcspmm_plan_export(const hcspmm_plan* plan, int32_t* ncols, int32_t* nnzw, uint8_t* route,
                                 int64_t* wptr, int32_t* wcols, int32_t* ecol,
                                 int32_t* mfma_windows, int32_t* csr_windows);

/*
 * Launch table of the run kernel (plans prepared with matrix_kernels = HCSPMM_MATRIX_RUNS; sizes from
 * hcspmm_plan_info: n_runs, run_union_cols, total_ncols).  Run r covers entries [4r, min(4r + 4, n_mfma_windows))
 * of mfma_windows.  Each pointer may be NULL:
 *   run_nu  int32[n_runs]          length of the run's merged column list
 *   ucols   int32[run_union_cols]  the merged lists, run after run, each ascending
 *   wslot   int32[total_ncols]     indexed like wcols: position of that window column in its run's merged
 *                                  list (-1 for columns of scalar-path windows)
 * HCSPMM_EINVAL when the plan has no run table.  Synchronises with the device.
 */
hcspmm_status hcspmm_plan_export_runs(const hcspmm_plan* plan, int32_t* run_nu, int32_t* ucols, int32_t* wslot);

/*
 * Y = A X on the hybrid paths (Eq. 1; Alg. 1/3 for route-0 windows, Alg. 2/4
 * for route-1 windows).  Y is overwritten (rows without entries become 0).
 *
 *   d_X      device, n_cols x d, row-major, leading dimension ldx >= d, dtype x_dtype
 *   d_Y      device, n_rows x d, row-major, leading dimension ldy >= d, dtype y_dtype
 *   x_dtype  HCSPMM_F32: fp32 arithmetic on both paths (true fp32 MFMA);
 *            HCSPMM_BF16 / HCSPMM_F16: the matrix path multiplies 16-bit
 *            operands (A values rounded to the same type) with fp32
 *            accumulation, the scalar path widens X to fp32.
 *   y_dtype  HCSPMM_F32, or HCSPMM_BF16 / HCSPMM_F16: the fp32 result of either path is rounded ONCE, to
 *            nearest even, when it is stored (the next layer can then gather 16-bit rows without a
 *            conversion pass in between).  ldy counts elements of that type.
 * X and Y must not overlap.  1 <= d <= 2^20.  Asynchronous on `stream`.
 *
 * A plan holds scratch buffers of its own (partial rows of long rows, partial tiles of wide
 * windows; allocated on the first call that needs them, which synchronises `stream` if it has to
 * grow them): calls that use the same plan must be ordered, i.e. issued on one stream or
 * otherwise serialised by the caller.  Different plans are independent.  Once a call with the
 * largest d in use has been made, later calls allocate nothing and can be captured in a HIP graph.
 * The same holds for hcspmm_gcn_layer(_ex), hcspmm_aggregate_update and hcspmm_layer_backward: after
 * one eager call of each with the shapes in use they only enqueue kernels on `stream`.
 * X must be finite.  On the matrix path the dense-tile product multiplies every gathered row with
 * explicit zeros, so a NaN or Inf in a gathered row reaches all 16 rows of its window.  The scalar path
 * pads a row's last batch of non-zeros with (the row's last column, value 0): an Inf in that X row
 * then gives NaN where exact arithmetic gives +-Inf (rows that do not reference a non-finite X row
 * are unaffected on this path).
 */
hcspmm_status hcspmm_spmm(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                          void* d_Y, int64_t ldy, int32_t y_dtype, void* stream);

/*
 * hcspmm_spmm for callers that must not allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result bits as
 * hcspmm_spmm; the difference is where the call's scratch lives (the partial rows of long rows cut
 * into segments and the partial tiles of wide matrix-path windows cut into slices): not in buffers the
 * plan allocates on first use, but in one fixed array of HCSPMM_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy until the process ends).
 * The call allocates and frees nothing, on the device or through any library.
 *
 *   HCSPMM_EUNSUPPORTED  when the plan needs more scratch at this d than the array holds
 *                        (256-byte-padded 4*d*(segments of multi-segment rows) plus 64*d*(slices of
 *                        multi-slice windows) bytes); nothing is launched then, use hcspmm_spmm
 *   HCSPMM_EINVAL        also when the current device is not the plan's
 *
 * Every call on a GPU shares that GPU's array, across plans and streams: calls of this entry point that
 * overlap in time on one GPU race on it and must be ordered by the caller (one stream, or events).
 * Nothing in the array has to start at zero (every partial row and tile is written before it is
 * read), so the previous call's contents need no clearing.
 */
#define HCSPMM_STATIC_SCRATCH_BYTES ((size_t)16 << 20)

hcspmm_status hcspmm_spmm_noalloc(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                                  void* d_Y, int64_t ldy, int32_t y_dtype, void* stream);

/* HCSPMM_STATIC_SCRATCH_BYTES as the loaded library was built with it. */
size_t hcspmm_spmm_noalloc_scratch_limit(void);

/*
 * Same as hcspmm_spmm, but brackets every kernel stage with HIP events on `stream`, waits for
 * completion and reports the elapsed milliseconds per stage (for benchmarks and profiling; the
 * stages run in this order).  A stage that launches nothing reports 0.
 */
typedef struct {
    float ms_total;
    float ms_mfma_big;        /* matrix path, workgroup per window */
    float ms_mfma_small;      /* matrix path, wave per window */
    float ms_csr;             /* scalar path: long-row segments, mid rows and short rows in one launch */
    float ms_csr_reduce;      /* sum of the partial rows of rows cut into several segments */
} hcspmm_stage_times;

hcspmm_status hcspmm_spmm_timed(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d, int32_t x_dtype,
                                void* d_Y, int64_t ldy, int32_t y_dtype, void* stream,
                                hcspmm_stage_times* times /* host, out */);

/*
 * GCN layer  Y = act(A (X W))  (Eq. 1 and Eq. 2; Section V-A couples the two
 * phases).  The update X W is formed first by an fp32 MFMA GEMM into the
 * workspace and the hybrid SpMM gathers its rows from there at once; the
 * activation (ReLU when apply_relu != 0) is applied in the SpMM epilogue, after
 * the complete row sum, so the call is two kernel families and no separate
 * activation or layout pass.  In this association every window needs arbitrary
 * rows of X W, so the intermediate cannot stay inside one kernel (Section V-A
 * says the same of update-before-aggregate), and at the benchmark's layer size
 * the call costs what the two stages cost separately (hcspmm_gcn_layer_ex can
 * store the intermediate in 16 bits, which halves the gather bytes).
 *
 *   d_X   device, n_cols x d_in fp32 (ldx >= d_in);  d_W  device, d_in x d_out fp32 (ldw >= d_out)
 *   d_Y   device, n_rows x d_out fp32 (ldy >= d_out)
 *   d_workspace  device, at least hcspmm_gcn_workspace_bytes(plan, d_in, d_out) bytes, 256-byte aligned
 * Asynchronous on `stream`.
 */
hcspmm_status hcspmm_gcn_layer(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in,
                               const void* d_W, int64_t ldw, int32_t d_out,
                               void* d_Y, int64_t ldy, int32_t apply_relu,
                               void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * The same layer with the intermediate T = X W stored as t_dtype: HCSPMM_F32 is hcspmm_gcn_layer;
 * HCSPMM_BF16 / HCSPMM_F16 round the fp32 MFMA accumulators of the update once (nearest even) and
 * let the aggregation gather half the bytes, with the arithmetic hcspmm_spmm documents for a
 * 16-bit X (the plan should then have been prepared with mfma_dtype = t_dtype, which selects the
 * selector coefficients fitted for 16-bit gathers).  y_dtype is the element type of Y as in
 * hcspmm_spmm (one rounding of the fp32 result when it is stored).  X and W stay fp32; the workspace
 * requirement is that of hcspmm_gcn_workspace_bytes.  HCSPMM_EUNSUPPORTED when the plan has
 * matrix-path windows and d_out / ldy do not fit the 16-bit matrix-path kernels (d_out % 4,
 * 16-byte aligned Y rows).
 */
hcspmm_status hcspmm_gcn_layer_ex(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in,
                                  const void* d_W, int64_t ldw, int32_t d_out,
                                  void* d_Y, int64_t ldy, int32_t y_dtype, int32_t apply_relu, int32_t t_dtype,
                                  void* d_workspace, size_t workspace_bytes, void* stream);

size_t hcspmm_gcn_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out);

/*
 * Aggregate-then-update layer  Y = act((A X) W)  -- the association of GIN's forward pass and of
 * GCN's backward pass, for which Section V-A describes the coupled kernel (aggregate a window,
 * then multiply its result tile by W).  With d_in a multiple of 16 up to 256 (and X aligned for
 * vector loads) the update
 * is fused into the aggregation kernels: short scalar-path rows and wave-per-window matrix-path
 * tiles stay in LDS and are multiplied by W on the fp32 matrix cores before anything is stored;
 * the remaining rows (long rows, very wide windows) pass through the workspace.  Otherwise, and when
 * those remaining rows are a quarter of the matrix or more, Z = A X is written to the workspace
 * and one fp32 MFMA kernel applies W and the activation (also for fp32 X with d_in of 48..128 and
 * d_out <= 64 on matrices of 32,768 rows or more, where that route measured faster).
 *
 *   d_X   device, n_cols x d_in, element type x_dtype (ldx >= d_in)
 *   d_W   device, d_in x d_out fp32 (ldw >= d_out)
 *   d_Y   device, n_rows x d_out of element type y_dtype (ldy >= d_out, in elements): fp32, or bf16 / fp16 with one
 *         rounding of the fp32 result when it is stored -- a chain of such layers with 16-bit X and Y needs no
 *         conversion pass between layers
 *   d_workspace  device, at least hcspmm_aggregate_update_workspace_bytes(plan, d_in, d_out) bytes,
 *                256-byte aligned; holds Z (n_rows x d_in fp32) on return when the update was not fused
 * Asynchronous on `stream`.  Errors as hcspmm_spmm.
 */
hcspmm_status hcspmm_aggregate_update(const hcspmm_plan* plan, const void* d_X, int64_t ldx, int32_t d_in,
                                      int32_t x_dtype, const void* d_W, int64_t ldw, int32_t d_out,
                                      void* d_Y, int64_t ldy, int32_t y_dtype, int32_t apply_relu,
                                      void* d_workspace, size_t workspace_bytes, void* stream);

size_t hcspmm_aggregate_update_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out);

/*
 * Backward pass of the layer  X_next = act(A_f (X W))  (Eq. 3 and Eq. 4), given G = dL/dX_next:
 *     Gm = G where Y_fwd > 0, else 0        (only with d_Yfwd; the derivative of max(0, .))
 *     S  = A Gm                             (Eq. 4; A is the plan's matrix: the transpose of the forward
 *                                            matrix A_f -- the same plan when A_f is symmetric, as the
 *                                            normalised adjacency of an undirected graph is)
 *     dX = S W^T                            (n_rows x d_in)
 *     dW = X^T S                            (d_in x d_out)
 * This is the stage of training where the update follows the aggregation (Section V-A): dX is
 * computed like hcspmm_aggregate_update computes its Y, the aggregated tile multiplied by W^T on the
 * matrix cores without a round trip (under the same conditions: d_out a multiple of 16 up to 256,
 * few long rows; with d_dW given, which makes the kernels store the tile as well, only for d_out <= 32,
 * where that measured faster), else by a GEMM.  dW is a reduction over all rows of the graph: S is also written
 * to the workspace, and one streaming fp32 MFMA kernel forms X^T S from contiguous row spans whose
 * partial products are added in span order (the result does not depend on scheduling).
 * Eq. 3 as printed, W' = Z^T X' with the aggregated Z = A X_k, is the same call with the dense
 * operands exchanged (d_G = X_k, d_X = X'): d_dW then holds W' transposed.
 *
 *   d_G     device, n_cols x d_out fp32 (ldg >= d_out): gradient with respect to the layer's output
 *   d_Yfwd  device, n_cols x d_out fp32 (ldyf >= d_out): the layer's forward output, or NULL when the
 *           layer had no activation
 *   d_X     device, n_rows x d_in fp32 (ldx >= d_in): the layer's forward input
 *   d_W     device, d_in x d_out fp32 (ldw >= d_out)
 *   d_dX    device, n_rows x d_in fp32 (lddx >= d_in), overwritten;  NULL: dX is not computed
 *   d_dW    device, d_in x d_out fp32 (lddw >= d_out), overwritten;  NULL: dW is not computed
 *   mask_dx_by_x  non-zero: d_dX receives dX where X > 0 and 0 elsewhere.  When the layer's input X is itself
 *           the output of the previous layer's max(0, .), that is the gradient the previous layer's
 *           backward call needs as its d_G, already masked (its d_Yfwd is then NULL): the mask is applied
 *           when dX is stored, which saves that call's separate masking pass over G.
 *   d_workspace  device, at least hcspmm_layer_backward_workspace_bytes(plan, d_in, d_out) bytes,
 *                256-byte aligned; its first n_rows x d_out floats hold S on return when d_dW was given
 * Outputs must not alias inputs.  Asynchronous on `stream`.  Errors as hcspmm_spmm.
 */
hcspmm_status hcspmm_layer_backward(const hcspmm_plan* plan, const void* d_G, int64_t ldg, int32_t d_out,
                                    const void* d_Yfwd, int64_t ldyf,
                                    const void* d_X, int64_t ldx, int32_t d_in,
                                    const void* d_W, int64_t ldw,
                                    void* d_dX, int64_t lddx, void* d_dW, int64_t lddw, int32_t mask_dx_by_x,
                                    void* d_workspace, size_t workspace_bytes, void* stream);

size_t hcspmm_layer_backward_workspace_bytes(const hcspmm_plan* plan, int32_t d_in, int32_t d_out);

/* Dense update alone, T = X W in fp32 MFMA (Eq. 2): d_X M x K, d_W K x N, d_T M x N, all fp32 device. */
hcspmm_status hcspmm_gemm_f32(int64_t m, int32_t k, int32_t n, const float* d_X, int64_t ldx,
                              const float* d_W, int64_t ldw, float* d_T, int64_t ldt, void* stream);

/*
 * Layout reformatting (Section V-B, Alg. 5/6, Eq. 5/6): an offline, host-side regrouping of the
 * vertices into row windows of higher computing intensity (#non-zeros / #non-zero columns), so
 * that more windows suit the matrix path.  Vertices are sorted by their smallest neighbour index;
 * each window is seeded with the first unplaced vertex of that list and grown window_rows - 1
 * times by the unplaced vertex, among the sorted positions seed .. seed + vw, that maximises the
 * window's intensity (ties: more neighbours, then the earlier position; intensities compared as
 * exact rationals).  If those positions hold no unplaced vertex the next unplaced vertex of the
 * list is taken.
 *
 *   h_rowptr, h_colind   host, CSR structure of the n_rows x n_cols matrix (rows need not be sorted)
 *   vw                   size of the vertices window (>= 0);  window_rows: 16 for hcspmm_prepare
 *   h_order              host, n_rows entries, out: h_order[i] = old id of the vertex placed i-th
 * Runs on the calling thread; touches no GPU.  HCSPMM_EBADCSR for an inconsistent CSR.
 */
hcspmm_status hcspmm_loa_order(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                               int32_t vw, int32_t window_rows, int32_t* h_order /* host, out */);

/*
 * hcspmm_loa_order plus its effect: h_total_ncols[0] receives the sum over all row windows of the number of
 * distinct columns for the layout as stored, h_total_ncols[1] the same sum for the returned order (the number of
 * non-zeros divided by these sums is the computing intensity of Eq. 5 over the whole matrix, before and after).
 * The greedy regrouping starts from the vertices sorted by their smallest neighbour, which can scatter a layout
 * that already had locality: apply the order only when h_total_ncols[1] < h_total_ncols[0].  The two sums are
 * computed by several host threads.
 */
hcspmm_status hcspmm_loa_order_checked(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                                       int32_t vw, int32_t window_rows, int32_t* h_order /* host, out */,
                                       int64_t* h_total_ncols /* host, out, 2 entries */);

/*
 * Applies a vertex order to a square CSR matrix on the host ("reorder G", Alg. 5): row and column
 * h_order[i] of the input become row and column i of the output, columns ascending within a row.
 * With P the permutation matrix of the order, the output is P A P^T, so Y' = A' X' holds for
 * X' = P X and Y' = P Y.  Output arrays are caller-allocated with the input's sizes.
 */
hcspmm_status hcspmm_permute_csr(int32_t n, const int32_t* h_rowptr, const int32_t* h_colind, const float* h_vals,
                                 const int32_t* h_order, int32_t* h_out_rowptr, int32_t* h_out_colind,
                                 float* h_out_vals);

/*
 * Transpose of a CSR matrix on the host: the backward aggregation (Eq. 4) multiplies by the
 * transpose of the forward matrix, which is the matrix itself only when it is symmetric; for a
 * directed graph prepare a second plan from this function's output.  The result is n_cols x n_rows
 * with ascending columns in every row.  h_out_rowptr has n_cols + 1 entries, h_out_colind and
 * h_out_vals as many as the input.  Runs on the calling thread; touches no GPU.
 */
hcspmm_status hcspmm_transpose_csr(int32_t n_rows, int32_t n_cols, const int32_t* h_rowptr, const int32_t* h_colind,
                                   const float* h_vals, int32_t* h_out_rowptr, int32_t* h_out_colind,
                                   float* h_out_vals);

/*
 * Measurement aid (no part of the method): the bare gather behind the scalar path of Alg. 1/3.  Reads
 * row d_index[i] of X for i = 0 .. n-1, in that order of the stream, with the scalar path's lane mapping
 * and eight row requests in flight per lane group, and does nothing else -- no row structure, no
 * values, no output rows.  Its duration is a floor for every kernel that fetches one X row per
 * non-zero of the same index stream (d_index = the CSR column array); bench.py reports the scalar
 * kernel against it.
 *
 *   d_index  device, int32[n]; values are clamped into [0, n_rows_x) before use
 *   d_X      device, n_rows_x x d fp32, ldx >= d; d a multiple of 4 in [4, 256], rows 16-byte aligned
 *   d_out    device, at least hcspmm_probe_gather_out_bytes(n, d) bytes, 16-byte aligned; receives
 *            per-lane sums of what was read (keeps the loads live; the values carry no meaning)
 * Asynchronous on `stream`.
 */
hcspmm_status hcspmm_probe_gather(const int32_t* d_index, int64_t n, const float* d_X, int64_t ldx, int32_t d,
                                  int32_t n_rows_x, float* d_out, size_t out_bytes, void* stream);
size_t hcspmm_probe_gather_out_bytes(int64_t n, int32_t d);

/* Changes options.update_fusion of an existing plan (hcspmm_update_fusion); calls already enqueued are not affected. */
hcspmm_status hcspmm_plan_set_update_fusion(hcspmm_plan* plan, int32_t update_fusion);

/* Frees everything the plan owns (not the borrowed CSR).  NULL is allowed. */
void hcspmm_plan_destroy(hcspmm_plan* plan);

const char* hcspmm_status_string(hcspmm_status s);
const char* hcspmm_last_error(void);
/* Library version: major*10000 + minor*100 + patch. */
int32_t hcspmm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HCSPMM_H */
