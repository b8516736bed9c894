/*
 * libra.h - C ABI of the MI355X (gfx950) hybrid SpMM / SDDMM library.
 *
 * The method follows arXiv 2506.22714 ("Libra"):
 *   - Section 2.2: rows are cut into windows of m rows; inside a window each
 *     column that holds a nonzero is an m x 1 nonzero column vector, and
 *     vectors are condensed k at a time into dense blocks.
 *   - Section 4.2 (Eq. 2-6): nonzeros are split between a matrix-unit path
 *     (here MFMA) and a scalar path (here VALU) by data reuse and utilisation.
 *   - Section 4.3: heavy windows and long rows are decomposed into bounded
 *     segments; decomposed segments accumulate with atomics.
 *   - Section 4.4: bitmap-encoded dense blocks decoded in registers, popcount
 *     offsets for SDDMM write-back, coalesced vector loads on the scalar path.
 *
 * Conventions
 *   - Every function returns LIBRA_OK (0) or a negative LIBRA_ERR_* code.
 *     Nothing throws or aborts across this boundary.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory on the current device.  The library never allocates device
 *     memory: the caller provides every device buffer and keeps it alive while
 *     any call that uses it may still be running.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Compute calls are asynchronous on that stream.
 *   - A is M x Kc in CSR (rowptr[M+1], col[nnz], val[nnz]); column indices are
 *     strictly increasing inside a row (no duplicates).
 */
#ifndef LIBRA_H
#define LIBRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LIBRA_VERSION 1

/* ---- error codes ---- */
#define LIBRA_OK                  0
#define LIBRA_ERR_NULL           -1   /* a required pointer is NULL */
#define LIBRA_ERR_SHAPE          -2   /* M, Kc, N, K, ld* out of range */
#define LIBRA_ERR_ROWPTR         -3   /* rowptr[0] != 0 or rowptr decreases */
#define LIBRA_ERR_COLUMN         -4   /* a column index is outside [0, Kc) */
#define LIBRA_ERR_UNSORTED       -5   /* columns in a row not strictly increasing */
#define LIBRA_ERR_TOO_LARGE      -6   /* nnz, M or Kc does not fit in 31 bits */
#define LIBRA_ERR_DTYPE          -7   /* unknown or unsupported value type */
#define LIBRA_ERR_OPTION         -8   /* an option is out of its documented range */
#define LIBRA_ERR_UNSUPPORTED    -9   /* valid request the kernels do not cover (e.g. N not a multiple of 32) */
#define LIBRA_ERR_NOT_UPLOADED  -10   /* compute call on a plan that has no device copy */
#define LIBRA_ERR_BUFFER        -11   /* device buffer too small or misaligned */
#define LIBRA_ERR_NOT_BUILT     -12   /* the sub-plan needed by the call was not built */
#define LIBRA_ERR_HIP           -13   /* a HIP runtime call or kernel launch failed */
#define LIBRA_ERR_NOMEM         -14   /* host allocation failed */

/* ---- value types (storage type of A's values and of the dense operands) ---- */
#define LIBRA_F16   0    /* IEEE binary16 in, fp32 accumulate (MFMA + VALU) */
#define LIBRA_BF16  1    /* bfloat16 in, fp32 accumulate (MFMA + VALU); beside the paper's FP16 / TF32 inputs (Section 4.4) */
#define LIBRA_F32   2    /* binary32 in, fp32 accumulate (MFMA 16x16x4 f32 + VALU): the paper's TF32 & FP32 mode with unrounded inputs */

/* ---- distribution modes (Section 5.3.2: matrix-unit-only, scalar-only, hybrid) ---- */
#define LIBRA_MODE_HYBRID       0
#define LIBRA_MODE_DENSE_ONLY   1
#define LIBRA_MODE_SCALAR_ONLY  2

/* ---- option flags ---- */
#define LIBRA_FLAG_NO_FILL_PADDING  1u  /* do not promote scalar-bound vectors into free slots of a window's last SpMM block */
#define LIBRA_FLAG_NO_SPMM          2u  /* skip the SpMM sub-plan */
#define LIBRA_FLAG_NO_SDDMM         4u  /* skip the SDDMM sub-plan */
#define LIBRA_FLAG_NATURAL_ORDER    8u  /* keep tasks in window order instead of heaviest-first */
#define LIBRA_FLAG_XCD_ORDER       16u  /* heaviest-first by groups of 4 neighbouring windows, one group per accelerator die
                                           (own L2): neighbours that read the same dense-operand rows share them; the
                                           task table then holds a few empty tasks (no work).  Without this flag and the
                                           next one the planner decides from the sampled neighbour_share statistic */
#define LIBRA_FLAG_NO_XCD_ORDER    32u  /* never use the die-aware order */
#define LIBRA_FLAG_SEGMENTS_BY_COLUMN 64u /* accepted, and what the planner does anyway (kept so that callers that ask for it
                                           still work): when the die-aware order is not in use, the segments of decomposed
                                           rows are sorted by their first column and cut into one run per die, so that a
                                           die fetches dense-operand rows of one column range only and its L2 holds eight
                                           times as many distinct hot rows; the flat SDDMM segments that lie inside one row are
                                           placed the same way */
#define LIBRA_FLAG_TWO_KERNELS    128u  /* libra_spmm runs the task table twice on the stream: first the dense blocks (MFMA), then the
                                           residual nonzeros (VALU), which add to what the first launch wrote - the paper's
                                           sequential schedule of its two kernels (Section 4.4.1).  Same results up to the order
                                           of additions; for debugging and as the baseline the fused task is measured against */

#define LIBRA_FLAG_SEGMENTS_BY_COST 256u /* leave the segments of decomposed rows where the heaviest-first order puts them */

typedef struct libra_plan_s libra_plan_t;   /* opaque; immutable after libra_plan() except for its values */

/*
 * Planner options.  A zero in any numeric field selects the default.
 * struct_size must be sizeof(libra_plan_opts_t) (versioning).
 */
typedef struct {
    uint32_t struct_size;
    int32_t  mode;               /* LIBRA_MODE_*                                                         */
    int32_t  window_rows;        /* m of Section 2.2. default 16; planner accepts 1..32, kernels need 16 */
    int32_t  block_cols;         /* k (SpMM) / n (SDDMM) of Section 2.2. default 16; planner accepts 1..64, kernels need 16 */
    int32_t  spmm_min_vec_nnz;   /* tau_spmm = ceil(eta_thr * m), Eq. 6: vector is dense iff NNZ_vector >= tau. default 3 */
    int32_t  sddmm_min_blk_nnz;  /* tau_sddmm = ceil(eta_thr * m * n), Eq. 6: block is dense iff NNZ_block >= tau. default 64 */
    int32_t  ts;                 /* Ts of Section 4.3 (SpMM sub-plan): a window's dense part is decomposed iff it has more than ts blocks. default 16 */
    int32_t  cs;                 /* Cs of Section 4.3: a residual row is decomposed iff it has more than cs nonzeros. default 128 */
    int32_t  short_len;          /* Short_len of Section 4.3: a residual row with fewer nonzeros is "short". default 3 */
    int32_t  sddmm_cs;           /* SDDMM residual nonzeros per scalar segment. default 128 */
    uint32_t flags;              /* LIBRA_FLAG_* */
    int32_t  threads;            /* host threads for planning; 0 = hardware concurrency */
    int32_t  sddmm_ts;           /* SDDMM: dense blocks of a window per task (Ts of Section 4.3 for the SDDMM sub-plan; its tasks
                                    write disjoint outputs, so cutting a window costs no atomics). default 4 */
    int32_t  sddmm_min_dense_pct;/* SDDMM, hybrid mode: the utilisation argument of Section 4.2.2 applied to the whole matrix.  If the
                                    blocks that pass tau_sddmm hold less than this percentage of the nonzeros, the sub-plan sends
                                    every nonzero to the scalar path (a few dense blocks cost more in outputs written twice, once
                                    by each kind of task, than they save).  1..100; default 0 = rule off */
} libra_plan_opts_t;

/* ---- task table entry (Section 4.3: WindowOffset/RowOffset, CurWindow/CurRow, Atomic) ---- */
#define LIBRA_TASK_WINDOW 0   /* dense blocks [blk_begin,blk_end) of window `id` plus residual nonzeros [res_begin,res_end) */
#define LIBRA_TASK_CHUNK  1   /* SpMM: residual nonzeros [res_begin,res_end) of the decomposed row `id`
                                 SDDMM: residual nonzeros [res_begin,res_end) of the residual list (id = 0) */
typedef struct {
    int32_t  kind;
    int32_t  id;
    int32_t  blk_begin, blk_end;
    int32_t  res_begin, res_end;
    uint32_t scalar_mask;   /* SpMM window task: bit r set = [res_begin,res_end) holds the residual nonzeros of row id*m + r */
    uint32_t atomic_mask;   /* SpMM window task: rows this task adds to C with atomics (they are zero-initialised first) */
    uint32_t store_mask;    /* SpMM window task: rows this task alone owns and writes with plain stores (zeros included) */
    uint32_t cost;          /* modelled rows of the dense operand this task fetches (ordering key) */
} libra_task_t;

/* ---- read-only host view of one sub-plan, for checkers ---- */
typedef struct {
    int64_t n_windows, n_blocks, n_dense_nnz, n_res_nnz, n_tasks, n_zero_rows;
    int32_t window_rows, block_cols, words_per_block, value_dtype;
    const int32_t  *win_blkptr;   /* [n_windows+1] first block of each window                                   */
    const int32_t  *blk_cols;     /* [n_blocks*block_cols] column of each slot, -1 = padding                     */
    const uint64_t *blk_bitmap;   /* [n_blocks*words_per_block] bit r*block_cols+s = nonzero at (row r, slot s)  */
    const int32_t  *blk_valptr;   /* [n_blocks+1] first packed value of each block                               */
    const void     *dense_val;    /* [n_dense_nnz] packed values in bit order, value_dtype                       */
    const int32_t  *dense_perm;   /* [n_dense_nnz] CSR position of each packed value                             */
    const int32_t  *win_resptr;   /* SpMM: [n_windows+1] first residual nonzero of each window; SDDMM: NULL      */
    const int32_t  *res_row;      /* [n_res_nnz] row of each residual nonzero                                    */
    const int32_t  *res_col;      /* [n_res_nnz]                                                                 */
    const void     *res_val;      /* [n_res_nnz] value_dtype                                                     */
    const int32_t  *res_perm;     /* [n_res_nnz] CSR position.  SDDMM: increasing.  SpMM: window by window, the
                                     rows that are not decomposed first (row order), then the decomposed rows     */
    const libra_task_t *tasks;    /* [n_tasks] in launch order                                                   */
    const int32_t  *zero_rows;    /* SpMM: [n_zero_rows] rows cleared before the kernel (rows with >1 writer)    */
} libra_subplan_view_t;

/* ---- planner statistics (Section 4.2 cost model evaluated on the plan) ---- */
typedef struct {
    int64_t M, Kc, nnz;
    int64_t n_windows;
    int64_t n_vectors;            /* nonzero column vectors over all windows                         */
    int64_t n_vectors_nnz1;       /* of which hold exactly one nonzero (Fig. 1's NNZ-1 ratio)        */
    /* SpMM sub-plan */
    int64_t spmm_dense_vectors, spmm_blocks, spmm_pad_slots, spmm_dense_nnz, spmm_res_nnz;
    int64_t spmm_tasks, spmm_chunk_tasks, spmm_zero_rows;
    int64_t spmm_short_rows, spmm_long_rows, spmm_split_rows;
    int64_t spmm_gather_rows;     /* dense vectors + residual nonzeros: dense-operand rows fetched (Eq. 2 numerator vs denominator, summed) */
    /* SDDMM sub-plan */
    int64_t sddmm_dense_vectors, sddmm_blocks, sddmm_pad_slots, sddmm_dense_nnz, sddmm_res_nnz;
    int64_t sddmm_tasks;
    int64_t sddmm_gather_rows;    /* per dense block m + real columns, per residual nonzero 2 (Eq. 4, summed) */
    double  plan_seconds;
    double  neighbour_share;      /* sampled: distinct columns of 4 neighbouring windows taken together / taken one by
                                     one (1 = neighbours share no dense-operand row, 0.25 = they read the same rows) */
    int64_t xcd_order;            /* 1 if the task tables are in the die-aware order */
    double  device_seconds;       /* libra_plan_device: time until the device passes had finished (0 for libra_plan) */
} libra_stats_t;

/*
 * libra_plan - build the distribution plan of A (Sections 4.2-4.3, host work only).
 *   M, Kc        in   matrix shape, 1 <= M, Kc < 2^31
 *   rowptr       in   host, int32[M+1], rowptr[0] = 0, non-decreasing, rowptr[M] = nnz < 2^31
 *   col          in   host, int32[nnz], strictly increasing inside each row, 0 <= col < Kc
 *   val          in   host, nnz values of type val_dtype (LIBRA_F16, LIBRA_BF16 or LIBRA_F32).  The split does not depend
 *                     on the type; fp32 dense tiles run on v_mfma_f32_16x16x4_f32 (CDNA4 has no TF32: nothing is rounded).
 *   opts         in   host, may be NULL (all defaults)
 *   out          out  receives a new plan; release with libra_plan_destroy.  The inputs are copied,
 *                     the caller may free them after the call.
 * Errors: NULL, SHAPE, ROWPTR, COLUMN, UNSORTED, TOO_LARGE, DTYPE, OPTION, NOMEM.
 */
int libra_plan(int64_t M, int64_t Kc, const int32_t *rowptr, const int32_t *col,
               const void *val, int val_dtype, const libra_plan_opts_t *opts, libra_plan_t **out);

/*
 * libra_plan_device - the same plan, bit for bit, built on the GPU from a CSR matrix that is already in device
 * memory (the paper's GPU-accelerated preprocessing, Section 4.5, Algorithm 1: per-window census by sorting,
 * prefix sums for every offset).  Only the kernels' shape is supported (window_rows = block_cols = 16).
 *   d_rowptr, d_col, d_val   device, as in libra_plan; nnz must equal d_rowptr[M]
 *   workspace                device, 256-byte aligned, at least libra_plan_device_workspace() bytes; only used
 *                            during the call, the caller may free it afterwards
 *   plan_buf, plan_bytes     device, 256-byte aligned, or NULL.  If given, the plan's device copy is written
 *                            there directly from the workspace (no trip through host memory) and the plan is
 *                            ready for the compute calls; it needs libra_plan_device_bytes() of the finished
 *                            plan, which libra_plan_device_buffer_bound() bounds from M and nnz beforehand.
 *                            The plan borrows it until libra_plan_destroy.  NULL: call libra_plan_upload later.
 *   keep_host_copy           nonzero: the arrays are also copied into the plan's host memory, so that
 *                            libra_plan_export and libra_plan_upload work as for a host-built plan.  Zero (only
 *                            with plan_buf): they are not; those two calls then return LIBRA_ERR_NOT_BUILT.
 *   stream                   the passes are enqueued on it; the call synchronises it several times
 * The task tables always pass through the host: their order and the statistics are made by the same code as in
 * libra_plan.  A matrix without nonzeros needs no device pass.
 * Errors: as libra_plan, plus UNSUPPORTED (window shape), BUFFER (workspace or plan buffer too small or
 * misaligned), HIP.
 */
int libra_plan_device_workspace(int64_t M, int64_t nnz, const libra_plan_opts_t *opts, size_t *bytes);
int libra_plan_device_buffer_bound(int64_t M, int64_t nnz, int val_dtype, const libra_plan_opts_t *opts, size_t *bytes);
int libra_plan_device(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                      const void *d_val, int val_dtype, const libra_plan_opts_t *opts,
                      void *workspace, size_t workspace_bytes, void *plan_buf, size_t plan_bytes,
                      int keep_host_copy, void *stream, libra_plan_t **out);

/*
 * libra_plan_device_bytes - bytes of device memory the plan's arrays need (256-byte aligned layout).  The plan is the
 * paper's one-off preprocessing result (Section 4.1: the matrix is translated once into bitmap blocks for the matrix
 * unit and a CSR-like residual for the scalar path, item 3, and reused by every later call); this is the size of that
 * translated form, which the caller allocates.  Errors: NULL.
 */
int libra_plan_device_bytes(const libra_plan_t *plan, size_t *bytes);

/*
 * libra_plan_upload - copy the plan's arrays (the translated formats of Section 4.1, item 3: bitmap blocks, packed
 * values, residual entries, task tables of Section 4.3) into caller-owned device memory, once per matrix.
 *   dev_buf  device pointer, 256-byte aligned, at least libra_plan_device_bytes() bytes;
 *            the plan borrows it until libra_plan_destroy or the next upload.
 * The copies are enqueued on `stream` and the stream is synchronised before returning
 * (the sources are pageable host memory).  Errors: NULL, BUFFER, HIP; UNSUPPORTED for a
 * plan with more than 2^27 columns (the device copy of a residual nonzero keeps its column
 * in 27 bits; libra_plan_device with a plan buffer returns the same).
 */
int libra_plan_upload(libra_plan_t *plan, void *dev_buf, size_t bytes, void *stream);

/*
 * libra_spmm - C = A * B (Section 2.2; Eq. 2 for what each path fetches).
 *   B    device, Kc x N row-major with row stride ldb elements (ldb >= N, ldb % 8 == 0), plan's value type
 *   C    device, M x N row-major fp32 with row stride ldc (ldc >= N, ldc % 4 == 0); fully overwritten
 *        (rows of A without nonzeros become zeros); must not alias B.
 *   N    multiple of 32 (fp16) or of 16 (fp32), 32 <= N <= 512
 * Dense blocks run on MFMA (operands of the plan's value type, fp32 accumulate), residual nonzeros on the VALU (fp32 FMA);
 * rows with one writer are stored once, rows with several writers are cleared and accumulated with
 * fp32 atomics (their summation order is not deterministic).
 * B must hold finite numbers: a dense block multiplies the empty slots of its tile (zeros) by the gathered rows of B, so
 * an Inf or NaN in row j of B reaches every row of a window that has a dense block with column j, not only the rows
 * with a nonzero in column j (0 * Inf = NaN), where the definition would leave them untouched.  The same holds for
 * X and Y in libra_sddmm only for outputs that exist (an output is always a sampled product).
 * ldb * (bytes per element) must be below 2^32.
 * Errors: NULL, SHAPE, UNSUPPORTED, NOT_UPLOADED, NOT_BUILT, HIP.
 */
int libra_spmm(const libra_plan_t *plan, const void *B, int32_t N, int64_t ldb,
               float *C, int64_t ldc, void *stream);

/*
 * libra_sddmm - out[p] = val[p] * <X[i,:], Y[col[p],:]> for every nonzero p of row i (Section 2.2; Eq. 4).
 *   X    device, M x K row-major, contiguous, plan's value type
 *   Y    device, Kc x K row-major, contiguous, plan's value type
 *   out  device, fp32[nnz] in A's CSR order; fully overwritten (may be NULL when nnz = 0)
 *   K    32, 64 or 128
 * Errors: NULL, UNSUPPORTED, NOT_UPLOADED, NOT_BUILT, HIP.
 */
int libra_sddmm(const libra_plan_t *plan, const void *X, const void *Y, int32_t K,
                float *out, void *stream);

/*
 * libra_sddmm_pattern - as libra_sddmm without A's values: out[p] = <X[i,:], Y[col[p],:]>.  The gradient of SpMM with
 * respect to A's values is this product of dC and B (the training use of the operators, Section 5.5).
 */
int libra_sddmm_pattern(const libra_plan_t *plan, const void *X, const void *Y, int32_t K,
                        float *out, void *stream);

/*
 * libra_edge_softmax - row-wise softmax over CSR-ordered scores (the step between SDDMM and SpMM in an
 * attention layer, Section 5.5): vals_out[p] = exp(scale*s[p] - mx_i) / sum_row exp(scale*s[q] - mx_i).
 *   scores    device, fp32[nnz], CSR order
 *   vals_out  device, nnz values of out_dtype (LIBRA_F16, LIBRA_BF16 or LIBRA_F32; rounded to nearest even), CSR order;
 *             may not alias scores
 * Errors: NULL, DTYPE, NOT_UPLOADED, HIP.
 */
int libra_edge_softmax(const libra_plan_t *plan, const float *scores, float scale,
                       void *vals_out, int out_dtype, void *stream);

/*
 * libra_edge_softmax_backward - gradient of libra_edge_softmax with respect to the scores:
 * dscores[p] = scale * alpha[p] * (dalpha[p] - sum over the row of alpha[q] * dalpha[q]).
 *   alpha     device, nnz values of alpha_dtype (what the forward call wrote), CSR order
 *   dalpha    device, fp32[nnz]; dscores  device, fp32[nnz], may not alias the inputs
 * Errors: NULL, DTYPE, NOT_UPLOADED, HIP.
 */
int libra_edge_softmax_backward(const libra_plan_t *plan, const void *alpha, int alpha_dtype, const float *dalpha,
                                float scale, float *dscores, void *stream);

/*
 * libra_csr_transpose_device - CSR pattern of the transposed matrix, on the device (the backward pass of SpMM,
 * dB = A^T dC, runs on a plan of A^T; Section 5.5 trains GNNs with these operators).
 *   d_rowptr, d_col      device, the M x Kc matrix (as in libra_plan_device; not validated here)
 *   d_rowptr_t           device, int32[Kc+1] out
 *   d_col_t, d_perm_t    device, int32[nnz] out: row index and CSR position in A of every nonzero of A^T, so that
 *                        values of A^T are values_of_A[d_perm_t[q]]
 *   workspace            device, 256-byte aligned, libra_csr_transpose_workspace(nnz) bytes, free after the call
 * The call synchronises the stream.  Errors: NULL, SHAPE, TOO_LARGE, BUFFER, HIP.
 */
int libra_csr_transpose_workspace(int64_t nnz, size_t *bytes);
int libra_csr_transpose_device(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                               int32_t *d_rowptr_t, int32_t *d_col_t, int32_t *d_perm_t,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * libra_csr_transpose_device_static - libra_csr_transpose_device for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): same inputs and outputs, no workspace
 * argument.  The workspace is a fixed array of LIBRA_TRANSPOSE_STATIC_MAX_NNZ * 40 bytes (40 MiB) in the library's device
 * image, which every GPU the process uses holds until the process ends.  The call allocates and frees nothing, only
 * enqueues kernels on `stream` and does not synchronise it: the outputs are valid once the stream has reached them.
 * All calls on one GPU share that array: calls on one stream run one after the other and are safe; calls that may overlap
 * (different streams or threads, same GPU) race and must be ordered by the caller.
 * Errors: as libra_csr_transpose_device without BUFFER; TOO_LARGE for nnz > LIBRA_TRANSPOSE_STATIC_MAX_NNZ.
 */
#define LIBRA_TRANSPOSE_STATIC_MAX_NNZ (1 << 20)
int libra_csr_transpose_device_static(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                                      int32_t *d_rowptr_t, int32_t *d_col_t, int32_t *d_perm_t, void *stream);

/*
 * libra_probe_coissue - the register-only concurrency experiment of Section 3.1 on this GPU: 1024 workgroups of 8 waves
 * (two per SIMD) run `iters` rounds of (a) 4 independent MFMA 16x16x16 chains on four of the waves, (b) 32 FMAs on
 * 8 independent chains on the other four, (c) both at once.  times_us[0..2] receive the best of three timed launches of
 * (a), (b), (c).  (c) close to max(a, b) means the two units work side by side.
 *   sink_dev  device, at least one float (never written in practice; keeps the loops alive)
 *   times_us  host out.  The call creates two events, synchronises on them, and destroys them.
 * Errors: NULL, SHAPE, HIP.
 */
int libra_probe_coissue(int iters, float *sink_dev, float times_us[3], void *stream);

/*
 * libra_probe_gather - the row fetches of a call and nothing else (measurement aid): lane groups fetch row idx[i]
 * (row_bytes = 64, 128 or 256: a row of B or Y at 32, 64 or 128 16-bit features) of `table`, 256 consecutive indices per
 * wave, 8 rows in flight per lane group, and fold what arrives into a register.  The time of this launch is the floor of
 * any kernel that must bring these rows, in this order, into a compute unit (Eq. 2 / Eq. 4 count exactly these fetches);
 * the benchmark reports the task kernels against it.
 *   table_dev  device, table_rows x row_bytes, 16-byte aligned; every idx[i] must lie in [0, table_rows) (not checked)
 *   idx_dev    device, int32[n];  sink_dev  device, one float, practically never written
 * Asynchronous on `stream`.  Errors: NULL, SHAPE, BUFFER, TOO_LARGE, UNSUPPORTED (row_bytes), HIP.
 */
int libra_probe_gather(const void *table_dev, int64_t table_rows, int32_t row_bytes, const int32_t *idx_dev, int64_t n,
                       float *sink_dev, void *stream);

/*
 * libra_probe_gather_hub - the same fetches with the most referenced rows held in LDS (measurement aid): what the data
 * reuse of Section 4.2.1 (Eq. 2-3) would gain if the rows of the dense operand that many nonzeros share were kept in a
 * compute unit's own memory instead of coming out of the L2 each time.  One persistent workgroup of 1024 threads per
 * compute unit copies rows hub_rows[0 .. n_hub) of the table into LDS once; then, as in libra_probe_gather, every wave
 * walks 256 consecutive indices at a time: idx[i] >= 0 is fetched from the table, idx[i] < 0 reads slot ~idx[i] of the
 * LDS copy (a slot >= n_hub reads the last slot; a row index outside the table reads zeros - the table is addressed
 * through range-checked buffer loads, so no index can leave it).
 *   table_dev     device, table_rows x row_bytes (64, 128 or 256), 16-byte aligned, smaller than 4 GiB
 *   idx_dev       device, int32[n];   hub_rows_dev  device, int32[n_hub] table rows (may be NULL when n_hub = 0)
 *   n_hub         n_hub * row_bytes <= LIBRA_PROBE_HUB_MAX_BYTES (LDS of one compute unit, less what the waves need)
 * Asynchronous on `stream`.  Errors: NULL, SHAPE, BUFFER, TOO_LARGE, UNSUPPORTED (row_bytes), HIP.
 */
#define LIBRA_PROBE_HUB_MAX_BYTES (128 * 1024)
int libra_probe_gather_hub(const void *table_dev, int64_t table_rows, int32_t row_bytes, const int32_t *idx_dev, int64_t n,
                           const int32_t *hub_rows_dev, int32_t n_hub, float *sink_dev, void *stream);

/*
 * libra_plan_set_values - replace A's values (same pattern): scatters CSR-ordered device values into the
 * packed dense-block and residual arrays of both sub-plans' device copies.  The distribution of Section 4.2 depends
 * on the pattern only, so the preprocessing of Section 4.1 is reused as it is when only the values change (an
 * attention layer writes new coefficients on a fixed graph in every pass, Section 5.5).  The host copy keeps the old
 * values.  `dtype` must equal the plan's value type.  Errors: NULL, DTYPE, NOT_UPLOADED, HIP.
 */
int libra_plan_set_values(libra_plan_t *plan, const void *vals_csr_dev, int dtype, void *stream);

/*
 * libra_plan_set_values_for - the same for the arrays of one operator only (`ops` = LIBRA_OP_SPMM, LIBRA_OP_SDDMM or
 * both or-ed together).  An attention layer (SDDMM with A's pattern -> softmax -> SpMM with the new coefficients,
 * Section 5.5) only needs the SpMM arrays refreshed; the other sub-plan then keeps its previous values, and what
 * libra_sddmm computes with them is the caller's business.  Errors as above, plus OPTION for an `ops` without a known bit
 * or with an unknown one.
 */
#define LIBRA_OP_SPMM  1
#define LIBRA_OP_SDDMM 2
int libra_plan_set_values_for(libra_plan_t *plan, const void *vals_csr_dev, int dtype, int ops, void *stream);

/* Host views for checkers; pointers stay valid until libra_plan_destroy.  which: 0 = SpMM, 1 = SDDMM. */
int libra_plan_export(const libra_plan_t *plan, int which, libra_subplan_view_t *view);
int libra_plan_stats(const libra_plan_t *plan, libra_stats_t *stats);

void        libra_plan_destroy(libra_plan_t *plan);
const char *libra_strerror(int code);
int         libra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LIBRA_H */
