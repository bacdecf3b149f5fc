/*
 * asyncsparse.h -- C ABI of the MI355X (gfx950) sparse-times-dense library.
 *
 * Computes C = A x B with A sparse (m x k), B dense (k x N), C dense (m x N)
 * (paper, Section II-C, problem statement), with A re-stored either as Block
 * Compressed Sparse Row (BCSR) or as Window Compressed Sparse Row (WCSR)
 * (Section II-C, "Sparse Formats"), and WCSR row-windows cut into fixed-size
 * sub-tasks for load balance (Section III-C, last paragraph).
 *
 * General rules
 *   - Every call returns an asp_status_t.  Nothing throws, nothing aborts.
 *     asp_last_error() gives a thread-local detail string for the last failure.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *     memory of the GPU that was current when the handle was created.
 *   - A handle is immutable after creation: concurrent asp_spmm calls on
 *     different streams with different C buffers are safe.  The one exception
 *     is a WCSR handle whose split windows go through the handle's scratch
 *     buffer (asp_reserve): those calls must be ordered on one stream; calls
 *     of asp_spmm_static_scratch share one scratch array per GPU in the same way.
 *   - asp_spmm, asp_spmm_xt and asp_spmm_static_scratch only launch kernels on
 *     the caller's stream (no allocation, no memset, no host synchronisation),
 *     so they may be recorded into a HIP graph; handle creation, asp_reserve
 *     and asp_destroy allocate or free and may not.
 *   - The library needs a gfx950 GPU for everything except the calls marked
 *     "host only".  There is no CPU fallback for the product.
 */
#ifndef ASYNCSPARSE_H
#define ASYNCSPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct asp_handle asp_handle_t; /* opaque, owned by the library */

typedef enum {
    ASP_OK = 0,
    ASP_ERR_INVALID_ARG = 1,      /* null pointer, non-positive size, misuse */
    ASP_ERR_INVALID_CSR = 2,      /* CSR arrays are not a valid sorted CSR matrix */
    ASP_ERR_UNSUPPORTED = 3,      /* block/window size, dtype or mode not built */
    ASP_ERR_OUT_OF_MEMORY = 4,
    ASP_ERR_HIP = 5,              /* a HIP runtime call failed (no GPU, launch error, ...) */
    ASP_ERR_BUFFER_TOO_SMALL = 6  /* asp_export: dst_bytes < *needed; asp_spmm: scratch not reserved for this N;
                                     asp_spmm_static_scratch: the static scratch is too small for this handle and N */
} asp_status_t;

typedef enum { ASP_FMT_BCSR = 0, ASP_FMT_WCSR = 1 } asp_format_t;

/* dtype of A's values, of B and of C.  Accumulation is always fp32 (MFMA). */
typedef enum { ASP_DT_BF16 = 0, ASP_DT_F32 = 1 } asp_dtype_t;

/* Convert on the host and keep host arrays only: no HIP call is made, so this works
 * without a GPU.  The handle can be inspected (info/export/plan) but asp_spmm refuses it. */
#define ASP_FLAG_HOST_CONVERT_ONLY 1u

/* Largest dense width N (columns of B and C; tokens of asp_spmm_xt) that any call accepts: 65535 column tiles
 * of 64.  Beyond it calls return ASP_ERR_UNSUPPORTED (asp_reserve, asp_plan_spmm: ASP_ERR_INVALID_ARG).
 * M x N (and K x N for asp_spmm_xt) must also stay below 2^40 elements. */
#define ASP_MAX_N (65535ll * 64)

typedef struct {
    int32_t format;    /* asp_format_t */
    int32_t dtype;     /* asp_dtype_t; both dtypes are built for both formats */
    int32_t b_row;     /* BCSR: block height in {32,64,128}; WCSR: window height in {16,32,64} */
    int32_t b_col;     /* BCSR: block width, = b_row; WCSR: column padding unit, = 8 */
    int32_t task_cols; /* WCSR: packed columns per sub-task, positive multiple of b_col up to 2^30; 0 = default (512) */
    uint32_t flags;    /* ASP_FLAG_* */
} asp_config_t;

typedef struct {
    int64_t m, k, nnz;
    int32_t format, dtype, b_row, b_col, task_cols;
    int32_t on_device;  /* 1 when the handle holds device arrays and asp_spmm can run */
    int64_t n_brows;    /* block-rows (BCSR) or windows (WCSR) = ceil(m / b_row) */
    int64_t n_units;    /* stored blocks (BCSR) or packed columns incl. pads (WCSR) */
    int64_t n_tasks;    /* WCSR sub-tasks; 0 for BCSR */
    int64_t n_zero_rows_units; /* WCSR: windows whose C rows are cleared before the kernel (empty or split) */
    double fill_ratio;  /* nnz / stored value slots (Section II-C, fill ratio) */
} asp_info_t;

/* Which array asp_export copies out.  Layouts (all row-major, int32 indices):
 *  BCSR (Section II-C):
 *    ROW_PTR  block_row_ptr[n_brows+1]      first stored block of each block-row
 *    COL_IDX  block_col_idx[n_units]        block column of each stored block, ascending in a block-row
 *    VALUES   blocks[n_units][b_row][b_col] dense blocks, +0.0 where CSR stores nothing
 *  WCSR (Section II-C):
 *    ROW_PTR  window_row_ptr[n_brows+1]     first packed column of each window (multiples of b_col)
 *    COL_IDX  window_col_idx[n_units]       original column of each packed column, ascending in a
 *                                           window, -1 for the (< b_col) pads at a window's tail
 *    VALUES   values[n_units/b_col][b_row][b_col]  one dense tile per b_col packed columns
 *    TASKS    tasks[n_tasks][4] = {window, col_begin, col_end, split}  (Section III-C); packed-column
 *             positions are absolute, col_end - col_begin = task_cols except for a window's last task,
 *             split = 1 when the window has more than one task.  Tasks are in window order.
 *  A block or a window column is stored when CSR holds an entry there, whatever its value.
 */
typedef enum { ASP_ARR_ROW_PTR = 0, ASP_ARR_COL_IDX = 1, ASP_ARR_VALUES = 2, ASP_ARR_TASKS = 3 } asp_array_t;

/* How asp_spmm would run for a dense width N (Section IV-C: tile-width selection).  bf16 BCSR picks, among its
 * tile widths 64 / 128 / 256 / 512 (512: tiles of 128 rows -- 128x128 blocks, or 128-row stacks of smaller blocks where
 * the handle keeps them -- with at least one tile per compute unit), the one with the
 * least padded width x cost per column, costs 135 / 96 / 74 / 64 (ties: the wider), and then the next narrower
 * width while non-empty block-rows x ceil(N / width) tiles are fewer than the GPU's compute units (256 assumed for
 * host-only handles); fp32 BCSR and WCSR take the widest of their widths that divides N, else the one that pads least. */
typedef struct {
    int32_t bn;          /* columns of B/C handled by one workgroup (BCSR) or one wave (WCSR) */
    int32_t n_tiles;     /* ceil(N / bn): tiles along N, the last one masked if bn does not divide N */
    int32_t vectorized;  /* 1: 16-byte row accesses (needs N*sizeof(dtype) % 16 == 0 and 16-byte aligned B, C) */
    int64_t workgroups;  /* output tiles of the main kernel (one workgroup each, or the work list of its resident workgroups) */
    int64_t padded_n;    /* n_tiles * bn: width actually computed on */
} asp_plan_t;

/*
 * Build a handle from CSR (Section II-C).  CSR arrays are HOST pointers and are only read during
 * the call.  Requirements: m, k >= 1; nnz >= 0; row_ptr[0] = 0, non-decreasing, row_ptr[m] = nnz;
 * 0 <= col_idx < k and strictly ascending inside every row (duplicates are rejected, not summed);
 * values are nnz elements of cfg->dtype (bf16 as uint16 bit patterns) and are only ever bit-copied.
 * stream: hipStream_t used for uploads and the task-partition kernels (NULL = default stream); the
 * call returns after they completed.  On error *out is NULL and nothing is leaked.
 */
asp_status_t asp_create_from_csr(const asp_config_t *cfg, int64_t m, int64_t k, int64_t nnz,
                                 const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                                 void *stream, asp_handle_t **out);

/*
 * C = A x B (Section II-C; kernels: Sections III-A..III-C re-designed for gfx950).
 * B: DEVICE, k x N row-major, leading dimension N.  C: DEVICE, m x N row-major, leading dimension N,
 * fully overwritten (rows of A without entries become zeros); C must not alias B.
 * 1 <= N <= ASP_MAX_N.  stream: hipStream_t (NULL = default).  Asynchronous: only enqueues kernels, never
 * synchronises, never allocates.  bf16: fp32 accumulation, round-to-nearest-even to bf16 on store.
 * f32: fp32 products and sums on the matrix cores (no reduced-precision operand formats).
 * WCSR windows that are split into several tasks: with scratch memory (asp_reserve) the tasks' fp32 partial
 * tiles are added in task order and rounded once; an f32 handle without scratch adds into C with fp32
 * atomics, and only then may those rows differ in the last bits from run to run.  Everything else is
 * bitwise reproducible.  The device the handle was created on must be the current one (ASP_ERR_INVALID_ARG otherwise)
 * and stream must belong to it.
 */
asp_status_t asp_spmm(const asp_handle_t *h, const void *B, void *C, int64_t N, void *stream);

/*
 * Scratch memory for asp_spmm calls of width up to N (Section III-C: the partial sums of a row-window that
 * is split into several tasks have to meet somewhere).  With scratch, every task of a split window stores
 * its fp32 partial tile (4 * b_row * N bytes per task) and a last kernel adds the tiles in task order: the
 * result is bitwise reproducible.  bf16 WCSR handles with split windows need it (bf16 C cannot take fp32
 * atomic adds); f32 WCSR handles use it when it is there and otherwise add into C with fp32 atomics.  BCSR
 * handles and WCSR handles without split windows use none: the call does nothing for them.
 * Allocates (and frees a smaller earlier buffer, which synchronises the device); asp_spmm itself never
 * allocates and returns ASP_ERR_BUFFER_TOO_SMALL when a bf16 call needs more scratch than was reserved.
 * Calls on one handle that use the scratch share it and must be ordered on one stream.
 */
asp_status_t asp_reserve(asp_handle_t *h, int64_t N);

/*
 * asp_spmm for callers that cannot allocate at all -- code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc -- and therefore cannot call asp_reserve either.  Same arguments, same result (bit for bit
 * that of asp_spmm on a handle with reserved scratch), but the fp32 partial tiles of split WCSR windows go into a
 * scratch array that is part of the library's device image (ASP_STATIC_SCRATCH_BYTES on every GPU the library
 * runs on, held until the process ends) instead of a buffer from asp_reserve.  Calls no hipMalloc, hipFree or other
 * allocating routine; its one piece of set-up, looking up the array's device address, happens when a WCSR handle with split
 * windows is created.  Returns ASP_ERR_BUFFER_TOO_SMALL when the handle's split tasks need more than the array
 * holds at this N (4 * b_row * N bytes per task of a split window): nothing is launched then.  BCSR handles and
 * WCSR handles without split windows use no scratch and run exactly as in asp_spmm.
 * Every call on one GPU shares that GPU's array, whatever the handle: calls that overlap in time on one GPU race
 * (order them on one stream, or with events).  Nothing in the array has to start at zero -- every slot a call
 * reads was written by that call first -- so contents left by earlier calls do no harm.
 */
#define ASP_STATIC_SCRATCH_BYTES (64ull << 20)
asp_status_t asp_spmm_static_scratch(const asp_handle_t *h, const void *B, void *C, int64_t N, void *stream);

/*
 * Y = X x A^T with K-contiguous dense operands: the same product as asp_spmm with B = X^T and C = Y^T, in
 * the layout of the paper's LLM case study (Section IV-D: C = W X^T, activations stored tokens x hidden),
 * so that projections can be chained without transposes.
 * X: DEVICE, N x k row-major (leading dimension k).  Y: DEVICE, N x m row-major (leading dimension m), fully
 * overwritten; Y must not alias X.  1 <= N <= ASP_MAX_N.  BCSR handles (bf16) only; others return ASP_ERR_UNSUPPORTED.
 * Asynchronous, never synchronises, never allocates.  fp32 accumulation, round-to-nearest-even to bf16;
 * bitwise reproducible.  128x128 blocks (and 64x64 / 32x32 blocks when k >= 32 and grouping their block-rows
 * into 128-row tiles adds at most 2.6x / 4.3x zero fill) with k % 8 == 0,
 * m % 8 == 0 and 16-byte aligned X and Y run on the matrix cores (128 outputs x 512 tokens per workgroup);
 * everything else takes a slow generic kernel.
 */
asp_status_t asp_spmm_xt(const asp_handle_t *h, const void *X, void *Y, int64_t N, void *stream);

/* host only: describe the handle */
asp_status_t asp_get_info(const asp_handle_t *h, asp_info_t *info);

/* host only: the launch shape asp_spmm would use for width N with 16-byte aligned B and C */
asp_status_t asp_plan_spmm(const asp_handle_t *h, int64_t N, asp_plan_t *plan);

/*
 * Copy one canonical array (see asp_array_t) to HOST memory.  *needed (may be NULL) receives the
 * size in bytes; when dst_bytes is smaller nothing is copied and ASP_ERR_BUFFER_TOO_SMALL returns
 * (call with host_dst = NULL, dst_bytes = 0 to query).  Synchronises the device if it must read back.
 */
asp_status_t asp_export(const asp_handle_t *h, asp_array_t which, void *host_dst, size_t dst_bytes,
                        size_t *needed);

/* Frees host and device memory of the handle.  NULL is allowed. */
asp_status_t asp_destroy(asp_handle_t *h);

/*
 * ---- host only: the preprocessing of the sparse-matrix evaluation (Section IV-A, "Baselines and datasets") ----
 *
 * Reverse Cuthill-McKee ordering of a square m x m matrix given as CSR structure (HOST arrays, valid sorted
 * CSR as for asp_create_from_csr).  The structure is taken as that of A + A^T.  perm (HOST, m entries,
 * written) receives perm[new] = old.  Every connected component is numbered breadth-first from its node of
 * least degree, neighbours in order of degree (ties: lower index), and the numbering is reversed.  A node's
 * degree is its number of neighbours in A + A^T, a stored diagonal entry counting twice (the convention of the
 * scipy routine the paper uses).
 */
asp_status_t asp_rcm(int64_t m, const int32_t *row_ptr, const int32_t *col_idx, int32_t *perm);

/*
 * A'[i][j] = A[row_perm[i]][col_perm[j]] as sorted CSR (col_perm NULL keeps the columns; the symmetric
 * reordering of Section IV-A passes the same permutation twice).  All arrays HOST; dtype is an asp_dtype_t,
 * values are bit-copied.  Outputs are caller-allocated: out_row_ptr m + 1 entries, out_col_idx and out_values
 * nnz entries; they must not alias the inputs.  Permutations that are not permutations are rejected.
 */
asp_status_t asp_permute_csr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                             int32_t dtype, const int32_t *row_perm, const int32_t *col_perm, int32_t *out_row_ptr,
                             int32_t *out_col_idx, void *out_values);

/*
 * Read a Matrix Market coordinate file (the format of the collection the paper evaluates on) into sorted CSR
 * with float values: fields real / integer / pattern (value 1), symmetries general / symmetric /
 * skew-symmetric (off-diagonal entries are mirrored); entries at equal positions are summed in fp64, explicit
 * zeros stay stored.  Array files, complex and hermitian matrices return ASP_ERR_UNSUPPORTED, malformed files
 * ASP_ERR_INVALID_CSR, a file that cannot be opened ASP_ERR_INVALID_ARG.  *out is owned by the library until
 * asp_mtx_free; asp_mtx_get hands out its sizes and HOST array pointers (any out-pointer may be NULL), valid
 * until the free.
 */
typedef struct asp_mtx asp_mtx_t;
asp_status_t asp_mtx_read(const char *path, asp_mtx_t **out);
asp_status_t asp_mtx_get(const asp_mtx_t *mx, int64_t *m, int64_t *k, int64_t *nnz, const int32_t **row_ptr,
                         const int32_t **col_idx, const float **values);
asp_status_t asp_mtx_free(asp_mtx_t *mx);

/* host only; any value is accepted (the name of an asp_status_t, "ASP_ERR_UNKNOWN" for everything else) */
const char *asp_status_string(int status);
const char *asp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCSPARSE_H */
