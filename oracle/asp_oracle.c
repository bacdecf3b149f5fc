/*
 * CPU oracle for sparse-times-dense multiplication C = A x B and for the two
 * sparse formats of the paper (Section II-C: problem statement, BCSR, WCSR;
 * Section III-C: splitting of long row-windows into fixed-size sub-tasks).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the library and the
 * library never calls it.  Everything is written as the definition reads:
 * no blocking, no fusion, no reordering.  The only parallelism is an OpenMP
 * loop over independent output rows in the product.
 *
 * Conventions (the paper leaves these open; they are this build's readings):
 *   - a block / a window column is "nonzero" when CSR stores an entry there,
 *     whatever its value (structural, like the textbook BSR conversion);
 *   - blocks of a block-row are in ascending block-column order, row-major
 *     inside a block; a window's columns are ascending, pads (-1) at the tail;
 *   - WCSR values are kept as dense tiles [b_row][b_col], one per group of
 *     b_col packed columns, tiles in packed-column order;
 *   - dimensions that do not divide are ceil-divided and zero padded;
 *   - padding zeros are +0.0 (all-zero bits); values are bit copies.
 *
 * dtype codes: 0 = bf16 carried as uint16 bit patterns, 1 = float32.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == 0) {
        uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16; /* bf16 = top half of an fp32 */
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    return (double)((const float *)base)[idx];
}

static size_t elem_size(int dtype) { return dtype == 0 ? 2 : 4; }

/* number of OpenMP threads the product will use */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * C[i][j] = sum over stored entries p of row i of  A.values[p] * B[A.col_idx[p]][j]   (Section II-C)
 * S[i][j] = the same sum over absolute values (the scale of the error bound); S may be NULL.
 * B is row-major with leading dimension ldb >= N, C and S are row-major m x N.
 * Accumulation is in fp64 in CSR order.
 */
int oracle_spmm(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                const void *values, int dtype, const void *B, int64_t N, int64_t ldb,
                double *C, double *S)
{
    (void)k;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < m; ++i) {
        double *c = C + i * N;
        double *s = S ? S + i * N : NULL;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        if (s) for (int64_t j = 0; j < N; ++j) s[j] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            double a = widen(values, p, dtype);
            int64_t brow = (int64_t)col_idx[p] * ldb;
            for (int64_t j = 0; j < N; ++j) {
                double b = widen(B, brow + j, dtype);
                c[j] += a * b;
                if (s) s[j] += fabs(a) * fabs(b);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ BCSR */

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* sorted distinct values of f(col) over the CSR rows [r0, r1); f(col) = col / div.  Returns count. */
static int64_t distinct_sorted(const int32_t *row_ptr, const int32_t *col_idx, int64_t r0, int64_t r1,
                               int32_t div, int32_t *out)
{
    int64_t n = 0;
    for (int64_t p = row_ptr[r0]; p < row_ptr[r1]; ++p) out[n++] = col_idx[p] / div;
    qsort(out, (size_t)n, sizeof(int32_t), cmp_i32);
    int64_t u = 0;
    for (int64_t t = 0; t < n; ++t)
        if (u == 0 || out[u - 1] != out[t]) out[u++] = out[t];
    return u;
}

static int64_t find_sorted(const int32_t *a, int64_t n, int32_t key)
{
    int64_t lo = 0, hi = n - 1;
    while (lo <= hi) {
        int64_t mid = (lo + hi) / 2;
        if (a[mid] == key) return mid;
        if (a[mid] < key) lo = mid + 1; else hi = mid - 1;
    }
    return -1;
}

static int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }

/*
 * BCSR, pass 1 (Section II-C): block_row_ptr[nbr+1], nbr = ceil(m / b_row).
 * A block is stored when CSR holds at least one entry inside it.  Returns nnz_blocks.
 */
int64_t oracle_bcsr_count(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                          int32_t b_row, int32_t b_col, int32_t *block_row_ptr)
{
    (void)k;
    int64_t nbr = (m + b_row - 1) / b_row;
    block_row_ptr[0] = 0;
    for (int64_t I = 0; I < nbr; ++I) {
        int64_t r0 = I * b_row, r1 = min64(m, r0 + b_row);
        int64_t cnt = row_ptr[r1] - row_ptr[r0];
        int32_t *tmp = (int32_t *)malloc((size_t)(cnt > 0 ? cnt : 1) * sizeof(int32_t));
        int64_t u = distinct_sorted(row_ptr, col_idx, r0, r1, b_col, tmp);
        free(tmp);
        block_row_ptr[I + 1] = block_row_ptr[I] + (int32_t)u;
    }
    return block_row_ptr[nbr];
}

/*
 * BCSR, pass 2: block_col_idx[nnz_blocks] ascending inside a block-row and
 * blocks[nnz_blocks][b_row][b_col] row-major, +0.0 where CSR stores nothing.
 */
int oracle_bcsr_fill(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                     const void *values, int dtype, int32_t b_row, int32_t b_col,
                     const int32_t *block_row_ptr, int32_t *block_col_idx, void *blocks)
{
    (void)k;
    size_t es = elem_size(dtype);
    int64_t nbr = (m + b_row - 1) / b_row;
    int64_t bsz = (int64_t)b_row * b_col;
    memset(blocks, 0, (size_t)block_row_ptr[nbr] * (size_t)bsz * es);
    for (int64_t I = 0; I < nbr; ++I) {
        int64_t r0 = I * b_row, r1 = min64(m, r0 + b_row);
        int64_t cnt = row_ptr[r1] - row_ptr[r0];
        int32_t *tmp = (int32_t *)malloc((size_t)(cnt > 0 ? cnt : 1) * sizeof(int32_t));
        int64_t u = distinct_sorted(row_ptr, col_idx, r0, r1, b_col, tmp);
        int64_t q0 = block_row_ptr[I];
        for (int64_t t = 0; t < u; ++t) block_col_idx[q0 + t] = tmp[t];
        for (int64_t i = r0; i < r1; ++i) {
            for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
                int32_t J = col_idx[p] / b_col;
                int64_t t = find_sorted(tmp, u, J);
                int64_t dst = (q0 + t) * bsz + (i - r0) * b_col + (col_idx[p] - (int64_t)J * b_col);
                memcpy((char *)blocks + (size_t)dst * es, (const char *)values + (size_t)p * es, es);
            }
        }
        free(tmp);
    }
    return 0;
}

/* fill ratio = nnz / (nnz_blocks * b_row * b_col)   (Section II-C) */
double oracle_fill_ratio(int64_t nnz, int64_t nnz_blocks, int32_t b_row, int32_t b_col)
{
    if (nnz_blocks == 0) return 0.0;
    return (double)nnz / ((double)nnz_blocks * (double)b_row * (double)b_col);
}

/* ------------------------------------------------------------------ WCSR */

/*
 * WCSR, pass 1 (Section II-C): window_row_ptr[nw+1], nw = ceil(m / b_row), in
 * units of packed columns.  Window w holds the distinct columns of its rows,
 * rounded up to a multiple of b_col.  Returns padded_nnz_cols.
 */
int64_t oracle_wcsr_count(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                          int32_t b_row, int32_t b_col, int32_t *window_row_ptr)
{
    (void)k;
    int64_t nw = (m + b_row - 1) / b_row;
    window_row_ptr[0] = 0;
    for (int64_t w = 0; w < nw; ++w) {
        int64_t r0 = w * b_row, r1 = min64(m, r0 + b_row);
        int64_t cnt = row_ptr[r1] - row_ptr[r0];
        int32_t *tmp = (int32_t *)malloc((size_t)(cnt > 0 ? cnt : 1) * sizeof(int32_t));
        int64_t u = distinct_sorted(row_ptr, col_idx, r0, r1, 1, tmp);
        free(tmp);
        int64_t padded = (u + b_col - 1) / b_col * b_col;
        window_row_ptr[w + 1] = window_row_ptr[w] + (int32_t)padded;
    }
    return window_row_ptr[nw];
}

/*
 * WCSR, pass 2: window_col_idx[padded] (original column of every packed
 * column, -1 for pads) and values as tiles: packed column p lives in tile
 * T = p / b_col at lane c = p % b_col, values[T][r][c] is the entry of row
 * (w*b_row + r) in column window_col_idx[p], or +0.0.
 */
int oracle_wcsr_fill(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx,
                     const void *values, int dtype, int32_t b_row, int32_t b_col,
                     const int32_t *window_row_ptr, int32_t *window_col_idx, void *out_values)
{
    (void)k;
    size_t es = elem_size(dtype);
    int64_t nw = (m + b_row - 1) / b_row;
    memset(out_values, 0, (size_t)window_row_ptr[nw] * (size_t)b_row * es);
    for (int64_t w = 0; w < nw; ++w) {
        int64_t r0 = w * b_row, r1 = min64(m, r0 + b_row);
        int64_t cnt = row_ptr[r1] - row_ptr[r0];
        int32_t *tmp = (int32_t *)malloc((size_t)(cnt > 0 ? cnt : 1) * sizeof(int32_t));
        int64_t u = distinct_sorted(row_ptr, col_idx, r0, r1, 1, tmp);
        int64_t p0 = window_row_ptr[w], p1 = window_row_ptr[w + 1];
        for (int64_t p = p0; p < p1; ++p) window_col_idx[p] = (p - p0 < u) ? tmp[p - p0] : -1;
        for (int64_t i = r0; i < r1; ++i) {
            for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
                int64_t p = p0 + find_sorted(tmp, u, col_idx[q]);
                int64_t T = p / b_col, c = p % b_col;
                int64_t dst = T * b_row * b_col + (i - r0) * b_col + c;
                memcpy((char *)out_values + (size_t)dst * es, (const char *)values + (size_t)q * es, es);
            }
        }
        free(tmp);
    }
    return 0;
}

/* ------------------------------------------------------------------ tasks */

/*
 * Sub-tasks of row-windows (Section III-C): a window of n packed columns
 * becomes ceil(n / task_cols) tasks that cover its packed-column range in
 * order, each task_cols wide except the last.  Tasks are listed in window
 * order; an empty window has none.  A task is 4 int32:
 *   { window, col_begin, col_end, split }   (absolute packed-column positions,
 *   split = 1 when its window has more than one task).
 * tasks may be NULL to only count.  Returns the number of tasks.
 */
int64_t oracle_wcsr_tasks(int64_t n_windows, const int32_t *window_row_ptr, int32_t task_cols,
                          int32_t *tasks)
{
    int64_t nt = 0;
    for (int64_t w = 0; w < n_windows; ++w) {
        int64_t p0 = window_row_ptr[w], p1 = window_row_ptr[w + 1];
        int64_t n = p1 - p0;
        int64_t parts = (n + task_cols - 1) / task_cols;
        for (int64_t t = 0; t < parts; ++t) {
            if (tasks) {
                tasks[4 * nt + 0] = (int32_t)w;
                tasks[4 * nt + 1] = (int32_t)(p0 + t * task_cols);
                tasks[4 * nt + 2] = (int32_t)min64(p1, p0 + (t + 1) * task_cols);
                tasks[4 * nt + 3] = parts > 1 ? 1 : 0;
            }
            ++nt;
        }
    }
    return nt;
}

/* ------------------------------------------------------------------ tile width */

/*
 * Width the dense operand is padded to when it is cut into tiles of BN
 * columns (Section IV-C): the next multiple of BN.
 */
int64_t oracle_padded_width(int64_t N, int64_t BN) { return (N + BN - 1) / BN * BN; }

/*
 * Tile-width rule of Section IV-C: among the candidate widths take the largest
 * one that divides N; when none divides, the one that pads N the least (ties:
 * the larger).  Returns the chosen width.
 */
int64_t oracle_choose_bn(int64_t N, const int64_t *candidates, int n_candidates)
{
    int64_t best = -1;
    for (int c = 0; c < n_candidates; ++c)
        if (N % candidates[c] == 0 && candidates[c] > best) best = candidates[c];
    if (best > 0) return best;
    int64_t best_pad = -1;
    for (int c = 0; c < n_candidates; ++c) {
        int64_t pad = oracle_padded_width(N, candidates[c]);
        if (best_pad < 0 || pad < best_pad || (pad == best_pad && candidates[c] > best)) {
            best_pad = pad;
            best = candidates[c];
        }
    }
    return best;
}

/*
 * Tile width by cost (Section IV-C: a wider tile does more work per loaded A tile, a tile that does not divide N
 * computes on padding): the candidate with the smallest  padded_width(N, BN) x cost_per_column(BN); ties: the
 * larger.  With equal costs this is oracle_choose_bn.
 * PARITY UNPINNED against the paper: this is not the rule Section IV-C states (that one is oracle_choose_bn, which
 * stays pinned to the paper's printed numbers) but the rule of the library under test, written out a second
 * time.  It is pinned only where the mathematics fixes it: equal costs reduce it to oracle_choose_bn, a widest
 * candidate that divides N wins under any non-increasing cost table, and hand arithmetic in the tests.
 */
int64_t oracle_choose_bn_weighted(int64_t N, const int64_t *candidates, const int64_t *cost, int n_candidates)
{
    int64_t best = -1, best_cost = -1;
    for (int c = 0; c < n_candidates; ++c) {
        int64_t total = oracle_padded_width(N, candidates[c]) * cost[c];
        if (best < 0 || total < best_cost || (total == best_cost && candidates[c] > best)) {
            best_cost = total;
            best = candidates[c];
        }
    }
    return best;
}

/*
 * The weighted choice followed by the launch-filling step of the library under test: while the chosen width
 * gives fewer tiles (rows x ceil(N / BN)) than the machine has units to run them on, and a narrower candidate
 * exists, take the next narrower candidate.  A widest candidate that is only admitted when it fills the machine
 * is the caller's business (it leaves it out of the list otherwise).
 * PARITY UNPINNED against the paper, which launches one thread block per tile and states no rule for launches
 * smaller than the machine (Section IV-C discusses the width only through work per loaded tile and padding):
 * pinned by hand arithmetic and by the properties that follow from the definition (never wider than the
 * weighted choice; equal to it when that already fills the machine; otherwise the widest narrower candidate
 * that fills it, or the narrowest).
 */
int64_t oracle_choose_bn_filled(int64_t N, const int64_t *candidates, const int64_t *cost, int n_candidates,
                                int64_t rows, int64_t units)
{
    int64_t bn = oracle_choose_bn_weighted(N, candidates, cost, n_candidates);
    for (;;) {
        if (rows * (oracle_padded_width(N, bn) / bn) >= units) return bn;
        int64_t narrower = -1;
        for (int c = 0; c < n_candidates; ++c)
            if (candidates[c] < bn && candidates[c] > narrower) narrower = candidates[c];
        if (narrower < 0) return bn;
        bn = narrower;
    }
}
