// WCSR x dense SpMM for gfx950 and the GPU-side split of row-windows into sub-tasks
// (paper, Section II-C for the format, Section III-B/III-C for the gather kernel and the task split).
//
// The work is bound by the gather of B rows from HBM, so the kernel is built around that stream:
// one wavefront owns one (task, N-tile).  For every packed column of its task a quarter (or half)
// of the wave reads a contiguous run of the addressed B row with 16-byte loads straight into the
// register layout of the fp32 MFMA B operand -- no LDS stage, no barrier -- while the matching A
// values come from the contiguous tile.  Loads for the next tile are issued before the MFMAs of the
// current one; many resident waves per CU keep the HBM queue full.  The columns of a 64-wide (or
// 128-wide) group are dealt to the MFMA's N index as n = 4*j + t (j = lane's N index, t = which of
// the lane's four loaded values), so that each lane ends with 4 adjacent output columns per row and
// C is written (or atomically accumulated, for split windows) 16 bytes at a time.
//
// The paper fixes the window height at 64 to fit the Hopper instruction; the CDNA fp32 MFMAs are
// 16 or 32 rows tall, so heights 16 (default), 32 and 64 are built.
#include <algorithm>
#include <cstdlib>
#include <mutex>

#include "asp_internal.h"

// Scratch for callers that cannot allocate (asp_spmm_static_scratch): the partial tiles of split windows go here
// instead of into a buffer from asp_reserve.  Every GPU the library runs on holds its own copy at its own address
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels and copies get
// the device address that wcsr_static_scratch() resolved.
static __device__ __align__(256) float scratch[ASP_STATIC_SCRATCH_BYTES / sizeof(float)];

namespace asp {

asp_status_t wcsr_static_scratch(int device, float **ptr, int64_t *floats) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static float *resolved[MAX_DEVICES] = {};
    if (device < 0 || device >= MAX_DEVICES) return fail(ASP_ERR_UNSUPPORTED, "device index beyond the static scratch table");
    std::lock_guard<std::mutex> lock(mu);
    if (!resolved[device]) {
        int cur = -1;
        ASP_HIP_TRY(hipGetDevice(&cur));
        if (cur != device) return fail(ASP_ERR_INVALID_ARG, "the static scratch of a device is resolved with that device current");
        float *p = nullptr;
        ASP_HIP_TRY(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ASP_ERR_HIP, "hipGetSymbolAddress returned no address for the static scratch");
        resolved[device] = p;
    }
    *ptr = resolved[device];
    *floats = (int64_t)(ASP_STATIC_SCRATCH_BYTES / sizeof(float));
    return ASP_OK;
}

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---- zero the C rows that the main kernel will not plainly overwrite -------------------------------
// (windows without columns; and, when they accumulate with atomics, windows split over several tasks)
// ws_slot != nullptr: split windows (slot >= 0) are left alone, their rows come from the partial tiles.
__global__ __launch_bounds__(256) void wcsr_zero_rows_kernel(const int32_t *__restrict__ zero_windows,
                                                             const int32_t *__restrict__ ws_slot, int b_row,
                                                             uint8_t *__restrict__ C, int esize, int M, int64_t N,
                                                             bool vec) {
    const int w = zero_windows[blockIdx.x];
    if (ws_slot && ws_slot[w] >= 0) return;
    const int64_t r0 = (int64_t)w * b_row;
    const int64_t r1 = r0 + b_row < M ? r0 + b_row : M;
    uint8_t *base = C + r0 * N * esize;
    const int64_t bytes = (r1 - r0) * N * esize;
    if (vec) {  // row size and base are multiples of 16 bytes
        uint4 *b4 = (uint4 *)base;
        for (int64_t i = threadIdx.x; i < bytes / 16; i += 256) b4[i] = make_uint4(0, 0, 0, 0);
    } else if (esize == 4) {
        for (int64_t i = threadIdx.x; i < bytes / 4; i += 256) ((uint32_t *)base)[i] = 0u;
    } else {
        for (int64_t i = threadIdx.x; i < bytes / 2; i += 256) ((uint16_t *)base)[i] = 0;
    }
}

// ---- rows of split windows from the partial tiles of their tasks (Section III-C) ---------------------
// Task j of a split window stored its fp32 partial tile [b_row][N] in slot ws_slot[w] + j of the scratch
// buffer.  One thread per output element adds the tiles in task order (fixed order: bitwise reproducible)
// and rounds once to the output type.
template <typename OutT, int U>  // U = elements per thread and access: 4 (16-byte loads) or 1
__global__ __launch_bounds__(256) void wcsr_sum_partials_kernel(const int32_t *__restrict__ zero_windows,
                                                                const int32_t *__restrict__ ws_slot,
                                                                const int32_t *__restrict__ window_row_ptr,
                                                                int task_cols, int b_row, OutT *__restrict__ C,
                                                                const float *__restrict__ ws, int M, int64_t N) {
    typedef float vec_t __attribute__((ext_vector_type(U)));
    typedef OutT out_t __attribute__((ext_vector_type(U)));
    const int w = zero_windows[blockIdx.x];
    const int slot0 = ws_slot[w];
    if (slot0 < 0) return;  // a window without columns
    const int parts = (int)(((int64_t)window_row_ptr[w + 1] - window_row_ptr[w] + task_cols - 1) / task_cols);
    const int64_t r0 = (int64_t)w * b_row, r1 = r0 + b_row < M ? r0 + b_row : M;
    const int64_t units = (r1 - r0) * N / U, tile = (int64_t)b_row * N / U;
    const vec_t *src = (const vec_t *)(ws + (int64_t)slot0 * b_row * N);
    out_t *dst = (out_t *)(C + r0 * N);
    for (int64_t i = (int64_t)blockIdx.y * 256 + threadIdx.x; i < units; i += (int64_t)gridDim.y * 256) {
        vec_t sum = src[i];
        int j = 1;
        for (; j + 8 <= parts; j += 8) {  // 8 independent loads in flight, added in task order
            vec_t t[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) t[e] = src[(j + e) * tile + i];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += t[e];
        }
        for (; j < parts; ++j) sum += src[j * tile + i];
        dst[i] = __builtin_convertvector(sum, out_t);  // bf16: round to nearest even
    }
}

__device__ __forceinline__ float4 gather4(const float *__restrict__ B, int col, int64_t N, int n, bool vec) {
    // 4 adjacent columns n..n+3 of row `col` of B; zeros for a pad column (col < 0) or past the edge
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col >= 0 && n < N) {
        const float *p = B + (int64_t)col * N + n;
        if (vec) {
            v = *(const float4 *)p;
        } else {
            v.x = p[0];
            if (n + 1 < N) v.y = p[1];
            if (n + 2 < N) v.z = p[2];
            if (n + 3 < N) v.w = p[3];
        }
    }
    return v;
}

__device__ __forceinline__ void put4(float *__restrict__ C, int64_t row, int M, int64_t N, int n, float4 v, bool split,
                                     bool vec) {
    if (row >= M || n >= N) return;
    float *p = C + row * N + n;
    if (split) {
        unsafeAtomicAdd(p, v.x);
        if (n + 1 < N) unsafeAtomicAdd(p + 1, v.y);
        if (n + 2 < N) unsafeAtomicAdd(p + 2, v.z);
        if (n + 3 < N) unsafeAtomicAdd(p + 3, v.w);
    } else if (vec) {
        *(float4 *)p = v;
    } else {
        p[0] = v.x;
        if (n + 1 < N) p[1] = v.y;
        if (n + 2 < N) p[2] = v.z;
        if (n + 3 < N) p[3] = v.w;
    }
}

// Where a task's tile goes.  An unsplit window writes its rows of C.  A split window (Section III-C) either
// adds into C with atomics (no scratch reserved) or stores its tile into its own slot of the scratch buffer:
// slot = first slot of the window + index of the task inside the window.
struct SplitTarget {
    float *base;
    int64_t row0;  // first row of the tile in base
    int64_t rows;  // rows that exist in base from its start (bound for the row check)
    bool atomic;
};
__device__ __forceinline__ SplitTarget split_target(int4 td, int b_row, float *C, int M, int64_t N, float *ws,
                                                    const int32_t *ws_slot, const int32_t *window_row_ptr,
                                                    int task_cols) {
    if (td.w != 0 && ws) {
        const int64_t slot = ws_slot[td.x] + (td.y - window_row_ptr[td.x]) / task_cols;
        return SplitTarget{ws + slot * b_row * N, 0, b_row, false};
    }
    return SplitTarget{C, (int64_t)td.x * b_row, M, td.w != 0};
}

// ---- window height 16: v_mfma_f32_16x16x4_f32 ----------------------------------------------------
// lane l: kq = l / 16 picks one of 4 packed columns of a k step, jl = l % 16 is the MFMA N index.
// NG = 64-column groups per wave (tile width BN = 64 * NG).
template <int NG, bool VEC>
__global__ __launch_bounds__(256) void wcsr16_spmm_kernel(const int4 *__restrict__ tasks, int n_tasks,
                                                          const int32_t *__restrict__ window_col_idx,
                                                          const float *__restrict__ values,
                                                          const float *__restrict__ B, float *__restrict__ C, int M,
                                                          int64_t N, int n_tiles, float *__restrict__ ws,
                                                          const int32_t *__restrict__ ws_slot,
                                                          const int32_t *__restrict__ window_row_ptr, int task_cols) {
    const int64_t wave_id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int task = (int)(wave_id / n_tiles), nt = (int)(wave_id % n_tiles);
    if (task >= n_tasks) return;  // whole wave leaves together
    const int lane = threadIdx.x & 63, kq = lane >> 4, jl = lane & 15;
    const int4 td = tasks[task];  // window, first packed column, end packed column, split flag
    const int n0 = nt * (64 * NG) + 4 * jl;

    f32x4 acc[NG][4];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[g][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline over chunks of D tiles (D*8 packed columns): while chunk c is multiplied, the B
    // rows and A values of chunk c+1 are in flight and the column indices of chunk c+2 are being read,
    // so neither the index -> address dependency nor the gather latency is waited for in the loop.
    constexpr int D = NG >= 2 ? 1 : 2;
    struct Chunk {
        float a[D][2];
        float4 b[D][2][NG];
    };
    const int tile0 = td.y >> 3, tile1 = td.z >> 3;
    // Which packed column a lane multiplies in which k step is free as long as A and B agree: lane group kq takes
    // columns 2 kq and 2 kq + 1 of a tile (k steps h = 0, 1), so its two indices and its two values of a row are
    // one 8-byte load each and the 16 x 4 lanes read a tile's 512 bytes of values as one contiguous span.
    auto load_idx = [&](int base, int (&idx)[D][2]) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            int2 c2 = make_int2(-1, -1);
            if (base + d < tile1) c2 = *(const int2 *)(window_col_idx + (int64_t)(base + d) * 8 + 2 * kq);
            idx[d][0] = c2.x;
            idx[d][1] = c2.y;
        }
    };
    auto gather = [&](int base, const int (&idx)[D][2], Chunk &c) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            float2 a2 = make_float2(0.f, 0.f);
            if (base + d < tile1) a2 = *(const float2 *)(values + (int64_t)(base + d) * 128 + jl * 8 + 2 * kq);
            c.a[d][0] = a2.x;
            c.a[d][1] = a2.y;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int g = 0; g < NG; ++g) c.b[d][h][g] = gather4(B, idx[d][h], N, n0 + 64 * g, VEC);
        }
    };
    auto multiply = [&](int base, const Chunk &c) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (base + d >= tile1) break;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    acc[g][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(c.a[d][h], c.b[d][h][g].x, acc[g][0], 0, 0, 0);
                    acc[g][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(c.a[d][h], c.b[d][h][g].y, acc[g][1], 0, 0, 0);
                    acc[g][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(c.a[d][h], c.b[d][h][g].z, acc[g][2], 0, 0, 0);
                    acc[g][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(c.a[d][h], c.b[d][h][g].w, acc[g][3], 0, 0, 0);
                }
        }
    };

    int idx[D][2];
    Chunk cur, nxt;
    load_idx(tile0, idx);
    gather(tile0, idx, cur);
    load_idx(tile0 + D, idx);
    for (int base = tile0; base < tile1; base += D) {
        const bool more = base + D < tile1;
        if (more) {
            gather(base + D, idx, nxt);
            load_idx(base + 2 * D, idx);
        }
        multiply(base, cur);
        if (more) cur = nxt;
    }

    // D layout: register r of lane l is row 4*(l/16) + r, MFMA column l%16 -> C column n0 + 64g + t
    const SplitTarget out = split_target(td, 16, C, M, N, ws, ws_slot, window_row_ptr, task_cols);
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float4 v = make_float4(acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]);
            put4(out.base, out.row0 + 4 * kq + r, out.rows, N, n0 + 64 * g, v, out.atomic, VEC);
        }
}

// ---- window heights 32 and 64: v_mfma_f32_32x32x2_f32 --------------------------------------------
// lane l: kq = l / 32 picks one of 2 packed columns of a k step, jl = l % 32 is the MFMA N index;
// the wave covers 128 columns.  MTW = window height / 32 MFMA row tiles share every gathered B value.
template <int MTW, bool VEC>
__global__ __launch_bounds__(256, 2) void wcsr32_spmm_kernel(const int4 *__restrict__ tasks, int n_tasks,
                                                          const int32_t *__restrict__ window_col_idx,
                                                          const float *__restrict__ values,
                                                          const float *__restrict__ B, float *__restrict__ C, int M,
                                                          int64_t N, int n_tiles, float *__restrict__ ws,
                                                          const int32_t *__restrict__ ws_slot,
                                                          const int32_t *__restrict__ window_row_ptr, int task_cols) {
    constexpr int BRW = 32 * MTW;
    const int64_t wave_id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int task = (int)(wave_id / n_tiles), nt = (int)(wave_id % n_tiles);
    if (task >= n_tasks) return;
    const int lane = threadIdx.x & 63, kq = lane >> 5, jl = lane & 31;
    const int4 td = tasks[task];
    const int n0 = nt * 128 + 4 * jl;

    f32x16 acc[MTW][4];
#pragma unroll
    for (int i = 0; i < MTW; ++i)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.f;

    struct Stage {
        float a[4][MTW];
        float4 b[4];
    };
    // lane group kq takes packed columns 4 kq .. 4 kq + 3 of a tile (k steps h = 0..3; any assignment works as long
    // as A and B agree): its four indices and its four values of a row are one 16-byte load each, and the 32 x 2
    // lanes read the 1 KB of values of a row tile as one contiguous span
    auto fetch = [&](int tile, Stage &s) {
        const int4 c4 = *(const int4 *)(window_col_idx + (int64_t)tile * 8 + 4 * kq);
        const int col[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            const float4 a4 = *(const float4 *)(values + (int64_t)tile * (BRW * 8) + (i * 32 + jl) * 8 + 4 * kq);
            s.a[0][i] = a4.x;
            s.a[1][i] = a4.y;
            s.a[2][i] = a4.z;
            s.a[3][i] = a4.w;
        }
#pragma unroll
        for (int h = 0; h < 4; ++h) s.b[h] = gather4(B, col[h], N, n0, VEC);
    };
    auto multiply = [&](const Stage &s) {
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
            for (int i = 0; i < MTW; ++i) {
                acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[h][i], s.b[h].x, acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[h][i], s.b[h].y, acc[i][1], 0, 0, 0);
                acc[i][2] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[h][i], s.b[h].z, acc[i][2], 0, 0, 0);
                acc[i][3] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[h][i], s.b[h].w, acc[i][3], 0, 0, 0);
            }
    };

    const int tile0 = td.y >> 3, tile1 = td.z >> 3;
    // two tiles in flight while a third is multiplied (three stages, walked with fixed register names): at this
    // register count the occupancy is the same as with one tile in flight, and the gather needs the bytes in flight
    Stage s0, s1, s2;
    fetch(tile0, s0);
    if (tile0 + 1 < tile1) fetch(tile0 + 1, s1);
    for (int tile = tile0; tile < tile1; tile += 3) {
        if (tile + 2 < tile1) fetch(tile + 2, s2);
        multiply(s0);
        if (tile + 3 < tile1) fetch(tile + 3, s0);
        if (tile + 1 < tile1) multiply(s1);
        if (tile + 4 < tile1) fetch(tile + 4, s1);
        if (tile + 2 < tile1) multiply(s2);
    }

    // D layout: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, MFMA column l%32
    const SplitTarget out = split_target(td, BRW, C, M, N, ws, ws_slot, window_row_ptr, task_cols);
#pragma unroll
    for (int i = 0; i < MTW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float4 v = make_float4(acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]);
            int row = i * 32 + 8 * (r >> 2) + 4 * kq + (r & 3);
            put4(out.base, out.row0 + row, out.rows, N, n0, v, out.atomic, VEC);
        }
}

// ---- sub-task list on the GPU (Section III-C) -----------------------------------------------------
// tasks_of(w) = ceil(width(w) / task_cols); an exclusive prefix sum over windows gives every window
// the index of its first task.  The sum is a wavefront scan (cross-lane shifts), stitched over the 4
// waves of a workgroup through LDS and over workgroups through a second, single-workgroup pass.

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(v, d, 64);
        if (lane >= d) v += up;
    }
    return v;
}

// inclusive scan over the 256 threads of a workgroup; returns the thread's inclusive value, *total = sum
__device__ __forceinline__ int block_inclusive_scan(int v, int *total) {
    __shared__ int wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = wave_inclusive_scan(v, lane);
    __syncthreads();  // protects wave_sum against the previous call
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    *total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
    return inc + base;
}

__global__ __launch_bounds__(256) void wcsr_task_count_kernel(const int32_t *__restrict__ window_row_ptr, int n_windows,
                                                              int task_cols, int32_t *__restrict__ local_excl,
                                                              int32_t *__restrict__ block_sums) {
    const int w = blockIdx.x * 256 + threadIdx.x;
    int cnt = 0;
    // (64-bit: width + task_cols may pass 2^31)
    if (w < n_windows) cnt = (int)(((int64_t)window_row_ptr[w + 1] - window_row_ptr[w] + task_cols - 1) / task_cols);
    int total;
    int inc = block_inclusive_scan(cnt, &total);
    if (w < n_windows) local_excl[w] = inc - cnt;
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// one workgroup: exclusive scan of block_sums in place, grand total to block_sums[n_blocks]
__global__ __launch_bounds__(256) void wcsr_task_block_scan_kernel(int32_t *__restrict__ block_sums, int n_blocks) {
    int carry = 0;
    for (int base = 0; base < n_blocks; base += 256) {
        const int i = base + threadIdx.x;
        const int v = i < n_blocks ? block_sums[i] : 0;
        int total;
        int inc = block_inclusive_scan(v, &total);
        if (i < n_blocks) block_sums[i] = carry + inc - v;
        carry += total;
    }
    if (threadIdx.x == 0) block_sums[n_blocks] = carry;
}

__global__ __launch_bounds__(256) void wcsr_task_offsets_kernel(const int32_t *__restrict__ local_excl,
                                                                const int32_t *__restrict__ block_sums, int n_windows,
                                                                int n_blocks, int32_t *__restrict__ task_offsets) {
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w < n_windows) task_offsets[w] = local_excl[w] + block_sums[blockIdx.x];
    if (w == 0) task_offsets[n_windows] = block_sums[n_blocks];
}

// one thread per task: find its window by bisection in the offsets, then cut the window's range
__global__ __launch_bounds__(256) void wcsr_task_emit_kernel(const int32_t *__restrict__ window_row_ptr,
                                                             const int32_t *__restrict__ task_offsets, int n_windows,
                                                             int n_tasks, int task_cols, int4 *__restrict__ tasks) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= n_tasks) return;
    int lo = 0, hi = n_windows;  // first window whose offset exceeds t lies in (lo, hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (task_offsets[mid] <= t) lo = mid; else hi = mid;
    }
    const int w = lo;
    const int64_t begin = window_row_ptr[w] + (int64_t)(t - task_offsets[w]) * task_cols;  // 64-bit: see above
    const int64_t wend = window_row_ptr[w + 1];
    int4 d;
    d.x = w;
    d.y = (int)begin;
    d.z = (int)(begin + task_cols < wend ? begin + task_cols : wend);
    d.w = (task_offsets[w + 1] - task_offsets[w]) > 1 ? 1 : 0;
    tasks[t] = d;
}

asp_status_t wcsr_build_tasks_device(asp_handle *h, hipStream_t stream) {
    const int nw = (int)h->n_brows;
    const int n_blocks = (int)ceil_div(nw, 256);
    int32_t *local_excl = nullptr, *block_sums = nullptr, *task_offsets = nullptr;
    asp_status_t st = ASP_OK;
    auto cleanup = [&]() {
        (void)hipFree(local_excl);
        (void)hipFree(block_sums);
        (void)hipFree(task_offsets);
    };
#define TRY_OR_CLEAN(expr)                                                                     \
    do {                                                                                       \
        hipError_t e__ = (expr);                                                               \
        if (e__ != hipSuccess) {                                                               \
            cleanup();                                                                         \
            return fail(e__ == hipErrorOutOfMemory ? ASP_ERR_OUT_OF_MEMORY : ASP_ERR_HIP,     \
                        std::string(#expr) + ": " + hipGetErrorString(e__));                  \
        }                                                                                      \
    } while (0)
    TRY_OR_CLEAN(hipMalloc((void **)&local_excl, (size_t)nw * 4));
    TRY_OR_CLEAN(hipMalloc((void **)&block_sums, (size_t)(n_blocks + 1) * 4));
    TRY_OR_CLEAN(hipMalloc((void **)&task_offsets, (size_t)(nw + 1) * 4));
    hipLaunchKernelGGL(wcsr_task_count_kernel, dim3(n_blocks), dim3(256), 0, stream, h->d_row_ptr, nw, h->task_cols,
                       local_excl, block_sums);
    hipLaunchKernelGGL(wcsr_task_block_scan_kernel, dim3(1), dim3(256), 0, stream, block_sums, n_blocks);
    hipLaunchKernelGGL(wcsr_task_offsets_kernel, dim3(n_blocks), dim3(256), 0, stream, local_excl, block_sums, nw,
                       n_blocks, task_offsets);
    TRY_OR_CLEAN(hipGetLastError());
    int32_t total = 0;
    TRY_OR_CLEAN(hipMemcpyAsync(&total, task_offsets + nw, 4, hipMemcpyDeviceToHost, stream));
    TRY_OR_CLEAN(hipStreamSynchronize(stream));
    h->n_tasks = total;
    TRY_OR_CLEAN(hipMalloc((void **)&h->d_tasks, total > 0 ? (size_t)total * 16 : 16));
    if (total > 0) {
        hipLaunchKernelGGL(wcsr_task_emit_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, stream,
                           h->d_row_ptr, task_offsets, nw, total, h->task_cols, (int4 *)h->d_tasks);
        TRY_OR_CLEAN(hipGetLastError());
        TRY_OR_CLEAN(hipStreamSynchronize(stream));
    }
#undef TRY_OR_CLEAN
    cleanup();
    return st;
}

// ---- host side ------------------------------------------------------------------------------------
WcsrPlan wcsr_plan(const asp_handle *h, int64_t N, bool aligned) {
    WcsrPlan p;
    if (h->dtype == ASP_DT_BF16) {  // one wavefront per (task, 128 columns), 4 to a workgroup; element-wise path: a workgroup per (window, 64 columns)
        p.vectorized = (aligned && N % 8 == 0) ? 1 : 0;
        p.bn = p.vectorized ? 128 : 64;
        p.n_tiles = (int32_t)ceil_div(N, p.bn);
        p.workgroups = p.vectorized ? ceil_div(h->n_tasks * p.n_tiles, 4) : h->n_brows * p.n_tiles;
        return p;
    }
    p.vectorized = (aligned && N % 4 == 0) ? 1 : 0;
    if (h->b_row == 16) {
        // Section IV-C rule over the built wave widths: widest that divides N, else least padding
        static const int cand[3] = {64, 128, 256};
        const int env_max = switches().wcsr_max_bn;  // benchmarking switch: widest wave tile to consider
        int best = -1;
        for (int c : cand)
            if (c <= env_max && N % c == 0 && c > best) best = c;
        if (best < 0) {
            int64_t best_pad = -1;
            for (int c : cand) {
                if (c > env_max) continue;
                int64_t pad = ceil_div(N, c) * c;
                if (best_pad < 0 || pad < best_pad || (pad == best_pad && c > best)) {
                    best_pad = pad;
                    best = c;
                }
            }
        }
        p.bn = best;
    } else {
        p.bn = 128;
    }
    p.n_tiles = (int32_t)ceil_div(N, p.bn);
    p.workgroups = ceil_div(h->n_tasks * p.n_tiles, 4);
    return p;
}

int64_t wcsr_scratch_floats(const asp_handle *h, int64_t N) { return h->n_split_tasks * h->b_row * N; }

void wcsr_clear_empty_windows(const asp_handle *h, void *C, int64_t N, bool keep_split, hipStream_t stream) {
    if (h->n_zero_windows == 0) return;
    const int es = (int)dtype_size(h->dtype);
    const bool vec = ((uintptr_t)C & 15) == 0 && (N * es) % 16 == 0;
    hipLaunchKernelGGL(wcsr_zero_rows_kernel, dim3((unsigned)h->n_zero_windows), dim3(256), 0, stream,
                       h->d_zero_windows, keep_split ? h->d_ws_slot : nullptr, h->b_row, (uint8_t *)C, es, (int)h->m, N,
                       vec);
}

void wcsr_sum_partial_tiles(const asp_handle *h, void *C, int64_t N, const float *ws, hipStream_t stream) {
    if (h->n_split_tasks == 0) return;
    const bool vec = N % 4 == 0 && ((uintptr_t)C & 15) == 0;
    const unsigned gy = (unsigned)std::min<int64_t>(64, ceil_div((int64_t)h->b_row * N, vec ? 1024 : 256));
    dim3 grid((unsigned)h->n_zero_windows, gy), block(256);
#define ASP_SUM(T, U)                                                                                              \
    hipLaunchKernelGGL((wcsr_sum_partials_kernel<T, U>), grid, block, 0, stream, h->d_zero_windows, h->d_ws_slot, \
                       h->d_row_ptr, h->task_cols, h->b_row, (T *)C, ws, (int)h->m, N)
    if (h->dtype == ASP_DT_BF16) {
        if (vec) ASP_SUM(__bf16, 4);
        else ASP_SUM(__bf16, 1);
    } else {
        if (vec) ASP_SUM(float, 4);
        else ASP_SUM(float, 1);
    }
#undef ASP_SUM
}

asp_status_t wcsr_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, float *ws_buf, int64_t ws_floats,
                              hipStream_t stream) {
    if (h->dtype == ASP_DT_BF16) return wcsr_bf16_spmm_launch(h, B, C, N, ws_buf, ws_floats, stream);
    const bool aligned = (((uintptr_t)B | (uintptr_t)C) & 15) == 0;
    const WcsrPlan p = wcsr_plan(h, N, aligned);
    const bool vec = p.vectorized != 0;
    if (p.workgroups >= (1ll << 31)) return fail(ASP_ERR_UNSUPPORTED, "too many wave tasks");
    // split windows: partial tiles in the scratch buffer when it is large enough, else atomic adds into C
    const bool partial = h->n_split_tasks > 0 && ws_buf && ws_floats >= wcsr_scratch_floats(h, N);
    float *ws = partial ? ws_buf : nullptr;
    wcsr_clear_empty_windows(h, C, N, partial, stream);
    if (h->n_tasks > 0) {
        dim3 grid((unsigned)p.workgroups), block(256);
        const int4 *tasks = (const int4 *)h->d_tasks;
        const float *vals = (const float *)h->d_values;
        const float *Bf = (const float *)B;
        float *Cf = (float *)C;
        const int nt = (int)h->n_tasks, M = (int)h->m;
#define ASP_W16(NG)                                                                                                   \
    do {                                                                                                              \
        if (vec)                                                                                                      \
            hipLaunchKernelGGL((wcsr16_spmm_kernel<NG, true>), grid, block, 0, stream, tasks, nt, h->d_col_idx, vals, \
                               Bf, Cf, M, N, p.n_tiles, ws, h->d_ws_slot, h->d_row_ptr, h->task_cols);                  \
        else                                                                                                          \
            hipLaunchKernelGGL((wcsr16_spmm_kernel<NG, false>), grid, block, 0, stream, tasks, nt, h->d_col_idx,      \
                               vals, Bf, Cf, M, N, p.n_tiles, ws, h->d_ws_slot, h->d_row_ptr, h->task_cols);          \
    } while (0)
#define ASP_W32(MTW)                                                                                                   \
    do {                                                                                                               \
        if (vec)                                                                                                       \
            hipLaunchKernelGGL((wcsr32_spmm_kernel<MTW, true>), grid, block, 0, stream, tasks, nt, h->d_col_idx, vals, \
                               Bf, Cf, M, N, p.n_tiles, ws, h->d_ws_slot, h->d_row_ptr, h->task_cols); \
        else                                                                                                           \
            hipLaunchKernelGGL((wcsr32_spmm_kernel<MTW, false>), grid, block, 0, stream, tasks, nt, h->d_col_idx,      \
                               vals, Bf, Cf, M, N, p.n_tiles, ws, h->d_ws_slot, h->d_row_ptr, h->task_cols); \
    } while (0)
        if (h->b_row == 16) {
            if (p.bn == 256) ASP_W16(4);
            else if (p.bn == 128) ASP_W16(2);
            else ASP_W16(1);
        } else if (h->b_row == 32) {
            ASP_W32(1);
        } else {
            ASP_W32(2);
        }
#undef ASP_W16
#undef ASP_W32
    }
    if (partial) wcsr_sum_partial_tiles(h, C, N, ws, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ASP_ERR_HIP, std::string("WCSR kernel launch: ") + hipGetErrorString(e));
    return ASP_OK;
}

}  // namespace asp
