// WCSR x dense SpMM in bf16 for gfx950 (paper, Section II-C for the format, Section III-B/III-C for the
// gather kernel and the split of long row-windows; Table I runs both formats at one precision).
//
// The work is bound by the gather of B rows, and the gather is bound by the bytes a compute unit keeps in
// flight (about 100 KB per compute unit are needed at the loaded memory latency of 3-4 us; measured with a
// plain gather loop).  LDS is too small a landing zone for that -- a direct-to-LDS ring of this kernel
// stalled at half the bandwidth with every ring depth -- so, as in the fp32 kernel, gathered rows land in
// registers: one wavefront owns one (task, 128-column tile), a quarter wave reads the 256 bytes of a row
// with 16-byte loads, 32 rows (8 loads per lane) per stage, issued one stage ahead, indices two stages ahead.
//
// The bf16 matrix-core instruction wants, per lane, 8 consecutive k of one column of B, while a gathered row
// is contiguous along N.  The stage therefore passes through 8 KB of wave-private LDS once: written as it
// arrives (ds_write_b128) and read back with the transposing read ds_read_b64_tr_b16, which hands each lane
// 4 consecutive k of one column.  A wave's LDS operations execute in order, so the single buffer needs no
// barrier and no wait beyond the data dependencies.
//
// v_mfma_f32_16x16x32_bf16 is issued with the operands swapped (B fragment first), so a lane ends with
// 4 consecutive columns per matrix instruction; the columns of the 8 instructions are dealt so that the lane
// owns 4 runs of 8 adjacent columns and writes C with 16-byte stores.  The tasks of a window that is split
// (Section III-C) store their fp32 partial tiles in the handle's scratch buffer (asp_reserve); a last kernel
// adds them up in task order and rounds to bf16 once.
#include "asp_bcsr_pipe.h"

namespace asp {

template <int MTW>
__global__ __launch_bounds__(256) void wcsr_bf16_spmm_kernel(const int4 *__restrict__ tasks, int n_tasks,
                                                             const int32_t *__restrict__ window_col_idx,
                                                             const uint16_t *__restrict__ values,
                                                             const uint16_t *__restrict__ B, uint16_t *__restrict__ C,
                                                             float *__restrict__ ws, const int32_t *__restrict__ ws_slot,
                                                             const int32_t *__restrict__ window_row_ptr, int task_cols,
                                                             int M, int64_t N, int n_tiles) {
    constexpr int BRW = 16 * MTW;
    constexpr int A_TILE = BRW * 8;  // elements of one value tile [BRW][8]
    __shared__ __attribute__((aligned(16))) uint8_t lds[4][32 * 256];  // per wave: 32 gathered rows x 128 columns

    const int64_t wave_id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int task = (int)(wave_id / n_tiles), nt = (int)(wave_id % n_tiles);
    if (task >= n_tasks) return;  // whole wave leaves together
    uint8_t *sb = lds[threadIdx.x >> 6];
    const int4 td = tasks[task];  // window, first packed column, end packed column, split flag
    const int lane = threadIdx.x & 63, h = lane >> 4, p = lane & 15;
    const int64_t n0 = (int64_t)nt * 128, n = n0 + p * 8;
    const int tile0 = td.y >> 3, tile1 = td.z >> 3;
    const int nst = (tile1 - tile0 + 3) >> 2;  // stages of 32 packed columns

    // lane (h, p) gathers the rows k = 8h .. 8h+7 of a stage (chunk p of each) and holds A's tile h, row p
    struct Idx {
        int c[8];
    };
    auto load_idx = [&](int st) {
        Idx ix;
        const int pos = td.y + 32 * st + 8 * h;
        if (pos < td.z) {  // tasks begin and end on multiples of 8 packed columns
            const int4 lo = *(const int4 *)(window_col_idx + pos), hi = *(const int4 *)(window_col_idx + pos + 4);
            ix = Idx{{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w}};
        } else {
            ix = Idx{{-1, -1, -1, -1, -1, -1, -1, -1}};
        }
        return ix;
    };
    auto load_b = [&](const Idx &ix, uint4 (&v)[8]) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            v[q] = make_uint4(0, 0, 0, 0);  // pads (index -1) and columns past N contribute zeros
            if (ix.c[q] >= 0 && n < N) v[q] = *(const uint4 *)(B + (int64_t)ix.c[q] * N + n);
        }
    };
    auto load_a = [&](int st, bf16x8 (&af)[MTW]) {
        const int tile = tile0 + 4 * st + h;
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            af[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (tile < tile1) af[i] = *(const bf16x8 *)(values + (int64_t)tile * A_TILE + (i * 16 + p) * 8);
        }
    };
    // LDS layout: row k = 8h + q sits in slot 4q + h (256 bytes each), so that one write instruction fills
    // 1 KB contiguously; the 16-byte chunks of a row are XOR-swizzled by (q % 4) * 4 against bank conflicts
    // of the transposing reads.
    auto stage_to_lds = [&](const uint4 (&v)[8]) {
#pragma unroll
        for (int q = 0; q < 8; ++q) *(uint4 *)(sb + (q * 4 + h) * 256 + ((p ^ ((q & 3) << 2)) * 16)) = v[q];
    };

    f32x4 acc[MTW][8];
#pragma unroll
    for (int i = 0; i < MTW; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](const bf16x8 (&af)[MTW]) {
        // transposing read: lane i of a 16-lane group addresses row i/4 of its k group and the 4 columns of
        // chunk i%4; it receives the 4 rows of column i of the 16 columns the group's chunks hold
        const int j4 = p >> 2, c = p & 3;
        const uint8_t *row = sb + (j4 * 4 + h) * 256;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint8_t *p0 = row + ((((j >> 1) * 4 + c) ^ (j4 << 2)) * 16) + (j & 1) * 8;
            short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3))) *)(p0));
            short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (short4v __attribute__((address_space(3))) *)(p0 + 16 * 256));
            bf16x8 bfr = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int i = 0; i < MTW; ++i)
                // operands swapped: D[n][m] = sum_k B[k][n] * A[m][k]
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr, af[i], acc[i][j], 0, 0, 0);
        }
    };

    Idx ix = load_idx(0), ix_next = load_idx(1);
    uint4 v[8];
    bf16x8 af[MTW], af_cur[MTW];
    load_b(ix, v);
    load_a(0, af);
    for (int s = 0; s < nst; ++s) {
        stage_to_lds(v);
#pragma unroll
        for (int i = 0; i < MTW; ++i) af_cur[i] = af[i];
        if (s + 1 < nst) {  // the next stage flies while this one is multiplied
            ix = ix_next;
            load_b(ix, v);
            load_a(s + 1, af);
            ix_next = load_idx(s + 2);
        }
        compute(af_cur);
    }

    // D layout: register r of lane l is MFMA row 4*(l/16) + r = column (j/2)*32 + 8*(l/16) + 4*(j%2) + r of the
    // tile, MFMA column l%16 = row of the window
    const int64_t row0 = (int64_t)td.x * BRW;
    if (td.w == 0) {
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            const int64_t grow = row0 + i * 16 + p;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t gcol = n0 + t * 32 + h * 8;
                if (grow < M && gcol < N) {
                    bf16x4 a = __builtin_convertvector(acc[i][2 * t], bf16x4);      // round to nearest even
                    bf16x4 b = __builtin_convertvector(acc[i][2 * t + 1], bf16x4);
                    bf16x8 v8 = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
                    *(bf16x8 *)(C + grow * N + gcol) = v8;
                }
            }
        }
    } else {
        // partial tile of this task: slot = first slot of the window + index of the task inside the window
        const int64_t slot = ws_slot[td.x] + (td.y - window_row_ptr[td.x]) / task_cols;
#pragma unroll
        for (int i = 0; i < MTW; ++i) {
            float *wr = ws + (slot * BRW + i * 16 + p) * N;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t gcol = n0 + t * 32 + h * 8;
                if (gcol < N) {
                    *(f32x4 *)(wr + gcol) = acc[i][2 * t];
                    *(f32x4 *)(wr + gcol + 4) = acc[i][2 * t + 1];
                }
            }
        }
    }
}

// ---- element-wise path: any N, any alignment; one thread per column, whole windows, no splitting, no scratch
template <int BRW>
__global__ __launch_bounds__(64) void wcsr_bf16_generic_kernel(const int32_t *__restrict__ window_row_ptr,
                                                               const int32_t *__restrict__ window_col_idx,
                                                               const uint16_t *__restrict__ values,
                                                               const uint16_t *__restrict__ B, uint16_t *__restrict__ C,
                                                               int M, int64_t N) {
    const int w = blockIdx.x;
    const int64_t n = (int64_t)blockIdx.y * 64 + threadIdx.x;
    if (n >= N) return;
    auto widen = [](uint16_t u) { return __uint_as_float((uint32_t)u << 16); };
    float acc[BRW];
#pragma unroll
    for (int r = 0; r < BRW; ++r) acc[r] = 0.f;
    for (int pc = window_row_ptr[w]; pc < window_row_ptr[w + 1]; ++pc) {
        const int col = window_col_idx[pc];
        if (col < 0) continue;
        const float b = widen(B[(int64_t)col * N + n]);
        const uint16_t *av = values + (int64_t)(pc >> 3) * (BRW * 8) + (pc & 7);
#pragma unroll
        for (int r = 0; r < BRW; ++r) acc[r] = __builtin_fmaf(widen(av[r * 8]), b, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < BRW; ++r) {
        const int64_t grow = (int64_t)w * BRW + r;
        if (grow < M) {
            const __bf16 v = (__bf16)acc[r];  // round to nearest even
            C[grow * N + n] = __builtin_bit_cast(uint16_t, v);
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------
asp_status_t wcsr_bf16_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, float *ws, int64_t ws_floats,
                                   hipStream_t stream) {
    const bool aligned = (((uintptr_t)B | (uintptr_t)C) & 15) == 0;
    const WcsrPlan p = wcsr_plan(h, N, aligned);
    const uint16_t *vals = (const uint16_t *)h->d_values, *Bh = (const uint16_t *)B;
    uint16_t *Ch = (uint16_t *)C;
    const int M = (int)h->m;
    if (!p.vectorized) {
        dim3 grid((unsigned)h->n_brows, (unsigned)ceil_div(N, 64)), block(64);
        if (grid.y > 65535) return fail(ASP_ERR_UNSUPPORTED, "N too large for the element-wise WCSR path");
        switch (h->b_row) {
            case 16: hipLaunchKernelGGL(wcsr_bf16_generic_kernel<16>, grid, block, 0, stream, h->d_row_ptr, h->d_col_idx, vals, Bh, Ch, M, N); break;
            case 32: hipLaunchKernelGGL(wcsr_bf16_generic_kernel<32>, grid, block, 0, stream, h->d_row_ptr, h->d_col_idx, vals, Bh, Ch, M, N); break;
            default: hipLaunchKernelGGL(wcsr_bf16_generic_kernel<64>, grid, block, 0, stream, h->d_row_ptr, h->d_col_idx, vals, Bh, Ch, M, N); break;
        }
    } else {
        if (p.workgroups >= (1ll << 31)) return fail(ASP_ERR_UNSUPPORTED, "too many wave tasks");
        if (h->n_split_tasks > 0 && ws_floats < wcsr_scratch_floats(h, N))
            return fail(ASP_ERR_BUFFER_TOO_SMALL,
                        "bf16 WCSR with split windows needs scratch memory for this width: call asp_reserve(handle, N) first");
        wcsr_clear_empty_windows(h, C, N, true, stream);
        if (h->n_tasks > 0) {
            dim3 grid((unsigned)p.workgroups), block(256);
            const int4 *tasks = (const int4 *)h->d_tasks;
            const int nt = (int)h->n_tasks;
#define ASP_WB(MTW)                                                                                                 \
    hipLaunchKernelGGL((wcsr_bf16_spmm_kernel<MTW>), grid, block, 0, stream, tasks, nt, h->d_col_idx, vals, Bh, Ch, \
                       ws, h->d_ws_slot, h->d_row_ptr, h->task_cols, M, N, p.n_tiles)
            if (h->b_row == 16) ASP_WB(1);
            else if (h->b_row == 32) ASP_WB(2);
            else ASP_WB(4);
#undef ASP_WB
        }
        wcsr_sum_partial_tiles(h, C, N, ws, stream);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ASP_ERR_HIP, std::string("WCSR bf16 kernel launch: ") + hipGetErrorString(e));
    return ASP_OK;
}

}  // namespace asp
