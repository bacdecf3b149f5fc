// BCSR x dense SpMM for gfx950: dispatch (tile-width rule of the paper's Section IV-C) and the
// register-staged kernel.
//
// The register-staged kernel is the synchronous-copy design (the analogue of the paper's Section III-A
// kernel with cooperative loads, plus one slice of prefetch): global loads go to VGPRs, then to LDS.  It
// serves operands that do not allow 16-byte accesses (element-wise path) and stays selectable for
// comparison runs; aligned operands take the direct-to-LDS ring kernel in asp_bcsr_dma.hip.
//
// One workgroup computes one (block-row, N-tile) output tile of b_row x BN: it walks the stored blocks
// of its block-row (Section II-C), and for each K slice of a block stages the A slice and the matching
// rows of B through LDS, double buffered, while the previous slice is multiplied on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Operand layouts
//   A  blocks are pre-permuted on the host into MFMA fragment order, so a slice is one contiguous,
//      fully coalesced run in memory and in LDS (ds_read_b128, lane-linear).
//   B  is row-major K x N: a K slice lands in LDS row by row (pitch BN*2+64 bytes so the four rows of a
//      transposing read fall in disjoint banks) and is read with ds_read_b64_tr_b16, which hands every
//      lane 4 consecutive k of one column -- the K-contiguous operand the MFMA wants.
//   The MFMA is issued with the operands swapped (B fragment first), so each lane ends with 4
//   consecutive columns of one output row: the tile is rounded to bf16, passed through LDS and written
//   to C with 16-byte row-contiguous stores.
#include <cstdlib>
#include <cstring>

#include "asp_internal.h"

namespace asp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // staging registers: a plain vector type, so that
                                                                 // arrays of it are split into registers

template <int BR, int BC, int BN, int WM, int WN, bool VEC>
struct BcsrCfg {
    static constexpr int KS = 32;                  // k rows per pipeline stage
    static constexpr int NT = WM * WN * 64;        // threads
    static constexpr int TM = BR / WM;             // wave tile rows
    static constexpr int TN = BN / WN;             // wave tile columns
    static constexpr int MT = TM / 32;             // 32x32 MFMA tiles per wave, along M
    static constexpr int NTL = TN / 32;            //   and along N
    static constexpr int KK = KS / 16;             // MFMA k steps per stage
    static constexpr int SPB = BC / KS;            // stages per block
    static constexpr int A_STAGE = BR * KS * 2;    // bytes
    static constexpr int PB = BN * 2 + 64;         // LDS pitch of a B row, bytes
    static constexpr int B_STAGE = KS * PB;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int A_CHUNKS = A_STAGE / 16;  // 16-byte units per stage
    static constexpr int B_CPR = BN / 8;           // 16-byte units per B row
    static constexpr int B_CHUNKS = KS * B_CPR;
    static constexpr int A_LD = (A_CHUNKS + NT - 1) / NT;
    static constexpr int B_LD = (B_CHUNKS + NT - 1) / NT;
    static constexpr int C_PITCH = TN * 2 + 16;    // epilogue staging pitch per wave, bytes
    static constexpr int C_WAVE = TM * C_PITCH;
    static constexpr int LDS_BYTES = (2 * STAGE > WM * WN * C_WAVE) ? 2 * STAGE : WM * WN * C_WAVE;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert(BC % KS == 0, "block width must be a multiple of the stage depth");
};

__device__ __forceinline__ u32x4 load_b_chunk_scalar(const uint16_t *__restrict__ B, int64_t row_off, int col, int N) {
    // slow path: N or the base pointers do not allow 16-byte accesses
    uint16_t e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = (col + i < N) ? B[row_off + col + i] : (uint16_t)0;
    u32x4 v;
    v.x = e[0] | ((uint32_t)e[1] << 16);
    v.y = e[2] | ((uint32_t)e[3] << 16);
    v.z = e[4] | ((uint32_t)e[5] << 16);
    v.w = e[6] | ((uint32_t)e[7] << 16);
    return v;
}

template <int BR, int BC, int BN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(WM *WN * 64, 2) void bcsr_spmm_kernel(
    const int32_t *__restrict__ block_row_ptr, const int32_t *__restrict__ block_col_idx,
    const uint16_t *__restrict__ a_packed, const uint16_t *__restrict__ B, uint16_t *__restrict__ C, int M, int K,
    int N, int n_brows, int n_tiles, int tiles_per_xcd) {
    using Cfg = BcsrCfg<BR, BC, BN, WM, WN, VEC>;
    constexpr int NT = Cfg::NT, KS = Cfg::KS, MT = Cfg::MT, NTL = Cfg::NTL;
    __shared__ __attribute__((aligned(16))) uint8_t lds[Cfg::LDS_BYTES];

    // Workgroups are handed to the 8 XCDs round-robin by flat id.  Give each XCD a contiguous run of
    // the (N-tile major, block-row minor) tile order so that the workgroups sharing one XCD's L2 work
    // on the same column slab of B.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int64_t total = (int64_t)n_brows * n_tiles;
    const int64_t u = (int64_t)xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || u >= total) return;
    const int nt = (int)(u / n_brows), br = (int)(u % n_brows);
    const int n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int blk0 = block_row_ptr[br], blk1 = block_row_ptr[br + 1];
    const int T = (blk1 - blk0) * Cfg::SPB;  // pipeline stages of this tile

    f32x16 acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 ra[Cfg::A_LD], rb[Cfg::B_LD];

    auto load_stage = [&](int t) {
        const int p = blk0 + t / Cfg::SPB, s = t % Cfg::SPB;
        const u32x4 *asrc = (const u32x4 *)(a_packed + (int64_t)p * (BR * BC) + (int64_t)s * (BR * KS));
#pragma unroll
        for (int i = 0; i < Cfg::A_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::A_CHUNKS % NT == 0 || c < Cfg::A_CHUNKS) ra[i] = asrc[c];
        }
        const int krow0 = block_col_idx[p] * BC + s * KS;
#pragma unroll
        for (int i = 0; i < Cfg::B_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::B_CHUNKS % NT == 0 || c < Cfg::B_CHUNKS) {
                int r = c / Cfg::B_CPR, cc = c % Cfg::B_CPR;
                int krow = krow0 + r, col = n0 + cc * 8;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (krow < K && col < N) {  // rows past K belong to the zero padding of the last block column
                    if (VEC)
                        v = *(const u32x4 *)(B + (int64_t)krow * N + col);
                    else
                        v = load_b_chunk_scalar(B, (int64_t)krow * N, col, N);
                }
                rb[i] = v;
            }
        }
    };
    auto store_stage = [&](int buf) {
        uint8_t *sa = lds + buf * Cfg::STAGE, *sb = sa + Cfg::A_STAGE;
#pragma unroll
        for (int i = 0; i < Cfg::A_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::A_CHUNKS % NT == 0 || c < Cfg::A_CHUNKS) *(u32x4 *)(sa + c * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < Cfg::B_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::B_CHUNKS % NT == 0 || c < Cfg::B_CHUNKS) {
                int r = c / Cfg::B_CPR, cc = c % Cfg::B_CPR;
                *(u32x4 *)(sb + r * Cfg::PB + cc * 16) = rb[i];
            }
        }
    };
    auto compute_stage = [&](int buf) {
        const uint8_t *sa = lds + buf * Cfg::STAGE, *sb = sa + Cfg::A_STAGE;
#pragma unroll
        for (int kk = 0; kk < Cfg::KK; ++kk) {
            bf16x8 af[MT], bfr[NTL];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                int mtg = wm * MT + i;
                af[i] = *(const bf16x8 *)(sa + ((kk * (BR / 32) + mtg) * 64 + lane) * 16);
            }
            // transposing read: lane i of a 16-lane group addresses row i/4, 4 columns at 4*(i%4);
            // it receives the 4 rows of column (i) of the group's 16 columns
            const int krow = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
#pragma unroll
            for (int j = 0; j < NTL; ++j) {
                int col = wn * Cfg::TN + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
                const uint8_t *p0 = sb + krow * Cfg::PB + col * 2;
                short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (short4v __attribute__((address_space(3))) *)(p0));
                short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (short4v __attribute__((address_space(3))) *)(p0 + 4 * Cfg::PB));
                short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bfr[j] = __builtin_bit_cast(bf16x8, both);
            }
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NTL; ++j)
                    // operands swapped: D[n][m] = sum_k B[k][n] * A[m][k]
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
        }
    };

    if (T > 0) {
        load_stage(0);
        store_stage(0);
        __syncthreads();
        for (int t = 0; t < T; ++t) {
            const int buf = t & 1;
            if (t + 1 < T) load_stage(t + 1);  // global loads fly while this stage is multiplied
            compute_stage(buf);
            if (t + 1 < T) store_stage(buf ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue: fp32 -> bf16, through LDS, 16-byte row stores --------------------------------
    uint8_t *sc = lds + wave * Cfg::C_WAVE;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                bf16x4 hv = __builtin_convertvector(v, bf16x4);  // round to nearest even
                int mrow = i * 32 + (lane & 31);
                int ncol = j * 32 + 8 * q + 4 * (lane >> 5);
                *(bf16x4 *)(sc + mrow * Cfg::C_PITCH + ncol * 2) = hv;
            }
    __syncthreads();
    constexpr int CPR = Cfg::TN / 8;   // 16-byte units per staged row
    constexpr int RPI = 64 / CPR;      // rows per wave instruction
#pragma unroll
    for (int it = 0; it < Cfg::TM / RPI; ++it) {
        int row = it * RPI + lane / CPR, cc = lane % CPR;
        uint4 v = *(const uint4 *)(sc + row * Cfg::C_PITCH + cc * 16);
        int grow = br * BR + wm * Cfg::TM + row;
        int gcol = n0 + wn * Cfg::TN + cc * 8;
        if (grow < M && gcol < N) {
            uint16_t *dst = C + (int64_t)grow * N + gcol;
            if (VEC) {
                *(uint4 *)dst = v;
            } else {
                uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (gcol + e < N) dst[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------

// Section IV-C: take the widest tile that divides N; when none does, the one that pads N the least.
static int choose_bn(int64_t N, const int *cand, int n) {
    int best = -1;
    for (int i = 0; i < n; ++i)
        if (N % cand[i] == 0 && cand[i] > best) best = cand[i];
    if (best > 0) return best;
    int64_t best_pad = -1;
    for (int i = 0; i < n; ++i) {
        int64_t pad = ceil_div(N, cand[i]) * cand[i];
        if (best_pad < 0 || pad < best_pad || (pad == best_pad && cand[i] > best)) {
            best_pad = pad;
            best = cand[i];
        }
    }
    return best;
}

// Section IV-C with both effects priced: a wider tile does more work per loaded A tile (cost per column falls
// with the width), a tile that does not divide N computes on padding.  Least padded width x cost; ties: wider.
static int choose_bn_weighted(int64_t N, const int *cand, const int *cost, int n) {
    int best = -1;
    int64_t best_total = -1;
    for (int i = 0; i < n; ++i) {
        const int64_t total = ceil_div(N, cand[i]) * cand[i] * cost[i];
        if (best < 0 || total < best_total || (total == best_total && cand[i] > best)) {
            best_total = total;
            best = cand[i];
        }
    }
    return best;
}

BcsrPlan bcsr_plan(const asp_handle *h, int64_t N, bool aligned) {
    BcsrPlan p;
    if (h->dtype == ASP_DT_F32) {  // fp32 kernel: 128- and 256-wide tiles, element-wise path at 128
        static const int cand32[2] = {128, 256};
        p.vectorized = (aligned && N % 4 == 0) ? 1 : 0;
        p.bn = p.vectorized ? choose_bn(N, cand32, 2) : 128;
        p.n_tiles = (int32_t)ceil_div(N, p.bn);
        p.workgroups = h->n_brows * p.n_tiles;
        return p;
    }
    p.vectorized = (aligned && N % 8 == 0) ? 1 : 0;
    static const int cand[4] = {64, 128, 256, 512};
    // time per column of a tile of that width relative to a 512-wide one, in 1/64 (measured on the 128x128-block
    // projection workload at steady clocks: 0.529 / 0.376 / 0.290 / 0.251 ms for the same work)
    static const int cost[4] = {135, 96, 74, 64};
    const int env_bn = switches().bcsr_bn;  // benchmarking switch: caps the tile width
    if (!p.vectorized) {
        p.bn = 64;  // the element-wise path is only built for BN = 64
    } else {
        // 512-wide tiles (one resident workgroup per compute unit) exist for 128x128 blocks and only pay
        // when every compute unit gets at least one tile
        int ncand = 3;
        const int64_t cus = h->n_cus > 0 ? h->n_cus : 256;
        // (smaller blocks: through the composite form with 128-row super-rows, when the handle has one)
        if (bcsr_wide_capable(h) && N < (1ll << 25)) {
            const int64_t rows = h->has_comp ? h->hc.n_nonempty : h->hb.n_nonempty > 0 ? h->hb.n_nonempty : h->n_brows;
            if (rows * ceil_div(N, 512) >= cus) ncand = 4;
        }
        if (env_bn == 64 || env_bn == 128 || env_bn == 256)
            while (ncand > 1 && cand[ncand - 1] > env_bn) --ncand;
        p.bn = choose_bn_weighted(N, cand, cost, ncand);
        // A launch with fewer tiles than compute units leaves part of the chip idle and every tile runs alone at
        // the latency of its K loop: take the next narrower width while that is so (the 28 block-rows of the case
        // study's down projection at N = 1024: 0.079 / 0.060 / 0.043 ms with 256- / 128- / 64-wide tiles).
        const int64_t rows_ne = h->hb.n_nonempty > 0 ? h->hb.n_nonempty : h->n_brows;
        while (p.bn > 64 && p.bn < 512 && rows_ne * ceil_div(N, p.bn) < cus) p.bn /= 2;
    }
    p.n_tiles = (int32_t)ceil_div(N, p.bn);
    p.workgroups = (p.bn == 512 && h->has_comp ? h->c_n_brows : h->n_brows) * p.n_tiles;
    return p;
}

template <int BR, int BN, int WM, int WN, bool VEC>
static void launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    const int64_t total = p.workgroups;
    const int tiles_per_xcd = (int)ceil_div(total, 8);
    dim3 grid((unsigned)(tiles_per_xcd * 8)), block(WM * WN * 64);
    hipLaunchKernelGGL((bcsr_spmm_kernel<BR, BR, BN, WM, WN, VEC>), grid, block, 0, stream, h->d_row_ptr, h->d_col_idx,
                       (const uint16_t *)h->d_values, (const uint16_t *)B, (uint16_t *)C, (int)h->m, (int)h->k, (int)N,
                       (int)h->n_brows, p.n_tiles, tiles_per_xcd);
}

asp_status_t bcsr_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, hipStream_t stream) {
    const bool aligned = (((uintptr_t)B | (uintptr_t)C) & 15) == 0;
    const BcsrPlan p = bcsr_plan(h, N, aligned);
    if (p.workgroups * 8 >= (1ll << 31)) return fail(ASP_ERR_UNSUPPORTED, "too many output tiles");
    if (h->dtype == ASP_DT_F32) {
        if (!bcsr_f32_launch(h, B, C, N, p, stream))
            return fail(ASP_ERR_UNSUPPORTED, "no fp32 kernel for this block size / tile width");
        hipError_t e32 = hipGetLastError();
        if (e32 != hipSuccess) return fail(ASP_ERR_HIP, std::string("BCSR fp32 kernel launch: ") + hipGetErrorString(e32));
        return ASP_OK;
    }
    const int key = h->b_row * 1000 + p.bn;
    const bool force_regstage = switches().bcsr_regstage;  // benchmarking switch: the synchronous-copy kernel
    if (p.vectorized && !force_regstage && N < (1ll << 25)) {
        if (!bcsr_wide_launch(h, B, C, N, p, stream) && !bcsr_dma_launch(h, B, C, N, p, stream))
            return fail(ASP_ERR_UNSUPPORTED, "no kernel for this block size / tile width");
    } else if (!p.vectorized) {  // element-wise path
        switch (h->b_row) {
            case 128: launch<128, 64, 2, 2, false>(h, B, C, N, p, stream); break;
            case 64: launch<64, 64, 2, 2, false>(h, B, C, N, p, stream); break;
            default: launch<32, 64, 1, 2, false>(h, B, C, N, p, stream); break;
        }
    } else {
        switch (key) {
            case 128256: launch<128, 256, 2, 2, true>(h, B, C, N, p, stream); break;
            case 128128: launch<128, 128, 2, 2, true>(h, B, C, N, p, stream); break;
            case 128064: launch<128, 64, 2, 2, true>(h, B, C, N, p, stream); break;
            case 64256: launch<64, 256, 1, 4, true>(h, B, C, N, p, stream); break;
            case 64128: launch<64, 128, 2, 2, true>(h, B, C, N, p, stream); break;
            case 64064: launch<64, 64, 2, 2, true>(h, B, C, N, p, stream); break;
            case 32256: launch<32, 256, 1, 4, true>(h, B, C, N, p, stream); break;
            case 32128: launch<32, 128, 1, 4, true>(h, B, C, N, p, stream); break;
            case 32064: launch<32, 64, 1, 2, true>(h, B, C, N, p, stream); break;
            default: return fail(ASP_ERR_UNSUPPORTED, "no kernel for this block size / tile width");
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ASP_ERR_HIP, std::string("BCSR kernel launch: ") + hipGetErrorString(e));
    return ASP_OK;
}

}  // namespace asp
