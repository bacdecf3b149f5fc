// BCSR x dense SpMM in fp32 for gfx950 (paper, Section II-C for the format; Table I runs both formats at
// one precision, which is why BCSR also exists in fp32 here).
//
// fp32 matrix-core throughput is 1/16 of bf16's while the operands are only twice as large, so this product
// is bound by the matrix cores by a wide margin and the data path can stay simple: one workgroup computes
// one (block-row, N-tile) output tile; per 16-k slice of a stored block the A slice and the matching rows
// of B go global -> registers -> LDS, double buffered, while the previous slice is multiplied
// (v_mfma_f32_32x32x2_f32, fp32 accumulation in hardware order).
//
// Operand layouts
//   A  blocks are pre-permuted on the host (bcsr_pack_fragments_f32): for every 32-row tile and group of
//      8 k, lane l holds 4 values A[l % 32][2t + l / 32], t = 0..3 -- the A operands of 4 consecutive MFMAs
//      as one ds_read_b128, lane-linear.
//   B  rows land in LDS as they are.  Lane l = 32*kq + j reads 4 adjacent columns 4j..4j+3 of row 2s + kq
//      (one ds_read_b128) and feeds them to four MFMAs that share the A value: MFMA t computes the columns
//      n = 4j + t of a 128-column group.  Every lane therefore ends with 4 adjacent output columns per row
//      and C is written straight from the accumulators with 16-byte stores.
#include "asp_internal.h"

namespace asp {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int BR, int BN, int WM, int WN>
struct BcsrF32Cfg {
    static constexpr int KS = 16;                  // k rows per pipeline stage
    static constexpr int NT = WM * WN * 64;        // threads
    static constexpr int TM = BR / WM;             // wave tile rows
    static constexpr int TN = BN / WN;             // wave tile columns
    static constexpr int MT = TM / 32;             // 32-row MFMA tiles per wave
    static constexpr int NG = TN / 128;            // 128-column groups per wave
    static constexpr int SPB = BR / KS;            // stages per (square) block
    static constexpr int A_STAGE = BR * KS * 4;    // bytes
    static constexpr int PB = BN * 4;              // LDS pitch of a B row, bytes
    static constexpr int B_STAGE = KS * PB;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int A_CHUNKS = A_STAGE / 16;  // 16-byte units per stage
    static constexpr int B_CPR = BN / 4;           // 16-byte units per B row
    static constexpr int B_CHUNKS = KS * B_CPR;
    static constexpr int A_LD = (A_CHUNKS + NT - 1) / NT;
    static constexpr int B_LD = (B_CHUNKS + NT - 1) / NT;
    static_assert(TM % 32 == 0 && TN % 128 == 0, "wave tile must be made of 32 x 128 pieces");
    static_assert(BR % KS == 0, "block width must be a multiple of the stage depth");
};

template <int BR, int BN, int WM, int WN, bool VEC>
__global__ __launch_bounds__(WM *WN * 64, 2) void bcsr_f32_spmm_kernel(
    const int32_t *__restrict__ rank_info, const int32_t *__restrict__ block_col_idx,
    const float *__restrict__ a_packed, const float *__restrict__ B, float *__restrict__ C, int M, int K, int64_t N,
    int n_brows, int n_tiles, int tiles_per_xcd) {
    using Cfg = BcsrF32Cfg<BR, BN, WM, WN>;
    constexpr int NT = Cfg::NT, KS = Cfg::KS, MT = Cfg::MT, NG = Cfg::NG;
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * Cfg::STAGE];

    // Workgroups go to the 8 XCDs round-robin by flat id: give each XCD a contiguous run of the
    // (N-tile major, block-row minor) order so that the tiles sharing an L2 read the same columns of B.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int64_t total = (int64_t)n_brows * n_tiles;
    const int64_t u = (int64_t)xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || u >= total) return;
    const int nt = (int)(u / n_brows);
    const int4 ri = ((const int4 *)rank_info)[u % n_brows];  // block-row, first block, blocks, -
    const int br = ri.x, blk0 = ri.y;
    const int64_t n0 = (int64_t)nt * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int kq = lane >> 5, jl = lane & 31;
    const int T = ri.z * Cfg::SPB;  // pipeline stages of this tile

    f32x16 acc[MT][NG][4];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][g][t][r] = 0.f;

    f32x4 ra[Cfg::A_LD], rb[Cfg::B_LD];

    auto load_stage = [&](int t) {
        const int p = blk0 + t / Cfg::SPB, s = t % Cfg::SPB;
        const f32x4 *asrc = (const f32x4 *)(a_packed + (int64_t)p * (BR * BR) + (int64_t)s * (BR * KS));
#pragma unroll
        for (int i = 0; i < Cfg::A_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::A_CHUNKS % NT == 0 || c < Cfg::A_CHUNKS) ra[i] = asrc[c];
        }
        const int krow0 = block_col_idx[p] * BR + s * KS;
#pragma unroll
        for (int i = 0; i < Cfg::B_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::B_CHUNKS % NT == 0 || c < Cfg::B_CHUNKS) {
                const int r = c / Cfg::B_CPR, cc = c % Cfg::B_CPR;
                const int krow = krow0 + r;
                const int64_t col = n0 + cc * 4;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (krow < K && col < N) {  // rows past K are the zero padding of the last block column
                    const float *src = B + (int64_t)krow * N + col;
                    if (VEC) {
                        v = *(const f32x4 *)src;
                    } else {
                        v.x = src[0];
                        if (col + 1 < N) v.y = src[1];
                        if (col + 2 < N) v.z = src[2];
                        if (col + 3 < N) v.w = src[3];
                    }
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
            if (Cfg::A_CHUNKS % NT == 0 || c < Cfg::A_CHUNKS) *(f32x4 *)(sa + c * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < Cfg::B_LD; ++i) {
            int c = i * NT + tid;
            if (Cfg::B_CHUNKS % NT == 0 || c < Cfg::B_CHUNKS) *(f32x4 *)(sb + c * 16) = rb[i];
        }
    };
    auto compute_stage = [&](int buf) {
        const uint8_t *sa = lds + buf * Cfg::STAGE, *sb = sa + Cfg::A_STAGE;
#pragma unroll
        for (int kg = 0; kg < KS / 8; ++kg) {
            f32x4 af[MT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                af[i] = *(const f32x4 *)(sa + (((wm * MT + i) * (KS / 8) + kg) * 64 + lane) * 16);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int krow = kg * 8 + 2 * t + kq;
                f32x4 bf[NG];
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    bf[g] = *(const f32x4 *)(sb + krow * Cfg::PB + (wn * Cfg::TN + g * 128 + 4 * jl) * 4);
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    const float a = af[i][t];
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        acc[i][g][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bf[g].x, acc[i][g][0], 0, 0, 0);
                        acc[i][g][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bf[g].y, acc[i][g][1], 0, 0, 0);
                        acc[i][g][2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bf[g].z, acc[i][g][2], 0, 0, 0);
                        acc[i][g][3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bf[g].w, acc[i][g][3], 0, 0, 0);
                    }
                }
            }
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

    // D layout of the MFMA: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32 (= jl), and
    // MFMA t of a group holds output column 4*jl + t: four adjacent columns per lane and row.
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t grow = (int64_t)br * BR + wm * Cfg::TM + i * 32 + 8 * (r >> 2) + 4 * kq + (r & 3);
                const int64_t gcol = n0 + wn * Cfg::TN + g * 128 + 4 * jl;
                if (grow < M && gcol < N) {
                    float *dst = C + grow * N + gcol;
                    const f32x4 v = {acc[i][g][0][r], acc[i][g][1][r], acc[i][g][2][r], acc[i][g][3][r]};
                    if (VEC) {
                        __builtin_nontemporal_store(v, (f32x4 *)dst);  // C is write-once: keep B in L2
                    } else {
                        dst[0] = v.x;
                        if (gcol + 1 < N) dst[1] = v.y;
                        if (gcol + 2 < N) dst[2] = v.z;
                        if (gcol + 3 < N) dst[3] = v.w;
                    }
                }
            }
}

// ---- host side ------------------------------------------------------------------------------------
template <int BR, int BN, int WM, int WN, bool VEC>
static void launch_f32(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    const int tiles_per_xcd = (int)ceil_div(p.workgroups, 8);
    dim3 grid((unsigned)(tiles_per_xcd * 8)), block(WM * WN * 64);
    hipLaunchKernelGGL((bcsr_f32_spmm_kernel<BR, BN, WM, WN, VEC>), grid, block, 0, stream, h->d_rank_info,
                       h->d_col_idx, (const float *)h->d_values, (const float *)B, (float *)C, (int)h->m, (int)h->k, N,
                       (int)h->n_brows, p.n_tiles, tiles_per_xcd);
}

bool bcsr_f32_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    const int key = h->b_row * 1000 + p.bn;
    if (p.vectorized) {
        switch (key) {
            case 128256: launch_f32<128, 256, 2, 2, true>(h, B, C, N, p, stream); return true;
            case 128128: launch_f32<128, 128, 2, 1, true>(h, B, C, N, p, stream); return true;
            case 64256: launch_f32<64, 256, 2, 2, true>(h, B, C, N, p, stream); return true;
            case 64128: launch_f32<64, 128, 2, 1, true>(h, B, C, N, p, stream); return true;
            case 32256: launch_f32<32, 256, 1, 2, true>(h, B, C, N, p, stream); return true;
            case 32128: launch_f32<32, 128, 1, 1, true>(h, B, C, N, p, stream); return true;
            default: return false;
        }
    }
    switch (key) {
        case 128128: launch_f32<128, 128, 2, 1, false>(h, B, C, N, p, stream); return true;
        case 64128: launch_f32<64, 128, 2, 1, false>(h, B, C, N, p, stream); return true;
        case 32128: launch_f32<32, 128, 1, 1, false>(h, B, C, N, p, stream); return true;
        default: return false;
    }
}

}  // namespace asp
