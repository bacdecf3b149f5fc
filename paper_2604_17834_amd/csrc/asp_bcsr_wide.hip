// BCSR x dense SpMM for 128x128 blocks, wide-tile kernel: 128 x 512 output tiles, one wave per SIMD.
//
// Why a second kernel.  With 64 x 128 wave tiles (two waves per SIMD) the multiply loop reads 6 KB of
// operand fragments from LDS per 8 MFMAs, which needs three quarters of the LDS read bandwidth at full
// matrix-core rate; the measured ceiling of that loop is about 1.6 PFLOP/s before any global traffic.
// A 128 x 128 wave tile reads 8 KB per 16 MFMAs (half of the LDS bandwidth), but its 256 accumulator
// registers leave room for only one wave per SIMD.  A lone wave issues about one instruction every
// 5-7 cycles (measured), i.e. 4-5 instructions per 32-cycle MFMA: the loop is bound by its instruction
// count, and everything here serves to keep that near 3 instructions per MFMA:
//   - the K loop runs block by block, 4 slices of 32 k each, fully unrolled: the ring of four LDS
//     buffers is walked in step with the slices of a block, so every LDS address and every M0 value is
//     an immediate offset from a register that never changes;
//   - the request cursor (which slice to fetch next, three slices ahead) advances by two 64-bit adds
//     per slice; the per-block and per-tile work sits in one place of the unrolled body;
//   - a direct-to-LDS load needs one wait state after the write of M0: the MFMA issued in between
//     provides it;
//   - accumulators are cleared by MFMAs (0 x 0 + 0) issued during the epilogue, when the matrix core
//     is idle, instead of 256 register writes or a second copy of the loop with a zero input.
//
// Structure of a step (one 32-wide K slice of a stored block, paper Section II-C, in a ring of four
// LDS buffers filled by direct-to-LDS loads, the role TMA plays in Section III-B):
//   phase A   read the fragments of the slice's second k16 half from LDS | 16 MFMAs on the first half
//   phase B   wait for the next slice's loads, one fence-free barrier, read the first-half fragments
//             of the NEXT slice, request the slice three steps ahead | 16 MFMAs on the second half
// so LDS reads, global requests and the barrier all sit under MFMAs issued by the same wave, and the
// fragments of a slice's first half are carried in registers across the step (and tile) boundary.
// After the barrier of phase B nobody reads the current slice's buffer any more: it is the ring's
// spare buffer until the next step's barrier, and a finished tile stages its output there, without
// an extra barrier.  Slices are requested two full steps before they are waited for.
//
// Tiles with no stored block are not part of the stream (their rows of C are cleared by the same
// workgroups once their streams have ended).  At the end of its stream a workgroup keeps requesting the last block again (into
// free buffers, never read), so every step issues the same loads and the wait counts are constants.
// Scheduling, swizzling, store accounting: as in the 64 x 128 kernel.
#include <cstdlib>
#include <cstring>

#include "asp_bcsr_pipe.h"

namespace asp {

namespace {

struct WideCfg {
    static constexpr int BR = 128, BN = 512, KS = 32, NS = 4, NW = 4;
    static constexpr int SPB = BR / KS;
    static constexpr int TN = BN / NW;              // wave tile: 128 rows x 128 columns
    static constexpr int MT = BR / 32, NTL = TN / 32;
    static constexpr int A_STAGE = BR * KS * 2, B_ROW = BN * 2, B_STAGE = KS * B_ROW, STAGE = A_STAGE + B_STAGE;
    static constexpr int A_LPW = A_STAGE / 1024 / NW, B_LPW = B_STAGE / 1024 / NW, LPW = A_LPW + B_LPW;
    // epilogue: a wave stages 32 rows x 128 columns at a time, privately
    static constexpr int C_PITCH = TN * 2 + 16, C_WAVE = 32 * C_PITCH;
    static constexpr int CPR = TN / 8, RPI = 64 / CPR;  // 16-byte units per staged row, rows per store
    static constexpr int NSTORE = MT * (32 / RPI);
    static constexpr int LDS_BYTES = NS * STAGE;
    static_assert(SPB == NS, "the ring is walked in step with the slices of a block");
    static_assert(A_LPW == 2 && B_LPW == 8 && MT == 4 && NTL == 4 && TN == 128 && BR == 128, "the step below is written out for these");
    static_assert(NW * C_WAVE <= STAGE, "epilogue staging must fit into one ring buffer");
    static_assert(NSTORE + LPW + LPW / 2 < 64 && LPW % 2 == 0, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 163840, "LDS of one compute unit");
};

}  // namespace

// rank_info[r] = {block-row, first stored block, number of stored blocks, block column of the first one} of the r-th
// block-row of the schedule; only the first n_rows (non-empty) ones are walked.  No slice of the dense operand
// reaches past K: K is a multiple of the block size, or the blocks come in the composite form (GATHER).
//
// XT = false: C[M x N] = A x B, B is K x N row-major (paper, Section II-C).
// XT = true:  Y[N x M] = X x A^T, X is N x K row-major -- the same product with both dense matrices
//   transposed, i.e. K-contiguous activations in and out (the layout of the paper's LLM case study,
//   Section IV-D: C = W X^T with X stored tokens x hidden).  In the argument list B is then X and C is Y; a
//   tile is still (block-row, 512 columns of the product) = 128 outputs x 512 tokens.  What changes: a slice
//   of X is 512 tokens x 64 bytes, laid out in LDS token-major (1 KB region = 16 tokens, the 16-byte chunk of
//   a token XOR-swizzled by (token / 4) % 4) and read with plain 16-byte reads (it already is k-contiguous);
//   the MFMA operands are not swapped, so a lane ends with 4 adjacent outputs of one token; the epilogue
//   transposes 32 tokens x 128 outputs at a time and stores 256-byte row segments of Y.
//
// GATHER = true: the composite form of a matrix with 64x64 or 32x32 blocks (asp_convert.cpp): a "block" is 128 rows
// x four 32-wide K slices that multiply four separately placed 32-row strips of the dense operand;
// block_col_idx then holds, per block, the first dense row of each slice (int4) instead of a block column, the
// block-row number in rank_info is a super-row number, and piece_rows gives, per super-row, the first row of C of
// each of the tile's four 32-row pieces (-1: the piece has no rows; its accumulators are zeros).
// The composite form keeps every slice inside K (the slices of a partly filled last block column start early
// enough to end at K), which is how 128x128 blocks with K % 128 != 0 run here too.
template <bool XT, bool GATHER>
__global__ __launch_bounds__(256, 1) void bcsr_spmm_wide_kernel(
    const int4 *__restrict__ rank_info, const int32_t *__restrict__ block_col_idx,
    const uint16_t *__restrict__ a_packed, const uint16_t *__restrict__ B, uint16_t *__restrict__ C, int M, int K,
    int N, int n_rows, int n_brows, int n_blocks, int n_tiles, int group_n, int xcd_aware, XcdRuns runs,
    const int4 *__restrict__ piece_rows) {
    using Cfg = WideCfg;
    constexpr int NS = Cfg::NS, NW = Cfg::NW, KS = Cfg::KS, BR = Cfg::BR, BN = Cfg::BN, MT = Cfg::MT, NTL = Cfg::NTL;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[Cfg::LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- this workgroup's tiles: every stride-th tile of its XCD's run.  The order of block-rows was
    // built (per handle) so that this deals every workgroup one weight-balanced list per group of
    // N-tiles. -----------------------------------------------------------------------------------------
    // (xcd_aware = 0, a benchmarking switch: one run for all workgroups, i.e. neighbouring tiles land on
    // different XCDs and share nothing in L2)
    const int xcd = xcd_aware ? blockIdx.x & 7 : 0, stride = xcd_aware ? gridDim.x >> 3 : gridDim.x;
    const int wg = xcd_aware ? blockIdx.x >> 3 : blockIdx.x;
    const int run_begin = __builtin_amdgcn_readfirstlane(runs.start[xcd]);
    const int run_end = __builtin_amdgcn_readfirstlane(runs.start[xcd + 1]);
    auto tile_of_round = [&](int r) __attribute__((always_inline)) {
        return run_begin + r * stride + wg;
    };
    // Rows of C of block-rows without stored blocks (ranks n_rows .. n_brows-1; GATHER: four pieces of 32 rows per
    // super-row, placed by piece_rows) are cleared by the workgroups when their streams have ended.  Every such
    // span of rows is cut into `parts` equal parts and workgroup b takes the (span, part) items b, b + grid, ...:
    // a part per workgroup when the spans are few (equal shares, as many steps as spans), else so many parts
    // that a workgroup gets at least eight items (hundreds of small spans: a step per span and workgroup would
    // cost more than its one store).  A lane looks up the first row of one of the workgroup's items, 64 items
    // at a time: looked up one by one, the two dependent loads per item cost more than its stores.
    // (XT: a span is up to 256 bytes in every row of Y, and a part is a range of tokens)
    auto clear_empty_rows = [&]() __attribute__((always_inline)) {
        const uint4 z = {0u, 0u, 0u, 0u};
        const int first = n_rows * (GATHER ? 4 : 1), count = n_brows * (GATHER ? 4 : 1) - first;
        if (count <= 0) return;
        const int grid = (int)gridDim.x, b = (int)blockIdx.x;
        constexpr int rows_full = GATHER ? 32 : Cfg::BR;
        // units of a part: 16 bytes (row-major C, whole rows are one contiguous span) or tokens (XT)
        const int64_t span_full = XT ? (int64_t)N : (int64_t)rows_full * N / 8;
        const int64_t chunks = (span_full + 63) / 64;  // a part is at least what one pass of the workgroup's waves stores
        int parts = count >= 8 * grid ? 1 : (8 * grid + count - 1) / count;
        if (2 * count <= grid && chunks >= grid) parts = grid;
        if (parts > chunks) parts = (int)chunks;
        const int items = count * parts;  // <= grid * grid / 2, < 16 * grid, or count
        if (b >= items) return;
        const int mine = (items - b + grid - 1) / grid;
        // (whole kilobytes, so that no store of a wave straddles two parts' cache lines)
        const int64_t per = XT ? (span_full + parts - 1) / parts : ((span_full + parts - 1) / parts + 63) / 64 * 64;
        for (int base = 0; base < mine; base += 64) {
            const int item = b + (base + lane) * grid;
            int r0_l = -1, part_l = 0;
            if (base + lane < mine) {
                const int e = first + item / parts;
                part_l = item % parts;
                const int br = rank_info[GATHER ? e >> 2 : e].x;
                if (GATHER) {
                    const int4 pr = piece_rows[br];
                    r0_l = (e & 3) == 0 ? pr.x : (e & 3) == 1 ? pr.y : (e & 3) == 2 ? pr.z : pr.w;
                } else {
                    r0_l = br * Cfg::BR;
                }
            }
            const int nb = mine - base < 64 ? mine - base : 64;
            for (int j = 0; j < nb; ++j) {
                const int r0 = __builtin_amdgcn_readlane(r0_l, j);
                const int part = __builtin_amdgcn_readlane(part_l, j);
                if (r0 < 0 || r0 >= M) continue;
                const int r1 = r0 + rows_full < M ? r0 + rows_full : M;
                if (!XT) {
                    uint16_t *dst = C + (int64_t)r0 * N;
                    const int64_t n16 = (int64_t)(r1 - r0) * N / 8;
                    const int64_t lo = per * part, hi = lo + per < n16 ? lo + per : n16;
                    for (int64_t i = lo + tid; i < hi; i += 256) store_c16(dst + i * 8, z);
                } else {
                    const int cpr = (r1 - r0) / 8;  // 16-byte units per row (M % 8 == 0)
                    const int64_t lo = per * part, hi = lo + per < N ? lo + per : N;
                    for (int64_t t = lo + (tid >> 4); t < hi; t += 16)
                        if ((tid & 15) < cpr) store_c16(C + t * M + r0 + (tid & 15) * 8, z);
                }
            }
        }
    };
    int round = 0;
    int idx_cur = tile_of_round(0);
    if (idx_cur >= run_end) {
        clear_empty_rows();
        return;
    }

    // ---- LDS read addresses: one register per ring buffer, everything else is an immediate ----------
    // A fragments: lane-linear 16 bytes.  B fragments, transposing read: lane i of a 16-lane group
    // addresses row (i/4), 4 columns at 4*(i%4); rows are XOR-swizzled in 64-byte units by (row & 3).
    const int krow_lane = 8 * (lane >> 5) + ((lane & 15) >> 2);   // + 16*kk (+4 for the upper half)
    const int sw = (krow_lane & 3) << 2;                           // same for krow_lane + 4 and + 16
    const int c_lane = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);  // chunk inside the 32-column tile
    const int sub = 8 * (lane & 1);                                // byte inside the chunk
    const uint32_t lds0 = lds_offset(lds);
    // XT: lane l reads token wave*128 + j*32 + l%32, chunk 2*kk + l/32 of its 64 bytes; the swizzle makes
    // the two k halves differ by more than an immediate, hence a second set of addresses (b_addr1).
    uint32_t a_addr[NS], b_addr[NS][NTL], b_addr1[XT ? NS : 1][NTL];
#pragma unroll
    for (int b = 0; b < NS; ++b) {
        a_addr[b] = lds0 + b * Cfg::STAGE + lane * 16;
#pragma unroll
        for (int j = 0; j < NTL; ++j) {
            if (!XT) {
                const int c = (wave * Cfg::TN + j * 32) / 8 + c_lane;
                b_addr[b][j] = lds0 + b * Cfg::STAGE + Cfg::A_STAGE + krow_lane * Cfg::B_ROW + ((c ^ sw) * 16) + sub;
            } else {
                const int t = wave * Cfg::TN + j * 32 + (lane & 31), f = (t >> 2) & 3, kg = lane >> 5;
                const uint32_t tok = lds0 + b * Cfg::STAGE + Cfg::A_STAGE + (t >> 4) * 1024 + (t & 15) * 64;
                b_addr[b][j] = tok + ((kg ^ f) * 16);
                b_addr1[b][j] = tok + (((2 + kg) ^ f) * 16);
            }
        }
        // opaque to the optimiser: otherwise it folds the buffer offset back into per-use additions
        asm volatile("" : "+v"(a_addr[b]), "+v"(b_addr[b][0]), "+v"(b_addr[b][1]), "+v"(b_addr[b][2]), "+v"(b_addr[b][3]));
        if (XT) asm volatile("" : "+v"(b_addr1[b][0]), "+v"(b_addr1[b][1]), "+v"(b_addr1[b][2]), "+v"(b_addr1[b][3]));
    }
    // B source: a 1 KB region is one whole row of the slice; the i-th load of this wave fills row
    // i*NW + wave, whose swizzle (row & 3) is the wave number for every i: lane l fetches chunk
    // l ^ (wave << 2) so that it lands at position l.
    // XT: a 1 KB region is 16 tokens x 64 bytes; the i-th load of this wave fills tokens 64*i + 16*wave
    // + l/4, and lane l fetches chunk (l % 4) ^ ((l / 16) % 4) of its token so that it lands swizzled.
    const int b_chunk = lane ^ (wave << 2);
    const int xt_chunk = (lane & 3) ^ ((lane >> 4) & 3), xt_token = 16 * wave + (lane >> 2);
    const uint32_t a_voff0 = (uint32_t)(wave * 1024 + lane * 16), a_voff1 = a_voff0 + NW * 1024;
    const int64_t row_bytes = XT ? (int64_t)K * 2 : (int64_t)N * 2;  // row of the dense input operand
    const uint32_t m0_base = __builtin_amdgcn_readfirstlane((int)(lds0 + wave * 1024));

    // ---- tile parameters, in named scalars: arrays or structs indexed at run time would be placed in
    // LDS or scratch by the compiler, and everything read back from there counts as lane-varying -------
    int c_br = 0, c_n0 = 0, c_nb = 0;                                   // tile being multiplied (nb: blocks)
    int n_br = 0, n_n0 = 0, n_nb = 0, n_blk0 = 0, n_bcol0 = 0, have_next = 0;  // the tile after it
    uint32_t n_col = 0;  // byte offset of this lane's 16-byte chunk inside a row of B
    int4 n_srow = {0, 0, 0, 0};  // GATHER: dense rows of the four slices of the tile's first block
    auto uniform4 = [&](int4 v) __attribute__((always_inline)) {
        return int4{__builtin_amdgcn_readfirstlane(v.x), __builtin_amdgcn_readfirstlane(v.y),
                    __builtin_amdgcn_readfirstlane(v.z), __builtin_amdgcn_readfirstlane(v.w)};
    };
    auto decode = [&](int idx, int &br, int &n0, int &nb, int &blk0, int &bcol0, uint32_t &colb, int4 &srow) __attribute__((always_inline)) {
        const int per_group = group_n * n_rows;
        const int grp = idx / per_group, in_grp = idx - grp * per_group;
        const int left = n_tiles - grp * group_n;
        const int gw = left < group_n ? left : group_n;  // the last group may be narrower
        // heaviest block-row first in even groups, lightest first in odd ones: neighbours in the order,
        // which run at the same time, then have similar weights across group boundaries too
        const int pos = in_grp / gw, nt = grp * group_n + (in_grp - pos * gw);
        const int rank = (grp & 1) ? n_rows - 1 - pos : pos;
        const int4 ri = rank_info[rank];
        br = __builtin_amdgcn_readfirstlane(ri.x);
        blk0 = __builtin_amdgcn_readfirstlane(ri.y);
        nb = __builtin_amdgcn_readfirstlane(ri.z);
        bcol0 = __builtin_amdgcn_readfirstlane(ri.w);
        if (GATHER) srow = uniform4(((const int4 *)block_col_idx)[blk0]);
        n0 = nt * BN;
        int col = n0 + 8 * b_chunk;
        col = col < N ? col : N - 8;  // chunks past N only feed columns that are never stored
        colb = XT ? (uint32_t)n0 : (uint32_t)col * 2;
    };

    // ---- the request cursor: block pf_b (of pf_nb) of its tile, stored block pf_blk; the slice to
    // request next is given by the position in the unrolled loop.  The cursor's tile is the current one
    // or (pf_in_next) the next one, never further: it runs three slices ahead and a tile has >= 4. ------
    int pf_nb = 0, pf_b = 0, pf_blk = 0, pf_in_next = 0;
    int pf_bcol = 0;      // block column of block pf_blk
    int pf_bcol_ld = 0;   // block column of stored block pf_blk + 1 (loaded one block early)
    int4 pf_srow = {0, 0, 0, 0}, pf_srow_ld = {0, 0, 0, 0};  // GATHER: the same for the slices' dense rows
    const uint8_t *pf_bb1 = nullptr, *pf_bb2 = nullptr, *pf_bb3 = nullptr;  // GATHER: dense operand of slices 1..3
    uint32_t pf_voff[Cfg::B_LPW];     // per-lane byte offsets of the 8 rows this wave loads of a slice of B
    const uint8_t *pf_abase = nullptr; // next A slice to request
    const uint8_t *pf_bbase = nullptr; // first row of B of the next slice to request
    int pf_n0 = 0;                      // XT: first token of the cursor's tile
    auto cursor_set_tile = [&](uint32_t colb) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < Cfg::B_LPW; ++i) {
            if (!XT) {
                pf_voff[i] = colb + (uint32_t)(i * NW + wave) * (uint32_t)row_bytes;
            } else {
                // tokens past N only feed columns of the product that are never stored: read the last one
                int t = 64 * i + xt_token;
                const int last = N - 1 - (int)colb;
                t = t < last ? t : last;
                pf_voff[i] = (uint32_t)t * (uint32_t)row_bytes + xt_chunk * 16;
            }
        }
        if (XT) pf_n0 = __builtin_amdgcn_readfirstlane((int)colb);
    };
    auto cursor_set_block = [&]() __attribute__((always_inline)) {
        // (made scalar here, well before the requests read them: a memory instruction may read a scalar
        // register only five wait states after a vector instruction wrote it, the compiler keeps such
        // wave-uniform values in vector registers at times, and it does not see the loads inside the asm)
        pf_abase = (const uint8_t *)uniform_ptr((const uint8_t *)a_packed + (int64_t)pf_blk * (BR * BR * 2));
        int nb_ = pf_blk + 1;
        nb_ = nb_ < n_blocks ? nb_ : n_blocks - 1;
        if (GATHER) {
            const uint8_t *origin = XT ? (const uint8_t *)B + (int64_t)pf_n0 * row_bytes : (const uint8_t *)B;
            const int64_t unit = XT ? 2 : row_bytes;  // one dense row (XT: one k) further
            pf_bbase = (const uint8_t *)uniform_ptr(origin + (int64_t)pf_srow.x * unit);
            pf_bb1 = (const uint8_t *)uniform_ptr(origin + (int64_t)pf_srow.y * unit);
            pf_bb2 = (const uint8_t *)uniform_ptr(origin + (int64_t)pf_srow.z * unit);
            pf_bb3 = (const uint8_t *)uniform_ptr(origin + (int64_t)pf_srow.w * unit);
            pf_srow_ld = uniform4(((const int4 *)block_col_idx)[nb_]);
            return;
        }
        pf_bbase = (const uint8_t *)uniform_ptr(
            XT ? (const uint8_t *)B + (int64_t)pf_n0 * row_bytes + (int64_t)pf_bcol * BR * 2
               : (const uint8_t *)B + (int64_t)pf_bcol * BR * row_bytes);
        pf_bcol_ld = __builtin_amdgcn_readfirstlane(block_col_idx[nb_]);
    };
    // dense operand of slice s_ of the cursor's block, s_ a compile-time constant in 1..3
    auto gather_base = [&](int s_) __attribute__((always_inline)) { return s_ == 1 ? pf_bb1 : s_ == 2 ? pf_bb2 : pf_bb3; };
    // once per block, before its slice 0 is requested
    auto cursor_next_block = [&]() __attribute__((always_inline)) {
        ++pf_b;
        if (pf_b < pf_nb) {
            ++pf_blk;
            pf_bcol = pf_bcol_ld;
            pf_srow = pf_srow_ld;
        } else if (have_next && !pf_in_next) {
            pf_in_next = 1;
            pf_nb = n_nb;
            pf_b = 0;
            pf_blk = n_blk0;
            pf_bcol = n_bcol0;
            pf_srow = n_srow;
            cursor_set_tile(n_col);
        } else {
            pf_b = pf_nb - 1;  // end of the stream: the same block again
        }
        pf_blk = __builtin_amdgcn_readfirstlane(pf_blk);
        pf_bcol = __builtin_amdgcn_readfirstlane(pf_bcol);
        cursor_set_block();
    };

    // MFMA operand fragments of one 16-wide k step
    struct Frags {
        bf16x8 a[MT], b[NTL];
    };
    typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
    typedef __attribute__((address_space(3))) short4v lds_short4v;
    auto load_a = [&](int buf, int kk, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MT; ++i) f.a[i] = *(const lds_bf16x8 *)(uintptr_t)(a_addr[buf] + (kk * MT + i) * 1024);
    };
    auto load_b = [&](int buf, int kk, Frags &f, int j) __attribute__((always_inline)) {
        if (XT) {
            f.b[j] = *(const lds_bf16x8 *)(uintptr_t)(kk ? b_addr1[buf][j] : b_addr[buf][j]);
            return;
        }
        const uint32_t p0 = b_addr[buf][j] + kk * 16 * Cfg::B_ROW;
        short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v *)(uintptr_t)(p0));
        short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v *)(uintptr_t)(p0 + 4 * Cfg::B_ROW));
        short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        f.b[j] = __builtin_bit_cast(bf16x8, both);
    };
    // The 256 accumulators fill the accumulation register file completely.  The MFMAs are written as
    // inline assembly with the accumulator tied to those registers, and there is exactly one copy of the
    // multiply loop: left to itself, or given several variants of the loop body to merge, the register
    // allocator moves accumulators between the register files or spills all of them at every merge.
    // Operands are swapped: D[n][m] = sum_k B[k][n] * A[m][k], so a lane ends with 4 adjacent columns.
    // The compiler does not see MFMAs here, so the wait states between the last MFMA of a tile and the
    // first read of its result are provided by hand (mfma_drain).
    f32x16 acc[MT][NTL];
    // (XT: not swapped, D[m][n]: a lane ends with 4 adjacent outputs of one token)
#define ASP_OP1(f, q) (XT ? f.a[(q) / NTL] : f.b[(q) % NTL])
#define ASP_OP2(f, q) (XT ? f.b[(q) % NTL] : f.a[(q) / NTL])
#define ASP_MFMA(f, q) \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[(q) / NTL][(q) % NTL]) : "v"(ASP_OP1(f, q)), "v"(ASP_OP2(f, q)))
    // the same with a direct-to-LDS load behind it: M0 = LDS destination of the wave's 1 KB region, then
    // the MFMA (the wait state the load needs after the write of M0), then the load of 16 bytes per lane
    // from sbase + voff
#define ASP_MFMA_DMA(f, q, region_off, voff, sbase)                                                              \
    asm volatile("s_add_u32 m0, %3, %4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\tglobal_load_lds_dwordx4 %5, %6" \
                 : "+a"(acc[(q) / NTL][(q) % NTL])                                                               \
                 : "v"(ASP_OP1(f, q)), "v"(ASP_OP2(f, q)), "s"(m0_base), "i"(region_off), "v"(voff),          \
                   "s"(uniform_ptr(sbase))                                                                       \
                 : "memory", "scc")
    // acc[i][j] = 0 x 0 + 0: clears a finished tile's accumulators on the matrix core, which is idle
    // during the epilogue anyway (256 register writes would cost more than a K slice)
    // (the compiler may set up the zero operand right in front of the first clear and knows nothing of
    // the wait states an MFMA needs after a vector-ALU write of its operands: they are part of the asm)
    const bf16x8 zero_frag = __builtin_bit_cast(bf16x8, short8v{0, 0, 0, 0, 0, 0, 0, 0});
    auto mfma_clear = [&](int i, int j) __attribute__((always_inline)) {
        asm volatile("s_nop 3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "+a"(acc[i][j]) : "v"(zero_frag));
    };
    auto mfma_drain = [&]() __attribute__((always_inline)) { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); };
#define ASP_FENCE() __builtin_amdgcn_sched_barrier(0)

    // B row i*NW + wave of the slice at pf_bbase (XT: the slice's 64 bytes of 16 tokens per load)
#define ASP_B_VOFF(s, i) pf_voff[i]
#define ASP_B_BASE(s) pf_bbase
    const int64_t slice_step = XT ? (int64_t)KS * 2 : (int64_t)KS * row_bytes;  // next slice of the dense operand

    // ---- one step: slice S of a block, in ring buffer S.  The instruction order is fixed by hand
    // (nothing moves across a fence).  HI: the previous tile's stores may still be outstanding. ---------
    Frags f0, f1;
    int vm_hi = 0;  // steps for which a tile's stores are still younger than the slice waited for
    // One phase: 16 MFMAs on fragments F (q = 4*i + j uses a[i], b[j]) while the fragments G of the next
    // phase are read from ring buffer GB, k half GK -- in the order in which they will be needed, one
    // or two reads per MFMA, so that the four waves' LDS traffic is spread over the phase instead of
    // arriving as one 32 KB burst that blocks the waves' issue -- and five loads of the request go out.
#define ASP_LOAD_A1(GB, GK, G, i) G.a[i] = *(const lds_bf16x8 *)(uintptr_t)(a_addr[GB] + ((GK) * MT + (i)) * 1024)
#define ASP_LOAD_B1(GB, GK, G, j) load_b(GB, GK, G, j)
#define ASP_PHASE(F, G, GB, GK, R0, R1, R2, R3, R4, EXTRA)                                       \
    do {                                                                                         \
        ASP_MFMA(F, 0);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_B1(GB, GK, G, 0);                                                                    \
        ASP_LOAD_A1(GB, GK, G, 0);                                                               \
        ASP_FENCE();                                                                             \
        ASP_MFMA(F, 1);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_B1(GB, GK, G, 1);                                                                    \
        ASP_FENCE();                                                                             \
        ASP_MFMA(F, 2);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_B1(GB, GK, G, 2);                                                                    \
        ASP_FENCE();                                                                             \
        ASP_MFMA(F, 3);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_B1(GB, GK, G, 3);                                                                    \
        EXTRA;                                                                                   \
        ASP_FENCE();                                                                             \
        ASP_MFMA(F, 4);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_A1(GB, GK, G, 1);                                                               \
        ASP_FENCE();                                                                             \
        R0(F, 5);                                                                                \
        ASP_MFMA(F, 6);                                                                          \
        R1(F, 7);                                                                                \
        ASP_MFMA(F, 8);                                                                          \
        ASP_FENCE();                                                                             \
        ASP_LOAD_A1(GB, GK, G, 2);                                                               \
        ASP_FENCE();                                                                             \
        R2(F, 9);                                                                                \
        ASP_MFMA(F, 10);                                                                         \
        R3(F, 11);                                                                               \
        ASP_MFMA(F, 12);                                                                         \
        ASP_FENCE();                                                                             \
        ASP_LOAD_A1(GB, GK, G, 3);                                                               \
        ASP_FENCE();                                                                             \
        R4(F, 13);                                                                               \
        ASP_MFMA(F, 14);                                                                         \
        ASP_MFMA(F, 15);                                                                         \
        ASP_FENCE();                                                                             \
    } while (0)
#define ASP_RQ_A0(F, q) ASP_MFMA_DMA(F, q, tb_ * Cfg::STAGE, a_voff0, pf_abase)
#define ASP_RQ_A1(F, q) ASP_MFMA_DMA(F, q, tb_ * Cfg::STAGE + NW * 1024, a_voff1, pf_abase)
#define ASP_RQ_B(F, q, i) \
    ASP_MFMA_DMA(F, q, tb_ * Cfg::STAGE + Cfg::A_STAGE + (i) * NW * 1024, ASP_B_VOFF(rs_, i), ASP_B_BASE(rs_))
#define ASP_RQ_B0(F, q) ASP_RQ_B(F, q, 0)
#define ASP_RQ_B1(F, q) ASP_RQ_B(F, q, 1)
#define ASP_RQ_B2(F, q) ASP_RQ_B(F, q, 2)
#define ASP_RQ_B3(F, q) ASP_RQ_B(F, q, 3)
#define ASP_RQ_B4(F, q) ASP_RQ_B(F, q, 4)
#define ASP_RQ_B5(F, q) ASP_RQ_B(F, q, 5)
#define ASP_RQ_B6(F, q) ASP_RQ_B(F, q, 6)
#define ASP_RQ_B7(F, q) ASP_RQ_B(F, q, 7)
#define ASP_WIDE_STEP(S, HI_POSSIBLE)                                                                              \
    do {                                                                                                           \
        constexpr int nb_ = ((S) + 1) % NS, tb_ = ((S) + 3) % NS; /* tb_: free since the previous barrier */      \
        constexpr int rs_ = ((S) + 3) % NS;                        /* slice of its block that is requested */      \
        /* ---- phase A: first k half | fragments of the second half, first half of the request ---- */           \
        /* (once per block, before its slice 0 is requested, the cursor moves on to the next block) */            \
        ASP_PHASE(f0, f1, S, 1, ASP_RQ_A0, ASP_RQ_A1, ASP_RQ_B0, ASP_RQ_B1, ASP_RQ_B2,                             \
                  if (rs_ == 0) cursor_next_block());                                                              \
        /* ---- phase B: second k half | fragments of the next slice's first half, rest of the request ---- */    \
        /* this wave's part of the next slice has landed (all but the newest one and a half requests and, */     \
        /* for two steps after an interior tile, its stores may be outstanding); f1 is complete           */     \
        if (HI_POSSIBLE && vm_hi > 0) wait_vmcnt_and_lds<Cfg::NSTORE + Cfg::LPW + Cfg::LPW / 2>();                               \
        else wait_vmcnt_and_lds<Cfg::LPW + Cfg::LPW / 2>();                                                                      \
        barrier_no_fence(); /* everybody's part has landed, nobody reads buffer S any more */                      \
        ASP_FENCE();                                                                                               \
        ASP_PHASE(f1, f0, nb_, 0, ASP_RQ_B3, ASP_RQ_B4, ASP_RQ_B5, ASP_RQ_B6, ASP_RQ_B7, (void)0);                 \
        pf_abase = (const uint8_t *)uniform_ptr(pf_abase + Cfg::A_STAGE);                                          \
        if (GATHER) { if (rs_ < NS - 1) pf_bbase = gather_base(rs_ + 1); }                                         \
        else pf_bbase = (const uint8_t *)uniform_ptr(pf_bbase + slice_step);                                       \
        if (HI_POSSIBLE) vm_hi = vm_hi > 0 ? vm_hi - 1 : 0;                                                        \
        ASP_FENCE();                                                                                               \
    } while (0)

    // ---- start of the stream: three slices requested, first-half fragments of slice 0 in registers ---
    {
        int blk0, bcol0;
        uint32_t colb;
        decode(idx_cur, c_br, c_n0, c_nb, blk0, bcol0, colb, pf_srow);
        pf_nb = c_nb;
        pf_blk = blk0;
        pf_bcol = bcol0;
        cursor_set_tile(colb);
        cursor_set_block();
        if (tile_of_round(1) < run_end) {
            have_next = 1;
            decode(tile_of_round(1), n_br, n_n0, n_nb, n_blk0, n_bcol0, n_col, n_srow);
        }
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j) {
            const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[i][j] = z;
        }
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
        dma16_to_lds(pf_abase, a_voff0, m0_base + s * Cfg::STAGE);
        dma16_to_lds(pf_abase, a_voff1, m0_base + s * Cfg::STAGE + NW * 1024);
#pragma unroll
        for (int i = 0; i < Cfg::B_LPW; ++i)
            dma16_to_lds(ASP_B_BASE(s), ASP_B_VOFF(s, i), m0_base + s * Cfg::STAGE + Cfg::A_STAGE + i * NW * 1024);
        pf_abase += Cfg::A_STAGE;
        if (GATHER) pf_bbase = gather_base(s + 1);
        else pf_bbase += slice_step;
    }
    wait_vmcnt_and_lds<2 * Cfg::LPW>();
    barrier_no_fence();
    load_a(0, 0, f0);
#pragma unroll
    for (int j = 0; j < NTL; ++j) load_b(0, 0, f0, j);

    for (;;) {
        // (in the first two steps of a tile the stores of the previous tile are younger than the slice
        // waited for; one copy of the loop only, see above)
        for (int blk = 0; blk < c_nb; ++blk) {
            ASP_WIDE_STEP(0, true);
            ASP_WIDE_STEP(1, true);
            ASP_WIDE_STEP(2, false);
            ASP_WIDE_STEP(3, false);
        }

        // ---- tile boundary ------------------------------------------------------------------------
        mfma_drain();
        // parameters of the tile after the next one: requested now, needed after the epilogue
        const int idx_nn = tile_of_round(round + 2);
        int nn_br = 0, nn_n0 = 0, nn_nb = 0, nn_blk0 = 0, nn_bcol0 = 0;
        uint32_t nn_col = 0;
        int4 nn_srow = {0, 0, 0, 0};
        if (idx_nn < run_end) decode(idx_nn, nn_br, nn_n0, nn_nb, nn_blk0, nn_bcol0, nn_col, nn_srow);

        // the buffer of the slice just finished (always the last one of the ring) is the spare one
        // until the next barrier
        // GATHER: where the tile's four 32-row pieces go (issued here, with the loads of decode)
        const int4 prow = GATHER ? piece_rows[c_br] : int4{0, 0, 0, 0};
        const int pmin = prow.x < prow.y ? (prow.x < prow.z ? (prow.x < prow.w ? prow.x : prow.w) : (prow.z < prow.w ? prow.z : prow.w))
                                         : (prow.y < prow.z ? (prow.y < prow.w ? prow.y : prow.w) : (prow.z < prow.w ? prow.z : prow.w));
        const int pmax = prow.x > prow.y ? (prow.x > prow.z ? (prow.x > prow.w ? prow.x : prow.w) : (prow.z > prow.w ? prow.z : prow.w))
                                         : (prow.y > prow.z ? (prow.y > prow.w ? prow.y : prow.w) : (prow.z > prow.w ? prow.z : prow.w));
        const bool rows_interior = GATHER ? __builtin_amdgcn_readfirstlane(pmin >= 0 && pmax + 32 <= M) : c_br * BR + BR <= M;
        const bool interior = rows_interior && c_n0 + BN <= N;
        uint8_t *sc = lds + (NS - 1) * Cfg::STAGE + wave * Cfg::C_WAVE;
        // a piece = 32 rows x 128 columns of the output matrix: rows of C and the wave's 128 columns, or
        // (XT) 32 of the wave's tokens = rows of Y and the block-row's 128 outputs
        const int out_ld = XT ? M : N, out_rows = XT ? N : M, out_cols = XT ? M : N;
        // GATHER: the tile's 128 rows of the product (rows of C, or XT: columns of Y) are four separately placed
        // pieces of 32; a 16-byte unit never straddles two of them
        const int xt_piece = (lane % Cfg::CPR) >> 2;  // XT: the piece this lane's 8 outputs belong to
        const int xt_pbase = xt_piece == 0 ? prow.x : xt_piece == 1 ? prow.y : xt_piece == 2 ? prow.z : prow.w;
        const int grow0 = (XT ? c_n0 + wave * Cfg::TN : GATHER ? 0 : c_br * BR) + lane / Cfg::CPR;
        const int gcol0 = XT ? (GATHER ? xt_pbase + ((lane % Cfg::CPR) & 3) * 8 : c_br * BR + (lane % Cfg::CPR) * 8)
                             : c_n0 + wave * Cfg::TN + (lane % Cfg::CPR) * 8;
        const bool xt_piece_ok = !(XT && GATHER) || xt_pbase >= 0;
        const uint8_t *scl = sc + (lane / Cfg::CPR) * Cfg::C_PITCH + (lane % Cfg::CPR) * 16;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            // fp32 -> bf16 (round to nearest even); lane holds row (lane & 31) of the piece, 4 adjacent columns per q
#pragma unroll
            for (int in = 0; in < 4; ++in) {
                f32x16 a = XT ? acc[in][o] : acc[o][in];
                asm volatile("" : "+v"(a));  // the copy sits in vector registers before the clear overwrites
                if (XT) mfma_clear(in, o);
                else mfma_clear(o, in);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                    bf16x4 hv = __builtin_convertvector(v, bf16x4);
                    *(bf16x4 *)(sc + (lane & 31) * Cfg::C_PITCH + (in * 32 + 8 * q + 4 * (lane >> 5)) * 2) = hv;
                }
            }
            // LDS is in order within a wave: the reads below see the writes above
            // first row of this piece: XT pieces are 32 tokens; otherwise rows of C
            const int prow_o = o == 0 ? prow.x : o == 1 ? prow.y : o == 2 ? prow.z : prow.w;
            const int rbase = (!XT && GATHER) ? prow_o : o * 32;
            const bool piece_ok = (!XT && GATHER) ? prow_o >= 0 : xt_piece_ok;
            uint16_t *cdst = C + (int64_t)(grow0 + rbase) * out_ld + gcol0;
            if (interior) {
#pragma unroll
                for (int it = 0; it < 32 / Cfg::RPI; ++it) {
                    uint4 v = *(const uint4 *)(scl + it * Cfg::RPI * Cfg::C_PITCH);
                    store_c16(cdst + (int64_t)it * Cfg::RPI * out_ld, v);
                }
            } else {
#pragma unroll
                for (int it = 0; it < 32 / Cfg::RPI; ++it) {
                    uint4 v = *(const uint4 *)(scl + it * Cfg::RPI * Cfg::C_PITCH);
                    if (piece_ok && grow0 + rbase + it * Cfg::RPI < out_rows && gcol0 < out_cols)
                        store_c16(cdst + (int64_t)it * Cfg::RPI * out_ld, v);
                }
            }
            ASP_FENCE();  // keeps the pieces apart: reading all 256 accumulators at once would spill
        }
        if (interior) {
            vm_hi = 2;  // exactly NSTORE stores were issued, none is waited for
        } else {
            // an edge tile issues a data-dependent number of stores: drain once so the counts are exact again
            wait_vmcnt_and_lds<0>();
            vm_hi = 0;
        }

        // ---- advance to the next tile ---------------------------------------------------------------
        if (!have_next) break;
        // the next step requests into the staging buffer before its own barrier: every wave must be done
        // reading its staging area first
        wait_vmcnt_and_lds<63>();
        barrier_no_fence();
        ++round;
        idx_cur = tile_of_round(round);
        c_br = n_br;
        c_n0 = n_n0;
        c_nb = n_nb;
        pf_in_next = 0;  // the cursor entered this tile three slices ago
        if (idx_nn < run_end) {
            n_br = nn_br;
            n_n0 = nn_n0;
            n_nb = nn_nb;
            n_blk0 = nn_blk0;
            n_bcol0 = nn_bcol0;
            n_col = nn_col;
            n_srow = nn_srow;
            have_next = 1;
        } else {
            have_next = 0;
        }
    }
    // the cursor's repeated requests at the end of the stream still write LDS: they must have landed
    // before the workgroup gives its LDS back
    wait_vmcnt_and_lds<0>();
    clear_empty_rows();
#undef ASP_FENCE
#undef ASP_WIDE_STEP
#undef ASP_MFMA
#undef ASP_MFMA_DMA
#undef ASP_OP1
#undef ASP_OP2
#undef ASP_B_VOFF
#undef ASP_B_BASE
}

// rows of C that belong to block-rows without stored blocks (ranks n_rows .. n_brows-1), for handles
// that have no stored block at all
__global__ __launch_bounds__(256) void bcsr_clear_empty_rows_kernel(const int4 *__restrict__ rank_info, int n_rows,
                                                                    uint16_t *__restrict__ C, int M, int N, int BR) {
    const int br = rank_info[n_rows + blockIdx.x].x;
    const int r0 = br * BR, r1 = r0 + BR < M ? r0 + BR : M;
    uint4 *dst = (uint4 *)(C + (int64_t)r0 * N);           // whole rows: one contiguous span, N % 8 == 0
    const int64_t n16 = (int64_t)(r1 - r0) * N / 8;
    const uint4 z = {0u, 0u, 0u, 0u};
    for (int64_t i = (int64_t)blockIdx.y * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.y * 256) dst[i] = z;
}

// What the kernel walks: the handle's own 128x128 blocks, or the composite form of a handle with smaller blocks.
struct WideOperand {
    const int4 *rank_info;
    const int32_t *cols;  // block columns, or (composite) four dense rows per block
    const uint16_t *values;
    const std::vector<int64_t> *weight_prefix;
    int64_t n_rows, n_brows, n_blocks;  // non-empty block-rows, all block-rows, blocks
    bool composite;
    const int4 *piece_rows;  // composite: first row of C of each 32-row piece of a super-row
};
static WideOperand wide_operand(const asp_handle *h) {
    if (!h->has_comp)
        return WideOperand{(const int4 *)h->d_rank_info, h->d_col_idx,          (const uint16_t *)h->d_values,
                           &h->hb.sorted_weight_prefix,  h->hb.n_nonempty,      h->n_brows,
                           h->n_units,                   false,                 nullptr};
    return WideOperand{(const int4 *)h->d_c_rank_info, h->d_c_slice_rows,     (const uint16_t *)h->d_c_values,
                       &h->hc.sorted_weight_prefix,    h->hc.n_nonempty,      h->c_n_brows,
                       h->c_n_units,                   true,                  (const int4 *)h->d_c_piece_rows};
}

template <bool XT>
static void launch_wide(const asp_handle *h, const void *B, void *C, int64_t N, int n_tiles, hipStream_t stream) {
    const int env_group = switches().bcsr_group_n;  // benchmarking switch
    // two N-tiles walked together: an A block is fetched once per pair while the pair's slab of B (K x 1024)
    // still has a chance in the 4 MB of L2 (measured: 1, 3 and 4 are 3-10 % slower on the 90 %-sparse projection)
    int group_n = env_group > 0 ? env_group : 2;
    if (group_n > n_tiles) group_n = n_tiles;
    const WideOperand op = wide_operand(h);
    const int64_t n_rows = op.n_rows;
    int64_t workers = h->n_cus;  // one resident workgroup per CU: the ring takes the whole LDS
    if (workers > n_rows * n_tiles) workers = n_rows * n_tiles;
    // benchmarking switch: fewer resident workgroups, i.e. part of the compute units idle (the schedule's 16 lists
    // per XCD stay balanced for 32, 16 or 8 workgroups per XCD)
    const int env_workers = switches().bcsr_workgroups;
    if (env_workers > 0 && env_workers < workers) workers = env_workers;
    workers = std::max<int64_t>(8, workers / 8 * 8);  // the same number of workgroups on every XCD
    const int env_xcd = switches().bcsr_xcd_aware ? 1 : 0;  // benchmarking switch: 0 = ignore the XCDs when dealing tiles
    XcdRuns runs = cut_runs(*op.weight_prefix, n_rows, n_tiles, group_n);
    if (!env_xcd)
        for (int x = 1; x <= 8; ++x) runs.start[x] = runs.start[8];
    dim3 grid((unsigned)workers), block(256);
#define ASP_LAUNCH_WIDE(GATHER)                                                                                        \
    hipLaunchKernelGGL((bcsr_spmm_wide_kernel<XT, GATHER>), grid, block, 0, stream, op.rank_info, op.cols, op.values,  \
                       (const uint16_t *)B, (uint16_t *)C, (int)h->m, (int)h->k, (int)N, (int)n_rows, (int)op.n_brows,  \
                       (int)op.n_blocks, n_tiles, group_n, env_xcd, runs, op.piece_rows)
    if (op.composite) ASP_LAUNCH_WIDE(true);
    else ASP_LAUNCH_WIDE(false);  // K % 128 == 0 (bcsr_wide_capable)
#undef ASP_LAUNCH_WIDE
}

// needs 128x128 blocks or the composite form, bn = 512, N % 8 == 0, 8 <= N < 2^25 and 16-byte aligned B and C
// (the caller checked)
bool bcsr_wide_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    if (!bcsr_wide_capable(h) || p.bn != 512) return false;
    const WideOperand op = wide_operand(h);
    const int64_t n_rows = op.n_rows, n_empty = op.n_brows - n_rows;
    if (n_empty > 0 && n_rows == 0) {  // nothing to multiply: the clearing is all there is
        dim3 grid((unsigned)n_empty, 16), block(256);
        hipLaunchKernelGGL(bcsr_clear_empty_rows_kernel, grid, block, 0, stream, op.rank_info, (int)n_rows,
                           (uint16_t *)C, (int)h->m, (int)N, 128);
    }
    if (n_rows == 0) return true;
    launch_wide<false>(h, B, C, N, p.n_tiles, stream);
    return true;
}

// ---- Y = X x A^T with K-contiguous X and Y (Section IV-D's layout) -------------------------------------

// Any block size, any alignment, any N: one thread per (token, quarter of the block-row's outputs), fp32
// multiply-adds over the stored blocks in order.  The safety net under the MFMA path below; two orders of
// magnitude slower.  grid = (block-rows, ceil(N / 64)), 256 threads.
template <int BR>
__global__ __launch_bounds__(256) void bcsr_xt_generic_kernel(const int32_t *__restrict__ block_row_ptr,
                                                              const int32_t *__restrict__ block_col_idx,
                                                              const uint16_t *__restrict__ a_packed,
                                                              const uint16_t *__restrict__ X, uint16_t *__restrict__ Y,
                                                              int M, int K, int64_t N) {
    constexpr int RPT = BR / 4;  // outputs per thread
    const int br = blockIdx.x, rg = threadIdx.x >> 6;
    const int64_t n = (int64_t)blockIdx.y * 64 + (threadIdx.x & 63);
    if (n >= N) return;
    float acc[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) acc[r] = 0.f;
    const uint16_t *x = X + n * K;
    for (int p = block_row_ptr[br]; p < block_row_ptr[br + 1]; ++p) {
        const int k0 = block_col_idx[p] * BR;
        const uint16_t *blk = a_packed + (int64_t)p * BR * BR;
        for (int k = 0; k < BR && k0 + k < K; ++k) {
            const float xv = __uint_as_float((uint32_t)x[k0 + k] << 16);
#pragma unroll
            for (int r = 0; r < RPT; ++r) {
                const int row = rg * RPT + r;
                // fragment order: [16-wide k slice][group of 32 rows][lane = row % 32 + 32 * (k % 16 / 8)][k % 8]
                const int idx = (((k >> 4) * (BR / 32) + (row >> 5)) * 64 + (row & 31) + 32 * ((k & 15) >> 3)) * 8 + (k & 7);
                acc[r] = fmaf(__uint_as_float((uint32_t)blk[idx] << 16), xv, acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int m = br * BR + rg * RPT + r;
        if (m < M) {
            // round to nearest even (inputs are finite sums; NaN payloads are not preserved)
            uint32_t u = __float_as_uint(acc[r]);
            u += 0x7FFFu + ((u >> 16) & 1u);
            Y[n * M + m] = (uint16_t)(u >> 16);
        }
    }
}

__global__ __launch_bounds__(256) void bcsr_fill_zero_kernel(uint16_t *__restrict__ p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0;
}

asp_status_t bcsr_spmm_xt_launch(const asp_handle *h, const void *X, void *Y, int64_t N, hipStream_t stream) {
    const bool wide_ok = bcsr_wide_capable(h);
    const int64_t n_rows = !h->has_comp ? h->hb.n_nonempty : h->hc.n_nonempty;
    if (n_rows == 0) {
        hipLaunchKernelGGL(bcsr_fill_zero_kernel, dim3(1024), dim3(256), 0, stream, (uint16_t *)Y, N * h->m);
    } else {
        const bool aligned = (((uintptr_t)X | (uintptr_t)Y) & 15) == 0;
        const int64_t n_tiles = ceil_div(N, 512);
        const bool force_generic = switches().xt_generic;  // benchmarking switch: forces the fallback
        // (no lower bound on the number of tiles: with fewer 128 x 512 tiles than compute units part of the chip
        // idles, which still is two orders of magnitude faster than the generic kernel -- the down projection of
        // the case study has 28 block-rows and would need 4600 tokens to give every compute unit a tile)
        if (!force_generic && wide_ok && aligned && h->k % 8 == 0 && h->m % 8 == 0 && N < (1ll << 25) &&
            h->k < (1ll << 22)) {
            launch_wide<true>(h, X, Y, N, (int)n_tiles, stream);
        } else {
            dim3 grid((unsigned)h->n_brows, (unsigned)ceil_div(N, 64)), block(256);
            if (grid.y > 65535) return fail(ASP_ERR_UNSUPPORTED, "N too large for the generic K-contiguous path");
#define ASP_XT_GENERIC(BR)                                                                                          \
    hipLaunchKernelGGL(bcsr_xt_generic_kernel<BR>, grid, block, 0, stream, h->d_row_ptr, h->d_col_idx,              \
                       (const uint16_t *)h->d_values, (const uint16_t *)X, (uint16_t *)Y, (int)h->m, (int)h->k, N)
            if (h->b_row == 128) ASP_XT_GENERIC(128);
            else if (h->b_row == 64) ASP_XT_GENERIC(64);
            else ASP_XT_GENERIC(32);
#undef ASP_XT_GENERIC
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ASP_ERR_HIP, std::string("BCSR K-contiguous kernel launch: ") + hipGetErrorString(e));
    return ASP_OK;
}

}  // namespace asp
