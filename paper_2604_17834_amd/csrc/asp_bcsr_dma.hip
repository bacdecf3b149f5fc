// BCSR x dense SpMM, main gfx950 kernel: resident workgroups that stream K slices through an LDS ring
// filled by direct-to-LDS loads, without ever waiting for their own stores.
//
// Decomposition: an output tile is one (block-row, N-tile) pair of b_row x BN; its K loop walks the
// stored blocks of the block-row (paper, Section II-C) in slices of 32 k; each slice is multiplied with
// v_mfma_f32_32x32x16_bf16 (fp32 accumulation), operands swapped so that a lane ends with 4 adjacent
// output columns; the finished tile is rounded to bf16, transposed through LDS and stored as full
// 128-byte row segments.
//
// Asynchronous copy (the role TMA plays in the paper's Section III-B): global->LDS traffic never
// touches VGPRs.  Each wave issues global_load_lds_dwordx4 instructions, each dropping 64 lanes x 16
// bytes into one contiguous 1 KB LDS region while the lanes' global source addresses are free.
// Because the LDS side of such a load is lane-linear, the B slice cannot be padded per row; instead the
// source chunk of every lane is permuted so that row r's 64-byte units land XOR-swizzled by (r & 3):
// the four rows touched by one transposing read (ds_read_b64_tr_b16) then fall into disjoint banks.
// Rows of B past K (zero padding of A's last block column) and 16-byte chunks past N are redirected to
// the last valid row / chunk: they meet zeros of A or feed columns that are never stored.
//
// One continuous pipeline per workgroup.  A workgroup owns a fixed sequence of tiles and treats their
// slices as one stream: the ring (NS buffers) is refilled one slice per step, and the prefetch cursor
// runs on into the next tile while the current one is finished, so a tile's first loads overlap the
// previous tile's last multiplications, its epilogue and its stores.  Per step there is one fence-free
// barrier and one exact s_waitcnt: the wave counts every vector-memory operation it issues (loads of
// each slice, stores of each epilogue) and waits only until the operations issued after the slice it
// needs are the only ones outstanding.  Nothing ever waits for stores to C; with tiles of 1-10 blocks
// the store drain time of a tile is comparable to its multiply time, so waiting for it (a fenced
// barrier, or the end of a one-tile workgroup) left the matrix cores idle most of the time.
// The epilogue stages 32 x 64 pieces of the wave's tile in the one ring buffer that is free at a tile
// boundary, wave-privately, so it needs a single extra barrier per tile.
//
// Scheduling (Sections III-E/III-F of the paper discuss persistent kernels and dynamic tile scheduling
// on Hopper and reject them there for imbalance and atomic traffic).  Here the assignment is static and
// balanced by construction: block-rows are sorted by length once per handle; the tile order walks
// group_n adjacent N-tiles together, heaviest block-rows first; the order is cut into 8 runs of equal
// weight, one per XCD (workgroup id mod 8 -- workgroups are dealt to XCDs round-robin), so the B column
// slabs of a group stay in that XCD's private L2 and A blocks are fetched once per group; inside a run
// the XCD's workgroups take tiles round-robin, which deals sorted weights evenly.
#include <cstdlib>
#include <cstring>

#include "asp_bcsr_pipe.h"

namespace asp {

template <int BR, int BN, int WM, int WN, int NS>
struct DmaCfg {
    static constexpr int KS = 32;
    static constexpr int NW = WM * WN;
    static constexpr int NT = NW * 64;
    static constexpr int TM = BR / WM, TN = BN / WN;
    static constexpr int MT = TM / 32, NTL = TN / 32;
    static constexpr int KK = KS / 16;
    static constexpr int SPB = BR / KS;             // slices per block (square blocks)
    static constexpr int A_STAGE = BR * KS * 2;     // bytes
    static constexpr int B_ROW = BN * 2;            // bytes per LDS row of B
    static constexpr int B_STAGE = KS * B_ROW;
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int A_R = A_STAGE / 1024, B_R = B_STAGE / 1024;  // 1 KB regions = wave-level loads
    static constexpr int A_LPW = A_R / NW, B_LPW = B_R / NW, LPW = A_LPW + B_LPW;
    static constexpr int CPRW = BN / 8;             // 16-byte chunks per B row
    // epilogue: a wave stages pieces of 32 rows x RW columns, privately, inside one ring buffer
    static constexpr int RW = (TN >= 64 && NW * 32 * (64 * 2 + 16) <= STAGE) ? 64 : 32;
    static constexpr int JR = RW / 32;              // MFMA tiles per piece
    static constexpr int C_PITCH = RW * 2 + 16;     // bytes
    static constexpr int C_WAVE = 32 * C_PITCH;
    static constexpr int CPR = RW / 8;              // 16-byte units per staged row
    static constexpr int RPI = 64 / CPR;            // rows per wave-level store
    static constexpr int NSTORE = MT * (TN / RW) * (32 / RPI);  // store instructions per wave and tile
    static constexpr int LDS_BYTES = NS * STAGE;
    static_assert(A_R % NW == 0 && B_R % NW == 0, "regions must split evenly over the waves");
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert(NW * C_WAVE <= STAGE, "epilogue staging must fit into one ring buffer");
    static_assert(NS == 3, "the wait table below is written for a ring of three");
    static_assert(NSTORE + 2 * LPW < 64, "vmcnt is a 6-bit counter");
    // swizzle of a row's 64-byte units: rows k..k+3 of a transposing read must not share banks
    __device__ static __forceinline__ int swz(int r) { return BN >= 128 ? (r & 3) : ((r >> 1) & 1); }
};

// rank_info[r] = {block-row, first stored block, number of stored blocks, block column of the first one} of the r-th heaviest block-row
//
// DYN = true (a benchmarking variant, ASP_BCSR_SCHEDULE=atomic: the dynamic tile scheduling that the paper's Sections
// III-E/III-F try on Hopper and reject): the resident workgroups of an XCD pull the tiles of its run from an atomic counter
// (sched[xcd], zeroed before the launch) instead of taking every stride-th one.  Thread 0 claims, the index travels
// through LDS under the barrier the tile boundary has anyway; the claim for the tile after the next one is made at each
// boundary, so its round trip is paid once per tile by wave 0.  Every workgroup leaves when its claim passes the end of
// the run.  Calls under this switch share the handle's counters and must be ordered on one stream.
template <int BR, int BN, int WM, int WN, int NS, bool DYN = false>
__global__ __launch_bounds__(WM *WN * 64, (BR / WM) * (BN / WN) > 8192 ? 1 : 2) void bcsr_spmm_dma_kernel(
    const int4 *__restrict__ rank_info, const int32_t *__restrict__ block_col_idx,
    const uint16_t *__restrict__ a_packed, const uint16_t *__restrict__ B, uint16_t *__restrict__ C, int M, int K,
    int N, int n_brows, int n_tiles, int group_n, XcdRuns runs, int *__restrict__ sched) {
    using Cfg = DmaCfg<BR, BN, WM, WN, NS>;
    constexpr int NW = Cfg::NW, KS = Cfg::KS, MT = Cfg::MT, NTL = Cfg::NTL, LPW = Cfg::LPW;
    __shared__ __attribute__((aligned(1024))) uint8_t lds[Cfg::LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- this workgroup's tiles: every stride-th tile of its XCD's run ------------------------------
    // (the order of block-rows was built so that this deals every workgroup one weight-balanced list per
    // group of N-tiles)
    const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3, wg = blockIdx.x >> 3;
    const int run_begin = __builtin_amdgcn_readfirstlane(runs.start[xcd]);
    const int run_end = __builtin_amdgcn_readfirstlane(runs.start[xcd + 1]);
    auto tile_of_round = [&](int r) { return run_begin + r * stride + wg; };
    int round = 0;
    int *s_claim = nullptr;  // two LDS words, only in the dynamic variant
    if constexpr (DYN) {
        __shared__ int claim_words[2];
        s_claim = claim_words;
    }
    int idx_cur = tile_of_round(0), idx_n1 = tile_of_round(1);
    if constexpr (DYN) {
        if (tid == 0) {
            s_claim[0] = run_begin + atomicAdd(&sched[xcd], 1);
            s_claim[1] = run_begin + atomicAdd(&sched[xcd], 1);
        }
        __syncthreads();
        idx_cur = __builtin_amdgcn_readfirstlane(s_claim[0]);
        idx_n1 = __builtin_amdgcn_readfirstlane(s_claim[1]);
        __syncthreads();  // s_claim[0] is written again at the first tile boundary
    }
    if (idx_cur >= run_end) return;

    // ---- lane-invariant parts of the LDS read addresses ------------------------------------------
    const int a_off = lane * 16;
    // transposing read: lane i of a 16-lane group addresses row (i/4), 4 columns at 4*(i%4)
    const int krow_lane = 8 * (lane >> 5) + ((lane & 15) >> 2);          // + 16*kk (+4 for the upper half)
    const int sw = Cfg::swz(krow_lane) << 2;                              // same for krow_lane + 4 and + 16
    const int c_lane = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);         // chunk inside the 32-column tile
    const int sub = 8 * (lane & 1);                                       // byte inside the chunk
    int b_off[NTL];
#pragma unroll
    for (int j = 0; j < NTL; ++j) {
        const int c = (wn * Cfg::TN + j * 32) / 8 + c_lane;
        b_off[j] = krow_lane * Cfg::B_ROW + ((c ^ sw) * 16) + sub;
    }
    // B source: region jb = i*NW + wave of a slice holds the 16-byte slots [jb*64, jb*64+64); slot s is
    // row s / CPRW, position s % CPRW; the position is the swizzled chunk index.
    int b_row_in_slice[Cfg::B_LPW], b_chunk[Cfg::B_LPW];
#pragma unroll
    for (int i = 0; i < Cfg::B_LPW; ++i) {
        const int s = (i * NW + wave) * 64 + lane;
        const int r = s / Cfg::CPRW, cp = s % Cfg::CPRW;
        b_row_in_slice[i] = r;
        b_chunk[i] = cp ^ (Cfg::swz(r) << 2);
    }
    const uint32_t a_voff = (uint32_t)(wave * 1024 + lane * 16);
    const uint32_t lds0 = lds_offset(lds);

    // ---- tile parameters ------------------------------------------------------------------------
    // (kept in named scalars: arrays indexed at run time would be placed in LDS or scratch by the
    // compiler, and everything read back from there counts as lane-varying)
    struct Tile {
        int br, n0, T;  // block-row, first column, number of K slices
        int blk0;       // first stored block of the block-row
        int bcol0;      // block column of that block (loaded early: no step waits for a dependent load)
    };
    auto decode = [&](int idx, Tile &t, uint32_t (&voff)[Cfg::B_LPW]) {
        const int per_group = group_n * n_brows;
        const int grp = idx / per_group, in_grp = idx - grp * per_group;
        const int left = n_tiles - grp * group_n;
        const int gw = left < group_n ? left : group_n;  // the last group may be narrower
        // heaviest block-row first in even groups, lightest first in odd ones: neighbours in the order,
        // which run at the same time, then have similar weights across group boundaries too
        const int pos = in_grp / gw, nt = grp * group_n + (in_grp - pos * gw);
        const int rank = (grp & 1) ? n_brows - 1 - pos : pos;
        const int4 ri = rank_info[rank];
        // the index is the same for the whole workgroup: tell the compiler, so that everything derived
        // from a tile's parameters stays in scalar registers
        t.br = __builtin_amdgcn_readfirstlane(ri.x);
        t.blk0 = __builtin_amdgcn_readfirstlane(ri.y);
        t.T = __builtin_amdgcn_readfirstlane(ri.z) * Cfg::SPB;
        t.bcol0 = t.T > 0 ? __builtin_amdgcn_readfirstlane(block_col_idx[t.blk0]) : 0;
        t.n0 = nt * BN;
#pragma unroll
        for (int i = 0; i < Cfg::B_LPW; ++i) {
            int col = t.n0 + 8 * b_chunk[i];
            col = col < N ? col : N - 8;  // chunks past N only feed columns that are never stored
            voff[i] = (uint32_t)(((int64_t)b_row_in_slice[i] * N + col) * 2);  // byte offset inside a slice of B
        }
    };

    // ---- the slice stream ---------------------------------------------------------------------------
    // cur_t is the tile being multiplied, nxt_t the one after it (if have_next).  The prefetch cursor is
    // the next slice to request; it carries its own copy of what it needs (pf_*), sits in the current tile
    // or, once that is fully requested, in the next one (pf_in_next), never further.
    // Buffers buf_c, buf_c+1, .. (mod NS) hold the `inflight` slices requested but not yet multiplied.
    // issued counts the vector-memory operations of this wave; mark[b] is its value right after the
    // loads into buffer b were issued, so issued - mark[b] operations may remain outstanding when the
    // content of b is needed (the counter retires in order).
    Tile cur_t, nxt_t;
    uint32_t nxt_voff[Cfg::B_LPW], pf_voff[Cfg::B_LPW];
    int have_next = 0;
    int pf_T = 0, pf_t = 0, pf_blk = 0, pf_s = 0, pf_in_next = 0;
    int pf_bcol = 0, pf_bcol_next = 0;  // block column of the cursor's block and of the block after it
    int buf_c = 0, inflight = 0;
    int issued = 0, mark0 = 0, mark1 = 0, mark2 = 0;
    auto mark_of = [&](int b) { return b == 0 ? mark0 : (b == 1 ? mark1 : mark2); };
    auto cursor_enter = [&](const Tile &t, const uint32_t (&voff)[Cfg::B_LPW]) {
        pf_T = t.T;
        pf_t = 0;
        pf_blk = t.blk0;
        pf_s = 0;
        pf_bcol_next = t.bcol0;
#pragma unroll
        for (int i = 0; i < Cfg::B_LPW; ++i) pf_voff[i] = voff[i];
    };

    decode(idx_cur, cur_t, nxt_voff);
    cursor_enter(cur_t, nxt_voff);
    nxt_t = cur_t;
    if (idx_n1 < run_end) {
        have_next = 1;
        decode(idx_n1, nxt_t, nxt_voff);
    }

    // request the cursor's slice into ring buffer buf and move the cursor on
    auto issue_slice = [&](int buf) {
        const uint32_t stage = lds0 + buf * Cfg::STAGE;
        // the blocks of a block-row, and the slices of a block, are consecutive in a_packed
        const uint8_t *abase = (const uint8_t *)a_packed + ((int64_t)pf_blk * (BR * BR) + pf_s * (BR * KS)) * 2;
#pragma unroll
        for (int i = 0; i < Cfg::A_LPW; ++i)
            dma16_to_lds(abase + i * NW * 1024, a_voff, stage + (i * NW + wave) * 1024);
        if (pf_s == 0) {
            pf_bcol = pf_bcol_next;
            if (pf_t + Cfg::SPB < pf_T) pf_bcol_next = __builtin_amdgcn_readfirstlane(block_col_idx[pf_blk + 1]);
        }
        const int krow0 = pf_bcol * BR + pf_s * KS;
        const uint8_t *bbase = (const uint8_t *)(B + (int64_t)krow0 * N);
        if (krow0 + KS <= K) {
#pragma unroll
            for (int i = 0; i < Cfg::B_LPW; ++i)
                dma16_to_lds(bbase, pf_voff[i], stage + Cfg::A_STAGE + (i * NW + wave) * 1024);
        } else {
            // the slice crosses K: rows past K are read from row K-1, they meet the zero padding of A
#pragma unroll
            for (int i = 0; i < Cfg::B_LPW; ++i) {
                int krow = krow0 + b_row_in_slice[i];
                int back = krow < K ? 0 : krow - (K - 1);
                dma16_to_lds(bbase + pf_voff[i] - (int64_t)back * N * 2, stage + Cfg::A_STAGE + (i * NW + wave) * 1024);
            }
        }
        ++pf_t;
        if (++pf_s == Cfg::SPB) {
            pf_s = 0;
            ++pf_blk;
        }
    };
    // request the next slice of the stream, if there is one within reach; returns whether it did
    auto prefetch_one = [&]() -> bool {
        if (pf_t >= pf_T) {  // this tile is fully requested: step into the next one
            if (pf_in_next || !have_next || nxt_t.T == 0) return false;
            cursor_enter(nxt_t, nxt_voff);
            pf_in_next = 1;
        }
        int buf = buf_c + inflight;
        buf = buf >= NS ? buf - NS : buf;
        issue_slice(buf);
        issued += LPW;
        mark0 = buf == 0 ? issued : mark0;
        mark1 = buf == 1 ? issued : mark1;
        mark2 = buf == 2 ? issued : mark2;
        ++inflight;
        return true;
    };
    // wait until at most `allowed` of this wave's vector-memory operations are outstanding (rounded
    // down to one of the counts that can occur), and until its LDS accesses and scalar loads are done
    auto wait_outstanding = [&](int allowed) {
        constexpr int S = Cfg::NSTORE;
        if (allowed >= S + 2 * LPW) wait_vmcnt_and_lds<S + 2 * LPW>();
        else if (allowed >= S + LPW) wait_vmcnt_and_lds<S + LPW>();
        else if (allowed >= S && S > 2 * LPW) wait_vmcnt_and_lds<S>();
        else if (allowed >= 2 * LPW) wait_vmcnt_and_lds<2 * LPW>();
        else if (allowed >= S) wait_vmcnt_and_lds<S>();
        else if (allowed >= LPW) wait_vmcnt_and_lds<LPW>();
        else wait_vmcnt_and_lds<0>();
    };

    // MFMA operand fragments of one 16-wide k step of the slice in ring buffer buf
    struct Frags {
        bf16x8 a[MT], b[NTL];
    };
    auto load_frags = [&](int buf, int kk, Frags &f) {
        const uint8_t *sa = lds + buf * Cfg::STAGE, *sb = sa + Cfg::A_STAGE;
#pragma unroll
        for (int i = 0; i < MT; ++i) f.a[i] = *(const bf16x8 *)(sa + (kk * (BR / 32) + wm * MT + i) * 1024 + a_off);
#pragma unroll
        for (int j = 0; j < NTL; ++j) {
            const uint8_t *p0 = sb + kk * 16 * Cfg::B_ROW + b_off[j];
            short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3))) *)(p0));
            short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (short4v __attribute__((address_space(3))) *)(p0 + 4 * Cfg::B_ROW));
            short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            f.b[j] = __builtin_bit_cast(bf16x8, both);
        }
    };
    auto multiply = [&](f32x16 (&acc)[MT][NTL], const Frags &f) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j)
                // operands swapped: D[n][m] = sum_k B[k][n] * A[m][k]
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
    };
    static_assert(Cfg::KK == 2, "the step below is written for two k steps per slice");
    const bool k_aligned = K % BR == 0;  // then no slice reaches past row K of B

    for (;;) {
        const Tile tc = cur_t;
        // (re)fill the ring up to NS-1 slices: the buffer behind buf_c may still be read as the previous
        // tile's staging area until the next barrier
        while (inflight < NS - 1 && prefetch_one()) {
        }
        f32x16 acc[MT][NTL];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        for (int t = 0; t < tc.T; ++t) {
            // Steady state: the NS-1 slices t .. t+NS-2 are in flight or landed, no store sits between them
            // (the previous tile's stores are older than slice NS-1), and the cursor is inside this tile at
            // slice t+NS-1.  Then the wait is a constant and the request code is straight-line.
            const bool steady = k_aligned && t >= NS - 1 && t + NS - 1 < tc.T && inflight == NS - 1 && !pf_in_next;
            if (steady) wait_vmcnt_and_lds<(NS - 2) * LPW>();
            else wait_outstanding(issued - mark_of(buf_c));  // this wave's part of the slice in buf_c has landed
            barrier_no_fence();  // everybody's part has landed; the buffer behind buf_c is free
            Frags f0, f1;
            load_frags(buf_c, 0, f0);  // LDS reads first: their latency runs under the request code below
            if (steady) {
                const int buf = buf_c == 0 ? NS - 1 : buf_c - 1;
                const uint32_t stage = lds0 + buf * Cfg::STAGE;
                const uint8_t *abase = (const uint8_t *)a_packed + ((int64_t)pf_blk * (BR * BR) + pf_s * (BR * KS)) * 2;
#pragma unroll
                for (int i = 0; i < Cfg::A_LPW; ++i)
                    dma16_to_lds(abase + i * NW * 1024, a_voff, stage + (i * NW + wave) * 1024);
                if (pf_s == 0) {
                    pf_bcol = pf_bcol_next;
                    if (pf_t + Cfg::SPB < pf_T) pf_bcol_next = __builtin_amdgcn_readfirstlane(block_col_idx[pf_blk + 1]);
                }
                const uint8_t *bbase = (const uint8_t *)(B + (int64_t)(pf_bcol * BR + pf_s * KS) * N);
#pragma unroll
                for (int i = 0; i < Cfg::B_LPW; ++i)
                    dma16_to_lds(bbase, pf_voff[i], stage + Cfg::A_STAGE + (i * NW + wave) * 1024);
                issued += LPW;
                mark0 = buf == 0 ? issued : mark0;
                mark1 = buf == 1 ? issued : mark1;
                mark2 = buf == 2 ? issued : mark2;
                ++pf_t;
                if (++pf_s == Cfg::SPB) {
                    pf_s = 0;
                    ++pf_blk;
                }
            } else {
                while (inflight < NS && prefetch_one()) {
                }
                --inflight;
            }
            load_frags(buf_c, 1, f1);
            multiply(acc, f0);
            multiply(acc, f1);
            buf_c = buf_c + 1 == NS ? 0 : buf_c + 1;
        }

        // ---- tile boundary ------------------------------------------------------------------------
        // parameters of the tile after the next one: requested now, needed after the epilogue
        int idx_nn = tile_of_round(round + 2);
        Tile tnn = tc;
        uint32_t voff_nn[Cfg::B_LPW];
#pragma unroll
        for (int i = 0; i < Cfg::B_LPW; ++i) voff_nn[i] = 0;
        if (!DYN && idx_nn < run_end) decode(idx_nn, tnn, voff_nn);
        if constexpr (DYN) {
            if (tid == 0) s_claim[0] = run_begin + atomicAdd(&sched[xcd], 1);  // read by all after the barrier below
        }

        // the buffer behind buf_c holds nothing that is still needed once every wave got here
        wait_vmcnt_and_lds<63>();
        barrier_no_fence();
        if constexpr (DYN) {
            idx_nn = __builtin_amdgcn_readfirstlane(s_claim[0]);
            if (idx_nn < run_end) decode(idx_nn, tnn, voff_nn);
        }
        const bool interior = tc.br * BR + BR <= M && tc.n0 + BN <= N;
        int sbuf = buf_c == 0 ? NS - 1 : buf_c - 1;
        uint8_t *sc = lds + sbuf * Cfg::STAGE + wave * Cfg::C_WAVE;
        const int grow0 = tc.br * BR + wm * Cfg::TM + lane / Cfg::CPR;
        const int gcol0 = tc.n0 + wn * Cfg::TN + (lane % Cfg::CPR) * 8;
        const uint8_t *scl = sc + (lane / Cfg::CPR) * Cfg::C_PITCH + (lane % Cfg::CPR) * 16;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int jh = 0; jh < NTL / Cfg::JR; ++jh) {
                // fp32 -> bf16 (round to nearest even); lane holds row (lane & 31), 4 adjacent columns per q
#pragma unroll
                for (int jj = 0; jj < Cfg::JR; ++jj)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x16 &a = acc[i][jh * Cfg::JR + jj];
                        f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                        bf16x4 hv = __builtin_convertvector(v, bf16x4);
                        *(bf16x4 *)(sc + (lane & 31) * Cfg::C_PITCH + (jj * 32 + 8 * q + 4 * (lane >> 5)) * 2) = hv;
                    }
                // LDS is in order within a wave: the reads below see the writes above
                uint16_t *cdst = C + (int64_t)(grow0 + i * 32) * N + gcol0 + jh * Cfg::RW;
                if (interior) {
#pragma unroll
                    for (int it = 0; it < 32 / Cfg::RPI; ++it) {
                        uint4 v = *(const uint4 *)(scl + it * Cfg::RPI * Cfg::C_PITCH);
                        store_c16(cdst + (int64_t)it * Cfg::RPI * N, v);
                    }
                } else {
#pragma unroll
                    for (int it = 0; it < 32 / Cfg::RPI; ++it) {
                        uint4 v = *(const uint4 *)(scl + it * Cfg::RPI * Cfg::C_PITCH);
                        if (grow0 + i * 32 + it * Cfg::RPI < M && gcol0 + jh * Cfg::RW < N)
                            store_c16(cdst + (int64_t)it * Cfg::RPI * N, v);
                    }
                }
            }
        if (interior) {
            issued += Cfg::NSTORE;  // exactly NSTORE stores were issued, none is waited for
        } else {
            // an edge tile issues a data-dependent number of stores: drain once so the count is exact again
            wait_vmcnt_and_lds<0>();
            mark0 = mark1 = mark2 = issued;
        }

        // ---- advance to the next tile ---------------------------------------------------------------
        if (!have_next) break;
        ++round;
        idx_cur = tile_of_round(round);
        cur_t = nxt_t;
        if (pf_in_next) pf_in_next = 0;          // the cursor's tile is now the current one
        else cursor_enter(nxt_t, nxt_voff);     // the cursor never left the finished tile: it follows
        if (idx_nn < run_end) {
            nxt_t = tnn;
#pragma unroll
            for (int i = 0; i < Cfg::B_LPW; ++i) nxt_voff[i] = voff_nn[i];
            have_next = 1;
        } else {
            have_next = 0;
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------

// Cut the tile order into 8 runs of equal weight.  Tile weight = stored blocks of its block-row + 1
// (the 1 stands for the epilogue).  Groups of N-tiles repeat the same sorted list of block-rows, so a
// cut is found from the per-handle prefix sums over that list.
XcdRuns cut_runs(const std::vector<int64_t> &pre, int64_t nbr, int n_tiles, int group_n) {
    const int64_t rows_weight = pre[nbr];
    const int64_t n_groups = ceil_div(n_tiles, group_n);
    const int64_t total_weight = rows_weight * n_tiles;
    XcdRuns r;
    r.start[0] = 0;
    for (int x = 1; x < 8; ++x) {
        const int64_t target = total_weight * x / 8;
        // whole groups before the cut
        int64_t g = 0, acc = 0;
        for (; g < n_groups; ++g) {
            const int64_t gw = std::min<int64_t>(group_n, n_tiles - g * group_n);
            if (acc + gw * rows_weight > target) break;
            acc += gw * rows_weight;
        }
        if (g >= n_groups) {
            r.start[x] = (int)(nbr * n_tiles);
            continue;
        }
        const int64_t gw = std::min<int64_t>(group_n, n_tiles - g * group_n);
        // first position whose prefix (times the group width) reaches the remainder; odd groups walk
        // the block-rows lightest first
        const int64_t rem = target - acc;
        auto prefix = [&](int64_t j) { return (g & 1) ? rows_weight - pre[nbr - j] : pre[j]; };
        int64_t lo = 0, hi = nbr;
        while (lo < hi) {
            int64_t mid = (lo + hi) / 2;
            if (prefix(mid) * gw < rem) lo = mid + 1; else hi = mid;
        }
        r.start[x] = (int)(g * group_n * nbr + lo * gw);
    }
    r.start[8] = (int)(nbr * n_tiles);
    for (int x = 1; x <= 8; ++x)
        if (r.start[x] < r.start[x - 1]) r.start[x] = r.start[x - 1];
    return r;
}

__global__ void bcsr_zero_sched_kernel(int *__restrict__ sched) {
    if (threadIdx.x < 8) sched[threadIdx.x] = 0;
}

template <int BR, int BN, int WM, int WN, int NS>
static void launch_dma(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    const int env_group = switches().bcsr_group_n, env_wgs = switches().bcsr_wgs_per_cu;  // benchmarking switches
    int group_n = env_group > 0 ? env_group : 4;
    if (group_n > p.n_tiles) group_n = p.n_tiles;
    // resident workgroups per CU: as many as LDS allows (the kernel is built for 2 waves per SIMD)
    const int fit = (int)(163840 / DmaCfg<BR, BN, WM, WN, NS>::LDS_BYTES);
    const int per_cu = std::max(1, std::min(fit, 8 / (WM * WN)));
    int64_t workers = (int64_t)h->n_cus * (env_wgs > 0 ? env_wgs : per_cu);
    if (workers > p.workgroups) workers = p.workgroups;
    workers = std::max<int64_t>(8, workers / 8 * 8);  // the same number of workgroups on every XCD
    const XcdRuns runs = cut_runs(h->hb.sorted_weight_prefix, h->n_brows, p.n_tiles, group_n);
    dim3 grid((unsigned)workers), block(WM * WN * 64);
    // benchmarking switch: tiles pulled from per-XCD atomic counters (built for the 128 x 256 tiles of the ladder;
    // everything else keeps the static schedule)
    const bool env_atomic = switches().bcsr_atomic;
    if constexpr (BR == 128 && BN == 256) {
        if (env_atomic && h->d_sched) {
            hipLaunchKernelGGL(bcsr_zero_sched_kernel, dim3(1), dim3(64), 0, stream, h->d_sched);
            hipLaunchKernelGGL((bcsr_spmm_dma_kernel<BR, BN, WM, WN, NS, true>), grid, block, 0, stream,
                               (const int4 *)h->d_rank_info, h->d_col_idx, (const uint16_t *)h->d_values,
                               (const uint16_t *)B, (uint16_t *)C, (int)h->m, (int)h->k, (int)N, (int)h->n_brows,
                               p.n_tiles, group_n, runs, h->d_sched);
            return;
        }
    }
    hipLaunchKernelGGL((bcsr_spmm_dma_kernel<BR, BN, WM, WN, NS>), grid, block, 0, stream, (const int4 *)h->d_rank_info,
                       h->d_col_idx, (const uint16_t *)h->d_values, (const uint16_t *)B, (uint16_t *)C, (int)h->m,
                       (int)h->k, (int)N, (int)h->n_brows, p.n_tiles, group_n, runs, (int *)nullptr);
}

// needs N % 8 == 0, 8 <= N < 2^25 and 16-byte aligned B and C (the caller checked)
bool bcsr_dma_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream) {
    switch (h->b_row * 1000 + p.bn) {
        case 128256: launch_dma<128, 256, 2, 2, 3>(h, B, C, N, p, stream); return true;
        case 128128: launch_dma<128, 128, 2, 2, 3>(h, B, C, N, p, stream); return true;
        case 128064: launch_dma<128, 64, 2, 2, 3>(h, B, C, N, p, stream); return true;
        case 64256: launch_dma<64, 256, 1, 4, 3>(h, B, C, N, p, stream); return true;
        case 64128: launch_dma<64, 128, 2, 2, 3>(h, B, C, N, p, stream); return true;
        case 64064: launch_dma<64, 64, 1, 2, 3>(h, B, C, N, p, stream); return true;
        case 32256: launch_dma<32, 256, 1, 2, 3>(h, B, C, N, p, stream); return true;
        case 32128: launch_dma<32, 128, 1, 2, 3>(h, B, C, N, p, stream); return true;
        case 32064: launch_dma<32, 64, 1, 2, 3>(h, B, C, N, p, stream); return true;
    }
    return false;
}


}  // namespace asp
