// Host-side format converters of the library: CSR -> BCSR and CSR -> WCSR (paper, Section II-C) and
// the host variant of the window sub-task list (Section III-C).  Values are bit-copied only.
//
// Work is spread over block-rows / windows with a shared atomic counter so that a few very long
// windows do not serialise the conversion.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <mutex>
#include <system_error>
#include <thread>

#include "asp_internal.h"

namespace asp {

namespace {

unsigned worker_count(int64_t items) {
    unsigned hw = std::thread::hardware_concurrency();
    if (hw == 0) hw = 1;
    hw = std::min(hw, 32u);
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>(hw, items / 64 + 1));
}

// run fn(worker_index, first, last) over [0, n) in dynamically claimed chunks
template <class F>
void parallel_chunks(int64_t n, int64_t chunk, F fn) {
    unsigned nw = worker_count(n);
    std::atomic<int64_t> next{0};
    // An exception inside a worker (an allocation that fails) must not leave its thread: the first one is kept,
    // the other workers stop claiming chunks, and it is thrown again on the calling thread after all have joined.
    std::exception_ptr first_error;
    std::mutex error_mu;
    auto body = [&](unsigned wi) {
        try {
            for (;;) {
                int64_t b = next.fetch_add(chunk);
                if (b >= n) break;
                fn(wi, b, std::min(n, b + chunk));
            }
        } catch (...) {
            std::lock_guard<std::mutex> lock(error_mu);
            if (!first_error) first_error = std::current_exception();
            next.store(n);
        }
    };
    std::vector<std::thread> th;
    for (unsigned w = 1; w < nw; ++w) {
        try {
            th.emplace_back(body, w);
        } catch (const std::system_error &) {
            break;  // no further thread to be had: the ones that run (at least the caller) do all the chunks
        }
    }
    body(0);
    for (auto &t : th) t.join();
    if (first_error) std::rethrow_exception(first_error);
}

}  // namespace

std::string validate_csr(int64_t m, int64_t k, int64_t nnz, const int32_t *row_ptr, const int32_t *col_idx) {
    if (row_ptr[0] != 0) return "row_ptr[0] != 0";
    for (int64_t i = 0; i < m; ++i)
        if (row_ptr[i + 1] < row_ptr[i]) return "row_ptr decreases at row " + std::to_string(i);
    if (row_ptr[m] != nnz) return "row_ptr[m] != nnz";
    std::atomic<int64_t> bad_row{-1};
    parallel_chunks(m, 4096, [&](unsigned, int64_t b, int64_t e) {
        for (int64_t i = b; i < e; ++i) {
            int64_t prev = -1;
            for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
                int64_t c = col_idx[p];
                if (c <= prev || c >= k) {
                    int64_t expect = -1;
                    bad_row.compare_exchange_strong(expect, i);
                    return;
                }
                prev = c;
            }
        }
    });
    if (bad_row.load() >= 0)
        return "row " + std::to_string(bad_row.load()) +
               ": column indices must be in [0,k) and strictly ascending (no duplicates)";
    return "";
}

// ------------------------------------------------------------------------------------------ BCSR
void csr_to_bcsr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                 size_t esize, int32_t b_row, int32_t b_col, HostBcsr &out) {
    const int64_t nbr = ceil_div(m, b_row), nbc = ceil_div(k, b_col);
    out.block_row_ptr.assign(nbr + 1, 0);
    unsigned nw = worker_count(nbr);
    // stamp[w][J] == I + 1 marks "block column J already seen in block-row I" for worker w
    std::vector<std::vector<int64_t>> stamp(nw, std::vector<int64_t>(nbc, 0));

    // pass 1: number of touched block columns per block-row
    parallel_chunks(nbr, 16, [&](unsigned wi, int64_t b, int64_t e) {
        auto &st = stamp[wi];
        for (int64_t I = b; I < e; ++I) {
            int64_t r1 = std::min<int64_t>(m, (I + 1) * b_row);
            int32_t cnt = 0;
            for (int64_t p = row_ptr[I * b_row]; p < row_ptr[r1]; ++p) {
                int64_t J = col_idx[p] / b_col;
                if (st[J] != I + 1) {
                    st[J] = I + 1;
                    ++cnt;
                }
            }
            out.block_row_ptr[I + 1] = cnt;
        }
    });
    for (int64_t I = 0; I < nbr; ++I) out.block_row_ptr[I + 1] += out.block_row_ptr[I];
    const int64_t nb = out.block_row_ptr[nbr];
    const int64_t bsz = (int64_t)b_row * b_col;
    out.block_col_idx.assign(nb, 0);
    out.blocks.assign((size_t)nb * bsz * esize, 0);  // +0.0 everywhere

    // pass 2: ascending block columns, then scatter the entries
    std::vector<std::vector<int32_t>> slot(nw, std::vector<int32_t>(nbc, -1));
    for (auto &s : stamp) std::fill(s.begin(), s.end(), 0);
    parallel_chunks(nbr, 16, [&](unsigned wi, int64_t b, int64_t e) {
        auto &st = stamp[wi];
        auto &sl = slot[wi];
        for (int64_t I = b; I < e; ++I) {
            int64_t r0 = I * b_row, r1 = std::min<int64_t>(m, r0 + b_row);
            int32_t *cols = out.block_col_idx.data() + out.block_row_ptr[I];
            int32_t cnt = 0;
            for (int64_t p = row_ptr[r0]; p < row_ptr[r1]; ++p) {
                int32_t J = col_idx[p] / b_col;
                if (st[J] != I + 1) {
                    st[J] = I + 1;
                    cols[cnt++] = J;
                }
            }
            std::sort(cols, cols + cnt);
            for (int32_t t = 0; t < cnt; ++t) sl[cols[t]] = out.block_row_ptr[I] + t;
            for (int64_t i = r0; i < r1; ++i) {
                for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
                    int32_t c = col_idx[p];
                    int32_t J = c / b_col;
                    size_t dst = ((size_t)sl[J] * bsz + (size_t)(i - r0) * b_col + (size_t)(c - J * b_col)) * esize;
                    std::memcpy(out.blocks.data() + dst, (const uint8_t *)values + (size_t)p * esize, esize);
                }
            }
        }
    });
}

// Scheduling data of the main BCSR kernel: block-rows ordered by their number of stored blocks,
// heaviest first (ties: lower block-row first), with prefix sums of the tile weights in that order.
void bcsr_build_schedule(HostBcsr &b) {
    const int64_t nbr = (int64_t)b.block_row_ptr.size() - 1;
    std::vector<int32_t> sorted(nbr);
    for (int64_t i = 0; i < nbr; ++i) sorted[i] = (int32_t)i;
    auto len = [&](int32_t r) { return b.block_row_ptr[r + 1] - b.block_row_ptr[r]; };
    std::stable_sort(sorted.begin(), sorted.end(), [&](int32_t x, int32_t y) { return len(x) > len(y); });
    int64_t n_nonempty = 0;
    while (n_nonempty < nbr && len(sorted[n_nonempty]) > 0) ++n_nonempty;

    // The kernels deal consecutive entries of this order to the workgroups of an XCD round-robin, LISTS
    // block-rows per round (each block-row repeated over the N-tiles of a group).  So entry j belongs to
    // list j % LISTS, and a workgroup walks one list per group of N-tiles.  The non-empty block-rows are
    // spread over the lists by the longest-processing-time rule (heaviest first, each to the list that is
    // lightest so far; weight = stored blocks + 1 for the tile's epilogue), which keeps the lists' sums
    // within one block-row of each other.  Empty block-rows follow.
    constexpr int LISTS = 16;
    std::vector<std::vector<int32_t>> lists(LISTS);
    std::vector<int64_t> load(LISTS, 0);
    for (int64_t r = 0; r < n_nonempty; ++r) {
        // among the lists with the fewest entries (the round being filled), the lightest one
        int best = -1;
        size_t fewest = lists[0].size();
        for (int l = 1; l < LISTS; ++l) fewest = std::min(fewest, lists[l].size());
        for (int l = 0; l < LISTS; ++l)
            if (lists[l].size() == fewest && (best < 0 || load[l] < load[best])) best = l;
        lists[best].push_back(sorted[r]);
        load[best] += len(sorted[r]) + 1;
    }
    // Lists with one entry more go first, so that the entries of the last, incomplete round are those of lists
    // 0, 1, ... and "entry j belongs to list j % LISTS" holds for every j.
    std::stable_sort(lists.begin(), lists.end(),
                     [](const std::vector<int32_t> &x, const std::vector<int32_t> &y) { return x.size() > y.size(); });
    // Inside a list the order is free (the sum stays).  Entries go by the block column of their first block:
    // the block-rows of one round then start in the same few block columns, their first slabs of B are requested
    // by several workgroups of the XCD at about the same time and cross the memory side of L2 once
    // (7 % less time on 90 % Bernoulli masks than lists in order of weight).
    for (auto &l : lists)
        std::stable_sort(l.begin(), l.end(), [&](int32_t x, int32_t y) {
            return b.block_col_idx[b.block_row_ptr[x]] < b.block_col_idx[b.block_row_ptr[y]];
        });
    std::vector<int32_t> order;
    order.reserve(nbr);
    for (size_t e = 0; order.size() < (size_t)n_nonempty; ++e)
        for (int l = 0; l < LISTS; ++l)
            if (e < lists[l].size()) order.push_back(lists[l][e]);
    for (int64_t r = n_nonempty; r < nbr; ++r) order.push_back(sorted[r]);

    b.rank_info.resize((size_t)nbr * 4);
    b.sorted_weight_prefix.assign(nbr + 1, 0);
    b.n_nonempty = n_nonempty;
    for (int64_t r = 0; r < nbr; ++r) {
        const int32_t br = order[r];
        b.rank_info[4 * r + 0] = br;
        b.rank_info[4 * r + 1] = b.block_row_ptr[br];
        b.rank_info[4 * r + 2] = len(br);
        b.rank_info[4 * r + 3] = len(br) > 0 ? b.block_col_idx[b.block_row_ptr[br]] : 0;  // column of its first block
        b.sorted_weight_prefix[r + 1] = b.sorted_weight_prefix[r] + len(br) + 1;
    }
}

// Composite form of a bf16 BCSR matrix with 64x64 or 32x32 blocks, for the kernel written for 128x128 blocks
// (Section II-C's block product, regrouped): R = 128 / b block-rows make one 128-row super-row; the union of their
// block columns is cut into groups of R; a composite block holds, for each of its R columns j, the b-wide column
// strip [block(r_0, j); ...; block(r_{R-1}, j)] of the super-row's members (zeros where a block is not stored) as
// b / 32 consecutive 32-wide K slices.  slice_rows gives, per composite block, the first row of B that each of
// its four K slices multiplies (for a plain 128x128 block these would be 128 J + 0, 32, 64, 96).  Strips that pad
// the last group are zeros and repeat the rows of the last real strip.
//
// Members of a super-row need not be adjacent: every absent block of a strip is computed as zeros, so block-rows
// with similar block columns are put together (greedy: longest unassigned block-row first, then R - 1 times the
// unassigned block-row with the largest Jaccard index against the group's union of columns; on 50-90 %-sparse
// random masks this stores 12-24 % fewer composite blocks than grouping neighbours).  piece_rows
// gives, per super-row, the first row of C of each of its four 32-row pieces, -1 for a member that does not
// exist.  Block-rows without blocks form super-rows of their own at the end (their rows of C are cleared).
// Returns the work inflation: composite blocks x 128 x 128 over stored blocks x b x b.
double bcsr_build_composite(const HostBcsr &in, int64_t m, int64_t k, int32_t b, HostBcsr &out) {
    const int64_t nbr = (int64_t)in.block_row_ptr.size() - 1;
    const int32_t R = 128 / b, spv = b / 32;  // members of a super-row = strips per composite block; K slices per strip
    (void)m;
    auto len = [&](int64_t r) { return in.block_row_ptr[r + 1] - in.block_row_ptr[r]; };
    auto cols = [&](int64_t r) { return in.block_col_idx.data() + in.block_row_ptr[r]; };

    // ---- grouping ----------------------------------------------------------------------------------------
    int32_t nbc = 0;
    for (int32_t c : in.block_col_idx) nbc = std::max(nbc, c + 1);
    std::vector<int32_t> inv_ptr((size_t)nbc + 1, 0), inv(in.block_col_idx.size());
    for (int32_t c : in.block_col_idx) ++inv_ptr[c + 1];
    for (int32_t c = 0; c < nbc; ++c) inv_ptr[c + 1] += inv_ptr[c];
    {
        std::vector<int32_t> fill(inv_ptr.begin(), inv_ptr.end() - 1);
        for (int64_t r = 0; r < nbr; ++r)
            for (int32_t t = 0; t < len(r); ++t) inv[fill[cols(r)[t]]++] = (int32_t)r;
    }
    std::vector<int32_t> order;
    for (int64_t r = 0; r < nbr; ++r)
        if (len(r) > 0) order.push_back((int32_t)r);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return len(x) > len(y); });
    std::vector<uint8_t> taken((size_t)nbr, 0), in_union((size_t)nbc, 0);
    std::vector<int32_t> shared((size_t)nbr, 0), touched, uni;
    std::vector<int32_t> members;  // R per super-row, -1 = none
    const int64_t budget = 1 << 18;  // shared-column counts examined per choice: bounds the work on dense matrices
    for (int32_t seed : order) {
        if (taken[seed]) continue;
        taken[seed] = 1;
        const size_t g0 = members.size();
        members.push_back(seed);
        uni.assign(cols(seed), cols(seed) + len(seed));
        for (int32_t c : uni) in_union[c] = 1;
        while (members.size() - g0 < (size_t)R) {
            touched.clear();
            int64_t spent = 0;
            for (int32_t c : uni) {
                for (int32_t q = inv_ptr[c]; q < inv_ptr[c + 1] && spent < budget; ++q, ++spent) {
                    const int32_t r = inv[q];
                    if (taken[r]) continue;
                    if (shared[r]++ == 0) touched.push_back(r);
                }
                if (spent >= budget) break;
            }
            // best Jaccard index with the group's union: shared / (union + own - shared), compared as fractions
            int32_t best = -1;
            int64_t best_num = 0, best_den = 1;
            const int64_t usize = (int64_t)uni.size();
            for (int32_t r : touched) {
                const int64_t num = shared[r], den = usize + len(r) - shared[r];
                const int64_t lhs = num * best_den, rhs = best_num * den;
                if (best < 0 || lhs > rhs || (lhs == rhs && r < best)) best = r, best_num = num, best_den = den;
                shared[r] = 0;
            }
            if (best < 0) break;  // nobody shares a column: the group stays short
            taken[best] = 1;
            members.push_back(best);
            for (int32_t t = 0; t < len(best); ++t) {
                const int32_t c = cols(best)[t];
                if (!in_union[c]) in_union[c] = 1, uni.push_back(c);
            }
        }
        for (int32_t c : uni) in_union[c] = 0;
        // members in ascending block-row order (rows of C of a tile ascend), padded with -1
        std::sort(members.begin() + g0, members.end());
        while (members.size() - g0 < (size_t)R) members.push_back(-1);
    }
    {   // block-rows without blocks
        size_t g0 = members.size();
        for (int64_t r = 0; r < nbr; ++r)
            if (len(r) == 0) {
                members.push_back((int32_t)r);
                if (members.size() - g0 == (size_t)R) g0 = members.size();
            }
        while ((members.size() - g0) % R != 0) members.push_back(-1);
    }
    const int64_t nsr = (int64_t)members.size() / R;

    // ---- composite blocks --------------------------------------------------------------------------------
    out = HostBcsr();
    out.block_row_ptr.assign(nsr + 1, 0);
    out.piece_rows.assign((size_t)nsr * 4, -1);
    std::vector<std::vector<int32_t>> unis((size_t)nsr);
    parallel_chunks(nsr, 16, [&](unsigned, int64_t lo, int64_t hi) {
        for (int64_t sr = lo; sr < hi; ++sr) {
            auto &u = unis[sr];
            for (int32_t t = 0; t < R; ++t) {
                const int32_t br = members[sr * R + t];
                if (br < 0) continue;
                u.insert(u.end(), cols(br), cols(br) + len(br));
                for (int32_t i = 0; i < spv; ++i) out.piece_rows[4 * sr + t * spv + i] = br * b + 32 * i;
            }
            std::sort(u.begin(), u.end());
            u.erase(std::unique(u.begin(), u.end()), u.end());
            out.block_row_ptr[sr + 1] = (int32_t)ceil_div((int64_t)u.size(), R);
        }
    });
    for (int64_t sr = 0; sr < nsr; ++sr) out.block_row_ptr[sr + 1] += out.block_row_ptr[sr];
    const int64_t nc = out.block_row_ptr[nsr];
    out.block_col_idx.assign(nc, 0);
    out.slice_rows.assign((size_t)nc * 4, 0);
    out.blocks.assign((size_t)nc * 128 * 128 * 2, 0);
    const uint16_t *src = (const uint16_t *)in.blocks.data();
    uint16_t *dst = (uint16_t *)out.blocks.data();
    parallel_chunks(nsr, 4, [&](unsigned, int64_t lo, int64_t hi) {
        for (int64_t sr = lo; sr < hi; ++sr) {
            const auto &u = unis[sr];
            for (int64_t c = out.block_row_ptr[sr]; c < out.block_row_ptr[sr + 1]; ++c) {
                const int64_t first = (c - out.block_row_ptr[sr]) * R;
                for (int32_t v = 0; v < R; ++v) {
                    const bool real = first + v < (int64_t)u.size();
                    const int32_t j = u[real ? first + v : u.size() - 1];
                    // a slice must not reach past K: in the last, partly filled block column it starts early enough
                    // to end at K, and its values move right by the same amount (the columns it then overlaps with
                    // an earlier slice stay zero here)
                    int32_t shift[4] = {0, 0, 0, 0};
                    for (int32_t t = 0; t < spv; ++t) {
                        const int64_t k0 = (int64_t)j * b + 32 * t;
                        const int64_t r0 = std::min<int64_t>(k0, k - 32);
                        shift[t] = (int32_t)(k0 - r0);
                        out.slice_rows[4 * c + v * spv + t] = (int32_t)r0;
                    }
                    if (!real) continue;
                    for (int32_t t = 0; t < R; ++t) {
                        const int32_t br = members[sr * R + t];
                        if (br < 0) continue;
                        const int32_t *cb = cols(br), *ce = cb + len(br);
                        const int32_t *hit = std::lower_bound(cb, ce, j);
                        if (hit == ce || *hit != j) continue;
                        const uint16_t *sb = src + (int64_t)(hit - in.block_col_idx.data()) * b * b;
                        for (int32_t r = 0; r < b; ++r)
                            for (int32_t sl = 0; sl < spv; ++sl) {
                                if (shift[sl] >= 32) continue;  // the slice lies past K altogether: zeros
                                std::memcpy(dst + c * 128 * 128 + ((int64_t)t * b + r) * 128 + v * b + 32 * sl + shift[sl],
                                            sb + (int64_t)r * b + 32 * sl, (size_t)(32 - shift[sl]) * 2);
                            }
                    }
                }
                out.block_col_idx[c] = out.slice_rows[4 * c] / 128;  // the schedule orders block-rows by this
            }
        }
    });
    bcsr_build_schedule(out);
    bcsr_pack_fragments_bf16(out, 128, 128, out.packed);
    out.blocks = std::vector<uint8_t>();  // only the packed form is used
    const double stored = (double)in.block_col_idx.size() * b * b;
    return stored > 0 ? (double)nc * 128 * 128 / stored : 0.0;
}

// Kernel-internal order of a bf16 block: for each 16-wide k slice, for each group of 32 rows, the 64
// lanes of a wavefront hold 8 consecutive k each (lane l: row l % 32, k offset 8 * (l / 32)), which
// is the A/B operand layout of v_mfma_f32_32x32x16_bf16.  A pure permutation of the canonical block.
void bcsr_pack_fragments_bf16(const HostBcsr &in, int32_t b_row, int32_t b_col, std::vector<uint8_t> &packed) {
    const int64_t nb = (int64_t)in.block_col_idx.size();
    const int64_t bsz = (int64_t)b_row * b_col;
    packed.resize(in.blocks.size());
    const uint16_t *src = (const uint16_t *)in.blocks.data();
    uint16_t *dst = (uint16_t *)packed.data();
    const int32_t mtiles = b_row / 32, kslices = b_col / 16;
    parallel_chunks(nb, 4, [&](unsigned, int64_t b, int64_t e) {
        for (int64_t q = b; q < e; ++q) {
            const uint16_t *s = src + q * bsz;
            uint16_t *d = dst + q * bsz;
            for (int32_t ks = 0; ks < kslices; ++ks)
                for (int32_t mt = 0; mt < mtiles; ++mt)
                    for (int32_t lane = 0; lane < 64; ++lane) {
                        int32_t row = mt * 32 + lane % 32, col = ks * 16 + 8 * (lane / 32);
                        std::memcpy(d, s + (int64_t)row * b_col + col, 16);
                        d += 8;
                    }
        }
    });
}

// Kernel-internal order of an fp32 block: for each 16-wide k slice, each group of 32 rows and each group of
// 8 k, lane l of a wavefront holds the 4 values A[l % 32][2t + l / 32], t = 0..3: the A operands of four
// consecutive v_mfma_f32_32x32x2_f32 (lane l feeds row l % 32, k index l / 32).  A pure permutation.
void bcsr_pack_fragments_f32(const HostBcsr &in, int32_t b_row, int32_t b_col, std::vector<uint8_t> &packed) {
    const int64_t nb = (int64_t)in.block_col_idx.size();
    const int64_t bsz = (int64_t)b_row * b_col;
    packed.resize(in.blocks.size());
    const uint32_t *src = (const uint32_t *)in.blocks.data();
    uint32_t *dst = (uint32_t *)packed.data();
    const int32_t mtiles = b_row / 32, kslices = b_col / 16;
    parallel_chunks(nb, 4, [&](unsigned, int64_t b, int64_t e) {
        for (int64_t q = b; q < e; ++q) {
            const uint32_t *s = src + q * bsz;
            uint32_t *d = dst + q * bsz;
            for (int32_t ks = 0; ks < kslices; ++ks)
                for (int32_t mt = 0; mt < mtiles; ++mt)
                    for (int32_t kg = 0; kg < 2; ++kg)
                        for (int32_t lane = 0; lane < 64; ++lane)
                            for (int32_t t = 0; t < 4; ++t) {
                                int32_t row = mt * 32 + lane % 32, col = ks * 16 + kg * 8 + 2 * t + lane / 32;
                                *d++ = s[(int64_t)row * b_col + col];
                            }
        }
    });
}

// ------------------------------------------------------------------------------------------ WCSR
namespace {

// Columns of one window, ascending with duplicates between rows removed: sort the window's CSR entries (they
// are one contiguous range of col_idx) by column.  A k-way merge of the sorted rows costs rows x distinct
// columns and was 30x slower for 64-row windows with ~1000 columns.
// key = column << 32 | entry index inside the window (the window's entries are fewer than 2^31).
struct WindowSorter {
    std::vector<uint64_t> key;
    std::vector<uint8_t> row_of;  // row inside the window of each entry

    // distinct columns only
    int64_t count(const int32_t *row_ptr, const int32_t *col_idx, int64_t r0, int64_t r1) {
        const int64_t p0 = row_ptr[r0], n = row_ptr[r1] - p0;
        if (r1 - r0 == 1) return n;  // a row's columns are distinct already
        key.resize((size_t)n);
        for (int64_t e = 0; e < n; ++e) key[e] = (uint32_t)col_idx[p0 + e];
        std::sort(key.begin(), key.end());
        return (int64_t)(std::unique(key.begin(), key.end()) - key.begin());
    }

    // emit(t, col) once per distinct column in ascending order with its rank t; hit(t, row_in_window, p) once
    // per CSR entry p that sits in that column
    template <class Emit, class Hit>
    void place(const int32_t *row_ptr, const int32_t *col_idx, int64_t r0, int64_t r1, Emit emit, Hit hit) {
        const int64_t p0 = row_ptr[r0], n = row_ptr[r1] - p0;
        key.resize((size_t)n);
        row_of.resize((size_t)n);
        for (int64_t r = r0; r < r1; ++r)
            for (int64_t p = row_ptr[r]; p < row_ptr[r + 1]; ++p) {
                key[p - p0] = ((uint64_t)(uint32_t)col_idx[p] << 32) | (uint64_t)(p - p0);
                row_of[p - p0] = (uint8_t)(r - r0);
            }
        std::sort(key.begin(), key.end());
        int64_t t = -1;
        int32_t prev = -1;
        for (int64_t i = 0; i < n; ++i) {
            const int32_t col = (int32_t)(key[i] >> 32);
            const int64_t e = (int64_t)(key[i] & 0xFFFFFFFFu);
            if (col != prev) {
                emit(++t, col);
                prev = col;
            }
            hit(t, (int)row_of[e], p0 + e);
        }
    }
};

}  // namespace

bool csr_to_wcsr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                 size_t esize, int32_t b_row, int32_t b_col, HostWcsr &out) {
    (void)k;
    const int64_t nw = ceil_div(m, b_row);
    out.window_row_ptr.assign(nw + 1, 0);
    parallel_chunks(nw, 64, [&](unsigned, int64_t b, int64_t e) {
        WindowSorter ws;
        for (int64_t w = b; w < e; ++w) {
            int64_t r0 = w * b_row, r1 = std::min<int64_t>(m, r0 + b_row);
            int64_t u = ws.count(row_ptr, col_idx, r0, r1);
            out.window_row_ptr[w + 1] = (int32_t)(ceil_div(u, b_col) * b_col);
        }
    });
    int64_t total = 0;  // packed positions are 32-bit: padding can push them past what the entries needed
    for (int64_t w = 0; w < nw; ++w) total += out.window_row_ptr[w + 1];
    if (total > INT32_MAX) return false;
    for (int64_t w = 0; w < nw; ++w) out.window_row_ptr[w + 1] += out.window_row_ptr[w];
    const int64_t padded = out.window_row_ptr[nw];
    out.window_col_idx.assign(padded, -1);
    out.values.reset((size_t)padded * b_row * esize);
    const int64_t tile = (int64_t)b_row * b_col;
    parallel_chunks(nw, 64, [&](unsigned, int64_t b, int64_t e) {
        WindowSorter ws;
        for (int64_t w = b; w < e; ++w) {
            int64_t r0 = w * b_row, r1 = std::min<int64_t>(m, r0 + b_row);
            const int64_t p0 = out.window_row_ptr[w];
            ws.place(
                row_ptr, col_idx, r0, r1, [&](int64_t t, int32_t col) { out.window_col_idx[p0 + t] = col; },
                [&](int64_t t, int r, int64_t p) {
                    int64_t pc = p0 + t;
                    size_t dst = (size_t)((pc / b_col) * tile + (int64_t)r * b_col + pc % b_col) * esize;
                    std::memcpy(out.values.data() + dst, (const uint8_t *)values + (size_t)p * esize, esize);
                });
        }
    });
    return true;
}

void wcsr_tasks_host(const std::vector<int32_t> &wrp, int32_t task_cols, std::vector<int32_t> &tasks) {
    tasks.clear();
    for (size_t w = 0; w + 1 < wrp.size(); ++w) {
        const int32_t lo = wrp[w], hi = wrp[w + 1];
        const int32_t split = (hi - lo > task_cols) ? 1 : 0;
        for (int64_t c = lo; c < hi; c += task_cols) {  // 64-bit: position + task_cols may pass 2^31
            tasks.push_back((int32_t)w);
            tasks.push_back((int32_t)c);
            tasks.push_back((int32_t)std::min<int64_t>(hi, c + task_cols));
            tasks.push_back(split);
        }
    }
}

void wcsr_zero_windows(const std::vector<int32_t> &wrp, int32_t task_cols, std::vector<int32_t> &zw) {
    zw.clear();
    for (size_t w = 0; w + 1 < wrp.size(); ++w) {
        int32_t n = wrp[w + 1] - wrp[w];
        if (n == 0 || n > task_cols) zw.push_back((int32_t)w);
    }
}

}  // namespace asp
