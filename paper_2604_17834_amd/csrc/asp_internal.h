// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <new>
#include <string>
#include <vector>

#include "asyncsparse.h"

namespace asp {

// thread-local detail string behind asp_last_error()
void set_error(const std::string &msg);
asp_status_t fail(asp_status_t s, const std::string &msg);

#define ASP_HIP_TRY(expr)                                                                        \
    do {                                                                                         \
        hipError_t e__ = (expr);                                                                 \
        if (e__ != hipSuccess)                                                                   \
            return ::asp::fail(e__ == hipErrorOutOfMemory ? ASP_ERR_OUT_OF_MEMORY : ASP_ERR_HIP, \
                               std::string(#expr) + ": " + hipGetErrorString(e__));             \
    } while (0)

// Benchmarking switches: environment variables that select among kernels and schedules which are all built and
// parity-tested, for the ladder and the tile-width study of bench.py.  Read once per process, in one place
// (asp_api.cpp); nothing else in the library looks at the environment.
struct Switches {
    int bcsr_bn;          // ASP_BCSR_BN=64|128|256: widest BCSR tile to consider (0: no cap)
    bool bcsr_regstage;   // ASP_BCSR_KERNEL=regstage: the synchronous register-staged kernel
    int bcsr_group_n;     // ASP_BCSR_GROUP_N=<n>: N-tiles walked together (0: the kernels' defaults, 2 and 4)
    int bcsr_wgs_per_cu;  // ASP_BCSR_WGS_PER_CU=<n>: resident workgroups of the ring kernel (0: as many as LDS allows)
    int bcsr_workgroups;  // ASP_BCSR_WORKGROUPS=<n>: resident workgroups of the 128x512-tile kernel (0: one per compute unit)
    bool bcsr_xcd_aware;  // ASP_BCSR_XCD_AWARE=0: deal tiles without regard to XCDs
    bool bcsr_atomic;     // ASP_BCSR_SCHEDULE=atomic: tiles pulled from per-XCD atomic counters (ring kernel, 128x256)
    bool xt_generic;      // ASP_BCSR_XT=generic: asp_spmm_xt without matrix cores
    int bcsr_composite;   // ASP_BCSR_COMPOSITE=0|1: never / always keep the 128-row stacks of smaller blocks (-1: by fill)
    int wcsr_max_bn;      // ASP_WCSR_MAX_BN=64|128|256: widest fp32 WCSR wave tile to consider
};
const Switches &switches();

inline size_t dtype_size(int32_t dt) { return dt == ASP_DT_BF16 ? 2 : 4; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- host-side converted forms -------------------------------------------------------------
// Zero-filled byte buffer taken from calloc: for gigabytes the pages arrive zeroed from the system and are first
// touched by the converter's worker threads, where a std::vector would fill them on one thread first.
class ZeroedBytes {
public:
    ZeroedBytes() = default;
    ZeroedBytes(const ZeroedBytes &) = delete;
    ZeroedBytes &operator=(const ZeroedBytes &) = delete;
    ZeroedBytes(ZeroedBytes &&o) noexcept : p_(o.p_), n_(o.n_) { o.p_ = nullptr, o.n_ = 0; }
    ZeroedBytes &operator=(ZeroedBytes &&o) noexcept {
        if (this != &o) {
            std::free(p_);
            p_ = o.p_, n_ = o.n_;
            o.p_ = nullptr, o.n_ = 0;
        }
        return *this;
    }
    ~ZeroedBytes() { std::free(p_); }
    void reset(size_t bytes) {
        std::free(p_);
        p_ = nullptr, n_ = 0;
        if (bytes == 0) return;
        p_ = (uint8_t *)std::calloc(bytes, 1);
        if (!p_) throw std::bad_alloc();
        n_ = bytes;
    }
    uint8_t *data() { return p_; }
    const uint8_t *data() const { return p_; }
    size_t size() const { return n_; }

private:
    uint8_t *p_ = nullptr;
    size_t n_ = 0;
};

struct HostBcsr {
    std::vector<int32_t> block_row_ptr;  // [n_brows + 1]
    std::vector<int32_t> block_col_idx;  // [nnz_blocks]
    std::vector<uint8_t> blocks;         // canonical [nnz_blocks][b_row][b_col], raw bytes
    std::vector<uint8_t> packed;         // same values in MFMA-fragment order (kernel-internal)
    // scheduling data of the main kernel: block-rows sorted by stored blocks (descending) and the
    // prefix sums of their tile weights (stored blocks + 1) in that order
    std::vector<int32_t> rank_info;            // [n_brows][4]
    std::vector<int64_t> sorted_weight_prefix; // [n_brows + 1]
    int64_t n_nonempty = 0;                    // block-rows with at least one stored block (they come first)
    std::vector<int32_t> slice_rows;           // composite form only: [blocks][4] first row of B of each K slice
    std::vector<int32_t> piece_rows;           // composite form only: [super-rows][4] first row of C of each 32-row piece, -1 = none
};

struct HostWcsr {
    std::vector<int32_t> window_row_ptr;  // [n_windows + 1]
    std::vector<int32_t> window_col_idx;  // [padded_cols]
    ZeroedBytes values;                   // [padded_cols / b_col][b_row][b_col], raw bytes
    std::vector<int32_t> tasks;           // [n_tasks][4]; filled on the host only in host-convert mode
    std::vector<int32_t> zero_windows;    // windows whose C rows must be cleared (empty or split)
    std::vector<int32_t> ws_slot;         // [n_windows] first scratch slot of a split window (one per task), -1 for the others
};

// converters (asp_convert.cpp); values are only bit-copied
void csr_to_bcsr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                 size_t esize, int32_t b_row, int32_t b_col, HostBcsr &out);
void bcsr_build_schedule(HostBcsr &b);
double bcsr_build_composite(const HostBcsr &in, int64_t m, int64_t k, int32_t b, HostBcsr &out);
void bcsr_pack_fragments_bf16(const HostBcsr &in, int32_t b_row, int32_t b_col, std::vector<uint8_t> &packed);
void bcsr_pack_fragments_f32(const HostBcsr &in, int32_t b_row, int32_t b_col, std::vector<uint8_t> &packed);
bool csr_to_wcsr(int64_t m, int64_t k, const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                 size_t esize, int32_t b_row, int32_t b_col, HostWcsr &out);
void wcsr_tasks_host(const std::vector<int32_t> &window_row_ptr, int32_t task_cols, std::vector<int32_t> &tasks);
void wcsr_zero_windows(const std::vector<int32_t> &window_row_ptr, int32_t task_cols,
                       std::vector<int32_t> &zero_windows);
// returns empty string when the CSR arrays are valid, else a description of the first problem
std::string validate_csr(int64_t m, int64_t k, int64_t nnz, const int32_t *row_ptr, const int32_t *col_idx);

}  // namespace asp

// ---- the opaque handle ---------------------------------------------------------------------------
struct asp_handle {
    int64_t m = 0, k = 0, nnz = 0;
    int32_t format = 0, dtype = 0, b_row = 0, b_col = 0, task_cols = 0;
    uint32_t flags = 0;
    int device = -1;  // HIP device that owns the d_* arrays, -1 in host-convert mode
    int64_t n_brows = 0, n_units = 0, n_tasks = 0, n_zero_windows = 0;
    int64_t n_split_windows = 0;  // WCSR: windows with more than one task
    int64_t n_split_tasks = 0;    // WCSR: tasks of those windows = scratch slots

    asp::HostBcsr hb;  // BCSR: canonical arrays stay on the host for export
    // bf16 BCSR with 64x64 / 32x32 blocks: the composite form (128-row super-rows, asp_convert.cpp) when it was
    // judged worth it at creation; hc keeps its scheduling data, the packed values live on the device only
    asp::HostBcsr hc;
    bool has_comp = false;
    double comp_inflation = 0.0;    // composite work over stored-block work
    int64_t c_n_brows = 0, c_n_units = 0;  // super-rows, composite blocks
    int32_t *d_c_rank_info = nullptr;
    int32_t *d_c_slice_rows = nullptr;     // [composite blocks][4]
    int32_t *d_c_piece_rows = nullptr;     // [super-rows][4]
    void *d_c_values = nullptr;
    asp::HostWcsr hw;  // WCSR: kept only in host-convert mode (device arrays are canonical)

    // device arrays
    int32_t *d_row_ptr = nullptr;   // block_row_ptr / window_row_ptr
    int32_t *d_col_idx = nullptr;   // block_col_idx / window_col_idx
    void *d_values = nullptr;       // BCSR: fragment-packed blocks; WCSR: canonical tiles
    int32_t *d_tasks = nullptr;     // WCSR tasks [n_tasks][4]
    int32_t *d_zero_windows = nullptr;
    int32_t *d_rank_info = nullptr; // BCSR: [n_brows][4] = {block-row, first block, stored blocks, block column of the first one}, heaviest first
    int n_cus = 0;                  // compute units of the owning device
    int32_t *d_sched = nullptr;     // BCSR: 8 tile counters of the dynamic-scheduling variant (a benchmarking switch)
    // WCSR: where the tasks of split windows put their partial tiles
    int32_t *d_ws_slot = nullptr;   // [n_windows] first scratch slot of a split window, -1 otherwise
    float *d_ws = nullptr;          // fp32 scratch, one [b_row][N] tile per slot (asp_reserve)
    int64_t ws_floats = 0;          // its capacity
};

namespace asp {
// kernels' host launchers (asp_bcsr.hip / asp_wcsr.hip)
struct BcsrPlan {
    int32_t bn;
    int32_t n_tiles;
    int32_t vectorized;
    int64_t workgroups;
};
BcsrPlan bcsr_plan(const asp_handle *h, int64_t N, bool aligned);
// the 128x512-tile kernel can take this handle: 128x128 blocks with K % 128 == 0, or a composite form
inline bool bcsr_wide_capable(const asp_handle *h) { return h->has_comp || (h->b_row == 128 && h->k % 128 == 0); }
bool bcsr_dma_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream);
bool bcsr_f32_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream);
bool bcsr_wide_launch(const asp_handle *h, const void *B, void *C, int64_t N, const BcsrPlan &p, hipStream_t stream);
asp_status_t bcsr_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, hipStream_t stream);
asp_status_t bcsr_spmm_xt_launch(const asp_handle *h, const void *X, void *Y, int64_t N, hipStream_t stream);

struct WcsrPlan {
    int32_t bn;
    int32_t n_tiles;
    int32_t vectorized;
    int64_t workgroups;
};
WcsrPlan wcsr_plan(const asp_handle *h, int64_t N, bool aligned);
// ws / ws_floats: the fp32 buffer that takes the partial tiles of split windows and its capacity (the handle's
// reserved buffer, or the library's static one; nullptr / 0: none)
asp_status_t wcsr_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, float *ws, int64_t ws_floats,
                              hipStream_t stream);
asp_status_t wcsr_bf16_spmm_launch(const asp_handle *h, const void *B, void *C, int64_t N, float *ws, int64_t ws_floats,
                                   hipStream_t stream);
// The library's static scratch array on `device` (which must be the current device): its device address, resolved
// once per device, and its capacity in floats.
asp_status_t wcsr_static_scratch(int device, float **ptr, int64_t *floats);
int64_t wcsr_scratch_floats(const asp_handle *h, int64_t N);  // fp32 scratch elements a call of width N uses
// clears the C rows of windows without columns (keep_split: and leaves split windows alone; else clears them too)
void wcsr_clear_empty_windows(const asp_handle *h, void *C, int64_t N, bool keep_split, hipStream_t stream);
// rows of split windows = sum of their tasks' partial tiles, in task order
void wcsr_sum_partial_tiles(const asp_handle *h, void *C, int64_t N, const float *ws, hipStream_t stream);
// GPU task partition: fills h->d_tasks / h->n_tasks from h->d_row_ptr (wavefront scans)
asp_status_t wcsr_build_tasks_device(asp_handle *h, hipStream_t stream);
}  // namespace asp
