// C ABI entry points: argument checking, handle life cycle, export.  See include/asyncsparse.h.
#include <cstring>
#include <new>

#include "asp_internal.h"

namespace asp {

static thread_local std::string g_last_error;

void set_error(const std::string &msg) { g_last_error = msg; }

asp_status_t fail(asp_status_t s, const std::string &msg) {
    g_last_error = msg;
    return s;
}

const Switches &switches() {
    static const Switches sw = [] {
        auto num = [](const char *name, int dflt) {
            const char *e = std::getenv(name);
            return e ? std::atoi(e) : dflt;
        };
        auto is = [](const char *name, const char *value) {
            const char *e = std::getenv(name);
            return e && std::strcmp(e, value) == 0;
        };
        Switches s;
        s.bcsr_bn = num("ASP_BCSR_BN", 0);
        s.bcsr_regstage = is("ASP_BCSR_KERNEL", "regstage");
        s.bcsr_group_n = num("ASP_BCSR_GROUP_N", 0);
        s.bcsr_wgs_per_cu = num("ASP_BCSR_WGS_PER_CU", 0);
        s.bcsr_workgroups = num("ASP_BCSR_WORKGROUPS", 0);
        s.bcsr_xcd_aware = num("ASP_BCSR_XCD_AWARE", 1) != 0;
        s.bcsr_atomic = is("ASP_BCSR_SCHEDULE", "atomic");
        s.xt_generic = is("ASP_BCSR_XT", "generic");
        s.bcsr_composite = num("ASP_BCSR_COMPOSITE", -1);
        s.wcsr_max_bn = num("ASP_WCSR_MAX_BN", 256);
        return s;
    }();
    return sw;
}

static void free_device(asp_handle *h) {
    if (h->device < 0) return;
    int cur = -1;
    (void)hipGetDevice(&cur);
    if (cur != h->device) (void)hipSetDevice(h->device);
    (void)hipFree(h->d_row_ptr);
    (void)hipFree(h->d_col_idx);
    (void)hipFree(h->d_values);
    (void)hipFree(h->d_tasks);
    (void)hipFree(h->d_zero_windows);
    (void)hipFree(h->d_rank_info);
    (void)hipFree(h->d_sched);
    (void)hipFree(h->d_ws_slot);
    (void)hipFree(h->d_ws);
    (void)hipFree(h->d_c_rank_info);
    (void)hipFree(h->d_c_slice_rows);
    (void)hipFree(h->d_c_piece_rows);
    (void)hipFree(h->d_c_values);
    if (cur >= 0 && cur != h->device) (void)hipSetDevice(cur);
}

template <class T>
static asp_status_t upload(T **dst, const void *src, size_t bytes, hipStream_t stream) {
    *dst = nullptr;
    ASP_HIP_TRY(hipMalloc((void **)dst, bytes > 0 ? bytes : 16));
    if (bytes > 0) ASP_HIP_TRY(hipMemcpyAsync(*dst, src, bytes, hipMemcpyHostToDevice, stream));
    return ASP_OK;
}

static asp_status_t create_impl(const asp_config_t *cfg, int64_t m, int64_t k, int64_t nnz,
                                const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                                hipStream_t stream, asp_handle *h) {
    h->m = m;
    h->k = k;
    h->nnz = nnz;
    h->format = cfg->format;
    h->dtype = cfg->dtype;
    h->b_row = cfg->b_row;
    h->b_col = cfg->b_col;
    h->flags = cfg->flags;
    h->n_brows = ceil_div(m, cfg->b_row);
    const bool host_only = (cfg->flags & ASP_FLAG_HOST_CONVERT_ONLY) != 0;
    const size_t es = dtype_size(cfg->dtype);

    if (cfg->format == ASP_FMT_BCSR) {
        h->task_cols = 0;
        csr_to_bcsr(m, k, row_ptr, col_idx, values, es, cfg->b_row, cfg->b_col, h->hb);
        h->n_units = (int64_t)h->hb.block_col_idx.size();
        // (the plan counts tiles of non-empty block-rows, also for host-only handles, which get no schedule)
        h->hb.n_nonempty = 0;
        for (size_t r = 0; r + 1 < h->hb.block_row_ptr.size(); ++r)
            h->hb.n_nonempty += h->hb.block_row_ptr[r + 1] > h->hb.block_row_ptr[r] ? 1 : 0;
        // Smaller blocks: the kernel for 128-row tiles on the composite form (asp_convert.cpp) beats the small-block
        // kernel, which reads twice / four times the LDS bytes per MFMA, until the zero fill outweighs that.
        // Measured on 8192 x 8192 matrices with geometric block-row lengths (N = 65536) at 50 / 75 / 90 / 95 / 99 %
        // block sparsity: 64x64 blocks, fill 1.22 / 1.44 / 1.70 / 1.78 / 2.04 -> 1.98 / 1.84 / 1.41 / 1.38 / 1.13
        // times faster; 32x32 blocks, fill 1.60 / 2.09 / 2.73 / 3.21 / 3.77 -> 2.72 / 2.44 / 1.68 / 1.22 / 1.08.
        // With super-rows of neighbouring block-rows (more fill) the break-even was at fill 2.6 / 4.3.
        // ASP_BCSR_COMPOSITE=0/1 is a benchmarking switch.
        // (128x128 blocks take the same form when K is not a multiple of 128: it keeps every K slice inside K)
        if (cfg->dtype == ASP_DT_BF16 && (cfg->b_row < 128 || k % 128 != 0) && k >= 32 && h->n_units > 0) {
            const int env_comp = switches().bcsr_composite;
            if (env_comp != 0) {
                h->comp_inflation = bcsr_build_composite(h->hb, m, k, cfg->b_row, h->hc);
                const double limit = cfg->b_row == 128 ? 1.0 : cfg->b_row == 64 ? 2.6 : 4.3;  // 128: no fill
                h->has_comp = env_comp == 1 || h->comp_inflation <= limit;
                h->c_n_brows = (int64_t)h->hc.block_row_ptr.size() - 1;
                h->c_n_units = (int64_t)h->hc.block_col_idx.size();
                if (!h->has_comp || host_only) h->hc.packed = std::vector<uint8_t>();
                if (!h->has_comp) h->hc = HostBcsr();
            }
        }
        if (host_only) return ASP_OK;
        if (cfg->dtype == ASP_DT_F32)
            bcsr_pack_fragments_f32(h->hb, cfg->b_row, cfg->b_col, h->hb.packed);
        else
            bcsr_pack_fragments_bf16(h->hb, cfg->b_row, cfg->b_col, h->hb.packed);
        ASP_HIP_TRY(hipGetDevice(&h->device));
        asp_status_t s;
        if ((s = upload(&h->d_row_ptr, h->hb.block_row_ptr.data(), h->hb.block_row_ptr.size() * 4, stream))) return s;
        if ((s = upload(&h->d_col_idx, h->hb.block_col_idx.data(), h->hb.block_col_idx.size() * 4, stream))) return s;
        if ((s = upload(&h->d_values, h->hb.packed.data(), h->hb.packed.size(), stream))) return s;
        ASP_HIP_TRY(hipDeviceGetAttribute(&h->n_cus, hipDeviceAttributeMultiprocessorCount, h->device));
        bcsr_build_schedule(h->hb);
        if ((s = upload(&h->d_rank_info, h->hb.rank_info.data(), h->hb.rank_info.size() * 4, stream))) return s;
        ASP_HIP_TRY(hipMalloc((void **)&h->d_sched, 64));
        if (h->has_comp) {
            if ((s = upload(&h->d_c_rank_info, h->hc.rank_info.data(), h->hc.rank_info.size() * 4, stream))) return s;
            if ((s = upload(&h->d_c_slice_rows, h->hc.slice_rows.data(), h->hc.slice_rows.size() * 4, stream))) return s;
            if ((s = upload(&h->d_c_piece_rows, h->hc.piece_rows.data(), h->hc.piece_rows.size() * 4, stream))) return s;
            if ((s = upload(&h->d_c_values, h->hc.packed.data(), h->hc.packed.size(), stream))) return s;
        }
        ASP_HIP_TRY(hipStreamSynchronize(stream));
        std::vector<uint8_t>().swap(h->hb.packed);  // the device copy is the only user
        std::vector<uint8_t>().swap(h->hc.packed);
        return ASP_OK;
    }

    // WCSR
    h->task_cols = cfg->task_cols > 0 ? cfg->task_cols : 512;
    if (!csr_to_wcsr(m, k, row_ptr, col_idx, values, es, cfg->b_row, cfg->b_col, h->hw)) {
        set_error("the packed columns of all windows, padded to multiples of b_col, exceed 2^31 - 1");
        return ASP_ERR_UNSUPPORTED;
    }
    h->n_units = (int64_t)h->hw.window_col_idx.size();
    wcsr_zero_windows(h->hw.window_row_ptr, h->task_cols, h->hw.zero_windows);
    h->n_zero_windows = (int64_t)h->hw.zero_windows.size();
    {
        const auto &wrp = h->hw.window_row_ptr;
        h->hw.ws_slot.assign(wrp.size() - 1, -1);
        for (size_t w = 0; w + 1 < wrp.size(); ++w)
            if (wrp[w + 1] - wrp[w] > h->task_cols) {
                h->hw.ws_slot[w] = (int32_t)h->n_split_tasks;
                h->n_split_tasks += ceil_div(wrp[w + 1] - wrp[w], h->task_cols);
                ++h->n_split_windows;
            }
    }
    if (host_only) {
        wcsr_tasks_host(h->hw.window_row_ptr, h->task_cols, h->hw.tasks);
        h->n_tasks = (int64_t)h->hw.tasks.size() / 4;
        return ASP_OK;
    }
    ASP_HIP_TRY(hipGetDevice(&h->device));
    asp_status_t s;
    if ((s = upload(&h->d_row_ptr, h->hw.window_row_ptr.data(), h->hw.window_row_ptr.size() * 4, stream))) return s;
    if ((s = upload(&h->d_col_idx, h->hw.window_col_idx.data(), h->hw.window_col_idx.size() * 4, stream))) return s;
    if ((s = upload(&h->d_values, h->hw.values.data(), h->hw.values.size(), stream))) return s;
    if ((s = upload(&h->d_zero_windows, h->hw.zero_windows.data(), h->hw.zero_windows.size() * 4, stream))) return s;
    if ((s = upload(&h->d_ws_slot, h->hw.ws_slot.data(), h->hw.ws_slot.size() * 4, stream))) return s;
    if ((s = wcsr_build_tasks_device(h, stream))) return s;  // wavefront-scan partition on the GPU
    if (h->n_split_tasks > 0) {
        // set-up for asp_spmm_static_scratch: the device address of the static scratch array, once per device
        float *p = nullptr;
        int64_t n = 0;
        if ((s = wcsr_static_scratch(h->device, &p, &n))) return s;
    }
    ASP_HIP_TRY(hipStreamSynchronize(stream));
    // the device arrays are the canonical ones; drop the host copies (values can be gigabytes)
    h->hw = HostWcsr();
    return ASP_OK;
}

}  // namespace asp

using namespace asp;

extern "C" {

asp_status_t asp_create_from_csr(const asp_config_t *cfg, int64_t m, int64_t k, int64_t nnz,
                                 const int32_t *row_ptr, const int32_t *col_idx, const void *values,
                                 void *stream, asp_handle_t **out) {
    if (out) *out = nullptr;
    if (!cfg || !out || !row_ptr) return fail(ASP_ERR_INVALID_ARG, "null cfg, out or row_ptr");
    if (m < 1 || k < 1 || nnz < 0) return fail(ASP_ERR_INVALID_ARG, "need m >= 1, k >= 1, nnz >= 0");
    if (m >= (1ll << 31) || k >= (1ll << 31) || nnz >= (1ll << 31))
        return fail(ASP_ERR_UNSUPPORTED, "m, k and nnz must fit int32");
    if (nnz > 0 && (!col_idx || !values)) return fail(ASP_ERR_INVALID_ARG, "null col_idx or values with nnz > 0");
    if (cfg->flags & ~ASP_FLAG_HOST_CONVERT_ONLY) return fail(ASP_ERR_INVALID_ARG, "unknown flag bits");
    if (cfg->format == ASP_FMT_BCSR) {
        if (cfg->dtype != ASP_DT_BF16 && cfg->dtype != ASP_DT_F32) return fail(ASP_ERR_INVALID_ARG, "unknown dtype");
        if (!(cfg->b_row == 32 || cfg->b_row == 64 || cfg->b_row == 128) || cfg->b_col != cfg->b_row)
            return fail(ASP_ERR_UNSUPPORTED, "BCSR blocks must be 32x32, 64x64 or 128x128");
    } else if (cfg->format == ASP_FMT_WCSR) {
        if (cfg->dtype != ASP_DT_BF16 && cfg->dtype != ASP_DT_F32) return fail(ASP_ERR_INVALID_ARG, "unknown dtype");
        if (!(cfg->b_row == 16 || cfg->b_row == 32 || cfg->b_row == 64) || cfg->b_col != 8)
            return fail(ASP_ERR_UNSUPPORTED, "WCSR needs b_row in {16,32,64} and b_col = 8");
        if (cfg->task_cols < 0 || cfg->task_cols % cfg->b_col != 0)
            return fail(ASP_ERR_INVALID_ARG, "task_cols must be 0 or a positive multiple of b_col");
        // (a window never has 2^31 packed columns: a larger task size means nothing; sums with it are taken in 64 bits)
        if (cfg->task_cols > (1 << 30)) return fail(ASP_ERR_INVALID_ARG, "task_cols must not exceed 2^30");
    } else {
        return fail(ASP_ERR_INVALID_ARG, "unknown format");
    }
    std::string why = validate_csr(m, k, nnz, row_ptr, col_idx);
    if (!why.empty()) return fail(ASP_ERR_INVALID_CSR, why);

    asp_handle *h = nullptr;
    asp_status_t s;
    try {
        h = new asp_handle();
        s = create_impl(cfg, m, k, nnz, row_ptr, col_idx, values, (hipStream_t)stream, h);
        // sizes that the kernels index with int32
        if (s == ASP_OK && h->n_units >= (1ll << 31)) s = fail(ASP_ERR_UNSUPPORTED, "too many blocks / packed columns");
    } catch (const std::bad_alloc &) {
        s = fail(ASP_ERR_OUT_OF_MEMORY, "host allocation failed during conversion");
    } catch (const std::exception &e) {
        s = fail(ASP_ERR_INVALID_ARG, std::string("conversion failed: ") + e.what());
    }
    if (s != ASP_OK) {
        if (h) {
            free_device(h);
            delete h;
        }
        return s;
    }
    *out = h;
    return ASP_OK;
}

// The handle's arrays live on one device; kernels go to the caller's stream, which must belong to it.
static asp_status_t check_current_device(const asp_handle *h) {
    int cur = -1;
    ASP_HIP_TRY(hipGetDevice(&cur));
    if (cur != h->device)
        return fail(ASP_ERR_INVALID_ARG, "the handle was created on device " + std::to_string(h->device) +
                                             ", the current device is " + std::to_string(cur));
    return ASP_OK;
}

asp_status_t asp_spmm(const asp_handle_t *h, const void *B, void *C, int64_t N, void *stream) {
    if (!h || !B || !C) return fail(ASP_ERR_INVALID_ARG, "null handle, B or C");
    if (N < 1) return fail(ASP_ERR_INVALID_ARG, "N must be >= 1");
    if (h->device < 0) return fail(ASP_ERR_UNSUPPORTED, "handle was converted on the host only; it has no device arrays");
    if (N > ASP_MAX_N || h->m * N >= (1ll << 40)) return fail(ASP_ERR_UNSUPPORTED, "N too large (ASP_MAX_N, and M x N below 2^40)");
    if (asp_status_t s = check_current_device(h)) return s;
    if (h->format == ASP_FMT_BCSR) return bcsr_spmm_launch(h, B, C, N, (hipStream_t)stream);
    return wcsr_spmm_launch(h, B, C, N, h->d_ws, h->ws_floats, (hipStream_t)stream);
}

asp_status_t asp_spmm_static_scratch(const asp_handle_t *h, const void *B, void *C, int64_t N, void *stream) {
    if (!h || !B || !C) return fail(ASP_ERR_INVALID_ARG, "null handle, B or C");
    if (N < 1) return fail(ASP_ERR_INVALID_ARG, "N must be >= 1");
    if (h->device < 0) return fail(ASP_ERR_UNSUPPORTED, "handle was converted on the host only; it has no device arrays");
    if (N > ASP_MAX_N || h->m * N >= (1ll << 40)) return fail(ASP_ERR_UNSUPPORTED, "N too large (ASP_MAX_N, and M x N below 2^40)");
    if (asp_status_t s = check_current_device(h)) return s;
    if (h->format == ASP_FMT_BCSR) return bcsr_spmm_launch(h, B, C, N, (hipStream_t)stream);  // uses no scratch
    float *ws = nullptr;
    int64_t ws_floats = 0;
    if (h->n_split_tasks > 0) {
        const int64_t need = wcsr_scratch_floats(h, N);
        if (need > (int64_t)(ASP_STATIC_SCRATCH_BYTES / sizeof(float)))
            return fail(ASP_ERR_BUFFER_TOO_SMALL,
                        "the partial tiles of this handle's split windows at this N take " + std::to_string(need * 4) +
                            " bytes, the static scratch holds " + std::to_string((long long)ASP_STATIC_SCRATCH_BYTES) +
                            ": use asp_reserve + asp_spmm");
        if (asp_status_t s = wcsr_static_scratch(h->device, &ws, &ws_floats)) return s;  // resolved at creation: no HIP call
    }
    return wcsr_spmm_launch(h, B, C, N, ws, ws_floats, (hipStream_t)stream);
}

asp_status_t asp_reserve(asp_handle_t *h, int64_t N) {
    if (!h) return fail(ASP_ERR_INVALID_ARG, "null handle");
    if (N < 1 || N > ASP_MAX_N) return fail(ASP_ERR_INVALID_ARG, "N out of range (1 .. ASP_MAX_N)");
    if (h->device < 0) return fail(ASP_ERR_UNSUPPORTED, "handle was converted on the host only; it has no device arrays");
    if (h->format != ASP_FMT_WCSR || h->n_split_tasks == 0) return ASP_OK;  // uses none
    const int64_t need = wcsr_scratch_floats(h, N);
    if (need <= h->ws_floats) return ASP_OK;
    int cur = -1;
    ASP_HIP_TRY(hipGetDevice(&cur));
    if (cur != h->device) ASP_HIP_TRY(hipSetDevice(h->device));
    (void)hipFree(h->d_ws);  // waits for the device, so no earlier call can still be using it
    h->d_ws = nullptr;
    h->ws_floats = 0;
    hipError_t e = hipMalloc((void **)&h->d_ws, (size_t)need * 4);
    if (cur != h->device) (void)hipSetDevice(cur);
    if (e != hipSuccess)
        return fail(e == hipErrorOutOfMemory ? ASP_ERR_OUT_OF_MEMORY : ASP_ERR_HIP,
                    std::string("hipMalloc of the scratch buffer: ") + hipGetErrorString(e));
    h->ws_floats = need;
    return ASP_OK;
}

asp_status_t asp_spmm_xt(const asp_handle_t *h, const void *X, void *Y, int64_t N, void *stream) {
    if (!h || !X || !Y) return fail(ASP_ERR_INVALID_ARG, "null handle, X or Y");
    if (N < 1) return fail(ASP_ERR_INVALID_ARG, "N must be >= 1");
    if (h->device < 0) return fail(ASP_ERR_UNSUPPORTED, "handle was converted on the host only; it has no device arrays");
    if (h->format != ASP_FMT_BCSR || h->dtype != ASP_DT_BF16)
        return fail(ASP_ERR_UNSUPPORTED, "the K-contiguous entry is built for bf16 BCSR handles only");
    if (N > ASP_MAX_N || h->m * N >= (1ll << 40) || h->k * N >= (1ll << 40))
        return fail(ASP_ERR_UNSUPPORTED, "N too large (ASP_MAX_N, and M x N, K x N below 2^40)");
    if (asp_status_t s = check_current_device(h)) return s;
    return bcsr_spmm_xt_launch(h, X, Y, N, (hipStream_t)stream);
}

asp_status_t asp_get_info(const asp_handle_t *h, asp_info_t *info) {
    if (!h || !info) return fail(ASP_ERR_INVALID_ARG, "null handle or info");
    info->m = h->m;
    info->k = h->k;
    info->nnz = h->nnz;
    info->format = h->format;
    info->dtype = h->dtype;
    info->b_row = h->b_row;
    info->b_col = h->b_col;
    info->task_cols = h->task_cols;
    info->on_device = h->device >= 0 ? 1 : 0;
    info->n_brows = h->n_brows;
    info->n_units = h->n_units;
    info->n_tasks = h->n_tasks;
    info->n_zero_rows_units = h->n_zero_windows;
    double slots = h->format == ASP_FMT_BCSR ? (double)h->n_units * h->b_row * h->b_col : (double)h->n_units * h->b_row;
    info->fill_ratio = slots > 0 ? (double)h->nnz / slots : 0.0;
    return ASP_OK;
}

asp_status_t asp_plan_spmm(const asp_handle_t *h, int64_t N, asp_plan_t *plan) {
    if (!h || !plan) return fail(ASP_ERR_INVALID_ARG, "null handle or plan");
    if (N < 1 || N > ASP_MAX_N) return fail(ASP_ERR_INVALID_ARG, "N out of range (1 .. ASP_MAX_N)");
    if (h->format == ASP_FMT_BCSR) {
        BcsrPlan p = bcsr_plan(h, N, true);
        plan->bn = p.bn;
        plan->n_tiles = p.n_tiles;
        plan->vectorized = p.vectorized;
        plan->workgroups = p.workgroups;
    } else {
        WcsrPlan p = wcsr_plan(h, N, true);
        plan->bn = p.bn;
        plan->n_tiles = p.n_tiles;
        plan->vectorized = p.vectorized;
        plan->workgroups = p.workgroups;
    }
    plan->padded_n = (int64_t)plan->n_tiles * plan->bn;
    return ASP_OK;
}

asp_status_t asp_export(const asp_handle_t *h, asp_array_t which, void *host_dst, size_t dst_bytes, size_t *needed) {
    if (!h) return fail(ASP_ERR_INVALID_ARG, "null handle");
    const size_t es = dtype_size(h->dtype);
    const bool bcsr = h->format == ASP_FMT_BCSR;
    const void *hsrc = nullptr;  // host source, when there is one
    const void *dsrc = nullptr;  // else device source
    size_t bytes = 0;
    switch (which) {
        case ASP_ARR_ROW_PTR:
            bytes = (size_t)(h->n_brows + 1) * 4;
            hsrc = bcsr ? (const void *)h->hb.block_row_ptr.data() : (const void *)h->hw.window_row_ptr.data();
            dsrc = h->d_row_ptr;
            break;
        case ASP_ARR_COL_IDX:
            bytes = (size_t)h->n_units * 4;
            hsrc = bcsr ? (const void *)h->hb.block_col_idx.data() : (const void *)h->hw.window_col_idx.data();
            dsrc = h->d_col_idx;
            break;
        case ASP_ARR_VALUES:
            bytes = bcsr ? (size_t)h->n_units * h->b_row * h->b_col * es : (size_t)h->n_units * h->b_row * es;
            hsrc = bcsr ? (const void *)h->hb.blocks.data() : (const void *)h->hw.values.data();
            dsrc = h->d_values;
            break;
        case ASP_ARR_TASKS:
            if (bcsr) return fail(ASP_ERR_INVALID_ARG, "BCSR has no task list");
            bytes = (size_t)h->n_tasks * 16;
            hsrc = h->hw.tasks.data();
            dsrc = h->d_tasks;
            break;
        default:
            return fail(ASP_ERR_INVALID_ARG, "unknown array id");
    }
    if (needed) *needed = bytes;
    if (dst_bytes < bytes || (!host_dst && bytes > 0)) return fail(ASP_ERR_BUFFER_TOO_SMALL, "destination too small");
    if (bytes == 0) return ASP_OK;
    // BCSR keeps canonical arrays on the host (the device holds a permuted copy of the blocks);
    // a WCSR device handle reads its canonical arrays back from the GPU.
    if (bcsr || h->device < 0) {
        std::memcpy(host_dst, hsrc, bytes);
        return ASP_OK;
    }
    int cur = -1;
    ASP_HIP_TRY(hipGetDevice(&cur));
    if (cur != h->device) ASP_HIP_TRY(hipSetDevice(h->device));
    hipError_t e = hipMemcpy(host_dst, dsrc, bytes, hipMemcpyDeviceToHost);
    if (cur != h->device) (void)hipSetDevice(cur);
    if (e != hipSuccess) return fail(ASP_ERR_HIP, std::string("hipMemcpy D2H: ") + hipGetErrorString(e));
    return ASP_OK;
}

asp_status_t asp_destroy(asp_handle_t *h) {
    if (!h) return ASP_OK;
    free_device(h);
    delete h;
    return ASP_OK;
}

const char *asp_status_string(int status) {
    switch (status) {
        case ASP_OK: return "ASP_OK";
        case ASP_ERR_INVALID_ARG: return "ASP_ERR_INVALID_ARG";
        case ASP_ERR_INVALID_CSR: return "ASP_ERR_INVALID_CSR";
        case ASP_ERR_UNSUPPORTED: return "ASP_ERR_UNSUPPORTED";
        case ASP_ERR_OUT_OF_MEMORY: return "ASP_ERR_OUT_OF_MEMORY";
        case ASP_ERR_HIP: return "ASP_ERR_HIP";
        case ASP_ERR_BUFFER_TOO_SMALL: return "ASP_ERR_BUFFER_TOO_SMALL";
    }
    return "ASP_ERR_UNKNOWN";
}

const char *asp_last_error(void) { return asp::g_last_error.c_str(); }

}  // extern "C"
