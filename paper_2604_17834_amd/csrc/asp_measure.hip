// Measurement support, NOT part of the product library: two probe kernels that give the rates this box sustains
// (matrix cores, read-only memory stream), beside the published peaks that the roofline fractions are quoted
// against.  Built into its own library (libasyncsparse_measure.so) with its own header
// (include/asyncsparse_measure.h); only bench.py and its test load it.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "asyncsparse_measure.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---- measurement support: the matrix-core rate this machine sustains ------------------------------------
// A loop of nothing but MFMAs on register operands, 8 independent accumulators per wave, two waves per SIMD:
// the ceiling that the roofline fraction of the product kernels can also be read against (published peaks
// assume the maximum clock; a box under its power limit runs slower).
template <bool BF16>
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    const float x = 1.0f + (float)(lane & 3), y = 0.5f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)x;
        b[e] = (__bf16)y;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (BF16) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
            else acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[j], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][15];
    if (s == -1.f) out[0] = s;  // never true: keeps the loop alive
}

// read-only stream over `bytes` of device memory: 16-byte loads, 8 in flight per lane, every wave on a contiguous span
__global__ __launch_bounds__(256) void read_probe_kernel(const uint4 *__restrict__ src, int64_t n16, uint32_t *__restrict__ out) {
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n16; i += stride) {
        uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) out[0] = acc;  // practically never: keeps the loads alive
}

}  // namespace

extern "C" {

int asp_probe_mfma(int32_t dtype, int64_t iters, void *out_device, void *stream, double *flop) {
    if (!out_device || !flop) return 1;
    if (dtype != 0 && dtype != 1) return 1;
    if (iters < 1 || iters > (1 << 24)) return 1;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 5;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 5;
    const unsigned wgs = 2u * (unsigned)cus;
    if (dtype == 0)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, (int)iters, (float *)out_device);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, (int)iters, (float *)out_device);
    if (hipGetLastError() != hipSuccess) return 5;
    *flop = (double)wgs * 4.0 * (double)iters * 8.0 * (dtype == 0 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2);
    return 0;
}

int asp_probe_read(const void *src_device, int64_t bytes, void *out_device, void *stream) {
    if (!src_device || !out_device) return 1;
    if (bytes < 16 || ((uintptr_t)src_device & 15)) return 1;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 5;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 5;
    hipLaunchKernelGGL(read_probe_kernel, dim3(8u * (unsigned)cus), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)src_device, bytes / 16, (uint32_t *)out_device);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

}  // extern "C"
