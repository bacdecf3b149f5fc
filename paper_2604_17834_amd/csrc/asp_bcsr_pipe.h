// Device-side helpers shared by the BCSR kernels that fill an LDS ring with direct-to-LDS loads.
#pragma once

#include "asp_internal.h"

namespace asp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(8))) short short8v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

// s_waitcnt vmcnt(N) lgkmcnt(0): at most N vector-memory operations (the newest ones) stay in flight,
// every LDS access and scalar load of this wave has completed
template <int N>
__device__ __forceinline__ void wait_vmcnt_and_lds() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would drain vmcnt to zero and
// with it the slices and stores that are meant to stay in flight.  Callers wait for what they need first.
__device__ __forceinline__ void barrier_no_fence() { __builtin_amdgcn_s_barrier(); }

// global_load_lds_dwordx4: LDS[lds_base + lane*16 .. +16) = 16 bytes at this lane's source address;
// lds_base is wave-uniform (it travels in M0).  Issued as inline assembly on purpose: for the builtin
// form the compiler cannot tell which LDS bytes the copy writes and drains vmcnt to zero before every
// later LDS read, which would serialise the ring.  Completion is tracked by hand.
// Form 1: per-lane 64-bit address.  Form 2: wave-uniform 64-bit base + per-lane 32-bit byte offset.
// The wave-uniform operands are passed through readfirstlane so that they sit in SGPRs even where the
// compiler's divergence analysis cannot prove that they are uniform.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ const void *uniform_ptr(const void *p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint64_t lo = uniform32((uint32_t)v), hi = uniform32((uint32_t)(v >> 32));
    return (const void *)(uintptr_t)(lo | (hi << 32));
}
__device__ __forceinline__ void dma16_to_lds(const void *gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(uniform32(lds_base))
                 : "memory", "m0");
}
__device__ __forceinline__ void dma16_to_lds(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(uniform_ptr(sbase)),
                 "s"(uniform32(lds_base))
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_offset(const void *p) { return (uint32_t)(uintptr_t)(lds_void_ptr)p; }

// 16-byte store of finished output, marked non-temporal: C is written once and never read here, and
// plain stores were measured ~10 % slower end to end because the written lines displace B slabs in L2
// (a store-only kernel with this access pattern is faster with plain stores; the product is not).
__device__ __forceinline__ void store_c16(uint16_t *dst, uint4 v) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
    u32x4 w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, (u32x4 *)dst);
}

// first tile of each XCD's run of the tile order, start[8] = number of tiles
struct XcdRuns {
    int start[9];
};

// Cut the tile order (groups of group_n N-tiles, inside a group the n_rows heaviest block-rows,
// heaviest first in even groups and lightest first in odd ones, each repeated over the group's N-tiles) into 8 runs of equal weight; pre[] are the prefix
// sums of the block-rows' tile weights in that order.
XcdRuns cut_runs(const std::vector<int64_t> &pre, int64_t n_rows, int n_tiles, int group_n);

}  // namespace asp
