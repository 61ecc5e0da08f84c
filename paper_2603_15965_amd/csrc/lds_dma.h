// LDS-direct loads and the explicit waits that go with them (gfx950), shared by the GEMM
// translation units.
#pragma once
#include "common.h"

namespace molora {
namespace {

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// 64 lanes x 16 bytes, HBM -> LDS; global address = base (scalar) + lane_off (per lane, 32 bit),
// LDS address = lds_base + lane * 16 (lds_base wave-uniform, goes to M0).  Written as inline assembly on purpose: the compiler then knows nothing of an
// outstanding LDS write and does not put a conservative vmcnt(0) wait in front of the operand
// reads of the tile being computed, which would serialise prefetch and compute.  The waits
// that order these loads against the LDS reads are the explicit wait_vmcnt + wg_barrier of
// the main loop.
__device__ __forceinline__ void load_to_lds16(const void *base, uint32_t lane_off,
                                              unsigned char *lds_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(MOLORA_LDS unsigned char *)lds_base;
    asm volatile(
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, %1"
        :
        : "v"(lane_off), "s"(base), "s"(lds_addr)
        : "memory", "m0");
}

// same, from a per-lane 64-bit address
__device__ __forceinline__ void load_to_lds16_ptr(const void *gptr, unsigned char *lds_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(MOLORA_LDS unsigned char *)lds_base;
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, off"
        :
        : "v"(gptr), "s"(lds_addr)
        : "memory", "m0");
}

// 256 bytes of zeros in device memory: the source of every operand chunk that must be zero
__device__ __attribute__((aligned(256))) uint32_t g_zero_page[64];  // one copy per translation unit

}  // namespace
}  // namespace molora
