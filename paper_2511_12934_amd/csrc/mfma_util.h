// Small device helpers shared by the MFMA kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aif {

typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

// Direct-to-LDS load of 16 bytes per lane: lane j's bytes land at lds_dst + 16 j
// (lds_dst = wave-uniform LDS byte address, handed over in M0).  Written as
// assembly so that the compiler does not see a store to LDS: with the builtin
// it makes later LDS reads of unrelated data wait for every outstanding load,
// which defeats any prefetch distance beyond one stage.  Completion is tracked
// by hand with wait_vmcnt<>() followed by a block barrier.
__device__ __forceinline__ void dma16(const char *gsrc, uint32_t lds_dst)
{
    uint32_t keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep)
                 : "s"(lds_dst), "v"(gsrc)
                 : "memory");
}

// The same with the address split into a wave-uniform base (scalar registers) and a per-lane byte offset:
// no 64-bit vector arithmetic and no vector register pair per load.
__device__ __forceinline__ void dma16_s(const char *sbase, uint32_t lane_off, uint32_t lds_dst)
{
    uint32_t keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep)
                 : "s"(lds_dst), "v"(lane_off), "s"(sbase)
                 : "memory");
}

// 16 * (lane id), computed on the spot: for a load in the middle of a long stream, where a value kept from the
// kernel's start would be spilled and its reload would wait for every load in flight.
__device__ __forceinline__ uint32_t lane_off16_now()
{
    uint32_t x;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0\n\tv_lshlrev_b32 %0, 4, %0" : "=v"(x));
    return x;
}

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

__device__ __forceinline__ uint32_t lds_address(const void *p) { return (uint32_t)(uintptr_t)(lptr_t)p; }

}  // namespace aif
