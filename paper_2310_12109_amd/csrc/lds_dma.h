// Direct-to-LDS loads (global_load_lds_dwordx4) and the waits that go with them (gfx950).
//
// Each lane's 16 bytes at its own global address go to LDS at a wave-uniform base + 16 * lane, without passing
// through registers.  The loads are written as assembly (M0 carries the LDS base and is saved / restored) so that
// the compiler does not put its own wait-for-everything in front of every later LDS read: a kernel that uses
// them waits by count (loads of all kinds share one in-order counter) and, if other waves read the data,
// publishes it with a barrier itself.
#pragma once

#include <stdint.h>

namespace monarch {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// LDS address of a pointer into shared memory, as a number
__device__ __forceinline__ uint32_t lds_address(const void *p) { return (uint32_t)(size_t)(lds_ptr_t)p; }

__device__ __forceinline__ void dma_16_at(const void *src, uint32_t lds_addr)   // lds_addr wave-uniform
{
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_addr), "v"(src)
                 : "memory");
}
__device__ __forceinline__ void dma_16(const void *src, void *lds_piece)
{
    dma_16_at(src, __builtin_amdgcn_readfirstlane(lds_address(lds_piece)));
}
// Two loads into consecutive 1 KB pieces with one save / restore of M0.
__device__ __forceinline__ void dma_16_pair(const void *src0, const void *src1, uint32_t lds_first)
{
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\t"
                 "s_add_u32 m0, m0, 0x400\n\tglobal_load_lds_dwordx4 %3, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_first), "v"(src0), "v"(src1)
                 : "memory", "scc");
}

// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt and lgkmcnt left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vm_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// The same wait as a compiler barrier too: no LDS read moves above it.
template <int N>
__device__ __forceinline__ void wait_loads_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Every LDS read issued so far has returned (needed before a direct-to-LDS load overwrites what was read).
__device__ __forceinline__ void wait_lds_reads()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

}  // namespace monarch
