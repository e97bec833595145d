// Direct global-to-LDS loads and the hand-kept wait that goes with them.  Internal.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ag {

// One wave-wide direct global-to-LDS load: lane l's 16 bytes at src land at LDS byte address lds_addr + l * 16
// (lds_addr is uniform and goes through M0).  One asm statement, so that nothing can come between the M0 write
// and its use; M0 is declared clobbered, so the compiler keeps nothing of its own there across the statement.
// The statement is deliberately NOT given a "memory" clobber or an LDS output operand: modelled as an LDS
// write, every later LDS operand read would wait for all outstanding tile loads.  Completion is tracked by
// hand instead: wait_vmcnt<N>() below, which ends in a compiler-level memory fence, so no ordinary LDS access that
// follows it in the source (the scrub of a landed tile, operand reads) can be moved above the wait.  The loops
// that use these loads contain no other vector memory instruction, so the counter holds exactly these loads.
// (M0 is a register the compiler reserves for itself; naming a reserved register as clobbered draws a generic
// warning, silenced here: the clobber is the truth, and tests/test_lds_dma_asm.py checks in the generated
// code that M0 is written only by these statements, each immediately before its load.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds(const void* src, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "m0");
}
// The 4-byte form: lane l's dword at src lands at lds_addr + l * 4 (a wave moves 256 bytes).
__device__ __forceinline__ void load_dword_to_lds(const void* src, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" : : "v"(src), "s"(lds_addr) : "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt 6:4 and lgkmcnt 11:8 left at
// their maximum), followed by a fence for the compiler: memory accesses are not moved across it in either
// direction.  The wait itself stays the builtin, which the compiler's own wait-count bookkeeping understands -
// written as opaque asm it would no longer know that loads it issued before (the Q fragments) have
// completed, and would wait for them again inside the tile loop, where its vmcnt(0) also covers the direct
// loads that are meant to stay in flight.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (0xF << 8));
    asm volatile("" ::: "memory");
}
#define AG_WAIT_VMCNT(n) ::ag::wait_vmcnt<(n)>()

}  // namespace ag
