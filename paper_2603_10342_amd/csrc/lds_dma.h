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
// hand instead: wait_vmcnt<N>() below, which IS a compiler-level memory fence, so no ordinary LDS access that
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
#pragma clang diagnostic pop
__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// s_waitcnt vmcnt(N) alone (the other counters are left alone), and a fence for the compiler: memory accesses
// are not moved across it in either direction.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}
#define AG_WAIT_VMCNT(n) ::ag::wait_vmcnt<(n)>()

}  // namespace ag
