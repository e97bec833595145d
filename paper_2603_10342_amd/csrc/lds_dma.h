// Direct global-to-LDS loads and the hand-kept wait that goes with them.  Internal.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ag {

// One wave-wide direct global-to-LDS load: lane l's 16 bytes at src land at LDS byte address lds_addr + l * 16
// (lds_addr is uniform and goes through M0).  Written as one asm statement so that nothing can come between the
// M0 write and its use (the compiler keeps nothing live in M0 on this target: it writes M0 immediately before each
// of its own uses), and so that the compiler does not model it: it would otherwise make every later LDS
// operand read wait for all outstanding tile loads.  Completion is tracked by hand with AG_WAIT_VMCNT; the
// loop contains no other vector memory instruction, so the counter holds exactly these loads.
__device__ __forceinline__ void load_to_lds(const void* src, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr));
}
__device__ __forceinline__ unsigned lds_address(const void* p)
{
    return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8 left at maximum).
#define AG_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (7 << 4) | (0xF << 8))

}  // namespace ag
