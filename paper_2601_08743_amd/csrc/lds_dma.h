// Direct global -> LDS loads (global_load_lds_dwordx4), shared by the kernels that stream K/V tiles
// into LDS without passing through registers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tc {

// 16 bytes per lane from (uniform base + per-lane offset) to LDS at lds_dst + 16 * lane.  The
// instruction takes its LDS address from M0 and its base from a scalar register pair; both are
// made uniform explicitly.  Completion is counted in vmcnt like any vector load; the compiler does
// not know about these loads, so the waits (s_waitcnt vmcnt) are the caller's.
//
// Because the load is hidden in assembly, the compiler's hazard recogniser does not see it either,
// and two rules of this hardware for vector-memory instructions have to be kept by hand:
//  * a scalar register written by a vector instruction (v_readfirstlane is one) must not be read
//    by a vector-memory instruction for 5 wait states.  Where the base is computed per lane and
//    made uniform, the compiler puts that v_readfirstlane directly in front of this statement;
//    the base is therefore copied with a scalar move inside the statement (scalar reads of such a
//    register are interlocked, and a scalar-written register may be used at once);
//  * one wait state between the write of M0 and the load (the s_nop).
// M0 cannot be named as clobbered (the compiler reserves it and warns that such a clobber is
// undefined); what must hold instead - that the compiler itself never keeps a value in M0 in a
// kernel that uses these loads - is checked on the emitted assembly by tests/test_kernel_schedule.py,
// which also checks that no such load reads a vector-written scalar register too early.
__device__ __forceinline__ void load_to_lds(uint32_t lds_dst, const char *base, uint32_t voff)
{
    const uint64_t b64 = (uint64_t)(uintptr_t)base;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b64), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b64 >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | lo;
    uint64_t sb_copy;
    asm volatile("s_mov_b64 %0, %3\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %0"
                 : "=&s"(sb_copy)
                 : "s"(__builtin_amdgcn_readfirstlane(lds_dst)), "v"(voff), "s"(sb) : "memory");
}

}  // namespace tc
