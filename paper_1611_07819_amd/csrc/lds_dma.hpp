// What the three MFMA pipelines (fp16, fp32, fp64) share: direct global -> LDS loads written as
// assembly, the explicit wait on them, and the XOR swizzle of 128-byte LDS rows.
#pragma once
#include <hip/hip_runtime.h>

namespace dm {
namespace ldsdma {

typedef __attribute__((address_space(3))) char lds_char;

// 16-byte chunk XOR of a k unit-stride LDS tile ([mn][128 bytes]): the eight chunks of row mn are
// rotated so that the 16 rows a 128-bit fragment read touches together hit 16 different chunks.
__device__ __forceinline__ int swz(int mn) { return (mn ^ (mn >> 3)) & 7; }

// Forces a wavefront-uniform pointer into scalar registers.  The registers are read by loads
// written as assembly, which the compiler does not recognise as memory instructions: the wait
// states the hardware wants between a vector instruction that writes a scalar register and a
// memory instruction that reads it are therefore spent here.
__device__ __forceinline__ const char* uniform_ptr(const char* p)
{
    uint64_t v = reinterpret_cast<uint64_t>(p);
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    asm volatile("s_nop 4" : "+s"(lo), "+s"(hi));
    return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// One direct global->LDS load: lane fetches 16 bytes at (sbase + voff), lands at m0 + 16*lane.
// The compiler is told what the assembly overwrites besides memory: M0, and in the second form
// the scalar condition code, which the add sets (a comparison whose result the compiler kept in
// SCC across such a load skipped a whole k-loop once).
__device__ __forceinline__ void dma16(uint32_t lds_addr, const void* sbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// The same with the LDS address given as a scalar base plus an offset: where the offset is a
// constant after unrolling it becomes a literal of the add that sets M0, so that neither a
// register nor a second instruction is spent on it.
__device__ __forceinline__ void dma16(uint32_t lds_base, int lds_off, const void* sbase, uint32_t voff)
{
    if (__builtin_constant_p(lds_off)) {
        asm volatile("s_add_i32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                     :
                     : "s"(lds_base), "i"(lds_off), "v"(voff), "s"(sbase)
                     : "memory", "m0", "scc");
    } else {
        dma16(lds_base + (uint32_t)lds_off, sbase, voff);
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }

}  // namespace ldsdma
}  // namespace dm
