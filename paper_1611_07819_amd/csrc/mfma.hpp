// Thin wrappers over the gfx950 matrix-core (MFMA) builtins and the register layouts of their
// operands and results.  One wavefront = 64 lanes.
#pragma once
#include <hip/hip_runtime.h>

namespace dm {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

// 32x32 result tile, 16 registers per lane (f32 accumulators, used by the f32 and f16 paths):
// register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
__device__ __forceinline__ int acc32_row(int lane, int r) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
__device__ __forceinline__ int acc32_col(int lane) { return lane & 31; }

// 16x16 fp64 result tile, 4 registers per lane: register r of lane l holds row 4*r + l/16,
// column l%16 (checked on the hardware with one-hot operands).
__device__ __forceinline__ int acc16d_row(int lane, int r) { return 4 * r + (lane >> 4); }
__device__ __forceinline__ int acc16d_col(int lane) { return lane & 15; }

// D += A(32x2) * B(2x32), fp32.  Lane l supplies A[l%32][l/32] and B[l/32][l%32].
__device__ __forceinline__ v16f mfma_f32_32x32x2(float a, float b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// D += A(32x16) * B(16x32), fp16 inputs, fp32 accumulate.  Lane l supplies 8 consecutive k of
// row/column l%32, k-group l/32.
__device__ __forceinline__ v16f mfma_f16_32x32x16(v8h a, v8h b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// D += A(16x32) * B(32x16), fp16 inputs, fp32 accumulate (half the result registers per flop of
// the 32x32x16 form: the chip sustains a higher clock on it).  Lane l supplies 8 consecutive k of
// row/column l%16, k-group l/16 (k = 8*(l/16) ...).  Result: 4 registers per lane, register r of
// lane l holds row 4*(l/16) + r, column l%16.
// Written as an instruction with the accumulator tied to its own registers: with 64 four-register
// accumulators per wavefront the compiler otherwise renames them from instruction to
// instruction and moves them between register files inside the k-loop.  The compiler does not
// know what the statement is, so it inserts none of the wait states the hardware leaves to
// software around matrix instructions:
//   - before: where two differently unrolled pieces of code keep an accumulator in different
//     registers, the compiler copies it (v_accvgpr_mov) directly in front of the statement, and a
//     matrix instruction must not read a register in the cycle after a vector instruction wrote
//     it (seen: the last-copied register of the tuple arrived stale) -- hence the wait
//     state in front, inside the statement, where nothing can be scheduled between;
//   - after: code that reads an accumulator written this way has to leave the matrix pipeline
//     time to drain first (mfma_drain() + pin()).
// WAIT = false leaves the wait state out: for code in which the compiler has been shown to put
// no copy in front of the statement (check_isa.py looks for exactly that).
template <bool WAIT = true> __device__ __forceinline__ void mfma_f16_16x16x32(v4f& c, v8h a, v8h b)
{
    if (WAIT)
        asm volatile("s_nop 0\n\tv_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else
        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
// More wait states than the longest matrix instruction needs before its result may be read.
// Volatile statements keep their order, so passing every accumulator through pin() after
// the drain keeps the compiler from reading it earlier.
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }
__device__ __forceinline__ void pin(v4f& c) { asm volatile("" : "+a"(c)); }

// D += A(16x4) * B(4x16), fp64.  Lane l supplies A[l%16][l/16] and B[l/16][l%16].
__device__ __forceinline__ v4d mfma_f64_16x16x4(double a, double b, v4d c)
{
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

}  // namespace dm
