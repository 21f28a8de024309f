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
// The pipelined fp64 kernels keep their accumulators in FIXED accumulation registers, a[8*idx ..
// 8*idx+7] for accumulator idx, which the compiler never sees as values: with the builtin, and
// also with an assembly statement whose accumulator is a tied operand, the register allocator kept
// part of the 8-register accumulators in VGPRs and copied them into and out of AGPRs around the
// instruction (128 v_accvgpr_write and 128 v_accvgpr_read per k-tile of a 128x128 tile), and every
// copy out waits for the 64-cycle instruction to finish: a third of the matrix cores' time.
//   acc_fixed_begin()  once, before anything else: tells the compiler that a0 .. a127 are taken
//                      (so that the kernel is given them and nothing of its own is kept there)
//   acc_f64_zero(idx)  accumulator idx = 0
//   mfma_f64_fixed(idx, a, b)   accumulator idx += A(16x4) * B(4x16); idx must be a constant after
//                      unrolling
//   acc_f64_read(idx)  the accumulator as a value; the caller drains the matrix cores first
//                      (mfma_drain_f64: the instruction takes 64 cycles, nothing interlocks the read)
// check_isa.py verifies on the compiler's output that nothing else touches these registers.
#define DM_A8(n) "a" #n "0", "a" #n "1", "a" #n "2", "a" #n "3", "a" #n "4", "a" #n "5", "a" #n "6", "a" #n "7", "a" #n "8", "a" #n "9"
__device__ __forceinline__ void acc_fixed_begin()
{
    asm volatile("" ::: "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", DM_A8(1), DM_A8(2), DM_A8(3),
                 DM_A8(4), DM_A8(5), DM_A8(6), DM_A8(7), DM_A8(8), DM_A8(9), DM_A8(10), DM_A8(11), "a120", "a121",
                 "a122", "a123", "a124", "a125", "a126", "a127");
}
#undef DM_A8
// (the register numbers are spelled out: an immediate operand above 64 would be printed in hex)
__device__ __forceinline__ void acc_f64_zero(int idx)
{
    switch (idx) {
    case 0: asm volatile("v_accvgpr_write_b32 a0, 0\n\tv_accvgpr_write_b32 a1, 0\n\tv_accvgpr_write_b32 a2, 0\n\tv_accvgpr_write_b32 a3, 0\n\tv_accvgpr_write_b32 a4, 0\n\tv_accvgpr_write_b32 a5, 0\n\tv_accvgpr_write_b32 a6, 0\n\tv_accvgpr_write_b32 a7, 0"); break;
    case 1: asm volatile("v_accvgpr_write_b32 a8, 0\n\tv_accvgpr_write_b32 a9, 0\n\tv_accvgpr_write_b32 a10, 0\n\tv_accvgpr_write_b32 a11, 0\n\tv_accvgpr_write_b32 a12, 0\n\tv_accvgpr_write_b32 a13, 0\n\tv_accvgpr_write_b32 a14, 0\n\tv_accvgpr_write_b32 a15, 0"); break;
    case 2: asm volatile("v_accvgpr_write_b32 a16, 0\n\tv_accvgpr_write_b32 a17, 0\n\tv_accvgpr_write_b32 a18, 0\n\tv_accvgpr_write_b32 a19, 0\n\tv_accvgpr_write_b32 a20, 0\n\tv_accvgpr_write_b32 a21, 0\n\tv_accvgpr_write_b32 a22, 0\n\tv_accvgpr_write_b32 a23, 0"); break;
    case 3: asm volatile("v_accvgpr_write_b32 a24, 0\n\tv_accvgpr_write_b32 a25, 0\n\tv_accvgpr_write_b32 a26, 0\n\tv_accvgpr_write_b32 a27, 0\n\tv_accvgpr_write_b32 a28, 0\n\tv_accvgpr_write_b32 a29, 0\n\tv_accvgpr_write_b32 a30, 0\n\tv_accvgpr_write_b32 a31, 0"); break;
    case 4: asm volatile("v_accvgpr_write_b32 a32, 0\n\tv_accvgpr_write_b32 a33, 0\n\tv_accvgpr_write_b32 a34, 0\n\tv_accvgpr_write_b32 a35, 0\n\tv_accvgpr_write_b32 a36, 0\n\tv_accvgpr_write_b32 a37, 0\n\tv_accvgpr_write_b32 a38, 0\n\tv_accvgpr_write_b32 a39, 0"); break;
    case 5: asm volatile("v_accvgpr_write_b32 a40, 0\n\tv_accvgpr_write_b32 a41, 0\n\tv_accvgpr_write_b32 a42, 0\n\tv_accvgpr_write_b32 a43, 0\n\tv_accvgpr_write_b32 a44, 0\n\tv_accvgpr_write_b32 a45, 0\n\tv_accvgpr_write_b32 a46, 0\n\tv_accvgpr_write_b32 a47, 0"); break;
    case 6: asm volatile("v_accvgpr_write_b32 a48, 0\n\tv_accvgpr_write_b32 a49, 0\n\tv_accvgpr_write_b32 a50, 0\n\tv_accvgpr_write_b32 a51, 0\n\tv_accvgpr_write_b32 a52, 0\n\tv_accvgpr_write_b32 a53, 0\n\tv_accvgpr_write_b32 a54, 0\n\tv_accvgpr_write_b32 a55, 0"); break;
    case 7: asm volatile("v_accvgpr_write_b32 a56, 0\n\tv_accvgpr_write_b32 a57, 0\n\tv_accvgpr_write_b32 a58, 0\n\tv_accvgpr_write_b32 a59, 0\n\tv_accvgpr_write_b32 a60, 0\n\tv_accvgpr_write_b32 a61, 0\n\tv_accvgpr_write_b32 a62, 0\n\tv_accvgpr_write_b32 a63, 0"); break;
    case 8: asm volatile("v_accvgpr_write_b32 a64, 0\n\tv_accvgpr_write_b32 a65, 0\n\tv_accvgpr_write_b32 a66, 0\n\tv_accvgpr_write_b32 a67, 0\n\tv_accvgpr_write_b32 a68, 0\n\tv_accvgpr_write_b32 a69, 0\n\tv_accvgpr_write_b32 a70, 0\n\tv_accvgpr_write_b32 a71, 0"); break;
    case 9: asm volatile("v_accvgpr_write_b32 a72, 0\n\tv_accvgpr_write_b32 a73, 0\n\tv_accvgpr_write_b32 a74, 0\n\tv_accvgpr_write_b32 a75, 0\n\tv_accvgpr_write_b32 a76, 0\n\tv_accvgpr_write_b32 a77, 0\n\tv_accvgpr_write_b32 a78, 0\n\tv_accvgpr_write_b32 a79, 0"); break;
    case 10: asm volatile("v_accvgpr_write_b32 a80, 0\n\tv_accvgpr_write_b32 a81, 0\n\tv_accvgpr_write_b32 a82, 0\n\tv_accvgpr_write_b32 a83, 0\n\tv_accvgpr_write_b32 a84, 0\n\tv_accvgpr_write_b32 a85, 0\n\tv_accvgpr_write_b32 a86, 0\n\tv_accvgpr_write_b32 a87, 0"); break;
    case 11: asm volatile("v_accvgpr_write_b32 a88, 0\n\tv_accvgpr_write_b32 a89, 0\n\tv_accvgpr_write_b32 a90, 0\n\tv_accvgpr_write_b32 a91, 0\n\tv_accvgpr_write_b32 a92, 0\n\tv_accvgpr_write_b32 a93, 0\n\tv_accvgpr_write_b32 a94, 0\n\tv_accvgpr_write_b32 a95, 0"); break;
    case 12: asm volatile("v_accvgpr_write_b32 a96, 0\n\tv_accvgpr_write_b32 a97, 0\n\tv_accvgpr_write_b32 a98, 0\n\tv_accvgpr_write_b32 a99, 0\n\tv_accvgpr_write_b32 a100, 0\n\tv_accvgpr_write_b32 a101, 0\n\tv_accvgpr_write_b32 a102, 0\n\tv_accvgpr_write_b32 a103, 0"); break;
    case 13: asm volatile("v_accvgpr_write_b32 a104, 0\n\tv_accvgpr_write_b32 a105, 0\n\tv_accvgpr_write_b32 a106, 0\n\tv_accvgpr_write_b32 a107, 0\n\tv_accvgpr_write_b32 a108, 0\n\tv_accvgpr_write_b32 a109, 0\n\tv_accvgpr_write_b32 a110, 0\n\tv_accvgpr_write_b32 a111, 0"); break;
    case 14: asm volatile("v_accvgpr_write_b32 a112, 0\n\tv_accvgpr_write_b32 a113, 0\n\tv_accvgpr_write_b32 a114, 0\n\tv_accvgpr_write_b32 a115, 0\n\tv_accvgpr_write_b32 a116, 0\n\tv_accvgpr_write_b32 a117, 0\n\tv_accvgpr_write_b32 a118, 0\n\tv_accvgpr_write_b32 a119, 0"); break;
    case 15: asm volatile("v_accvgpr_write_b32 a120, 0\n\tv_accvgpr_write_b32 a121, 0\n\tv_accvgpr_write_b32 a122, 0\n\tv_accvgpr_write_b32 a123, 0\n\tv_accvgpr_write_b32 a124, 0\n\tv_accvgpr_write_b32 a125, 0\n\tv_accvgpr_write_b32 a126, 0\n\tv_accvgpr_write_b32 a127, 0"); break;
    }
}
__device__ __forceinline__ void mfma_f64_fixed(int idx, double a, double b)
{
    switch (idx) {
    case 0: asm volatile("v_mfma_f64_16x16x4_f64 a[0:7], %0, %1, a[0:7]" ::"v"(a), "v"(b)); break;
    case 1: asm volatile("v_mfma_f64_16x16x4_f64 a[8:15], %0, %1, a[8:15]" ::"v"(a), "v"(b)); break;
    case 2: asm volatile("v_mfma_f64_16x16x4_f64 a[16:23], %0, %1, a[16:23]" ::"v"(a), "v"(b)); break;
    case 3: asm volatile("v_mfma_f64_16x16x4_f64 a[24:31], %0, %1, a[24:31]" ::"v"(a), "v"(b)); break;
    case 4: asm volatile("v_mfma_f64_16x16x4_f64 a[32:39], %0, %1, a[32:39]" ::"v"(a), "v"(b)); break;
    case 5: asm volatile("v_mfma_f64_16x16x4_f64 a[40:47], %0, %1, a[40:47]" ::"v"(a), "v"(b)); break;
    case 6: asm volatile("v_mfma_f64_16x16x4_f64 a[48:55], %0, %1, a[48:55]" ::"v"(a), "v"(b)); break;
    case 7: asm volatile("v_mfma_f64_16x16x4_f64 a[56:63], %0, %1, a[56:63]" ::"v"(a), "v"(b)); break;
    case 8: asm volatile("v_mfma_f64_16x16x4_f64 a[64:71], %0, %1, a[64:71]" ::"v"(a), "v"(b)); break;
    case 9: asm volatile("v_mfma_f64_16x16x4_f64 a[72:79], %0, %1, a[72:79]" ::"v"(a), "v"(b)); break;
    case 10: asm volatile("v_mfma_f64_16x16x4_f64 a[80:87], %0, %1, a[80:87]" ::"v"(a), "v"(b)); break;
    case 11: asm volatile("v_mfma_f64_16x16x4_f64 a[88:95], %0, %1, a[88:95]" ::"v"(a), "v"(b)); break;
    case 12: asm volatile("v_mfma_f64_16x16x4_f64 a[96:103], %0, %1, a[96:103]" ::"v"(a), "v"(b)); break;
    case 13: asm volatile("v_mfma_f64_16x16x4_f64 a[104:111], %0, %1, a[104:111]" ::"v"(a), "v"(b)); break;
    case 14: asm volatile("v_mfma_f64_16x16x4_f64 a[112:119], %0, %1, a[112:119]" ::"v"(a), "v"(b)); break;
    case 15: asm volatile("v_mfma_f64_16x16x4_f64 a[120:127], %0, %1, a[120:127]" ::"v"(a), "v"(b)); break;
    }
}
__device__ __forceinline__ void mfma_drain_f64()
{
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
}
__device__ __forceinline__ v4d acc_f64_read(int idx)
{
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    switch (idx) {
    case 0: asm volatile("v_accvgpr_read_b32 %0, a0\n\tv_accvgpr_read_b32 %1, a1\n\tv_accvgpr_read_b32 %2, a2\n\tv_accvgpr_read_b32 %3, a3\n\tv_accvgpr_read_b32 %4, a4\n\tv_accvgpr_read_b32 %5, a5\n\tv_accvgpr_read_b32 %6, a6\n\tv_accvgpr_read_b32 %7, a7" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 1: asm volatile("v_accvgpr_read_b32 %0, a8\n\tv_accvgpr_read_b32 %1, a9\n\tv_accvgpr_read_b32 %2, a10\n\tv_accvgpr_read_b32 %3, a11\n\tv_accvgpr_read_b32 %4, a12\n\tv_accvgpr_read_b32 %5, a13\n\tv_accvgpr_read_b32 %6, a14\n\tv_accvgpr_read_b32 %7, a15" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 2: asm volatile("v_accvgpr_read_b32 %0, a16\n\tv_accvgpr_read_b32 %1, a17\n\tv_accvgpr_read_b32 %2, a18\n\tv_accvgpr_read_b32 %3, a19\n\tv_accvgpr_read_b32 %4, a20\n\tv_accvgpr_read_b32 %5, a21\n\tv_accvgpr_read_b32 %6, a22\n\tv_accvgpr_read_b32 %7, a23" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 3: asm volatile("v_accvgpr_read_b32 %0, a24\n\tv_accvgpr_read_b32 %1, a25\n\tv_accvgpr_read_b32 %2, a26\n\tv_accvgpr_read_b32 %3, a27\n\tv_accvgpr_read_b32 %4, a28\n\tv_accvgpr_read_b32 %5, a29\n\tv_accvgpr_read_b32 %6, a30\n\tv_accvgpr_read_b32 %7, a31" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 4: asm volatile("v_accvgpr_read_b32 %0, a32\n\tv_accvgpr_read_b32 %1, a33\n\tv_accvgpr_read_b32 %2, a34\n\tv_accvgpr_read_b32 %3, a35\n\tv_accvgpr_read_b32 %4, a36\n\tv_accvgpr_read_b32 %5, a37\n\tv_accvgpr_read_b32 %6, a38\n\tv_accvgpr_read_b32 %7, a39" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 5: asm volatile("v_accvgpr_read_b32 %0, a40\n\tv_accvgpr_read_b32 %1, a41\n\tv_accvgpr_read_b32 %2, a42\n\tv_accvgpr_read_b32 %3, a43\n\tv_accvgpr_read_b32 %4, a44\n\tv_accvgpr_read_b32 %5, a45\n\tv_accvgpr_read_b32 %6, a46\n\tv_accvgpr_read_b32 %7, a47" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 6: asm volatile("v_accvgpr_read_b32 %0, a48\n\tv_accvgpr_read_b32 %1, a49\n\tv_accvgpr_read_b32 %2, a50\n\tv_accvgpr_read_b32 %3, a51\n\tv_accvgpr_read_b32 %4, a52\n\tv_accvgpr_read_b32 %5, a53\n\tv_accvgpr_read_b32 %6, a54\n\tv_accvgpr_read_b32 %7, a55" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 7: asm volatile("v_accvgpr_read_b32 %0, a56\n\tv_accvgpr_read_b32 %1, a57\n\tv_accvgpr_read_b32 %2, a58\n\tv_accvgpr_read_b32 %3, a59\n\tv_accvgpr_read_b32 %4, a60\n\tv_accvgpr_read_b32 %5, a61\n\tv_accvgpr_read_b32 %6, a62\n\tv_accvgpr_read_b32 %7, a63" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 8: asm volatile("v_accvgpr_read_b32 %0, a64\n\tv_accvgpr_read_b32 %1, a65\n\tv_accvgpr_read_b32 %2, a66\n\tv_accvgpr_read_b32 %3, a67\n\tv_accvgpr_read_b32 %4, a68\n\tv_accvgpr_read_b32 %5, a69\n\tv_accvgpr_read_b32 %6, a70\n\tv_accvgpr_read_b32 %7, a71" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 9: asm volatile("v_accvgpr_read_b32 %0, a72\n\tv_accvgpr_read_b32 %1, a73\n\tv_accvgpr_read_b32 %2, a74\n\tv_accvgpr_read_b32 %3, a75\n\tv_accvgpr_read_b32 %4, a76\n\tv_accvgpr_read_b32 %5, a77\n\tv_accvgpr_read_b32 %6, a78\n\tv_accvgpr_read_b32 %7, a79" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 10: asm volatile("v_accvgpr_read_b32 %0, a80\n\tv_accvgpr_read_b32 %1, a81\n\tv_accvgpr_read_b32 %2, a82\n\tv_accvgpr_read_b32 %3, a83\n\tv_accvgpr_read_b32 %4, a84\n\tv_accvgpr_read_b32 %5, a85\n\tv_accvgpr_read_b32 %6, a86\n\tv_accvgpr_read_b32 %7, a87" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 11: asm volatile("v_accvgpr_read_b32 %0, a88\n\tv_accvgpr_read_b32 %1, a89\n\tv_accvgpr_read_b32 %2, a90\n\tv_accvgpr_read_b32 %3, a91\n\tv_accvgpr_read_b32 %4, a92\n\tv_accvgpr_read_b32 %5, a93\n\tv_accvgpr_read_b32 %6, a94\n\tv_accvgpr_read_b32 %7, a95" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 12: asm volatile("v_accvgpr_read_b32 %0, a96\n\tv_accvgpr_read_b32 %1, a97\n\tv_accvgpr_read_b32 %2, a98\n\tv_accvgpr_read_b32 %3, a99\n\tv_accvgpr_read_b32 %4, a100\n\tv_accvgpr_read_b32 %5, a101\n\tv_accvgpr_read_b32 %6, a102\n\tv_accvgpr_read_b32 %7, a103" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 13: asm volatile("v_accvgpr_read_b32 %0, a104\n\tv_accvgpr_read_b32 %1, a105\n\tv_accvgpr_read_b32 %2, a106\n\tv_accvgpr_read_b32 %3, a107\n\tv_accvgpr_read_b32 %4, a108\n\tv_accvgpr_read_b32 %5, a109\n\tv_accvgpr_read_b32 %6, a110\n\tv_accvgpr_read_b32 %7, a111" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 14: asm volatile("v_accvgpr_read_b32 %0, a112\n\tv_accvgpr_read_b32 %1, a113\n\tv_accvgpr_read_b32 %2, a114\n\tv_accvgpr_read_b32 %3, a115\n\tv_accvgpr_read_b32 %4, a116\n\tv_accvgpr_read_b32 %5, a117\n\tv_accvgpr_read_b32 %6, a118\n\tv_accvgpr_read_b32 %7, a119" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    case 15: asm volatile("v_accvgpr_read_b32 %0, a120\n\tv_accvgpr_read_b32 %1, a121\n\tv_accvgpr_read_b32 %2, a122\n\tv_accvgpr_read_b32 %3, a123\n\tv_accvgpr_read_b32 %4, a124\n\tv_accvgpr_read_b32 %5, a125\n\tv_accvgpr_read_b32 %6, a126\n\tv_accvgpr_read_b32 %7, a127" : "=v"(w[0]), "=v"(w[1]), "=v"(w[2]), "=v"(w[3]), "=v"(w[4]), "=v"(w[5]), "=v"(w[6]), "=v"(w[7])); break;
    }
    v4d c;
#pragma unroll
    for (int e = 0; e < 4; ++e) c[e] = __builtin_bit_cast(double, ((uint64_t)w[2 * e + 1] << 32) | w[2 * e]);
    return c;
}

// The same for the fp16 16x16x32 instruction where the compiler cannot be kept from renaming tied
// accumulators (the convolution's weight gradient: its walk holds many per-lane values, and the
// copies between renamed accumulators landed right behind the matrix instructions that write
// them): accumulator idx < 32 lives in a[4*idx .. 4*idx+3].  acc_fixed_begin() reserves a0 .. a127
// for these as well; acc_fixed_marker() leaves a comment in the assembly by which check_isa.py
// knows that in this kernel nothing but the three statements below may name an accumulation
// register.
#define DM_ACC4_LIST(X) \
    X(0, 0, 1, 2, 3) X(1, 4, 5, 6, 7) X(2, 8, 9, 10, 11) X(3, 12, 13, 14, 15) \
    X(4, 16, 17, 18, 19) X(5, 20, 21, 22, 23) X(6, 24, 25, 26, 27) X(7, 28, 29, 30, 31) \
    X(8, 32, 33, 34, 35) X(9, 36, 37, 38, 39) X(10, 40, 41, 42, 43) X(11, 44, 45, 46, 47) \
    X(12, 48, 49, 50, 51) X(13, 52, 53, 54, 55) X(14, 56, 57, 58, 59) X(15, 60, 61, 62, 63) \
    X(16, 64, 65, 66, 67) X(17, 68, 69, 70, 71) X(18, 72, 73, 74, 75) X(19, 76, 77, 78, 79) \
    X(20, 80, 81, 82, 83) X(21, 84, 85, 86, 87) X(22, 88, 89, 90, 91) X(23, 92, 93, 94, 95) \
    X(24, 96, 97, 98, 99) X(25, 100, 101, 102, 103) X(26, 104, 105, 106, 107) X(27, 108, 109, 110, 111) \
    X(28, 112, 113, 114, 115) X(29, 116, 117, 118, 119) X(30, 120, 121, 122, 123) X(31, 124, 125, 126, 127)
__device__ __forceinline__ void acc_fixed_marker() { asm volatile("; dmath: fixed accumulation registers"); }
__device__ __forceinline__ void acc_f16_zero(int idx)
{
    switch (idx) {
#define X(I, R0, R1, R2, R3)                                                                                   \
    case I:                                                                                                    \
        asm volatile("v_accvgpr_write_b32 a" #R0 ", 0\n\tv_accvgpr_write_b32 a" #R1 ", 0\n\tv_accvgpr_write_b32 a" #R2 \
                     ", 0\n\tv_accvgpr_write_b32 a" #R3 ", 0");                                                \
        break;
        DM_ACC4_LIST(X)
#undef X
    }
}
__device__ __forceinline__ void mfma_f16_fixed(int idx, v8h a, v8h b)
{
    switch (idx) {
#define X(I, R0, R1, R2, R3)                                                                                    \
    case I:                                                                                                     \
        asm volatile("v_mfma_f32_16x16x32_f16 a[" #R0 ":" #R3 "], %0, %1, a[" #R0 ":" #R3 "]" ::"v"(a), "v"(b)); \
        break;
        DM_ACC4_LIST(X)
#undef X
    }
}
__device__ __forceinline__ v4f acc_f16_read(int idx)
{
    v4f c = {0.f, 0.f, 0.f, 0.f};
    switch (idx) {
#define X(I, R0, R1, R2, R3)                                                                                  \
    case I:                                                                                                   \
        asm volatile("v_accvgpr_read_b32 %0, a" #R0 "\n\tv_accvgpr_read_b32 %1, a" #R1 "\n\tv_accvgpr_read_b32 %2, a" #R2 \
                     "\n\tv_accvgpr_read_b32 %3, a" #R3                                                       \
                     : "=v"(c[0]), "=v"(c[1]), "=v"(c[2]), "=v"(c[3]));                                         \
        break;
        DM_ACC4_LIST(X)
#undef X
    }
    return c;
}
#undef DM_ACC4_LIST

}  // namespace dm
