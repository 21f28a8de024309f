// MFMA-only micro-kernel: measures the matrix-core throughput the chip sustains (clocks under
// load are below the nominal 2.4 GHz), reported beside the nominal peak by the benchmark.
// Every wavefront issues independent chains of MFMA instructions on registers only; the
// operands rotate through pseudo-random values so that the inputs change from instruction to
// instruction as in a real GEMM (constant operands draw less power and sustain higher clocks:
// fp16 2450 TFLOP/s with constants, 1680 with changing random operands).
#include <hip/hip_runtime.h>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {
namespace {

__global__ __launch_bounds__(256) void peak_f32(float* out, int iters)
{
    v16f c[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    float a[4], b[4];
    uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q) {
        seed = seed * 1664525u + 1013904223u;
        a[q] = (float)(seed >> 8) * (1.0f / 16777216.0f);
        seed = seed * 1664525u + 1013904223u;
        b[q] = (float)(seed >> 8) * (1.0f / 16777216.0f) - 0.5f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] = mfma_f32_32x32x2(a[(u + i) & 3], b[u], c[i]);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 12345.678f) out[0] = s;  // keeps the chains alive; practically never true
}

// The operands rotate through eight different pseudo-random fragments per lane, so that the
// matrix cores see inputs that change from instruction to instruction as in a real GEMM
// (constant operands draw less power and sustain a higher clock).  The instruction is the one
// the large fp16 GEMM tiles use, v_mfma_f32_16x16x32_f16, sixteen independent chains.
__global__ __launch_bounds__(256) void peak_f16(float* out, int iters)
{
    v4f c[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 4; ++r) c[i][r] = 0.f;
    v8h a[4], b[4];
    uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q)
        for (int e = 0; e < 8; ++e) {
            seed = seed * 1664525u + 1013904223u;
            a[q][e] = (_Float16)((float)(seed >> 16) * (1.0f / 65536.0f));
            seed = seed * 1664525u + 1013904223u;
            b[q][e] = (_Float16)((float)(seed >> 16) * (1.0f / 65536.0f) - 0.5f);
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                c[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[(u + i) & 3], b[(u + (i >> 2)) & 3], c[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 4; ++r) s += c[i][r];
    if (s == 12345.678f) out[0] = s;
}

// The same on v_mfma_f32_32x32x16_f16 (the instruction of the fp16 convolution kernels and of
// the 64-row GEMM tiles): four chains of 16 accumulator registers, the same flops per iteration.
__global__ __launch_bounds__(256) void peak_f16_wide(float* out, int iters)
{
    v16f c[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    v8h a[4], b[4];
    uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q)
        for (int e = 0; e < 8; ++e) {
            seed = seed * 1664525u + 1013904223u;
            a[q][e] = (_Float16)((float)(seed >> 16) * (1.0f / 65536.0f));
            seed = seed * 1664525u + 1013904223u;
            b[q][e] = (_Float16)((float)(seed >> 16) * (1.0f / 65536.0f) - 0.5f);
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] = mfma_f16_32x32x16(a[(u + i) & 3], b[u], c[i]);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 12345.678f) out[0] = s;
}

// fp64: sixteen chains on accumulators in fixed accumulation registers, as in the pipelined
// kernels (mfma.hpp); with the builtin the compiler moved accumulators between register files
// around the instructions and the probe read 60 TFLOP/s where the GEMM kernel now runs at 67.
__global__ __launch_bounds__(256) void peak_f64(float* out, int iters)
{
    acc_fixed_begin();
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_f64_zero(i);
    double a[4], b[4];
    uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int q = 0; q < 4; ++q) {
        seed = seed * 1664525u + 1013904223u;
        a[q] = (double)seed * (1.0 / 4294967296.0) + (double)(seed >> 7) * 1e-12;
        seed = seed * 1664525u + 1013904223u;
        b[q] = (double)seed * (1.0 / 4294967296.0) - 0.5 + (double)(seed >> 9) * 1e-13;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) mfma_f64_fixed(i, a[i & 3], b[(i >> 2) & 3]);
    }
    mfma_drain_f64();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const v4d c = acc_f64_read(i);
        for (int r = 0; r < 4; ++r) s += c[r];
    }
    if (s == 12345.678) out[0] = (float)s;
}

}  // namespace

// Enqueues the micro-kernel; *flops receives the floating-point operations it performs.
// wide_f16: fp16 on the 32x32x16 instruction instead of 16x16x32.
hipError_t launch_mfma_peak(dmath_dtype_t dt, int iters, void* scratch, hipStream_t st, double* flops, bool wide_f16)
{
    const int blocks = 256 * 8, threads = 256;  // 8 workgroups of 4 wavefronts per CU
    const double waves = (double)blocks * threads / 64;
    float* out = static_cast<float*>(scratch);
    if (dt == DMATH_F32) {
        peak_f32<<<blocks, threads, 0, st>>>(out, iters);
        *flops = waves * iters * 16.0 * (2.0 * 32 * 32 * 2);
    } else if (dt == DMATH_F16 && wide_f16) {
        peak_f16_wide<<<blocks, threads, 0, st>>>(out, iters);
        *flops = waves * iters * 16.0 * (2.0 * 32 * 32 * 16);
    } else if (dt == DMATH_F16) {
        peak_f16<<<blocks, threads, 0, st>>>(out, iters);
        *flops = waves * iters * 64.0 * (2.0 * 16 * 16 * 32);
    } else {
        peak_f64<<<blocks, threads, 0, st>>>(out, iters);
        *flops = waves * iters * 16.0 * (2.0 * 16 * 16 * 4);
    }
    return hipGetLastError();
}

}  // namespace dm
