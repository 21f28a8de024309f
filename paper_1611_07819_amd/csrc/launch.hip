// Kernel selection and launch.  The chooser sits beside the kernels because it encodes their
// preconditions (tile shapes, k-step divisibility, 16-byte alignment).
#include <hip/hip_runtime.h>

#include "context.hpp"

namespace dm {

hipError_t launch_gemm_generic(const GemmPlan& p, double alpha, double beta, hipStream_t st);
hipError_t launch_conv_generic(const ConvPlan& p, int mode, double alpha, double beta, hipStream_t st);

GemmChoice choose_gemm(const SegView& v)
{
    GemmChoice ch;  // generic 64x64x16
    // Few C tiles and a deep K: split K so that the chip is filled.  The partial sums are
    // reduced in a fixed order by a second kernel.
    int64_t tiles = 0;
    for (int64_t m : *v.mlen)
        for (int64_t n : *v.nlen) tiles += ((m + ch.tile_m - 1) / ch.tile_m) * ((n + ch.tile_n - 1) / ch.tile_n);
    if (tiles < 128 && v.K >= 2048) {
        int64_t want = (512 + tiles - 1) / tiles;
        int64_t max_by_k = v.K / 512;
        ch.split_k = (int32_t)std::max<int64_t>(1, std::min<int64_t>({want, max_by_k, 32}));
    }
    return ch;
}

hipError_t launch_gemm(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    return launch_gemm_generic(p, alpha, beta, st);
}

hipError_t launch_conv(const ConvPlan& p, int mode, double alpha, double beta, hipStream_t st)
{
    return launch_conv_generic(p, mode, alpha, beta, st);
}

}  // namespace dm
