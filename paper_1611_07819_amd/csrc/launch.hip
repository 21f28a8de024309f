// Kernel selection and launch.  The chooser sits beside the kernels because it encodes their
// preconditions (tile shapes, k-step divisibility, 16-byte alignment).
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>

#include "context.hpp"

namespace dm {

hipError_t launch_gemm_generic(const GemmPlan& p, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_reduce(const GemmPlan& p, int n_partials, double alpha, double beta, hipStream_t st);
hipError_t launch_conv_generic(const ConvPlan& p, int mode, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f32(const GemmPlan& p, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f64(const GemmPlan& p, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f16(const GemmPlan& p, double alpha, double beta, hipStream_t st);

namespace {

constexpr int kCUs = 256;

// Few tiles and a deep K: split K over workgroups so that the chip is filled; every split keeps
// at least 8 k-steps of 64.  The partial sums are reduced in a fixed order by a second kernel.
int32_t split_for(int64_t tiles, int64_t K)
{
    if (tiles * 2 > kCUs || K < 1024) return 1;
    int64_t want = kCUs / tiles, max_by_k = K / 512;
    return (int32_t)std::max<int64_t>(1, std::min<int64_t>({want, max_by_k, 32}));
}

bool all_multiple(const std::vector<int64_t>& v, int64_t q)
{
    for (int64_t x : v)
        if (x % q) return false;
    return true;
}

int64_t count_tiles(const SegView& v, int bm, int bn)
{
    int64_t tiles = 0;
    for (int64_t m : *v.mlen)
        for (int64_t n : *v.nlen) tiles += ((m + bm - 1) / bm) * ((n + bn - 1) / bn);
    return tiles;
}

// Optional "BMxBN" override for experiments, e.g. DMATH_TILE=128x64.
bool env_tile(int* bm, int* bn)
{
    const char* e = std::getenv("DMATH_TILE");
    if (!e) return false;
    return std::sscanf(e, "%dx%d", bm, bn) == 2;
}

}  // namespace

GemmChoice choose_gemm(const SegView& v)
{
    GemmChoice ch;  // generic 64x64x16
    const bool f32 = v.in_dtype == DMATH_F32 && all_multiple(*v.klen, 32);
    const bool f64 = v.in_dtype == DMATH_F64 && all_multiple(*v.klen, 16);
    if (v.policy == 0 && v.aligned16 && (f32 || f64)) {
        // Candidate shapes; take the one with the least serialised work per CU.  fp32: smaller
        // tiles move more bytes per flop, which costs clock at the power limit: 3 % handicap
        // (measured on configuration 2: 128x128 beats 128x64 when both fill the chip evenly).
        // fp64: the register-staged kernel runs two 128x64 workgroups per CU and is 14 % faster
        // that way on configuration 4, so there the larger tile carries the handicap.
        struct Shape {
            int bm, bn;
            bool needs_b_kcontig, f32_only;
        };
        const Shape shapes[] = {{128, 128, false, false}, {128, 64, false, false}, {128, 96, true, true}};
        double best_cost = -1;
        int ebm = 0, ebn = 0;
        const bool forced = env_tile(&ebm, &ebn);
        for (auto& s : shapes) {
            if (forced && (s.bm != ebm || s.bn != ebn)) continue;
            if ((s.needs_b_kcontig && !v.b_kcontig) || (s.f32_only && !f32)) continue;
            int64_t tiles = count_tiles(v, s.bm, s.bn);  // ragged last tiles count as whole ones
            double cost = (double)((tiles + kCUs - 1) / kCUs) * s.bm * s.bn;
            if (f32 && s.bm * s.bn < 128 * 128) cost *= 1.03;
            if (f64 && s.bm * s.bn >= 128 * 128) cost *= 1.03;
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                ch.kernel = f32 ? KERNEL_F32_128 : KERNEL_F64_128;
                ch.tile_m = s.bm;
                ch.tile_n = s.bn;
                ch.tile_k = f32 ? 32 : 16;
                ch.split_k = split_for(tiles, v.K);
            }
        }
        if (ch.kernel != KERNEL_GENERIC) return ch;
    }
    if (v.policy == 0 && v.aligned16 && v.in_dtype == DMATH_F16 && all_multiple(*v.klen, 64)) {
        const int shapes[][2] = {{256, 256}, {256, 128}, {128, 128}};
        int64_t best_cost = -1;
        int ebm = 0, ebn = 0;
        const bool forced = env_tile(&ebm, &ebn);
        for (auto& s : shapes) {
            if (forced && (s[0] != ebm || s[1] != ebn)) continue;
            int64_t tiles = count_tiles(v, s[0], s[1]);
            int64_t cost = ((tiles + kCUs - 1) / kCUs) * s[0] * s[1];
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                ch.kernel = KERNEL_F16_256;
                ch.tile_m = s[0];
                ch.tile_n = s[1];
                ch.tile_k = 64;
                ch.split_k = split_for(tiles, v.K);
            }
        }
        if (ch.kernel != KERNEL_GENERIC) return ch;
    }
    // Generic kernel.  Few C tiles and a deep K: split K so that the chip is filled.  The
    // partial sums are reduced in a fixed order by a second kernel.
    int64_t tiles = count_tiles(v, ch.tile_m, ch.tile_n);
    if (tiles < 128 && v.K >= 2048) {
        int64_t want = (512 + tiles - 1) / tiles;
        int64_t max_by_k = v.K / 512;
        ch.split_k = (int32_t)std::max<int64_t>(1, std::min<int64_t>({want, max_by_k, 32}));
    }
    return ch;
}

hipError_t launch_gemm(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    if (alpha == 0.0) return launch_gemm_reduce(p, 0, 0.0, beta, st);
    hipError_t e;
    switch (p.info.kernel) {
    case KERNEL_F32_128: e = launch_gemm_f32(p, alpha, beta, st); break;
    case KERNEL_F64_128: e = launch_gemm_f64(p, alpha, beta, st); break;
    case KERNEL_F16_256: e = launch_gemm_f16(p, alpha, beta, st); break;
    default: return launch_gemm_generic(p, alpha, beta, st);  // does its own reduction
    }
    if (e != hipSuccess || p.t.split_k == 1) return e;
    return launch_gemm_reduce(p, p.t.split_k, alpha, beta, st);
}

hipError_t launch_conv(const ConvPlan& p, int mode, double alpha, double beta, unsigned rewrite, hipStream_t st)
{
    if (p.kernel == 1 && alpha != 0.0) return launch_conv_f16(p, mode, alpha, beta, rewrite, st);
    return launch_conv_generic(p, mode, alpha, beta, st);
}

}  // namespace dm
