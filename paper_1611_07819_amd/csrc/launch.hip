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

// Few rows (a small batch against a large weight matrix): every m-segment fits a 64-row tile.
bool few_rows(const SegView& v)
{
    for (int64_t m : *v.mlen)
        if (m > 64) return false;
    return true;
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

namespace {

struct Shape {
    int32_t kernel, bm, bn, bk;
};

// Tile shapes of the specialised kernels whose preconditions this GEMM meets.
std::vector<Shape> specialised_shapes(const SegView& v)
{
    std::vector<Shape> out;
    if (v.policy != 0 || !v.aligned16 || !v.offsets32) return out;
    const bool f32 = v.in_dtype == DMATH_F32 && all_multiple(*v.klen, 32);
    const bool f64 = v.in_dtype == DMATH_F64 && all_multiple(*v.klen, 16);
    const bool f16 = v.in_dtype == DMATH_F16 && all_multiple(*v.klen, 64);
    if (f32 || f64) {
        const int32_t kern = f32 ? KERNEL_F32_128 : KERNEL_F64_128, bk = f32 ? 32 : 16;
        out.push_back({kern, 128, 128, bk});
        out.push_back({kern, 128, 64, bk});
        if (f32 && v.b_kcontig) out.push_back({kern, 128, 96, bk});  // wavefronts 4x1, k-major B only
        // few rows: 64-row tiles do half the matrix instructions of 128-row ones on padding
        if (few_rows(v)) {
            out.push_back({kern, 64, 128, bk});
            if (f32) out.push_back({kern, 64, 256, bk});
        }
    }
    if (f16) {
        out.push_back({KERNEL_F16_256, 256, 256, 64});
        out.push_back({KERNEL_F16_256, 256, 128, 64});
        out.push_back({KERNEL_F16_256, 128, 128, 64});
    }
    return out;
}

// Generic kernel.  Few C tiles and a deep K: split K so that the chip is filled.
int32_t generic_split(const SegView& v)
{
    const int64_t tiles = count_tiles(v, 64, 64);
    if (tiles >= 128 || v.K < 2048) return 1;
    const int64_t want = (512 + tiles - 1) / tiles, max_by_k = v.K / 512;
    return (int32_t)std::max<int64_t>(1, std::min<int64_t>({want, max_by_k, 32}));
}

}  // namespace

// The cost model: among the specialised shapes the one with the least serialised work per CU.
// fp32: smaller tiles move more bytes per flop, which costs clock at the power limit: 3 %
// handicap (measured on configuration 2: 128x128 beats 128x64 when both fill the chip evenly),
// except when neither operand is k unit-stride (TN): there every fragment is a 4-byte LDS read
// per MFMA, two 128x64 workgroups per CU hide those better and win by 2 %.
// fp64: 128x64 runs two workgroups per CU and is faster on configuration 4, so there the larger
// tile carries the handicap.  Ragged last tiles count as whole ones.
GemmChoice choose_gemm(const SegView& v)
{
    GemmChoice ch;  // generic 64x64x16
    double best_cost = -1;
    int ebm = 0, ebn = 0;
    const bool forced = env_tile(&ebm, &ebn);
    for (const Shape& s : specialised_shapes(v)) {
        if (forced && (s.bm != ebm || s.bn != ebn)) continue;
        const int64_t tiles = count_tiles(v, s.bm, s.bn);
        double cost = (double)((tiles + kCUs - 1) / kCUs) * s.bm * s.bn;
        const bool f32_strided = !v.a_kcontig && !v.b_kcontig;
        if (s.kernel == KERNEL_F32_128 && (s.bm * s.bn < 128 * 128) != f32_strided) cost *= 1.03;
        if (s.kernel == KERNEL_F64_128 && s.bm * s.bn >= 128 * 128) cost *= 1.03;
        // few rows: a 128-row tile multiplies 64 rows of padding (one or two workgroups per CU
        // measured the same, so the split stays at one round: half the partial sums)
        const bool short_tile = s.bm == 64;
        if (few_rows(v) && !short_tile) cost *= 2;
        if (short_tile && s.bn > 128) cost *= 1.03;
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            ch.kernel = s.kernel;
            ch.tile_m = s.bm;
            ch.tile_n = s.bn;
            ch.tile_k = s.bk;
            ch.split_k = split_for(tiles, v.K);
        }
    }
    if (ch.kernel == KERNEL_GENERIC) ch.split_k = generic_split(v);
    return ch;
}

// Every configuration worth a timing sample: each shape unsplit, with the cost model's split,
// and with the power-of-two splits that keep at least 512 of K per part and at most two rounds
// of workgroups; the generic kernel unsplit and with its own split.
std::vector<GemmChoice> gemm_candidates(const SegView& v)
{
    std::vector<GemmChoice> out;
    auto add = [&](int32_t kernel, int bm, int bn, int bk, int32_t split) {
        for (const GemmChoice& c : out)
            if (c.kernel == kernel && c.tile_m == bm && c.tile_n == bn && c.split_k == split) return;
        GemmChoice c;
        c.kernel = kernel;
        c.tile_m = bm;
        c.tile_n = bn;
        c.tile_k = bk;
        c.split_k = split;
        out.push_back(c);
    };
    for (const Shape& s : specialised_shapes(v)) {
        const int64_t tiles = count_tiles(v, s.bm, s.bn);
        add(s.kernel, s.bm, s.bn, s.bk, 1);
        add(s.kernel, s.bm, s.bn, s.bk, split_for(tiles, v.K));
        for (int32_t sp = 2; sp <= 32; sp *= 2)
            if (v.K / sp >= 512 && tiles * sp <= 2 * kCUs) add(s.kernel, s.bm, s.bn, s.bk, sp);
    }
    add(KERNEL_GENERIC, 64, 64, 16, 1);
    add(KERNEL_GENERIC, 64, 64, 16, generic_split(v));
    return out;
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
