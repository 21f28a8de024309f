// Kernel selection and launch.  The chooser sits beside the kernels because it encodes their
// preconditions (tile shapes, k-step divisibility, 16-byte alignment).
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>

#include "context.hpp"

namespace dm {

hipError_t launch_gemm_generic(const GemmPlan& p, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_reduce(const GemmPlan& p, const GemmTables& t, int n_partials, double alpha, double beta,
                              hipStream_t st);
hipError_t launch_conv_generic(const ConvPlan& p, int mode, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f32(const GemmPlan& p, const GemmTables& t, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f64(const GemmPlan& p, const GemmTables& t, double alpha, double beta, hipStream_t st);
hipError_t launch_gemm_f16(const GemmPlan& p, const GemmTables& t, double alpha, double beta, hipStream_t st);

namespace {

constexpr int kCUs = 256;

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

// A tile shape of a specialised kernel: how many of its workgroups fit on a CU (LDS), and the
// fraction of the precision's practical rate it reaches when the chip is full (measured).
struct Shape {
    int32_t kernel, bm, bn, bk;
    int32_t per_cu;
    double efficiency;
};

// Tile shapes of the specialised kernels whose preconditions this GEMM meets.
std::vector<Shape> specialised_shapes(const SegView& v)
{
    std::vector<Shape> out;
    if (v.policy != 0 || !v.aligned16 || !v.offsets32) return out;
    const bool f32 = v.in_dtype == DMATH_F32 && all_multiple(*v.klen, 32);
    const bool f64 = v.in_dtype == DMATH_F64 && all_multiple(*v.klen, 16);
    const bool f16 = v.in_dtype == DMATH_F16 && all_multiple(*v.klen, 64);
    const bool strided = !v.a_kcontig && !v.b_kcontig;  // neither operand k unit-stride (TN)
    if (f32) {
        // on a full chip the two run level (configuration 2); where the chip is not full, and for
        // TN (every fragment a 4-byte LDS read per MFMA), two 128x64 workgroups per CU cover each
        // other's fill, drain and LDS latency: 6-9 % on batch sizes of 256-1024
        // (128x128 against 128x64 on twelve shapes whose last round is split: 1.5-7 % slower)
        out.push_back({KERNEL_F32_128, 128, 128, 32, 1, strided ? 0.94 : 0.95});
        out.push_back({KERNEL_F32_128, 128, 64, 32, 2, 1.0});
        if (v.b_kcontig) out.push_back({KERNEL_F32_128, 128, 96, 32, 1, 0.97});  // wavefronts 4x1, k-major B only
    }
    if (f64) {  // two 128x64 workgroups per CU are faster than one 128x128: 3 % on configuration 4,
                // 11-18 % on shapes with a partial last round
        out.push_back({KERNEL_F64_128, 128, 128, 16, 1, 0.9});
        out.push_back({KERNEL_F64_128, 128, 64, 16, 2, 1.0});
    }
    // few rows: 64-row tiles do half the matrix instructions of 128-row ones on padding
    if ((f32 || f64) && few_rows(v)) {
        out.push_back({f32 ? KERNEL_F32_128 : KERNEL_F64_128, 64, 128, f32 ? 32 : 16, 2, 0.95});
        if (f32) out.push_back({KERNEL_F32_128, 64, 256, 32, 1, 0.92});
    }
    if (f16) {  // 128x128 reads twice the LDS bytes per flop of the 256-wide tiles
        out.push_back({KERNEL_F16_256, 256, 256, 64, 1, 1.0});
        out.push_back({KERNEL_F16_256, 256, 128, 64, 1, 1.0});
        out.push_back({KERNEL_F16_256, 128, 128, 64, 2, 0.7});
        if (few_rows(v)) {  // half the padding rows and half the partial sums of a 128-row tile
            out.push_back({KERNEL_F16_256, 64, 128, 64, 2, 0.5});
            out.push_back({KERNEL_F16_256, 64, 64, 64, 3, 0.4});
        }
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

// The cost model.  Time of a (shape, split) pair =
//     workgroups on the busiest CU x work of one workgroup / (CU rate x shape efficiency x occupancy)
//   + the reduction kernel (launch + reading the partial sums and writing C) when split > 1,
// with the practical per-CU rates measured on configurations 2-4, occupancy 0.9 (fp32) or 0.8 (fp64) when an fp32 /
// fp64 shape that wants two workgroups per CU gets only one, ragged tiles counted as whole ones.
// Checked against timing samples on 30 shapes per precision: within 10 % of the best sample.
double modelled_seconds(const SegView& v, const Shape& s, int32_t split)
{
    const double cu_flops = s.kernel == KERNEL_F16_256 ? 3.9e12 : s.kernel == KERNEL_F32_128 ? 0.512e12 : 0.23e12;
    const int64_t wgs = count_tiles(v, s.bm, s.bn) * split;
    // workgroups are dispatched in rounds that fill every slot of the chip (per_cu per CU)
    const int64_t slots = (int64_t)kCUs * s.per_cu;
    const int64_t busiest = wgs <= kCUs ? 1 : (wgs + slots - 1) / slots * s.per_cu;
    const double alone = s.kernel == KERNEL_F32_128 ? 0.9 : 0.8;  // a CU with one workgroup of a shape that fits two
    const double occupancy = s.kernel != KERNEL_F16_256 && s.per_cu > 1 && busiest < s.per_cu ? alone : 1.0;
    const double wg_flops = 2.0 * s.bm * s.bn * ((double)v.K / split);
    // + what a workgroup spends outside its k-loop (filling the load ring, storing its tile),
    // which the workgroups that share a CU overlap
    const int64_t rounds = (busiest + s.per_cu - 1) / s.per_cu;
    double t = busiest * wg_flops / (cu_flops * s.efficiency * occupancy) + rounds * 1.5e-6;
    if (split > 1) {
        const double acc_bytes = v.in_dtype == DMATH_F64 ? 8 : 4;
        t += 3e-6 + (split + 1.0) * v.M * v.N * acc_bytes / 3e12;
    }
    return t;
}

// Several rounds of workgroups and a last round that is not full: the tiles of the full rounds
// run the whole k-loop (one launch), only the tiles left over are split (a second launch and the
// reduction over those tiles) into 2, 4, 8 or 16 parts of at least 128 of K each; the parts may
// take several rounds of their own, each 1/parts as long (measured, fp32 1280x4096x4096: 512 us
// unsplit, 353 / 328 / 335 / 345 us with 2 / 4 / 8 / 16 parts).  Returns the tiles of the full
// rounds (0: does not apply) and the best part count with the model's time.
int32_t tail_split(const SegView& v, const Shape& s, int32_t* split, double* seconds)
{
    const int64_t tiles = count_tiles(v, s.bm, s.bn), slots = (int64_t)kCUs * s.per_cu;
    const int64_t full = tiles / slots * slots, left = tiles - full;
    if (full == 0 || left == 0) return 0;
    const double cu_flops = s.kernel == KERNEL_F16_256 ? 3.9e12 : s.kernel == KERNEL_F32_128 ? 0.512e12 : 0.23e12;
    const double wg_flops = 2.0 * s.bm * s.bn * (double)v.K;
    const int64_t rounds = full / slots;
    const double t_full = rounds * s.per_cu * wg_flops / (cu_flops * s.efficiency) + rounds * 1.5e-6;
    const double alone = s.kernel == KERNEL_F32_128 ? 0.9 : 0.8;
    const double acc_bytes = v.in_dtype == DMATH_F64 ? 8 : 4;
    double best = -1;
    for (int32_t sp = 2; sp <= 16 && v.K / sp >= 128; sp *= 2) {
        const int64_t wgs = left * sp;
        const int64_t busiest = wgs <= kCUs ? 1 : (wgs + slots - 1) / slots * s.per_cu;
        const double occupancy = s.kernel != KERNEL_F16_256 && s.per_cu > 1 && busiest < s.per_cu ? alone : 1.0;
        const int64_t tail_rounds = (busiest + s.per_cu - 1) / s.per_cu;
        double t = t_full + busiest * wg_flops / sp / (cu_flops * s.efficiency * occupancy) + tail_rounds * 1.5e-6;
        t += 2e-6 + 3e-6 + (sp + 1.0) * left * s.bm * s.bn * acc_bytes / 3e12;  // second launch, reduction
        if (best < 0 || t < best) {
            best = t;
            *split = sp;
        }
    }
    if (best < 0) return 0;
    *seconds = best;
    return (int32_t)full;
}

// Splits are powers of two that leave at least 128 of K per part (64 where K itself is at most
// 256: a 256^3 fp32 product on 8 tiles takes 12.2 us unsplit, 9.6 us in two parts and 7.4 us in
// four, each part two k-tiles deep); a split has to be 3 % better than the one before to pay for
// its workspace.
int32_t best_split(const SegView& v, const Shape& s, double* seconds)
{
    int32_t best = 1;
    double best_t = modelled_seconds(v, s, 1);
    const int64_t min_k = v.K <= 256 ? 64 : 128;
    for (int32_t sp = 2; sp <= 32; sp *= 2) {
        if (v.K / sp < min_k) break;
        const double t = modelled_seconds(v, s, sp);
        if (t < best_t * 0.97) {
            best_t = t;
            best = sp;
        }
    }
    if (seconds) *seconds = best_t;
    return best;
}

}  // namespace

GemmChoice choose_gemm(const SegView& v)
{
    GemmChoice ch;  // generic 64x64x16
    double best_t = -1;
    int ebm = 0, ebn = 0;
    const bool forced = env_tile(&ebm, &ebn);
    for (const Shape& s : specialised_shapes(v)) {
        if (forced && (s.bm != ebm || s.bn != ebn)) continue;
        double t;
        const int32_t split = best_split(v, s, &t);
        if (best_t < 0 || t < best_t) {
            best_t = t;
            ch.kernel = s.kernel;
            ch.tile_m = s.bm;
            ch.tile_n = s.bn;
            ch.tile_k = s.bk;
            ch.split_k = split;
            ch.full_tiles = 0;
        }
        // (a split of the last round only takes little workspace: it replaces another such
        // choice as soon as it is faster, anything else when it is 3 % faster)
        int32_t tsplit = 1;
        double tt = 0;
        const int32_t full = tail_split(v, s, &tsplit, &tt);
        if (full > 0 && tt < (ch.full_tiles > 0 ? 1.0 : 0.97) * best_t) {
            best_t = tt;
            ch.kernel = s.kernel;
            ch.tile_m = s.bm;
            ch.tile_n = s.bn;
            ch.tile_k = s.bk;
            ch.split_k = tsplit;
            ch.full_tiles = full;
        }
    }
    if (ch.kernel == KERNEL_GENERIC) ch.split_k = generic_split(v);
    // optional override for experiments and tests: DMATH_GEMM_SPLIT=4 (every tile) or =4t (only
    // the tiles after the last full round of workgroups)
    if (const char* e = std::getenv("DMATH_GEMM_SPLIT")) {
        const int forced_split = std::atoi(e);
        if (ch.kernel != KERNEL_GENERIC && forced_split >= 1 && forced_split <= 32 && v.K / forced_split >= 64) {
            ch.split_k = forced_split;
            ch.full_tiles = 0;
            if (std::strchr(e, 't'))
                for (const Shape& s : specialised_shapes(v))
                    if (s.kernel == ch.kernel && s.bm == ch.tile_m && s.bn == ch.tile_n) {
                        const int64_t slots = (int64_t)kCUs * s.per_cu;
                        ch.full_tiles = (int32_t)(count_tiles(v, s.bm, s.bn) / slots * slots);
                    }
        }
    }
    return ch;
}

// Every configuration worth a timing sample: each shape unsplit, with the cost model's split,
// with the power-of-two splits that keep at least 128 of K per part and at most four rounds
// of workgroups, and with only the tiles after the last full round split; the generic kernel unsplit and with its own split.
std::vector<GemmChoice> gemm_candidates(const SegView& v)
{
    std::vector<GemmChoice> out;
    auto add = [&](int32_t kernel, int bm, int bn, int bk, int32_t split, int32_t full_tiles = 0) {
        for (const GemmChoice& c : out)
            if (c.kernel == kernel && c.tile_m == bm && c.tile_n == bn && c.split_k == split &&
                c.full_tiles == full_tiles)
                return;
        GemmChoice c;
        c.kernel = kernel;
        c.tile_m = bm;
        c.tile_n = bn;
        c.tile_k = bk;
        c.split_k = split;
        c.full_tiles = full_tiles;
        out.push_back(c);
    };
    for (const Shape& s : specialised_shapes(v)) {
        const int64_t tiles = count_tiles(v, s.bm, s.bn);
        add(s.kernel, s.bm, s.bn, s.bk, 1);
        add(s.kernel, s.bm, s.bn, s.bk, best_split(v, s, nullptr));
        for (int32_t sp = 2; sp <= 32; sp *= 2)
            if (v.K / sp >= 128 && tiles * sp <= 4 * kCUs * s.per_cu) add(s.kernel, s.bm, s.bn, s.bk, sp);
        int32_t tsplit = 1;
        double tt = 0;
        const int32_t full = tail_split(v, s, &tsplit, &tt);  // only the last round split
        for (int32_t sp = 2; full > 0 && sp <= 16 && v.K / sp >= 128; sp *= 2) add(s.kernel, s.bm, s.bn, s.bk, sp, full);
    }
    add(KERNEL_GENERIC, 64, 64, 16, 1);
    add(KERNEL_GENERIC, 64, 64, 16, generic_split(v));
    return out;
}

hipError_t launch_gemm(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    if (alpha == 0.0) return launch_gemm_reduce(p, p.t, 0, 0.0, beta, st);
    hipError_t e;
    if (p.n_tail_cells) {  // refresh the zero-padded copies of the k-tails
        e = launch_reblock(p.in_dtype, p.in_dtype, p.tail_cells, p.n_tail_cells, p.tail_rows, false, st);
        if (e != hipSuccess) return e;
    }
    auto specialised = [&](const GemmTables& t) {
        switch (p.info.kernel) {
        case KERNEL_F32_128: return launch_gemm_f32(p, t, alpha, beta, st);
        case KERNEL_F64_128: return launch_gemm_f64(p, t, alpha, beta, st);
        default: return launch_gemm_f16(p, t, alpha, beta, st);
        }
    };
    if (p.info.kernel == KERNEL_GENERIC) return launch_gemm_generic(p, alpha, beta, st);  // does its own reduction
    if (p.full_tiles > 0) {
        // the tiles of the full rounds of workgroups run the whole k-loop and store C; the tiles
        // after them are split, with a compact workspace of their own
        GemmTables full = p.t;
        full.n_tiles = p.full_tiles;
        full.split_k = 1;
        full.ksplit = p.ksplit_whole;
        e = specialised(full);
        if (e != hipSuccess) return e;
        GemmTables rest = p.t;
        rest.tiles += p.full_tiles;
        rest.n_tiles -= p.full_tiles;
        rest.M = (int64_t)rest.n_tiles * p.info.tile_m;
        rest.N = p.info.tile_n;
        e = specialised(rest);
        if (e != hipSuccess) return e;
        return launch_gemm_reduce(p, rest, rest.split_k, alpha, beta, st);
    }
    e = specialised(p.t);
    if (e != hipSuccess || p.t.split_k == 1) return e;
    return launch_gemm_reduce(p, p.t, p.t.split_k, alpha, beta, st);
}

hipError_t launch_conv(const ConvPlan& p, int mode, double alpha, double beta, unsigned rewrite, hipStream_t st)
{
    if (p.kernel == 2 && alpha != 0.0 && p.gemm) return launch_gemm(*p.gemm, alpha, beta, st);
    if (p.kernel == 1 && alpha != 0.0) return launch_conv_fast(p, mode, alpha, beta, rewrite, st);
    return launch_conv_generic(p, mode, alpha, beta, st);
}

}  // namespace dm
