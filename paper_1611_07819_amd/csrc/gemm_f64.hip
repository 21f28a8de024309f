// Specialised fp64 GEMM for gfx950: C <- alpha * op(A) * op(B) + beta * C on full tiles, on
// the v_mfma_f64_16x16x4_f64 matrix-core instruction.
//
// Same structure as the fp32 kernel: one workgroup of 4 wavefronts (2 x 2) per BM x BN tile of
// C inside one block, k-panels walked 16 at a time (128-byte rows), 128-bit global loads one
// tile ahead, double-buffered LDS, fused alpha/beta epilogue.  A wavefront owns a
// (BM/2) x (BN/2) tile as a grid of 16 x 16 result tiles.
//
// LDS layouts:
//   k unit-stride operand  : [mn][16 k], 16-byte chunks (2 doubles) XOR-swizzled by ((mn ^ (mn >> 3)) & 7);
//                            one 128-bit read gives a lane its values for two MFMA steps
//   m/n unit-stride operand: [k][mn]; one 64-bit read per MFMA step, lanes on consecutive
//                            addresses
// Inside a group of 8 k the order is permuted identically for A and B: lane group g = lane/16
// supplies k = 8u + 2g + j at step j of group u.
//
// Preconditions (checked by the chooser): full tiles, k-segments multiples of 16, 16-byte
// aligned panel origins and leading dimensions.
#include <hip/hip_runtime.h>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

namespace {

constexpr int BK = 16;
constexpr int NT = 256;

// XOR applied to the 16-byte chunk index of row mn: rows 8 apart differ too, so that the 16 lanes
// served per LDS cycle never meet in a bank.
__device__ __forceinline__ int swz(int mn) { return (mn ^ (mn >> 3)) & 7; }
typedef double v2d __attribute__((ext_vector_type(2)));

template <int BMN, bool KC> struct OperandTile {
    static constexpr int kLoads = BMN * BK / 2 / NT;
    static constexpr int kChunksPerRow = KC ? BK / 2 : BMN / 2;
    static constexpr int kRowsPerPass = NT / kChunksPerRow;

    __device__ __forceinline__ static void load(const double* base, int64_t ld, int mn0, int k0,
                                                int tid, v2d (&r)[kLoads])
    {
        const int chunk = tid % kChunksPerRow, row0 = tid / kChunksPerRow;
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int row = row0 + q * kRowsPerPass;
            const double* p = KC ? base + (int64_t)(mn0 + row) * ld + k0 + chunk * 2
                                 : base + (int64_t)(k0 + row) * ld + mn0 + chunk * 2;
            r[q] = *reinterpret_cast<const v2d*>(p);
        }
    }

    __device__ __forceinline__ static void store(double* lds, int tid, const v2d (&r)[kLoads])
    {
        const int chunk = tid % kChunksPerRow, row0 = tid / kChunksPerRow;
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int row = row0 + q * kRowsPerPass;
            double* p = KC ? lds + row * BK + ((chunk ^ swz(row)) << 1) : lds + row * BMN + chunk * 2;
            *reinterpret_cast<v2d*>(p) = r[q];
        }
    }

    // values of steps j = 0, 1 of group u for lane (mn, g)
    __device__ __forceinline__ static v2d fragment(const double* lds, int mn, int g, int u)
    {
        if (KC) return *reinterpret_cast<const v2d*>(lds + mn * BK + ((((u << 2) + g) ^ swz(mn)) << 1));
        v2d f;
        const double* p = lds + (8 * u + 2 * g) * BMN + mn;
        f[0] = p[0];
        f[1] = p[BMN];
        return f;
    }
};

template <int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(NT) void gemm_f64_kernel(GemmTables t, double alpha, double beta)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int MT = WM / 16, NTL = WN / 16;
    __shared__ __attribute__((aligned(16))) double lds_a[2][BM * BK];
    __shared__ __attribute__((aligned(16))) double lds_b[2][BN * BK];

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, g = lane >> 4, l16 = lane & 15;

    v4d acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0;

    const int ks_end = t.n_kseg;
    int ks = 0, k0 = 0;
    int n_ktiles = 0;
    for (int s = 0; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    Panel pa = t.a[tile.mseg * t.n_kseg], pb = t.b[tile.nseg];
    int klen = t.klen[0];

    v2d ra[TA::kLoads], rb[TB::kLoads];
    auto fetch = [&]() {
        TA::load(static_cast<const double*>(pa.ptr), pa.ld, tile.m_off, k0, tid, ra);
        TB::load(static_cast<const double*>(pb.ptr), pb.ld, tile.n_off, k0, tid, rb);
        k0 += BK;
        if (k0 >= klen && ks + 1 < ks_end) {
            ++ks;
            k0 = 0;
            pa = t.a[tile.mseg * t.n_kseg + ks];
            pb = t.b[ks * t.n_nseg + tile.nseg];
            klen = t.klen[ks];
        }
    };

    fetch();
    TA::store(lds_a[0], tid, ra);
    TB::store(lds_b[0], tid, rb);
    __syncthreads();
    if (n_ktiles > 1) fetch();

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int cur = kt & 1;
        const double* sa = lds_a[cur];
        const double* sb = lds_b[cur];
#pragma unroll
        for (int u = 0; u < BK / 8; ++u) {
            v2d fa[MT], fb[NTL];
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[i] = TA::fragment(sa, wm * WM + i * 16 + l16, g, u);
#pragma unroll
            for (int j = 0; j < NTL; ++j) fb[j] = TB::fragment(sb, wn * WN + j * 16 + l16, g, u);
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NTL; ++j)
                        acc[i][j] = mfma_f64_16x16x4(fa[i][s], fb[j][s], acc[i][j]);
        }
        if (kt + 1 < n_ktiles) {
            TA::store(lds_a[cur ^ 1], tid, ra);
            TB::store(lds_b[cur ^ 1], tid, rb);
            __syncthreads();
            if (kt + 2 < n_ktiles) fetch();
        }
    }

    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    double* c = static_cast<double*>(const_cast<void*>(pc.ptr));
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = tile.m_off + wm * WM + i * 16 + acc16d_row(lane, r);
                const int col = tile.n_off + wn * WN + j * 16 + l16;
                double* p = c + (int64_t)row * pc.ld + col;
                double v = alpha * acc[i][j][r];
                if (beta != 0.0) v += beta * *p;
                *p = v;
            }
}

template <int BM, int BN>
hipError_t launch_shape(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    const GemmTables& t = p.t;
    dim3 grid(t.n_tiles), block(NT);
    if (t.a_kcontig && t.b_kcontig)
        gemm_f64_kernel<BM, BN, true, true><<<grid, block, 0, st>>>(t, alpha, beta);
    else if (t.a_kcontig && !t.b_kcontig)
        gemm_f64_kernel<BM, BN, true, false><<<grid, block, 0, st>>>(t, alpha, beta);
    else if (!t.a_kcontig && t.b_kcontig)
        gemm_f64_kernel<BM, BN, false, true><<<grid, block, 0, st>>>(t, alpha, beta);
    else
        gemm_f64_kernel<BM, BN, false, false><<<grid, block, 0, st>>>(t, alpha, beta);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f64(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 128 && bn == 128) return launch_shape<128, 128>(p, alpha, beta, st);
    if (bm == 128 && bn == 64) return launch_shape<128, 64>(p, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace dm
