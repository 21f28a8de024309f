// Specialised fp32 GEMM for gfx950: C <- alpha * op(A) * op(B) + beta * C on full tiles.
//
// One workgroup (256 threads = 4 wavefronts in a 2 x 2 arrangement) owns one BM x BN tile of C
// that lies inside one block of C, and walks the k-panels of its block row / block column
// (paper section 2.1: blocks; section 1: the transposed variants of back-propagation).
// Per k-tile of 32: 128-bit global loads into registers (issued one tile ahead), 128-bit
// stores into a double-buffered LDS stage, fragments read back in the order the
// v_mfma_f32_32x32x2_f32 instruction wants them, fused alpha/beta epilogue.
//
// LDS layouts (both conflict-free for the accesses used):
//   operand whose unit-stride axis is k  : [mn][32 k], 16-byte chunks XOR-swizzled by (mn & 7);
//                                          a lane reads 4 consecutive k with one 128-bit read
//   operand whose unit-stride axis is m/n: [k][mn] as in memory; a lane reads one value per
//                                          MFMA with lanes on consecutive addresses
// The k index inside a group of 8 is permuted identically for A and B (lanes 0-31 take
// k = 8u+j, lanes 32-63 take k = 8u+4+j at step j), which the sum over k does not notice.
//
// Preconditions (checked by the chooser): every tile is full, every k-segment is a multiple of
// 32, every panel origin and leading dimension is 16-byte aligned.
#include <hip/hip_runtime.h>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

namespace {

constexpr int BK = 32;
constexpr int NT = 256;

template <int BMN, bool KC> struct OperandTile {
    // number of 128-bit loads per thread and k-tile
    static constexpr int kLoads = BMN * BK / 4 / NT;
    static constexpr int kChunksPerRow = KC ? BK / 4 : BMN / 4;
    static constexpr int kRowsPerPass = NT / kChunksPerRow;

    // global -> registers.  base points at the panel origin (element (0,0) of the panel);
    // mn0 = offset of the tile inside the panel, k0 = offset of the k-tile inside the panel.
    __device__ __forceinline__ static void load(const float* base, int64_t ld, int mn0, int k0,
                                                int tid, v4f (&r)[kLoads])
    {
        const int chunk = tid % kChunksPerRow, row0 = tid / kChunksPerRow;
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int row = row0 + q * kRowsPerPass;
            const float* p = KC ? base + (int64_t)(mn0 + row) * ld + k0 + chunk * 4
                                : base + (int64_t)(k0 + row) * ld + mn0 + chunk * 4;
            r[q] = *reinterpret_cast<const v4f*>(p);
        }
    }

    // registers -> LDS stage
    __device__ __forceinline__ static void store(float* lds, int tid, const v4f (&r)[kLoads])
    {
        const int chunk = tid % kChunksPerRow, row0 = tid / kChunksPerRow;
#pragma unroll
        for (int q = 0; q < kLoads; ++q) {
            const int row = row0 + q * kRowsPerPass;
            float* p = KC ? lds + row * BK + ((chunk ^ (row & 7)) << 2) : lds + row * BMN + chunk * 4;
            *reinterpret_cast<v4f*>(p) = r[q];
        }
    }

    // The four values (steps j = 0..3 of group u) that lane (mn, h) feeds to the MFMA.
    __device__ __forceinline__ static v4f fragment(const float* lds, int mn, int h, int u)
    {
        if (KC) return *reinterpret_cast<const v4f*>(lds + mn * BK + ((((u << 1) + h) ^ (mn & 7)) << 2));
        v4f f;
        const float* p = lds + (8 * u + 4 * h) * BMN + mn;
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = p[j * BMN];
        return f;
    }
};

template <int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(NT) void gemm_f32_kernel(GemmTables t, float alpha, float beta)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WM = BM / 2, WN = BN / 2;  // wavefront tile
    constexpr int MT = WM / 32, NTL = WN / 32;
    __shared__ __attribute__((aligned(16))) float lds_a[2][BM * BK];
    __shared__ __attribute__((aligned(16))) float lds_b[2][BN * BK];

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, h = lane >> 5, l32 = lane & 31;

    v16f acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // walk of the k-panels: position of the next k-tile to fetch
    const int ks_end = t.n_kseg;
    int ks = 0, k0 = 0;
    int n_ktiles = 0;
    for (int s = 0; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    Panel pa = t.a[tile.mseg * t.n_kseg], pb = t.b[tile.nseg];
    int klen = t.klen[0];

    v4f ra[TA::kLoads], rb[TB::kLoads];
    auto fetch = [&]() {
        TA::load(static_cast<const float*>(pa.ptr), pa.ld, tile.m_off, k0, tid, ra);
        TB::load(static_cast<const float*>(pb.ptr), pb.ld, tile.n_off, k0, tid, rb);
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
        const float* sa = lds_a[cur];
        const float* sb = lds_b[cur];
#pragma unroll
        for (int u = 0; u < BK / 8; ++u) {
            v4f fa[MT], fb[NTL];
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[i] = TA::fragment(sa, wm * WM + i * 32 + l32, h, u);
#pragma unroll
            for (int j = 0; j < NTL; ++j) fb[j] = TB::fragment(sb, wn * WN + j * 32 + l32, h, u);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NTL; ++j)
                        acc[i][j] = mfma_f32_32x32x2(fa[i][s], fb[j][s], acc[i][j]);
        }
        if (kt + 1 < n_ktiles) {
            TA::store(lds_a[cur ^ 1], tid, ra);
            TB::store(lds_b[cur ^ 1], tid, rb);
            __syncthreads();
            if (kt + 2 < n_ktiles) fetch();
        }
    }

    // epilogue: register r of a 32x32 result tile holds row 8*(r/4) + 4*h + r%4, column l32
    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    float* c = static_cast<float*>(const_cast<void*>(pc.ptr));
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile.m_off + wm * WM + i * 32 + acc32_row(lane, r);
                const int col = tile.n_off + wn * WN + j * 32 + l32;
                float* p = c + (int64_t)row * pc.ld + col;
                float v = alpha * acc[i][j][r];
                if (beta != 0.f) v += beta * *p;
                *p = v;
            }
}

template <int BM, int BN>
hipError_t launch_shape(const GemmPlan& p, float alpha, float beta, hipStream_t st)
{
    const GemmTables& t = p.t;
    dim3 grid(t.n_tiles), block(NT);
    if (t.a_kcontig && t.b_kcontig)
        gemm_f32_kernel<BM, BN, true, true><<<grid, block, 0, st>>>(t, alpha, beta);
    else if (t.a_kcontig && !t.b_kcontig)
        gemm_f32_kernel<BM, BN, true, false><<<grid, block, 0, st>>>(t, alpha, beta);
    else if (!t.a_kcontig && t.b_kcontig)
        gemm_f32_kernel<BM, BN, false, true><<<grid, block, 0, st>>>(t, alpha, beta);
    else
        gemm_f32_kernel<BM, BN, false, false><<<grid, block, 0, st>>>(t, alpha, beta);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f32(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 128 && bn == 128) return launch_shape<128, 128>(p, (float)alpha, (float)beta, st);
    if (bm == 128 && bn == 64) return launch_shape<128, 64>(p, (float)alpha, (float)beta, st);
    return hipErrorInvalidValue;
}

}  // namespace dm
