// Specialised fp64 GEMM for gfx950 on the pipeline of f64_pipeline.hpp:
// C <- alpha * op(A) * op(B) + beta * C on full and ragged tiles (paper abstract: matrix
// multiplication; section 1, feature d: double precision).
//
// One workgroup per BM x BN tile of C inside one block; the k-panels of the block row / block
// column are walked 16 at a time.
//
// Preconditions (checked by the chooser): k-segments multiples of 16, 16-byte
// aligned panel origins and leading dimensions, blocks smaller than 4 GiB.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "context.hpp"
#include "epilogue.hpp"
#include "f64_pipeline.hpp"

namespace dm {

namespace {

using namespace f64p;

// The k-panels of one tile's block row of op(A) and block column of op(B), in k order.
template <int BM, int BN, bool AKC, bool BKC> struct PanelWalk {
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    const GemmTables& t;
    const Tile& tile;
    const char *abase, *bbase;
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];
    Panel pa, pb;
    int ks, ks_end, kleft, wave, lane;

    __device__ __forceinline__ PanelWalk(const GemmTables& t_, const Tile& tile_, int ks_, int ks_end_, int wave_,
                                         int lane_)
        : t(t_), tile(tile_), ks(ks_), ks_end(ks_end_), wave(wave_), lane(lane_)
    {
        enter();
    }
    __device__ __forceinline__ void enter()
    {
        pa = t.a[tile.mseg * t.n_kseg + ks];
        pb = t.b[ks * t.n_nseg + tile.nseg];
        kleft = t.klen[ks] / BK;
        abase = static_cast<const char*>(pa.ptr);
        bbase = static_cast<const char*>(pb.ptr);
        TA::offsets(pa.ld, tile.m_off, tile.m_len, wave, lane, aoff);
        TB::offsets(pb.ld, tile.n_off, tile.n_len, wave, lane, boff);
    }
    __device__ __forceinline__ void advance()
    {
        abase += TA::step(pa.ld);
        bbase += TB::step(pb.ld);
        if (--kleft == 0 && ks + 1 < ks_end) {
            ++ks;
            enter();
        }
    }
};

// WVM x WVN = 4: arrangement of the wavefronts over the tile.
template <int BM, int BN, int WVM, bool AKC, bool BKC, int NS>
__global__ __launch_bounds__(NT) void gemm_f64_kernel(GemmTables t, double alpha, double beta)
{
    constexpr int WVN = 4 / WVM;
    constexpr int WM = BM / WVM, WN = BN / WVN;  // wavefront tile
    constexpr int MT = WM / 16, NTL = WN / 16;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WVN, wn = wave % WVN;

    v4d acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0;

    // split-K: blockIdx.y owns the k-segments [ksplit[y], ksplit[y+1])
    const int split = blockIdx.y;
    const int ks = t.ksplit[split], ks_end = t.ksplit[split + 1];
    int n_ktiles = 0;
    for (int s = ks; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    PanelWalk<BM, BN, AKC, BKC> walk(t, tile, ks, ks_end, wave, lane);
    run<BM, BN, WVM, AKC, BKC, NS>(walk, n_ktiles, smem, acc);

    store_tile<16, BM, BN, double>(t, tile, split, wm * WM, wn * WN, lane, acc, alpha, beta);
}

template <int BM, int BN, int WVM, bool AKC, bool BKC, int NS>
hipError_t launch_one(const GemmTables& t, double alpha, double beta, hipStream_t st)
{
    constexpr int lds_bytes = NS * (BM + BN) * BK * 8;
    auto kern = gemm_f64_kernel<BM, BN, WVM, AKC, BKC, NS>;
    static bool configured = false;
    if (!configured) {  // more than 64 KiB of LDS has to be asked for once per kernel
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<dim3(t.n_tiles, t.split_k), dim3(NT), lds_bytes, st>>>(t, alpha, beta);
    return hipGetLastError();
}

template <int BM, int BN, int WVM, int NS = STAGES>
hipError_t launch_shape(const GemmTables& t, double alpha, double beta, hipStream_t st)
{
    if (t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, WVM, true, true, NS>(t, alpha, beta, st);
    if (!t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, WVM, false, true, NS>(t, alpha, beta, st);
    if constexpr (64 % (BN / 2) == 0) {  // an m/n-major B tile must fill whole 1 KiB LDS segments
        if (t.a_kcontig) return launch_one<BM, BN, WVM, true, false, NS>(t, alpha, beta, st);
        return launch_one<BM, BN, WVM, false, false, NS>(t, alpha, beta, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_f64(const GemmPlan& p, const GemmTables& t, double alpha, double beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 128 && bn == 128) return launch_shape<128, 128, 2>(t, alpha, beta, st);
    if (bm == 128 && bn == 64) return launch_shape<128, 64, 2>(t, alpha, beta, st);
    if (bm == 64 && bn == 128) return launch_shape<64, 128, 2>(t, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace dm
