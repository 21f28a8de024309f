// Specialised fp16-input / fp32-accumulate GEMM for gfx950:
// C <- alpha * op(A) * op(B) + beta * C on full tiles, C stored as fp32 or fp16 (paper
// section 4.2: values stored in half, arithmetic in float).
//
// One workgroup per BM x BN tile of C inside one block; the k-panels of the block row / block
// column (paper section 2.1) are walked by the loader below and multiplied by the shared
// pipeline of f16_pipeline.hpp (direct global->LDS loads, LDS ring, pinned MFMA schedule).
//
// Preconditions (checked by the chooser): k-segments multiples of 64, 16-byte
// aligned panel origins and leading dimensions, blocks smaller than 4 GiB.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "context.hpp"
#include "epilogue.hpp"
#include "f16_pipeline.hpp"

namespace dm {

// Opt-in cycle probe (a separate build with -DDMATH_CYCLE_PROBE, never the product library): the
// workgroup that owns the C tile at (0, 0) records, for wavefront 0, the shader-clock cycles of
// its prologue (until the first k-tile is in registers), k-loop and epilogue, the cycles spent
// waiting at the per-k-tile barrier, and the elapsed 100 MHz reference ticks, from which the
// clock the kernel really ran at follows.
#ifdef DMATH_CYCLE_PROBE
__device__ uint64_t g_cycle_probe[6];
#endif

bool read_cycle_probe(uint64_t* out6)
{
#ifdef DMATH_CYCLE_PROBE
    return hipMemcpyFromSymbol(out6, HIP_SYMBOL(g_cycle_probe), 6 * sizeof(uint64_t)) == hipSuccess;
#else
    (void)out6;
    return false;
#endif
}

namespace {

using namespace f16p;

#ifdef DMATH_CYCLE_PROBE
struct CycleProbe {
    uint64_t t_prologue = 0, t_wait = 0, w0 = 0;
    __device__ __forceinline__ void prologue_done() { t_prologue = __builtin_amdgcn_s_memtime(); }
    __device__ __forceinline__ void wait_begin() { w0 = __builtin_amdgcn_s_memtime(); }
    __device__ __forceinline__ void wait_end() { t_wait += __builtin_amdgcn_s_memtime() - w0; }
};
#endif

// Walks the k-panels of one C tile: dense panels, pointer + leading dimension per k-segment.
template <int BM, int BN, bool AKC, bool BKC, int MF> struct PanelWalk {
    using TA = OperandTile<BM, AKC, MF>;
    using TB = OperandTile<BN, BKC, MF>;
    const GemmTables& t;
    const Tile& tile;
    int wave, lane, ks, ks_end, kleft;
    Panel pa, pb;
    const char *abase, *bbase;
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];

    // walks the k-segments [ks_begin, ks_end_) (one split of a split-K plan, or all of them)
    __device__ __forceinline__ PanelWalk(const GemmTables& t_, const Tile& tile_, int wave_, int lane_,
                                         int ks_begin, int ks_end_)
        : t(t_), tile(tile_), wave(wave_), lane(lane_), ks(ks_begin), ks_end(ks_end_)
    {
        load_panel();
    }
    __device__ __forceinline__ void load_panel()
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
            load_panel();
        }
    }
    // The same for a pipeline that keeps issuing loads to the end of its k-loop: on the last
    // k-tile the walk stays, and what is then fetched again is valid memory that nobody reads.
    __device__ __forceinline__ void advance_or_stay()
    {
        if (kleft > 1) {
            --kleft;
            abase += TA::step(pa.ld);
            bbase += TB::step(pb.ld);
        } else if (ks + 1 < ks_end) {
            ++ks;
            load_panel();
        }
    }
};

// MF: 32 = v_mfma_f32_32x32x16_f16 fragments (every tile shape), 16 = v_mfma_f32_16x16x32_f16
// (2 x 2 wavefronts on tiles of 128 or more rows and columns).
template <int BM, int BN, int STAGES, bool AKC, bool BKC, class TC, int MF>
__global__ __launch_bounds__(NT) void gemm_f16_kernel(GemmTables t, float alpha, float beta)
{
    using TS = std::conditional_t<MF == 16, TileShape16<BM, BN>, TileShape<BM, BN>>;
    using Acc = std::conditional_t<MF == 16, v4f, v16f>;
    constexpr int WM = TS::WM, WN = TS::WN, MT = TS::MT, NTL = TS::NTL;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = TS::wm(wave), wn = TS::wn(wave);

    Acc acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < (MF == 16 ? 4 : 16); ++r) acc[i][j][r] = 0.f;

    const int split = blockIdx.y, ks0 = t.ksplit[split], ks1 = t.ksplit[split + 1];
    int n_ktiles = 0;
    for (int s = ks0; s < ks1; ++s) n_ktiles += t.klen[s] / BK;
    PanelWalk<BM, BN, AKC, BKC, MF> walk(t, tile, wave, lane, ks0, ks1);
#ifdef DMATH_CYCLE_PROBE
    const uint64_t t_start = __builtin_amdgcn_s_memtime(), r_start = __builtin_amdgcn_s_memrealtime();
    CycleProbe probe;
#else
    NoProbe probe;
#endif
    if constexpr (MF == 16)
        // tiles with at most 32 accumulators keep them in fixed registers, out of the compiler's
        // reach (no copies between differently scheduled iterations, hence nothing to drain for)
        run16<BM, BN, STAGES, AKC, BKC, MT * NTL <= 32>(walk, n_ktiles, smem, acc, probe);
    else
        run<BM, BN, STAGES, AKC, BKC>(walk, n_ktiles, smem, acc, probe);
#ifdef DMATH_CYCLE_PROBE
    const uint64_t t_loop_end = __builtin_amdgcn_s_memtime();
    auto record_probe = [&] {
        __syncthreads();
        if (tid == 0 && tile.m_glob == 0 && tile.n_glob == 0 && blockIdx.y == 0) {
            const uint64_t t_end = __builtin_amdgcn_s_memtime(), r_end = __builtin_amdgcn_s_memrealtime();
            g_cycle_probe[0] = probe.t_prologue - t_start;
            g_cycle_probe[1] = t_loop_end - probe.t_prologue;
            g_cycle_probe[2] = t_end - t_loop_end;
            g_cycle_probe[3] = probe.t_wait;
            g_cycle_probe[4] = r_end - r_start;
            g_cycle_probe[5] = (uint64_t)n_ktiles;
        }
    };
#endif
    store_tile<MF, BM, BN, TC, MF == 16>(t, tile, split, wm * WM, wn * WN, lane, acc, alpha, beta);
#ifdef DMATH_CYCLE_PROBE
    record_probe();
#endif
}

template <int BM, int BN, int STAGES, bool AKC, bool BKC, class TC, int MF>
hipError_t launch_one(const GemmTables& t, float alpha, float beta, hipStream_t st)
{
    constexpr int lds_bytes = STAGES * (BM + BN) * BK * 2;
    auto kern = gemm_f16_kernel<BM, BN, STAGES, AKC, BKC, TC, MF>;
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

template <int BM, int BN, int STAGES, class TC, int MF = 32>
hipError_t launch_shape(const GemmTables& t, float alpha, float beta, hipStream_t st)
{
    if (t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, STAGES, true, true, TC, MF>(t, alpha, beta, st);
    if (t.a_kcontig && !t.b_kcontig) return launch_one<BM, BN, STAGES, true, false, TC, MF>(t, alpha, beta, st);
    if (!t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, STAGES, false, true, TC, MF>(t, alpha, beta, st);
    return launch_one<BM, BN, STAGES, false, false, TC, MF>(t, alpha, beta, st);
}

// Tile shapes: 256x256 (two 64 KiB stages), 256x128 (three 48 KiB stages), 128x128 (two 32 KiB
// stages, so that two workgroups share a CU); 64x128 and 64x64 (three stages) for batches of at
// most 64 rows, which are bound by streaming the other operand from HBM.
template <class TC>
hipError_t launch_out(const GemmPlan& p, const GemmTables& t, float alpha, float beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    // The three large tiles run on 16x16x32 fragments; DMATH_F16_MFMA32=1 switches them back to
    // 32x32x16 (A/B measurements).
    static const bool mf32 = std::getenv("DMATH_F16_MFMA32") != nullptr;
    if (!mf32) {
        if (bm == 256 && bn == 256) return launch_shape<256, 256, 2, TC, 16>(t, alpha, beta, st);
        if (bm == 256 && bn == 128) return launch_shape<256, 128, 3, TC, 16>(t, alpha, beta, st);
        if (bm == 128 && bn == 128) return launch_shape<128, 128, 2, TC, 16>(t, alpha, beta, st);
    }
    if (bm == 256 && bn == 256) return launch_shape<256, 256, 2, TC>(t, alpha, beta, st);
    if (bm == 256 && bn == 128) return launch_shape<256, 128, 3, TC>(t, alpha, beta, st);
    if (bm == 128 && bn == 128) return launch_shape<128, 128, 2, TC>(t, alpha, beta, st);
    if (bm == 64 && bn == 128) return launch_shape<64, 128, 3, TC>(t, alpha, beta, st);
    if (bm == 64 && bn == 64) return launch_shape<64, 64, 3, TC>(t, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_f16(const GemmPlan& p, const GemmTables& t, double alpha, double beta, hipStream_t st)
{
    if (p.out_dtype == DMATH_F16) return launch_out<_Float16>(p, t, (float)alpha, (float)beta, st);
    return launch_out<float>(p, t, (float)alpha, (float)beta, st);
}

}  // namespace dm
