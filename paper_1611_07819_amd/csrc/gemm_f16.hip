// Specialised fp16-input / fp32-accumulate GEMM for gfx950 on v_mfma_f32_32x32x16_f16:
// C <- alpha * op(A) * op(B) + beta * C on full tiles, C stored as fp32 or fp16 (paper
// section 4.2: values stored in half, arithmetic in float).
//
// One workgroup of 4 wavefronts (2 x 2) per BM x BN tile of C inside one block; k-panels are
// walked 64 at a time.  Both operands end up in LDS in one layout, [mn][64 k] with 128-byte
// rows whose 16-byte chunks are XOR-swizzled by ((mn ^ (mn >> 3)) & 7), so that the MFMA
// fragment of a lane (8 consecutive k of one row) is a single 128-bit read:
//   k unit-stride operand  : 128-bit global loads along k, stored as they are;
//   m/n unit-stride operand: each thread loads an 8(k) x 8(mn) block with eight 128-bit loads
//                            along mn, transposes it in registers (32 byte-permutes) and
//                            stores eight 128-bit rows.
// The swizzle keeps both store patterns and the fragment reads free of bank conflicts.
// Global loads run one k-tile ahead of the MFMAs; LDS is double-buffered; alpha/beta and the
// conversion to the output type are fused into the epilogue.
//
// Preconditions (checked by the chooser): full tiles, k-segments multiples of 64, 16-byte
// aligned panel origins and leading dimensions.
#include <hip/hip_runtime.h>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

namespace {

constexpr int BK = 64;
constexpr int NT = 256;
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int swz(int mn) { return (mn ^ (mn >> 3)) & 7; }

template <int BMN, bool KC> struct OperandTile {
    // k unit-stride: BMN rows x 8 chunks; m/n unit-stride: 8 x (BMN/8) blocks of 8x8
    static constexpr int kLoads = KC ? BMN / 32 : 8;
    static constexpr int kBlocks = 8 * (BMN / 8);

    __device__ __forceinline__ static bool active(int tid) { return KC || tid < kBlocks; }

    __device__ __forceinline__ static void load(const _Float16* base, int64_t ld, int mn0, int k0,
                                                int tid, v4u (&r)[kLoads])
    {
        if (KC) {
            const int chunk = tid & 7, row0 = tid >> 3;
#pragma unroll
            for (int q = 0; q < kLoads; ++q) {
                const _Float16* p = base + (int64_t)(mn0 + row0 + q * 32) * ld + k0 + chunk * 8;
                r[q] = *reinterpret_cast<const v4u*>(p);
            }
        } else if (tid < kBlocks) {
            const int mb = tid % (BMN / 8), kb = tid / (BMN / 8);
            const _Float16* p = base + (int64_t)(k0 + kb * 8) * ld + mn0 + mb * 8;
#pragma unroll
            for (int q = 0; q < 8; ++q) r[q] = *reinterpret_cast<const v4u*>(p + q * ld);
        }
    }

    __device__ __forceinline__ static void store(_Float16* lds, int tid, const v4u (&r)[kLoads])
    {
        if (KC) {
            const int chunk = tid & 7, row0 = tid >> 3;
#pragma unroll
            for (int q = 0; q < kLoads; ++q) {
                const int row = row0 + q * 32;
                *reinterpret_cast<v4u*>(lds + row * BK + ((chunk ^ swz(row)) << 3)) = r[q];
            }
        } else if (tid < kBlocks) {
            const int mb = tid % (BMN / 8), kb = tid / (BMN / 8);
            // r[i][d] = values (mn = 2d, 2d+1) at k = i  ->  o[e] of row j = values (k = 2e, 2e+1)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v4u o;
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = __builtin_amdgcn_perm(r[2 * e + 1][j >> 1], r[2 * e][j >> 1], sel);
                const int row = mb * 8 + j;
                *reinterpret_cast<v4u*>(lds + row * BK + ((kb ^ swz(row)) << 3)) = o;
            }
        }
    }

    // 8 consecutive k (chunk 2s + h) of row mn
    __device__ __forceinline__ static v8h fragment(const _Float16* lds, int mn, int h, int s)
    {
        return *reinterpret_cast<const v8h*>(lds + mn * BK + ((((s << 1) + h) ^ swz(mn)) << 3));
    }
};

template <class TC> __device__ __forceinline__ TC to_out(float v);
template <> __device__ __forceinline__ float to_out<float>(float v) { return v; }
template <> __device__ __forceinline__ _Float16 to_out<_Float16>(float v) { return (_Float16)v; }

template <int BM, int BN, bool AKC, bool BKC, class TC>
__global__ __launch_bounds__(NT) void gemm_f16_kernel(GemmTables t, float alpha, float beta)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int MT = WM / 32, NTL = WN / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // two stages, each [A tile][B tile]
    constexpr int kStage = (BM + BN) * BK;
    _Float16* const lds = reinterpret_cast<_Float16*>(smem);

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

    const int ks_end = t.n_kseg;
    int ks = 0, k0 = 0;
    int n_ktiles = 0;
    for (int s = 0; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    Panel pa = t.a[tile.mseg * t.n_kseg], pb = t.b[tile.nseg];
    int klen = t.klen[0];

    v4u ra[TA::kLoads], rb[TB::kLoads];
    auto fetch = [&]() {
        TA::load(static_cast<const _Float16*>(pa.ptr), pa.ld, tile.m_off, k0, tid, ra);
        TB::load(static_cast<const _Float16*>(pb.ptr), pb.ld, tile.n_off, k0, tid, rb);
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
    TA::store(lds, tid, ra);
    TB::store(lds + BM * BK, tid, rb);
    __syncthreads();
    if (n_ktiles > 1) fetch();

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int cur = kt & 1;
        const _Float16* sa = lds + cur * kStage;
        const _Float16* sb = sa + BM * BK;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            v8h fa[MT], fb[NTL];
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[i] = TA::fragment(sa, wm * WM + i * 32 + l32, h, s);
#pragma unroll
            for (int j = 0; j < NTL; ++j) fb[j] = TB::fragment(sb, wn * WN + j * 32 + l32, h, s);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NTL; ++j) acc[i][j] = mfma_f16_32x32x16(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < n_ktiles) {
            _Float16* na = lds + (cur ^ 1) * kStage;
            TA::store(na, tid, ra);
            TB::store(na + BM * BK, tid, rb);
            __syncthreads();
            if (kt + 2 < n_ktiles) fetch();
        }
    }

    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    TC* c = static_cast<TC*>(const_cast<void*>(pc.ptr));
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile.m_off + wm * WM + i * 32 + acc32_row(lane, r);
                const int col = tile.n_off + wn * WN + j * 32 + l32;
                TC* p = c + (int64_t)row * pc.ld + col;
                float v = alpha * acc[i][j][r];
                if (beta != 0.f) v += beta * (float)*p;
                *p = to_out<TC>(v);
            }
}

template <int BM, int BN, bool AKC, bool BKC, class TC>
hipError_t launch_one(const GemmTables& t, float alpha, float beta, hipStream_t st)
{
    constexpr int lds_bytes = 2 * (BM + BN) * BK * 2;
    auto kern = gemm_f16_kernel<BM, BN, AKC, BKC, TC>;
    static bool configured = false;
    if (!configured) {  // more than 64 KiB of LDS has to be asked for once per kernel
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<dim3(t.n_tiles), dim3(NT), lds_bytes, st>>>(t, alpha, beta);
    return hipGetLastError();
}

template <int BM, int BN, class TC>
hipError_t launch_shape(const GemmPlan& p, float alpha, float beta, hipStream_t st)
{
    const GemmTables& t = p.t;
    if (t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, true, true, TC>(t, alpha, beta, st);
    if (t.a_kcontig && !t.b_kcontig) return launch_one<BM, BN, true, false, TC>(t, alpha, beta, st);
    if (!t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, false, true, TC>(t, alpha, beta, st);
    return launch_one<BM, BN, false, false, TC>(t, alpha, beta, st);
}

template <class TC>
hipError_t launch_out(const GemmPlan& p, float alpha, float beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 256 && bn == 128) return launch_shape<256, 128, TC>(p, alpha, beta, st);
    if (bm == 128 && bn == 128) return launch_shape<128, 128, TC>(p, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_f16(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    if (p.out_dtype == DMATH_F16) return launch_out<_Float16>(p, (float)alpha, (float)beta, st);
    return launch_out<float>(p, (float)alpha, (float)beta, st);
}

}  // namespace dm
