// Specialised fp16-input / fp32-accumulate GEMM for gfx950 on v_mfma_f32_32x32x16_f16:
// C <- alpha * op(A) * op(B) + beta * C on full tiles, C stored as fp32 or fp16 (paper
// section 4.2: values stored in half, arithmetic in float).
//
// One workgroup of 4 wavefronts (2 x 2) per BM x BN tile of C inside one block; the k-panels of
// the block row / block column are walked 64 at a time through a three-stage LDS ring.
//
// Global -> LDS without registers: every wavefront issues global_load_lds_dwordx4, which
// writes the 16 bytes fetched by lane p to (LDS base in M0) + 16*p.  A 1 KiB LDS segment is
// therefore filled per instruction, and the swizzles below are applied by choosing WHICH global
// chunk each lane fetches.  Two tiles are in flight while a third is being multiplied; the
// loads are inline assembly with explicit s_waitcnt vmcnt(), so that the compiler neither sees
// nor serialises them.
//
// LDS layouts, both as the operand lies in memory:
//   k unit-stride operand  : [mn][64 k], 128-byte rows, 16-byte chunk index XOR ((mn^(mn>>3))&7);
//                            the MFMA fragment of a lane (8 consecutive k of one row) is one
//                            ds_read_b128, conflict-free
//   m/n unit-stride operand: [k][mn], 16-byte chunk index XOR ((k&3)<<1); fragments come from
//                            two ds_read_b64_tr_b16 (the gfx950 transposing LDS read: inside a
//                            16-lane group, lane i receives element i%4 of the 8 bytes fetched
//                            by lanes i/4, i/4+4, i/4+8, i/4+12), so a group fetches a 4(k) x
//                            16(mn) patch and every lane ends up with 4 consecutive k of its
//                            own column; the XOR spreads the four k rows over the banks
//
// Preconditions (checked by the chooser): full tiles, k-segments multiples of 64, 16-byte
// aligned panel origins and leading dimensions, blocks smaller than 4 GiB.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

namespace {

constexpr int BK = 64;
constexpr int NT = 256;
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ int swz(int mn) { return (mn ^ (mn >> 3)) & 7; }

// Forces a wavefront-uniform pointer into scalar registers.
__device__ __forceinline__ const char* uniform_ptr(const char* p)
{
    uint64_t v = reinterpret_cast<uint64_t>(p);
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// One direct global->LDS load: lane fetches 16 bytes at (sbase + voff), lands at m0 + 16*lane.
__device__ __forceinline__ void dma16(uint32_t lds_addr, const void* sbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory");
}

template <int BMN, bool KC> struct OperandTile {
    static constexpr int kInstr = BMN / 32;           // 1 KiB segments per wavefront and k-tile
    static constexpr int kBytes = BMN * BK * 2;       // one stage of this operand
    static constexpr int kChunksPerRow = KC ? 8 : BMN / 8;
    static constexpr int kRowsPerSeg = 64 / kChunksPerRow;

    // byte offsets (relative to the panel origin) of the chunks this lane fetches at k-tile 0
    __device__ __forceinline__ static void offsets(int64_t ld, int mn0, int wave, int lane,
                                                   uint32_t (&off)[kInstr])
    {
#pragma unroll
        for (int q = 0; q < kInstr; ++q) {
            const int seg = q * 4 + wave;
            const int row = seg * kRowsPerSeg + lane / kChunksPerRow;
            const int cpos = lane % kChunksPerRow;
            if (KC) {
                const int chunk = cpos ^ swz(row);
                off[q] = (uint32_t)((((int64_t)(mn0 + row)) * ld + chunk * 8) * 2);
            } else {
                const int chunk = cpos ^ ((row & 3) << 1);
                off[q] = (uint32_t)(((int64_t)row * ld + mn0 + chunk * 8) * 2);
            }
        }
    }
    // bytes the panel pointer advances per k-tile
    __device__ __forceinline__ static int64_t step(int64_t ld) { return KC ? BK * 2 : BK * 2 * ld; }

    __device__ __forceinline__ static void issue(uint32_t lds_stage, const char* base, int wave,
                                                 const uint32_t (&off)[kInstr])
    {
#pragma unroll
        for (int q = 0; q < kInstr; ++q) dma16(lds_stage + (q * 4 + wave) * 1024, base, off[q]);
    }

    // Per-lane LDS byte offset (inside the operand's stage) of the fragment for k-step 0 of the
    // 32-row tile starting at mn_base; k-step s adds frag_step * s.
    __device__ __forceinline__ static uint32_t frag_base(int mn_base, int lane)
    {
        if (KC) return (uint32_t)((mn_base + (lane & 31)) * 128);
        const int g = lane >> 4, i = lane & 15;
        const int row = 8 * (g >> 1) + (i >> 2);
        const int col = mn_base + 16 * (g & 1) + 4 * (i & 3);
        return (uint32_t)(row * (BMN * 2) + (((col >> 3) ^ ((row & 3) << 1)) << 4) + (col & 7) * 2);
    }

    __device__ __forceinline__ static v8h fragment(const lds_char* tile, uint32_t fb, int mn_row,
                                                   int h, int s)
    {
        if (KC) {
            const int chunk = ((s << 1) + h) ^ swz(mn_row);
            return *reinterpret_cast<const __attribute__((address_space(3))) v8h*>(tile + fb + (chunk << 4));
        }
        const lds_char* p = tile + fb + s * (16 * BMN * 2);
        v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)p);
        v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)(p + 4 * BMN * 2));
        typedef short v8s __attribute__((ext_vector_type(8)));
        v8s both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(v8h, both);
    }
};

template <class TC> __device__ __forceinline__ TC to_out(float v);
template <> __device__ __forceinline__ float to_out<float>(float v) { return v; }
template <> __device__ __forceinline__ _Float16 to_out<_Float16>(float v) { return (_Float16)v; }

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BM, int BN, int STAGES, bool AKC, bool BKC, class TC>
__global__ __launch_bounds__(NT) void gemm_f16_kernel(GemmTables t, float alpha, float beta)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int MT = WM / 32, NTL = WN / 32;
    constexpr int kStage = TA::kBytes + TB::kBytes;
    constexpr int kPerTile = TA::kInstr + TB::kInstr;  // loads per wavefront and k-tile
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const lds_char* lds = (const lds_char*)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1, h = lane >> 5, l32 = lane & 31;

    v16f acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint32_t fa_base[MT], fb_base[NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i) fa_base[i] = TA::frag_base(wm * WM + i * 32, lane);
#pragma unroll
    for (int j = 0; j < NTL; ++j) fb_base[j] = TB::frag_base(wn * WN + j * 32, lane);

    // walk of the k-panels by the loader
    const int ks_end = t.n_kseg;
    int ks = 0, kleft;
    int n_ktiles = 0;
    for (int s = 0; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    Panel pa = t.a[tile.mseg * t.n_kseg], pb = t.b[tile.nseg];
    kleft = t.klen[0] / BK;
    const char* abase = static_cast<const char*>(pa.ptr);
    const char* bbase = static_cast<const char*>(pb.ptr);
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];
    TA::offsets(pa.ld, tile.m_off, wave, lane, aoff);
    TB::offsets(pb.ld, tile.n_off, wave, lane, boff);

    // The loads of one k-tile are numbered 0 .. kPerTile-1 (A segments first).  issue_one()
    // enqueues one of them; advance() moves the loader to the next k-tile.
    auto issue_one = [&](uint32_t sbase, const char* ab, const char* bb, int idx) {
        if (idx < TA::kInstr)
            dma16(sbase + (idx * 4 + wave) * 1024, ab, aoff[idx]);
        else
            dma16(sbase + TA::kBytes + ((idx - TA::kInstr) * 4 + wave) * 1024, bb, boff[idx - TA::kInstr]);
    };
    auto advance = [&]() {
        abase += TA::step(pa.ld);
        bbase += TB::step(pb.ld);
        if (--kleft == 0 && ks + 1 < ks_end) {
            ++ks;
            pa = t.a[tile.mseg * t.n_kseg + ks];
            pb = t.b[ks * t.n_nseg + tile.nseg];
            kleft = t.klen[ks] / BK;
            abase = static_cast<const char*>(pa.ptr);
            bbase = static_cast<const char*>(pb.ptr);
            TA::offsets(pa.ld, tile.m_off, wave, lane, aoff);
            TB::offsets(pb.ld, tile.n_off, wave, lane, boff);
        }
    };
    auto issue_all = [&](int stage) {
        const uint32_t sbase = lds0 + stage * kStage;
        const char* ab = uniform_ptr(abase);
        const char* bb = uniform_ptr(bbase);
#pragma unroll
        for (int idx = 0; idx < kPerTile; ++idx) issue_one(sbase, ab, bb, idx);
        advance();
    };

    // Multiplies the tile in `stage`.  The instruction order is pinned: after every MFMA comes
    // one fragment read for the NEXT k-step (register double buffer) and, when PREFETCH, every
    // few MFMAs one load of the tile two ahead into `next_stage` -- so neither the LDS nor the
    // memory pipeline ever holds up the matrix instructions queued behind it.
    auto multiply = [&](int stage, int next_stage, auto prefetch) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        constexpr int kSteps = BK / 16, kMfma = MT * NTL, kReads = MT + NTL;
        static_assert(kReads <= kMfma, "one fragment read per MFMA slot");
        static_assert(kSteps * kMfma >= kPerTile, "not enough slots to spread the loads");
        const lds_char* sa = lds + stage * kStage;
        const lds_char* sb = sa + TA::kBytes;
        const uint32_t nbase = lds0 + next_stage * kStage;
        const char* ab = uniform_ptr(abase);
        const char* bb = uniform_ptr(bbase);
        v8h fa[2][MT], fb[2][NTL];
        // read order: what the first MFMAs need comes first (A0, all B, then the other A)
        auto read_frag = [&](int buf, int r, int s) {
            if (r == 0)
                fa[buf][0] = TA::fragment(sa, fa_base[0], wm * WM + l32, h, s);
            else if (r <= NTL)
                fb[buf][r - 1] = TB::fragment(sb, fb_base[r - 1], wn * WN + (r - 1) * 32 + l32, h, s);
            else
                fa[buf][r - NTL] = TA::fragment(sa, fa_base[r - NTL], wm * WM + (r - NTL) * 32 + l32, h, s);
        };
#pragma unroll
        for (int r = 0; r < kReads; ++r) read_frag(0, r, 0);
        int issued = 0;
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const int cur = s & 1;
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NTL; ++j) {
                    const int m = i * NTL + j;
#ifndef DM_DBG_NO_MFMA
                    acc[i][j] = mfma_f16_32x32x16(fa[cur][i], fb[cur][j], acc[i][j]);
#else
                    acc[i][j][0] += (float)fa[cur][i][0] * (float)fb[cur][j][0];
#endif
                    __builtin_amdgcn_sched_barrier(0);
                    if (s + 1 < kSteps && m < kReads) read_frag(cur ^ 1, m, s + 1);
                    // spread kPerTile loads evenly over the kSteps * kMfma slots
                    const int slot = s * kMfma + m;
                    if (PREFETCH && issued < kPerTile && slot * kPerTile >= issued * (kSteps * kMfma)) {
#ifndef DM_DBG_NO_DMA
                        issue_one(nbase, ab, bb, issued);
#endif
                        ++issued;
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        if (PREFETCH) advance();
    };

#ifdef DM_DBG_TIMING
    uint64_t dbg_t0 = __builtin_amdgcn_s_memtime(), dbg_r0 = __builtin_amdgcn_s_memrealtime();
    uint64_t dbg_wait = 0, dbg_tw;
#define DBG_W0 dbg_tw = __builtin_amdgcn_s_memtime();
#define DBG_W1 dbg_wait += __builtin_amdgcn_s_memtime() - dbg_tw;
#else
#define DBG_W0
#define DBG_W1
#endif
    // Prologue: STAGES-1 tiles in flight.
#pragma unroll
    for (int p = 0; p < STAGES - 1; ++p)
        if (p < n_ktiles) issue_all(p);
#ifdef DM_DBG_TIMING
    uint64_t dbg_t1 = __builtin_amdgcn_s_memtime();
#endif

    // k-tile kt is multiplied from stage kt % STAGES.  Before that, its loads must have landed
    // (only the loads of the STAGES-2 younger tiles may still be outstanding) and every
    // wavefront must be past tile kt-1, whose stage then receives tile kt+STAGES-1.
    int stage = 0;
    int kt = 0;
    for (; kt + STAGES - 1 < n_ktiles; ++kt) {
        DBG_W0
        wait_vmcnt<kPerTile * (STAGES - 2)>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        DBG_W1
        multiply(stage, stage == 0 ? STAGES - 1 : stage - 1, std::true_type{});
        asm volatile("" ::: "memory");
        stage = stage == STAGES - 1 ? 0 : stage + 1;
    }
    // drain: no more loads to issue; the number of younger tiles in flight shrinks to zero
    if (STAGES == 3 && kt + 1 < n_ktiles) {
        wait_vmcnt<kPerTile>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        multiply(stage, 0, std::false_type{});
        asm volatile("" ::: "memory");
        stage = stage == STAGES - 1 ? 0 : stage + 1;
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    multiply(stage, 0, std::false_type{});
#ifdef DM_DBG_TIMING
    uint64_t dbg_t2 = __builtin_amdgcn_s_memtime();
#endif

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
#ifdef DM_DBG_TIMING
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint64_t dbg_t3 = __builtin_amdgcn_s_memtime(), dbg_r3 = __builtin_amdgcn_s_memrealtime();
    if (tid == 0 && tile.m_off == 0 && tile.n_off == 0 && tile.mseg == 0 && tile.nseg == 0) {
        float* o = reinterpret_cast<float*>(c);
        o[0] = (float)(dbg_t1 - dbg_t0);  // prologue issue
        o[1] = (float)(dbg_t2 - dbg_t1);  // main loop
        o[2] = (float)(dbg_t3 - dbg_t2);  // epilogue
        o[3] = (float)dbg_wait;           // wait + barrier inside the loop
        o[4] = (float)(dbg_r3 - dbg_r0);  // 100 MHz ticks
        o[5] = (float)n_ktiles;
    }
#endif
}

template <int BM, int BN, int STAGES, bool AKC, bool BKC, class TC>
hipError_t launch_one(const GemmTables& t, float alpha, float beta, hipStream_t st)
{
    constexpr int lds_bytes = STAGES * (BM + BN) * BK * 2;
    auto kern = gemm_f16_kernel<BM, BN, STAGES, AKC, BKC, TC>;
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

template <int BM, int BN, int STAGES, class TC>
hipError_t launch_shape(const GemmPlan& p, float alpha, float beta, hipStream_t st)
{
    const GemmTables& t = p.t;
    if (t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, STAGES, true, true, TC>(t, alpha, beta, st);
    if (t.a_kcontig && !t.b_kcontig) return launch_one<BM, BN, STAGES, true, false, TC>(t, alpha, beta, st);
    if (!t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, STAGES, false, true, TC>(t, alpha, beta, st);
    return launch_one<BM, BN, STAGES, false, false, TC>(t, alpha, beta, st);
}

// Tile shapes: 256x256 (two 64 KiB stages), 256x128 (three 48 KiB stages), 128x128 (two 32 KiB
// stages, so that two workgroups share a CU).
template <class TC>
hipError_t launch_out(const GemmPlan& p, float alpha, float beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 256 && bn == 256) return launch_shape<256, 256, 2, TC>(p, alpha, beta, st);
    if (bm == 256 && bn == 128) return launch_shape<256, 128, 3, TC>(p, alpha, beta, st);
    if (bm == 128 && bn == 128) return launch_shape<128, 128, 2, TC>(p, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_f16(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    if (p.out_dtype == DMATH_F16) return launch_out<_Float16>(p, (float)alpha, (float)beta, st);
    return launch_out<float>(p, (float)alpha, (float)beta, st);
}

}  // namespace dm
