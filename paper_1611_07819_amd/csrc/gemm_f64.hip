// Specialised fp64 GEMM for gfx950 on v_mfma_f64_16x16x4_f64:
// C <- alpha * op(A) * op(B) + beta * C on full tiles (paper abstract: matrix multiplication;
// section 1, feature d: double precision).
//
// Same pipeline as the fp32 kernel: one workgroup of 4 wavefronts (2 x 2) per BM x BN tile of C
// inside one block; the k-panels are walked 16 at a time (128-byte rows) through a three-stage
// LDS ring filled by global_load_lds_dwordx4 (16 bytes per lane straight into LDS), two tiles
// in flight while a third is multiplied, explicit s_waitcnt vmcnt(), pinned instruction order.
// A wavefront owns a (BM/2) x (BN/2) tile as a grid of 16 x 16 result tiles.
//
// LDS layouts, both as the operand lies in memory:
//   k unit-stride operand  : [mn][16 k], 128-byte rows, 16-byte chunk (2 doubles) index XOR
//                            ((mn ^ (mn>>3)) & 7); one ds_read_b128 gives a lane its values for
//                            two MFMA steps
//   m/n unit-stride operand: [k][mn]; one ds_read_b64 per MFMA step, lanes on consecutive
//                            addresses
// Inside a group of 8 k the order is permuted identically for A and B: lane group g = lane/16
// supplies k = 8u + 2g + j at step j of group u.
//
// Preconditions (checked by the chooser): k-segments multiples of 16, 16-byte
// aligned panel origins and leading dimensions, blocks smaller than 4 GiB.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

namespace {

constexpr int BK = 16;
typedef double v2d __attribute__((ext_vector_type(2)));
constexpr int NT = 256;
constexpr int STAGES = 3;
typedef __attribute__((address_space(3))) char lds_char;

__device__ __forceinline__ int swz(int mn) { return (mn ^ (mn >> 3)) & 7; }

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

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BMN, bool KC> struct OperandTile {
    static constexpr int kInstr = BMN / 32;      // 1 KiB segments per wavefront and k-tile
    static constexpr int kBytes = BMN * BK * 8;  // one stage of this operand
    static constexpr int kChunksPerRow = KC ? 8 : BMN / 2;
    static constexpr int kRowsPerSeg = 64 / kChunksPerRow;
    static constexpr int kReadsPerFrag = KC ? 1 : 2;

    // byte offsets (relative to the panel origin) of the chunks this lane fetches at k-tile 0
    // Only `len` (<= BMN) rows/columns of the tile exist (ragged last tile): loads for the rest are
    // redirected to the last existing row / 16-byte chunk, so every address stays inside the
    // operand; what they bring in only reaches accumulators that the epilogue does not store.
    __device__ __forceinline__ static void offsets(int64_t ld, int mn0, int len, int wave, int lane,
                                                   uint32_t (&off)[kInstr])
    {
#pragma unroll
        for (int q = 0; q < kInstr; ++q) {
            const int seg = q * 4 + wave;
            const int row = seg * kRowsPerSeg + lane / kChunksPerRow;
            const int cpos = lane % kChunksPerRow;
            if (KC)
                off[q] = (uint32_t)((((int64_t)(mn0 + min(row, len - 1))) * ld + (cpos ^ swz(row)) * 2) * 8);
            else
                off[q] = (uint32_t)(((int64_t)row * ld + mn0 + min(cpos, (len - 1) >> 1) * 2) * 8);
        }
    }
    __device__ __forceinline__ static int64_t step(int64_t ld) { return KC ? BK * 8 : BK * 8 * ld; }

    // Part `part` of the fragment of group u (2 MFMA steps) for the lane whose row/column is mn
    // and whose k-group is g = lane/16.
    __device__ __forceinline__ static void read(const lds_char* tile, int mn, int g, int u, int part,
                                                v2d& frag)
    {
        if (KC) {
            frag = *reinterpret_cast<const __attribute__((address_space(3))) v2d*>(
                tile + mn * 128 + ((((u << 2) + g) ^ swz(mn)) << 4));
        } else {
            frag[part] = *reinterpret_cast<const __attribute__((address_space(3))) double*>(
                tile + ((8 * u + 2 * g + part) * BMN + mn) * 8);
        }
    }
};

template <int BMN, bool KC> struct KCheck {
    static constexpr bool ok = KC || (64 % (BMN / 2) == 0);
};

// WVM x WVN = 4: arrangement of the wavefronts over the tile.
template <int BM, int BN, int WVM, bool AKC, bool BKC>
__global__ __launch_bounds__(NT) void gemm_f64_kernel(GemmTables t, double alpha, double beta)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WVN = 4 / WVM;
    constexpr int WM = BM / WVM, WN = BN / WVN;  // wavefront tile
    static_assert(KCheck<BM, AKC>::ok && KCheck<BN, BKC>::ok, "m/n-major tiles must fill whole LDS segments");
    constexpr int MT = WM / 16, NTL = WN / 16;
    constexpr int kStage = TA::kBytes + TB::kBytes;
    constexpr int kPerTile = TA::kInstr + TB::kInstr;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const lds_char* lds = (const lds_char*)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    const Tile tile = t.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WVN, wn = wave % WVN, h = lane >> 4, l32 = lane & 15;

    v4d acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0;

    // walk of the k-panels by the loader
    // split-K: blockIdx.y owns the k-segments [ksplit[y], ksplit[y+1])
    const int split = blockIdx.y;
    const int ks_end = t.ksplit[split + 1];
    int ks = t.ksplit[split], kleft;
    int n_ktiles = 0;
    for (int s = ks; s < ks_end; ++s) n_ktiles += t.klen[s] / BK;
    Panel pa = t.a[tile.mseg * t.n_kseg + ks], pb = t.b[ks * t.n_nseg + tile.nseg];
    kleft = t.klen[ks] / BK;
    const char* abase = static_cast<const char*>(pa.ptr);
    const char* bbase = static_cast<const char*>(pb.ptr);
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];
    TA::offsets(pa.ld, tile.m_off, tile.m_len, wave, lane, aoff);
    TB::offsets(pb.ld, tile.n_off, tile.n_len, wave, lane, boff);

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
            TA::offsets(pa.ld, tile.m_off, tile.m_len, wave, lane, aoff);
            TB::offsets(pb.ld, tile.n_off, tile.n_len, wave, lane, boff);
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

    // Multiplies the tile in `stage`: 4 groups of 8 k, each group 4 MFMA steps on every pair of
    // fragments.  While group u is multiplied the fragments of group u+1 are read (register
    // double buffer), one read unit after each MFMA, and -- when PREFETCH -- the loads of the
    // tile two ahead are spread over the MFMA slots.
    auto multiply = [&](int stage, int next_stage, auto prefetch) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        constexpr int kGroups = BK / 8, kMfma = 2 * MT * NTL;
        constexpr int kUnitsA = MT * TA::kReadsPerFrag, kUnits = kUnitsA + NTL * TB::kReadsPerFrag;
        constexpr int kPerSlot = (kUnits + kMfma - 1) / kMfma;
        static_assert(kGroups * kMfma >= kPerTile, "not enough slots to spread the loads");
        const lds_char* sa = lds + stage * kStage;
        const lds_char* sb = sa + TA::kBytes;
        const uint32_t nbase = lds0 + next_stage * kStage;
        const char* ab = uniform_ptr(abase);
        const char* bb = uniform_ptr(bbase);
        v2d fa[2][MT], fb[2][NTL];
        auto read_unit = [&](int buf, int r, int u) {
            if (r < kUnitsA)
                TA::read(sa, wm * WM + (r / TA::kReadsPerFrag) * 16 + l32, h, u, r % TA::kReadsPerFrag,
                         fa[buf][r / TA::kReadsPerFrag]);
            else
                TB::read(sb, wn * WN + ((r - kUnitsA) / TB::kReadsPerFrag) * 16 + l32, h, u,
                         (r - kUnitsA) % TB::kReadsPerFrag, fb[buf][(r - kUnitsA) / TB::kReadsPerFrag]);
        };
#pragma unroll
        for (int r = 0; r < kUnits; ++r) read_unit(0, r, 0);
        int issued = 0;
#pragma unroll
        for (int u = 0; u < kGroups; ++u) {
            const int cur = u & 1;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NTL; ++j) {
                        const int m = (s * MT + i) * NTL + j;
                        acc[i][j] = mfma_f64_16x16x4(fa[cur][i][s], fb[cur][j][s], acc[i][j]);
                        __builtin_amdgcn_sched_barrier(0);
                        if (u + 1 < kGroups) {
#pragma unroll
                            for (int q = 0; q < kPerSlot; ++q)
                                if (m * kPerSlot + q < kUnits) read_unit(cur ^ 1, m * kPerSlot + q, u + 1);
                        }
                        const int slot = u * kMfma + m;
                        if (PREFETCH && issued < kPerTile && slot * kPerTile >= issued * (kGroups * kMfma)) {
                            issue_one(nbase, ab, bb, issued);
                            ++issued;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
        }
        if (PREFETCH) advance();
    };

    // Prologue: STAGES-1 tiles in flight.
#pragma unroll
    for (int p = 0; p < STAGES - 1; ++p)
        if (p < n_ktiles) issue_all(p);

    // k-tile kt is multiplied from stage kt % STAGES.  Before that, its loads must have landed
    // (only the loads of the younger tile may still be outstanding) and every wavefront must be
    // past tile kt-1, whose stage then receives tile kt+2.
    int stage = 0;
    int kt = 0;
    for (; kt + STAGES - 1 < n_ktiles; ++kt) {
        wait_vmcnt<kPerTile>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        multiply(stage, stage == 0 ? STAGES - 1 : stage - 1, std::true_type{});
        asm volatile("" ::: "memory");
        stage = stage == STAGES - 1 ? 0 : stage + 1;
    }
    if (kt + 1 < n_ktiles) {
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

    if (t.split_k > 1) {  // partial sums; the fixed-order reduction kernel finishes the job
        double* ws = static_cast<double*>(t.workspace) + (int64_t)split * t.M * t.N;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = wm * WM + i * 16 + acc16d_row(lane, r);
                    const int col = wn * WN + j * 16 + l32;
                    if (row < tile.m_len && col < tile.n_len)
                        ws[(int64_t)(tile.m_glob + row) * t.N + tile.n_glob + col] = acc[i][j][r];
                }
        return;
    }
    // epilogue: register r of a 16x16 result tile holds row 4*r + lane/16, column lane%16
    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    double* c = static_cast<double*>(const_cast<void*>(pc.ptr));
    // full tiles (the common case) store unmasked; a ragged last tile masks every element
    auto store = [&](auto ragged) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = wm * WM + i * 16 + acc16d_row(lane, r);
                    const int col = wn * WN + j * 16 + l32;
                    if constexpr (decltype(ragged)::value)
                        if (row >= tile.m_len || col >= tile.n_len) continue;
                    double* p = c + (int64_t)(tile.m_off + row) * pc.ld + tile.n_off + col;
                    double v = alpha * acc[i][j][r];
                    if (beta != 0.0) v += beta * *p;
                    *p = v;
                }
    };
    if (tile.m_len == BM && tile.n_len == BN) store(std::false_type{});
    else store(std::true_type{});
}

template <int BM, int BN, int WVM, bool AKC, bool BKC>
hipError_t launch_one(const GemmTables& t, double alpha, double beta, hipStream_t st)
{
    constexpr int lds_bytes = STAGES * (BM + BN) * BK * 8;
    auto kern = gemm_f64_kernel<BM, BN, WVM, AKC, BKC>;
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

template <int BM, int BN, int WVM>
hipError_t launch_shape(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    const GemmTables& t = p.t;
    if (t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, WVM, true, true>(t, alpha, beta, st);
    if (!t.a_kcontig && t.b_kcontig) return launch_one<BM, BN, WVM, false, true>(t, alpha, beta, st);
    if constexpr (64 % (BN / 2) == 0) {  // an m/n-major B tile must fill whole 1 KiB LDS segments
        if (t.a_kcontig) return launch_one<BM, BN, WVM, true, false>(t, alpha, beta, st);
        return launch_one<BM, BN, WVM, false, false>(t, alpha, beta, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm_f64(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    const int bm = p.info.tile_m, bn = p.info.tile_n;
    if (bm == 128 && bn == 128) return launch_shape<128, 128, 2>(p, alpha, beta, st);
    if (bm == 128 && bn == 64) return launch_shape<128, 64, 2>(p, alpha, beta, st);
    if (bm == 64 && bn == 128) return launch_shape<64, 128, 2>(p, alpha, beta, st);
    return hipErrorInvalidValue;
}

}  // namespace dm
