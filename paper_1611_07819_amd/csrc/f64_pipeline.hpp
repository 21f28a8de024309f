// The fp64 MFMA pipeline for gfx950 on v_mfma_f64_16x16x4_f64, shared by the fp64 GEMM and the
// fp64 convolution kernels (paper section 1, feature d: double precision).
//
// Same structure as the fp32 pipeline: one workgroup of 4 wavefronts per BM x BN tile of C; k is
// walked 16 at a time (128-byte rows) through a three-stage LDS ring filled by
// global_load_lds_dwordx4 (16 bytes per lane straight into LDS), two tiles in flight while a
// third is multiplied, explicit s_waitcnt vmcnt(), pinned instruction order.  A wavefront owns
// its part of the tile as a grid of 16 x 16 result tiles.
//
// LDS layouts, both as the operand lies in memory:
//   k unit-stride operand  : [mn][16 k], 128-byte rows, 16-byte chunk (2 doubles) index XOR
//                            ((mn ^ (mn>>3)) & 7); one ds_read_b128 gives a lane its values for
//                            two MFMA steps
//   m/n unit-stride operand: [k][mn]; one ds_read_b64 per MFMA step, lanes on consecutive
//                            addresses
// Inside a group of 8 k the order is permuted identically for A and B: lane group g = lane/16
// supplies k = 8u + 2g + j at step j of group u.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "lds_dma.hpp"
#include "mfma.hpp"

namespace dm {
namespace f64p {

using ldsdma::cdiv;
using ldsdma::dma16;
using ldsdma::lds_char;
using ldsdma::swz;
using ldsdma::uniform_ptr;
using ldsdma::wait_vmcnt;

constexpr int BK = 16;
typedef double v2d __attribute__((ext_vector_type(2)));
constexpr int NT = 256;
constexpr int STAGES = 3;


template <int BMN, bool KC> struct OperandTile {
    static constexpr int kInstr = BMN / 32;      // 1 KiB segments per wavefront and k-tile
    static constexpr int kBytes = BMN * BK * 8;  // one stage of this operand
    static constexpr int kChunksPerRow = KC ? 8 : BMN / 2;
    static constexpr int kRowsPerSeg = 64 / kChunksPerRow;
    static constexpr int kReadsPerFrag = KC ? 1 : 2;

    // Chunk XOR of an m/n unit-stride tile ([k][mn], rows of 512 or 1024 bytes: every row starts on
    // the same bank).  A 64-bit fragment read serves 32 lanes at a time, the 16 doubles of one k row
    // and those of a row 2 or 4 further on: moving rows by 128 bytes according to the parity of row
    // bits 1 and 2 puts any such two on different bank halves (without it the counters showed
    // every such read taking two turns).
    __device__ __forceinline__ static int mswz(int row) { return (((row >> 1) ^ (row >> 2)) & 1) << 3; }

    // Which pair of k indices of an 8-deep group the 16-lane group g supplies.  The instruction sums
    // over k, so any order serves as long as both operands use the same one; pairs 1 and 2 are
    // exchanged because a 128-bit read serves lanes of two groups in one turn, and with the natural
    // order those read chunks 2 apart of rows of equal parity: the same banks.
    __device__ __forceinline__ static constexpr int kgroup(int g) { return ((g & 1) << 1) | (g >> 1); }

    // Row (k unit-stride: m/n index; otherwise: k index) inside the tile, and 16-byte chunk of
    // that row in memory, which this lane fetches with segment q (operands whose rows are gathered).
    __device__ __forceinline__ static void lane_slot(int q, int wave, int lane, int& row, int& chunk)
    {
        const int seg = q * 4 + wave;
        row = seg * kRowsPerSeg + lane / kChunksPerRow;
        const int cpos = lane % kChunksPerRow;
        chunk = KC ? (cpos ^ swz(row)) : (cpos ^ mswz(row));
    }

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
                off[q] = (uint32_t)(((int64_t)row * ld + mn0 + min(cpos ^ mswz(row), (len - 1) >> 1) * 2) * 8);
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
                tile + mn * 128 + ((((u << 2) + kgroup(g)) ^ swz(mn)) << 4));
        } else {
            const int row = 8 * u + 2 * kgroup(g) + part;
            frag[part] = *reinterpret_cast<const __attribute__((address_space(3))) double*>(
                tile + row * (BMN * 8) + (((mn >> 1) ^ mswz(row)) << 4) + (mn & 1) * 8);
        }
    }
};

template <int BMN, bool KC> struct KCheck {
    static constexpr bool ok = KC || (64 % (BMN / 2) == 0);
};

// Runs the whole k-loop of one workgroup tile (wavefronts arranged WVM x 4/WVM).  `walk` must
// provide
//   const char *abase, *bbase;  uint32_t aoff[BM/32], boff[BN/32];  void advance();
// describing the k-tile that is fetched next.  acc receives the sums (what it holds on entry is ignored).
// NS: stages of the LDS ring (k-tiles NS-1 ahead are in flight).
template <int BM, int BN, int WVM, bool AKC, bool BKC, int NS = STAGES, class Walk>
__device__ __forceinline__ void run(Walk& walk, int n_ktiles, char* smem,
                                    v4d (&acc)[BM / WVM / 16][BN / (4 / WVM) / 16])
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    constexpr int WVN = 4 / WVM;
    constexpr int WM = BM / WVM, WN = BN / WVN;  // wavefront tile
    static_assert(KCheck<BM, AKC>::ok && KCheck<BN, BKC>::ok, "m/n-major tiles must fill whole LDS segments");
    constexpr int MT = WM / 16, NTL = WN / 16;
    constexpr int kStage = TA::kBytes + TB::kBytes;
    constexpr int kPerTile = TA::kInstr + TB::kInstr;
    const lds_char* lds = (const lds_char*)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WVN, wn = wave % WVN, h = lane >> 4, l32 = lane & 15;

    static_assert(MT * NTL * 8 <= 128, "accumulators in a0 .. a127");
    acc_fixed_begin();
#pragma unroll
    for (int idx = 0; idx < MT * NTL; ++idx) acc_f64_zero(idx);

    auto issue_one = [&](uint32_t sbase, const char* ab, const char* bb, int idx) {
        if (idx < TA::kInstr)
            dma16(sbase + (idx * 4 + wave) * 1024, ab, walk.aoff[idx]);
        else
            dma16(sbase + TA::kBytes + ((idx - TA::kInstr) * 4 + wave) * 1024, bb, walk.boff[idx - TA::kInstr]);
    };
    auto issue_all = [&](int stage) {
        const uint32_t sbase = lds0 + stage * kStage;
        const char* ab = uniform_ptr(walk.abase);
        const char* bb = uniform_ptr(walk.bbase);
#pragma unroll
        for (int idx = 0; idx < kPerTile; ++idx) issue_one(sbase, ab, bb, idx);
        walk.advance();
    };

    // Ring protocol.  k-tile kt lives in stage kt % STAGES and is multiplied in groups of 8 k, each
    // group 2 MFMA steps on every pair of fragments; the fragments of group u+1 are read from LDS
    // while group u is multiplied (register double buffer), one read unit after each MFMA.
    // Before the LAST group of tile kt every wavefront
    //   - waits until its own loads of tile kt+1 have landed (s_waitcnt vmcnt),
    //   - waits for its last fragment reads of tile kt (s_waitcnt lgkmcnt(0)),
    //   - meets the others at the workgroup barrier.
    // After that barrier tile kt+1 is visible to everybody and nobody reads tile kt's stage any
    // more, so the last group of tile kt already reads the first fragments of tile kt+1 (no LDS
    // latency is exposed at tile boundaries).  Tile kt+2 is fetched during the groups before
    // that barrier into the stage of tile kt-1 (freed by the barrier of iteration kt-1); at the
    // barrier only those loads may still be outstanding.
    constexpr int kGroups = BK / 8, kMfma = 2 * MT * NTL;
    constexpr int kUnitsA = MT * TA::kReadsPerFrag, kUnits = kUnitsA + NTL * TB::kReadsPerFrag;
    constexpr int kPerSlot = (kUnits + kMfma - 1) / kMfma;
    constexpr int kDmaSlots = (kGroups - 1) * kMfma;
    static_assert(kGroups % 2 == 0, "the fragment double buffer returns to buffer 0 every tile");
    static_assert(kDmaSlots >= kPerTile, "not enough slots to spread the loads");

    v2d fa[2][MT], fb[2][NTL];
    auto read_unit = [&](const lds_char* sa, int buf, int r, int u) {
        const lds_char* sb = sa + TA::kBytes;
        if (r < kUnitsA)
            TA::read(sa, wm * WM + (r / TA::kReadsPerFrag) * 16 + l32, h, u, r % TA::kReadsPerFrag,
                     fa[buf][r / TA::kReadsPerFrag]);
        else
            TB::read(sb, wn * WN + ((r - kUnitsA) / TB::kReadsPerFrag) * 16 + l32, h, u,
                     (r - kUnitsA) % TB::kReadsPerFrag, fb[buf][(r - kUnitsA) / TB::kReadsPerFrag]);
    };

    // One iteration.  HAS_NEXT: tile kt+1 exists; HAS_DMA: tile kt+NS-1 exists and is fetched.
    // The accumulators live in fixed accumulation registers (mfma.hpp) from the first iteration to
    // the read-out after the last.
    auto iteration = [&](int stage, auto has_next, auto has_dma) __attribute__((always_inline)) {
        constexpr bool HAS_NEXT = decltype(has_next)::value, HAS_DMA = decltype(has_dma)::value;
        const int stage1 = stage + 1 == NS ? 0 : stage + 1;   // tile kt+1
        const int stage2 = stage == 0 ? NS - 1 : stage - 1;   // tile kt+NS-1 (= stage of tile kt-1)
        const lds_char* sa = lds + stage * kStage;
        const lds_char* sa1 = lds + stage1 * kStage;
        const uint32_t dbase = lds0 + stage2 * kStage;
        const char* ab = uniform_ptr(walk.abase);
        const char* bb = uniform_ptr(walk.bbase);
        int issued = 0;
#pragma unroll
        for (int u = 0; u < kGroups; ++u) {
            const int cur = u & 1;
            if (u == kGroups - 1 && HAS_NEXT) {
                if (HAS_DMA)
                    wait_vmcnt<(NS - 2) * kPerTile>();  // the tiles after the next one may still be on their way
                else
                    wait_vmcnt<0>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NTL; ++j) {
                        const int m = (s * MT + i) * NTL + j;
                        mfma_f64_fixed(i * NTL + j, fa[cur][i][s], fb[cur][j][s]);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int q = 0; q < kPerSlot; ++q) {
                            const int r = m * kPerSlot + q;
                            if (r < kUnits) {
                                if (u + 1 < kGroups)
                                    read_unit(sa, cur ^ 1, r, u + 1);
                                else if (HAS_NEXT)
                                    read_unit(sa1, cur ^ 1, r, 0);
                            }
                        }
                        const int slot = u * kMfma + m;
                        if (HAS_DMA && u < kGroups - 1 && issued < kPerTile && slot * kPerTile >= issued * kDmaSlots) {
                            issue_one(dbase, ab, bb, issued);
                            ++issued;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
        }
        if (HAS_DMA) walk.advance();
    };

    // Prologue: tiles 0 .. NS-2 in flight, tile 0 landed and visible, its first fragments read.
    static_assert(NS >= 3 && (NS - 1) * kPerTile <= 63, "ring length (the counter of outstanding loads has 6 bits)");
    issue_all(0);
#pragma unroll
    for (int t = 1; t <= NS - 2; ++t)
        if (n_ktiles > t) issue_all(t);
    if (n_ktiles > NS - 2)
        wait_vmcnt<(NS - 2) * kPerTile>();
    else
        wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < kUnits; ++r) read_unit(lds, 0, r, 0);

    int stage = 0;
    int kt = 0;
    for (; kt + NS - 1 < n_ktiles; ++kt) {
        iteration(stage, std::true_type{}, std::true_type{});
        stage = stage + 1 == NS ? 0 : stage + 1;
    }
    for (; kt + 1 < n_ktiles; ++kt) {
        iteration(stage, std::true_type{}, std::false_type{});
        stage = stage + 1 == NS ? 0 : stage + 1;
    }
    iteration(stage, std::false_type{}, std::false_type{});
    // hand the sums to the caller: the last matrix instruction has 64 cycles to go
    mfma_drain_f64();
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j) acc[i][j] = acc_f64_read(i * NTL + j);
}

}  // namespace f64p
}  // namespace dm
