// The fp16-input / fp32-accumulate MFMA pipeline shared by the GEMM and the implicit-GEMM
// convolution kernels (v_mfma_f32_32x32x16_f16, gfx950).
//
// A workgroup of 4 wavefronts (2 x 2, or 1 x 4 for the 224-row tile) multiplies a BM x BN tile; k is walked 64 at a time
// through a ring of STAGES LDS stages.
//
// Global -> LDS without registers: every wavefront issues global_load_lds_dwordx4, which
// writes the 16 bytes fetched by lane p to (LDS base in M0) + 16*p.  A 1 KiB LDS segment is
// filled per instruction; the swizzles below are applied by choosing WHICH global chunk each
// lane fetches.  The loads are inline assembly with explicit s_waitcnt vmcnt(), so that the
// compiler neither sees nor serialises them; STAGES-1 tiles are in flight while one is
// multiplied.
//
// LDS layouts, both as the operand lies in memory:
//   k unit-stride operand  : [mn][64 k], 128-byte rows, 16-byte chunk index XOR ((mn^(mn>>3))&7);
//                            the MFMA fragment of a lane (8 consecutive k of one row) is one
//                            ds_read_b128, conflict-free
//   m/n unit-stride operand: [k][mn], 16-byte chunk index XOR ((k&3)<<2) (64-column tiles:
//                            XOR (((k>>1)&1)<<2)); fragments come from
//                            two ds_read_b64_tr_b16 (the gfx950 transposing LDS read: inside a
//                            16-lane group, lane i receives element i%4 of the 8 bytes fetched
//                            by lanes i/4, i/4+4, i/4+8, i/4+12), so a group fetches a 4(k) x
//                            16(mn) patch and every lane ends up with 4 consecutive k of its
//                            own column; the XOR puts the four k rows x two 16-column groups
//                            that 32 lanes fetch together into eight different 32-byte bank
//                            groups
//
// What a kernel supplies is a "walk": for the k-tile about to be fetched, a wavefront-uniform
// base pointer and one 32-bit byte offset per lane and 1 KiB segment for each operand, plus
// advance() to move to the next k-tile.  Operand rows need not be equidistant (the convolution
// gathers them), only 16-byte aligned and 128 bytes long per k-tile.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "lds_dma.hpp"
#include "mfma.hpp"

namespace dm {
namespace f16p {

using ldsdma::cdiv;
using ldsdma::dma16;
using ldsdma::lds_char;
using ldsdma::swz;
using ldsdma::uniform_ptr;
using ldsdma::wait_vmcnt;

constexpr int BK = 64;
constexpr int NT = 256;
typedef short v4s __attribute__((ext_vector_type(4)));


// MF: edge of the matrix instruction the fragments are read for (32: 32x32x16, 16: 16x16x32).
template <int BMN, bool KC, int MF = 32> struct OperandTile {
    static_assert(MF == 32 || (MF == 16 && BMN >= 128), "16-row fragments: tiles of 128 or more only");
    static constexpr int kInstr = BMN / 32;      // 1 KiB segments per wavefront and k-tile
    static constexpr int kBytes = BMN * BK * 2;  // one stage of this operand
    static constexpr int kChunksPerRow = KC ? 8 : BMN / 8;
    static constexpr int kRowsPerSeg = 64 / kChunksPerRow;

    // Chunk XOR of an m/n unit-stride tile for k row `row`: rows of 256 bytes or more all start
    // on the same bank, so the four rows a transposing read touches are spread by two chunk bits;
    // 128-byte rows (64 columns) alternate between two bank halves already and need one bit,
    // taken from the row pair.  Both are the same for rows 4 and 16 apart.
    // 16-row fragments: the four 16-lane groups of a transposing read touch k rows r .. r+3 of the
    // four 8-row blocks of a 32-deep k-step, all in one 16-column group; a third chunk bit, the
    // parity of row bits 3 and 4, differs between any two blocks that are 8 or 16 rows apart, so
    // whichever two groups the LDS serves together land on different banks.
    __device__ __forceinline__ static int mswz(int row)
    {
        if (MF == 16) return ((row & 3) << 2) | ((((row >> 3) ^ (row >> 4)) & 1) << 1);
        return BMN >= 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
    }

    // Row (k unit-stride: m/n index; otherwise: k index) inside the tile, and 16-byte chunk of
    // that row in memory, which this lane fetches with segment q.
    __device__ __forceinline__ static void lane_slot(int q, int wave, int lane, int& row, int& chunk)
    {
        const int seg = q * 4 + wave;
        row = seg * kRowsPerSeg + lane / kChunksPerRow;
        const int cpos = lane % kChunksPerRow;
        chunk = KC ? (cpos ^ swz(row)) : (cpos ^ mswz(row));
    }

    // byte offsets (relative to the panel origin) for a dense panel with leading dimension ld.
    // Only `len` (<= BMN) rows/columns of the tile exist (ragged last tile of a segment): loads
    // for the rest are redirected to the last existing row / 16-byte chunk, so every address
    // stays inside the operand; what they bring in only reaches accumulators that the
    // epilogue does not store.
    __device__ __forceinline__ static void offsets(int64_t ld, int mn0, int len, int wave, int lane,
                                                   uint32_t (&off)[kInstr])
    {
#pragma unroll
        for (int q = 0; q < kInstr; ++q) {
            int row, chunk;
            lane_slot(q, wave, lane, row, chunk);
            if (KC)
                off[q] = (uint32_t)((((int64_t)(mn0 + min(row, len - 1))) * ld + chunk * 8) * 2);
            else
                off[q] = (uint32_t)(((int64_t)row * ld + mn0 + min(chunk, (len - 1) >> 3) * 8) * 2);
        }
    }
    // bytes a dense panel pointer advances per k-tile
    __device__ __forceinline__ static int64_t step(int64_t ld) { return KC ? BK * 2 : BK * 2 * ld; }

    // 16-row fragments: which 8-deep block of a 32-deep k-step the 16-lane group g supplies.
    // The instruction sums over k, so any order serves as long as both operands use the same one;
    // blocks 1 and 2 are exchanged because a 128-bit read serves lanes of groups g and g+2 (or
    // g and g+1 -- the counters cannot tell which) in one turn: with the natural order the two read
    // chunks 2 apart of rows of equal parity, the same banks (counted: 40 to 50 % of the LDS
    // cycles were conflicts); exchanged, chunks 1 or 2 apart never coincide under the row XOR.
    __device__ __forceinline__ static constexpr int kgroup(int g) { return ((g & 1) << 1) | (g >> 1); }

    // Per-lane LDS byte offset (inside the operand's stage) of the fragment for k-step 0 of the
    // MF-row tile starting at mn_base.
    __device__ __forceinline__ static uint32_t frag_base(int mn_base, int lane)
    {
        if (KC) return (uint32_t)((mn_base + (lane & (MF - 1))) * 128);
        const int g = lane >> 4, i = lane & 15;
        // the 16-lane group g reads a 4 (k) x 16 (mn) patch: 32-row fragments have two column
        // groups and two k-groups of 8, 16-row fragments one column group and four k-groups
        const int row = (MF == 32 ? 8 * (g >> 1) : 8 * kgroup(g)) + (i >> 2);
        const int col = mn_base + (MF == 32 ? 16 * (g & 1) : 0) + 4 * (i & 3);
        return (uint32_t)(row * (BMN * 2) + (((col >> 3) ^ mswz(row)) << 4) + (col & 7) * 2);
    }

    // The fragment of k-step s (16 deep for 32-row fragments, 32 deep for 16-row ones); h is the
    // lane's k-group (lane / MF), mn_row its row of the tile.
    __device__ __forceinline__ static v8h fragment(const lds_char* tile, uint32_t fb, int mn_row,
                                                   int h, int s)
    {
        if (KC) {
            const int chunk = (MF == 32 ? (s << 1) + h : (s << 2) + kgroup(h)) ^ swz(mn_row);
            return *reinterpret_cast<const __attribute__((address_space(3))) v8h*>(tile + fb + (chunk << 4));
        }
        const lds_char* p = tile + fb + s * ((MF == 32 ? 16 : 32) * BMN * 2);
        v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)p);
        v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)(p + 4 * BMN * 2));
        typedef short v8s __attribute__((ext_vector_type(8)));
        v8s both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(v8h, both);
    }

    // 16-row fragments, addressed so that a read is ONE instruction: a loop-invariant lane address
    // out of a small table plus an immediate.  f: which of the wavefront's 16-row blocks, s: which
    // 32-deep k-step; the wavefront's first row mn0 is a multiple of 64.
    //   k unit-stride: chunk = (4s + g) ^ swz(row) = [g ^ (l&7) ^ (l>>3)] ^ [(4s) ^ (2f & 7)] (g = kgroup(lane/16),
    //     l = lane%16): the bracket on the right is one of eight constants, so eight lane addresses
    //     serve every fragment, the block's row offset 2048*f goes into the immediate;
    //   m/n unit-stride: the chunk XOR depends on the lane only, one lane address per block, the
    //     k-step goes into the immediate.
    static constexpr int kAddr = KC ? 8 : BMN / 32;
    __device__ __forceinline__ static void lane_addrs(int mn0, int lane, uint32_t (&x)[kAddr])
    {
        const int g = lane >> 4, l = lane & 15;
#pragma unroll
        for (int k = 0; k < kAddr; ++k) {
            if (KC)
                x[k] = (uint32_t)((mn0 + l) * 128 + (((kgroup(g) ^ (l & 7) ^ (l >> 3)) ^ k) << 4));
            else
                x[k] = frag_base(mn0 + 16 * k, lane);
        }
    }
    __device__ __forceinline__ static constexpr int addr_index(int f, int s) { return KC ? (((4 * s) ^ (2 * f)) & 7) : f; }
    __device__ __forceinline__ static constexpr int addr_imm(int f, int s) { return KC ? 2048 * f : s * (32 * BMN * 2); }
    __device__ __forceinline__ static v8h fragment16(const lds_char* at)
    {
        if (KC) return *reinterpret_cast<const __attribute__((address_space(3))) v8h*>(at);
        v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)at);
        v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3)))*)(at + 4 * BMN * 2));
        typedef short v8s __attribute__((ext_vector_type(8)));
        v8s both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(v8h, both);
    }
};

template <class TC> __device__ __forceinline__ TC to_out(float v);
template <> __device__ __forceinline__ float to_out<float>(float v) { return v; }
template <> __device__ __forceinline__ _Float16 to_out<_Float16>(float v) { return (_Float16)v; }

// The four wavefronts tile BM x BN as 2 x 2, or as 1 x 4 where BM is not a multiple of 64
// (224 rows: seven 32-row blocks per wavefront).
template <int BM, int BN> struct TileShape {
    static constexpr int WVM = BM % 64 == 0 ? 2 : 1, WVN = 4 / WVM;  // wavefronts along m and n
    static constexpr int WM = BM / WVM, WN = BN / WVN;               // wavefront tile
    static constexpr int MT = WM / 32, NTL = WN / 32;
    __device__ __forceinline__ static int wm(int wave) { return wave / WVN; }
    __device__ __forceinline__ static int wn(int wave) { return wave % WVN; }
};

// Measurement hooks of run(): nothing by default.  CycleProbe (gemm_f16.hip, opt-in build) reads
// the shader clock at these points.
struct NoProbe {
    __device__ __forceinline__ void prologue_done() {}
    __device__ __forceinline__ void wait_begin() {}
    __device__ __forceinline__ void wait_end() {}
};

// Runs the whole k-loop of one workgroup tile.  `walk` must provide
//   const char *abase, *bbase;  uint32_t aoff[BM/32], boff[BN/32];  void advance();
// describing the k-tile that is fetched next.  acc must be zeroed by the caller.
template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Probe>
__device__ __forceinline__ void run(Walk& walk, int n_ktiles, char* smem,
                                    v16f (&acc)[TileShape<BM, BN>::MT][TileShape<BM, BN>::NTL], Probe& probe)
{
    using TA = OperandTile<BM, AKC>;
    using TB = OperandTile<BN, BKC>;
    using TS = TileShape<BM, BN>;
    constexpr int WM = TS::WM, WN = TS::WN, MT = TS::MT, NTL = TS::NTL;
    constexpr int kStage = TA::kBytes + TB::kBytes;
    constexpr int kPerTile = TA::kInstr + TB::kInstr;  // loads per wavefront and k-tile
    static_assert(STAGES == 2 || STAGES == 3, "ring of two or three stages");
    const lds_char* lds = (const lds_char*)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = TS::wm(wave), wn = TS::wn(wave), h = lane >> 5, l32 = lane & 31;

    uint32_t fa_base[MT], fb_base[NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i) fa_base[i] = TA::frag_base(wm * WM + i * 32, lane);
#pragma unroll
    for (int j = 0; j < NTL; ++j) fb_base[j] = TB::frag_base(wn * WN + j * 32, lane);

    // The loads of one k-tile are numbered 0 .. kPerTile-1 (A segments first).
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

    // Ring protocol.  k-tile kt lives in stage kt % STAGES and is multiplied in 4 k-steps; the
    // fragments of step s+1 are read from LDS while step s is multiplied (register double
    // buffer).  Before the LAST step of tile kt every wavefront
    //   - waits until its own loads of tile kt+1 have landed (s_waitcnt vmcnt),
    //   - waits for its last fragment reads of tile kt (s_waitcnt lgkmcnt(0)),
    //   - meets the others at the workgroup barrier.
    // After that barrier tile kt+1 is visible to everybody and nobody reads tile kt's stage
    // any more.  So the last step of tile kt already prefetches the first fragments of tile
    // kt+1 (no LDS latency is exposed at tile boundaries), and the stage of tile kt is free for
    // tile kt+STAGES.  The loads of that tile are spread over a whole iteration, because the
    // four wavefronts run in lockstep and share one address unit that takes 16 cycles per
    // 1 KiB load: bunched into one k-step they queue behind each other and the matrix
    // instructions behind them (a 256x256 tile lost a quarter of its cycles that way).  Its
    // first kFirst loads are issued during the last step of iteration kt (right after the
    // barrier that freed the stage), the others during the first kRestSteps steps of iteration
    // kt+1:
    //   STAGES == 3: all four steps are used; the tile has until the barrier of iteration kt+2
    //                to land, and at a barrier only the loads of the tile after the next one may
    //                still be outstanding;
    //   STAGES == 2: the tile must have landed at the barrier of iteration kt+1, so its last
    //                loads are issued no later than step kRestSteps-1 of that iteration and at
    //                the barrier nothing may be outstanding.
    // The instruction order inside a step is pinned: after every MFMA one fragment read (two in
    // the narrow tiles, which have more fragments than MFMAs per step) and at most one load, so
    // neither LDS nor the memory pipeline holds up the matrix instructions.
    constexpr int kSteps = BK / 16, kMfma = MT * NTL, kReads = MT + NTL;
    constexpr int kReadsPerSlot = (kReads + kMfma - 1) / kMfma;  // 1 except for the narrow tiles
    constexpr int kRestSteps = STAGES == 3 ? kSteps - 1 : 2;
    constexpr int kFirst = (kPerTile + kRestSteps) / (kRestSteps + 1);  // loads issued in the last step
    constexpr int kRest = kPerTile - kFirst;                            // ... in steps 0 .. kRestSteps-1
    constexpr int kRestSlots = kRestSteps * kMfma;
    constexpr int kRestPerSlot = (kRest + kRestSlots - 1) / kRestSlots;
    constexpr int kFirstPerSlot = (kFirst + kMfma - 1) / kMfma;

    v8h fa[2][MT], fb[2][NTL];
    // read order: what the first MFMAs need comes first (A0, all B, then the other A)
    auto read_frag = [&](const lds_char* sa, int buf, int r, int s) {
        const lds_char* sb = sa + TA::kBytes;
        if (r == 0)
            fa[buf][0] = TA::fragment(sa, fa_base[0], wm * WM + l32, h, s);
        else if (r <= NTL)
            fb[buf][r - 1] = TB::fragment(sb, fb_base[r - 1], wn * WN + (r - 1) * 32 + l32, h, s);
        else
            fa[buf][r - NTL] = TA::fragment(sa, fa_base[r - NTL], wm * WM + (r - NTL) * 32 + l32, h, s);
    };

    // One iteration (tile kt in `stage`).  HAS_NEXT: tile kt+1 exists; DMA_REST: tile
    // kt+STAGES-1 exists (its first loads are in flight, `walk` describes it, the others are
    // issued now); DMA_FIRST: tile kt+STAGES exists (its first loads are issued in the last step).
    auto iteration = [&](int stage, auto has_next, auto dma_rest, auto dma_first) __attribute__((always_inline)) {
        constexpr bool HAS_NEXT = decltype(has_next)::value, DMA_REST = decltype(dma_rest)::value,
                       DMA_FIRST = decltype(dma_first)::value;
        const int stage1 = stage + 1 == STAGES ? 0 : stage + 1;    // tile kt+1
        const int stage_rest = stage == 0 ? STAGES - 1 : stage - 1;  // tile kt+STAGES-1
        const lds_char* sa = lds + stage * kStage;
        const lds_char* sa1 = lds + stage1 * kStage;
        const uint32_t rest_base = lds0 + stage_rest * kStage, first_base = lds0 + stage * kStage;
        const char *ab = nullptr, *bb = nullptr;
        if (DMA_REST) {
            ab = uniform_ptr(walk.abase);
            bb = uniform_ptr(walk.bbase);
        }
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            const int cur = s & 1;
            if (s == kSteps - 1) {
                if (DMA_REST) walk.advance();  // every load of tile kt+STAGES-1 has been issued
                if (DMA_FIRST) {
                    ab = uniform_ptr(walk.abase);
                    bb = uniform_ptr(walk.bbase);
                }
            }
            if (s == kSteps - 1 && HAS_NEXT) {
                probe.wait_begin();
                if (DMA_REST && STAGES == 3)
                    wait_vmcnt<kPerTile>();
                else
                    wait_vmcnt<0>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                probe.wait_end();
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NTL; ++j) {
                    const int m = i * NTL + j;
                    acc[i][j] = mfma_f16_32x32x16(fa[cur][i], fb[cur][j], acc[i][j]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int q = 0; q < kReadsPerSlot; ++q) {
                        const int r = m * kReadsPerSlot + q;
                        if (r < kReads) {
                            if (s + 1 < kSteps)
                                read_frag(sa, cur ^ 1, r, s + 1);
                            else if (HAS_NEXT)
                                read_frag(sa1, cur ^ 1, r, 0);
                        }
                    }
                    // load d of a window of n slots goes into slot floor(d * n / count): a pure
                    // function of the slot, so that every index is a constant after unrolling
                    if (DMA_REST && s < kRestSteps) {
                        const int slot = s * kMfma + m;
#pragma unroll
                        for (int q = 0; q < kRestPerSlot; ++q) {
                            const int d = cdiv(slot * kRest, kRestSlots) + q;
                            if (d < cdiv((slot + 1) * kRest, kRestSlots)) issue_one(rest_base, ab, bb, kFirst + d);
                        }
                    }
                    if (DMA_FIRST && s == kSteps - 1) {
#pragma unroll
                        for (int q = 0; q < kFirstPerSlot; ++q) {
                            const int d = cdiv(m * kFirst, kMfma) + q;
                            if (d < cdiv((m + 1) * kFirst, kMfma)) issue_one(first_base, ab, bb, d);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
    };

    // Prologue: tiles 0 .. STAGES-2 and the first loads of tile STAGES-1 in flight, tile 0 landed
    // and visible, its first fragments read.
    issue_all(0);
    if (STAGES == 3 && n_ktiles > 1) issue_all(1);
    if (n_ktiles > STAGES - 1) {
        const uint32_t sbase = lds0 + (STAGES - 1) * kStage;
        const char* ab = uniform_ptr(walk.abase);
        const char* bb = uniform_ptr(walk.bbase);
#pragma unroll
        for (int idx = 0; idx < kFirst; ++idx) issue_one(sbase, ab, bb, idx);
        wait_vmcnt<(STAGES - 2) * kPerTile + kFirst>();
    } else if (STAGES == 3 && n_ktiles > 1) {
        wait_vmcnt<kPerTile>();
    } else {
        wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < kReads; ++r) read_frag(lds, 0, r, 0);

    probe.prologue_done();
    int stage = 0;
    int kt = 0;
    auto next_stage = [&] { stage = stage + 1 == STAGES ? 0 : stage + 1; };
    for (; kt + STAGES < n_ktiles; ++kt) {
        iteration(stage, std::true_type{}, std::true_type{}, std::true_type{});
        next_stage();
    }
    for (; kt + 1 < n_ktiles; ++kt) {
        if (kt + STAGES - 1 < n_ktiles)
            iteration(stage, std::true_type{}, std::true_type{}, std::false_type{});
        else
            iteration(stage, std::true_type{}, std::false_type{}, std::false_type{});
        next_stage();
    }
    iteration(stage, std::false_type{}, std::false_type{}, std::false_type{});
}

template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk>
__device__ __forceinline__ void run(Walk& walk, int n_ktiles, char* smem,
                                    v16f (&acc)[TileShape<BM, BN>::MT][TileShape<BM, BN>::NTL])
{
    NoProbe none;
    run<BM, BN, STAGES, AKC, BKC>(walk, n_ktiles, smem, acc, none);
}

// ---------------------------------------------------------------------------------------------
// The same ring on v_mfma_f32_16x16x32_f16 fragments (2 x 2 wavefronts, tiles of 128 rows and
// columns or more).  A k-tile is two 32-deep k-steps; each step's matrix instructions are cut
// into two halves (the first and the second half of the wavefront's 16-row blocks), which gives
// the four phases that the load schedule and the barrier are laid over: the fragments of k-step 1
// are read during phases 0 and 1, the barrier sits before phase 3, and phase 3 reads the first
// fragments of the next tile.
// The four wavefronts tile BM x BN as 2 x 2, or as 1 x 4 where BM is not a multiple of 128
// (224 rows: fourteen 16-row blocks per wavefront; k unit-stride A only, whose lane addresses do
// not depend on how many blocks a wavefront has).
template <int BM, int BN> struct TileShape16 {
    static constexpr int WVM = BM % 128 == 0 ? 2 : 1, WVN = 4 / WVM;
    static constexpr int WM = BM / WVM, WN = BN / WVN;  // wavefront tile
    static constexpr int MT = WM / 16, NTL = WN / 16;
    static_assert(MT % 2 == 0, "two halves of row blocks");
    static_assert(WM % 64 == 0 || WVM == 1, "a wavefront's first row is a multiple of 64");
    static_assert(WN % 64 == 0, "a wavefront's first column is a multiple of 64");
    __device__ __forceinline__ static int wm(int wave) { return wave / WVN; }
    __device__ __forceinline__ static int wn(int wave) { return wave % WVN; }
};

// FIXED: the accumulators live in fixed accumulation registers that the compiler never sees
// (mfma.hpp: acc_f16_zero / mfma_f16_fixed / acc_f16_read; at most 32 of them); `acc` only
// receives the sums at the end.  For kernels in which the compiler renames tied accumulators.
template <int BM, int BN, int STAGES, bool AKC, bool BKC, bool FIXED = false, class Walk, class Probe>
__device__ __forceinline__ void run16(Walk& walk, int n_ktiles, char* smem,
                                      v4f (&acc)[TileShape16<BM, BN>::MT][TileShape16<BM, BN>::NTL], Probe& probe)
{
    using TA = OperandTile<BM, AKC, 16>;
    using TB = OperandTile<BN, BKC, 16>;
    using TS = TileShape16<BM, BN>;
    constexpr int WM = TS::WM, WN = TS::WN, MT = TS::MT, NTL = TS::NTL;
    constexpr int kPerTile = TA::kInstr + TB::kInstr;
    static_assert(STAGES == 2 || STAGES == 3, "ring of two or three stages");
    static_assert((AKC || TS::WVM == 2) && (BKC || TS::WVN == 2), "m/n unit-stride operands: 2 x 2 wavefronts");
    // LDS: the STAGES stages of A, then those of B.  A 16x16x32 instruction takes 16 cycles, and a
    // wavefront issues one instruction every four: between two of them there is room for three
    // others.  So in the steady state the stage of every iteration is a compile-time constant
    // (the loop is unrolled by STAGES): a fragment read is one instruction, a lane's loop-invariant
    // address plus an immediate offset (which must stay below 64 KiB: hence the two regions, with
    // B's origin inside the lane address), and the LDS address of a load is one scalar add.
    constexpr int kAStage = TA::kBytes, kBStage = TB::kBytes, kBRegion = STAGES * kAStage;
    const lds_char* lds = (const lds_char*)smem;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wave_lds = lds0 + wave * 1024;  // where this wavefront's segments start (scalar)
    // A wavefront tile of 128 x 128 (or 224 x 64) fills the accumulator register file, or nearly: the
    // compiler then has no register to spare where differently scheduled iterations meet, and spills.  So
    // there every iteration is the full one: loads are issued to the very end (the walk stays on
    // the last k-tile; what is fetched again lands in stages nobody reads any more), and the
    // last iteration reads "next" fragments it never uses.
    constexpr bool kAlwaysFull = MT * NTL * 4 >= 224;
    static_assert(!FIXED || MT * NTL <= 32, "fixed accumulators: a0 .. a127");
    if constexpr (FIXED) {
        acc_fixed_begin();
        acc_fixed_marker();
#pragma unroll
        for (int idx = 0; idx < MT * NTL; ++idx) acc_f16_zero(idx);
    }
    auto next_tile = [&]() __attribute__((always_inline)) {
        if constexpr (kAlwaysFull)
            walk.advance_or_stay();
        else
            walk.advance();
    };
    const int wm = TS::wm(wave), wn = TS::wn(wave), g = lane >> 4, l16 = lane & 15;

    // lane addresses of the fragment reads (see OperandTile::lane_addrs); B's carry the origin of
    // its region, and a second copy 32 KiB up serves the stages a 16-bit immediate cannot reach
    constexpr bool kFarA = (STAGES - 1) * kAStage + 16384 + 2048 >= 65536,
                   kFarB = (STAGES - 1) * kBStage + 16384 + 2048 >= 65536;
    uint32_t xa[TA::kAddr], xb[TB::kAddr], xa_far[kFarA ? TA::kAddr : 1], xb_far[kFarB ? TB::kAddr : 1];
    TA::lane_addrs(wm * WM, lane, xa);
    TB::lane_addrs(wn * WN, lane, xb);
#pragma unroll
    for (int k = 0; k < TB::kAddr; ++k) xb[k] += kBRegion;
    if (kFarA)
#pragma unroll
        for (int k = 0; k < TA::kAddr; ++k) xa_far[k] = xa[k] + 32768;
    if (kFarB)
#pragma unroll
        for (int k = 0; k < TB::kAddr; ++k) xb_far[k] = xb[k] + 32768;

    // load idx of a k-tile (A segments first) into `stage`
    auto issue_one = [&](int stage, const char* ab, const char* bb, int idx) {
        if (idx < TA::kInstr)
            dma16(wave_lds, stage * kAStage + idx * 4096, ab, walk.aoff[idx]);
        else
            dma16(wave_lds, kBRegion + stage * kBStage + (idx - TA::kInstr) * 4096, bb, walk.boff[idx - TA::kInstr]);
    };
    auto issue_all = [&](int stage) {
        const char* ab = uniform_ptr(walk.abase);
        const char* bb = uniform_ptr(walk.bbase);
#pragma unroll
        for (int idx = 0; idx < kPerTile; ++idx) issue_one(stage, ab, bb, idx);
        next_tile();
    };

    constexpr int kPhases = 4, kMfma = MT * NTL / 2, kReads = MT + NTL;  // per phase / per k-step
    constexpr int kRestSteps = STAGES == 3 ? kPhases - 1 : 2;
    constexpr int kFirst = (kPerTile + kRestSteps) / (kRestSteps + 1);
    constexpr int kRest = kPerTile - kFirst;
    constexpr int kRestSlots = kRestSteps * kMfma;
    constexpr int kRestPerSlot = (kRest + kRestSlots - 1) / kRestSlots;
    constexpr int kFirstPerSlot = (kFirst + kMfma - 1) / kMfma;

    v8h fa[2][MT], fb[2][NTL];
    // read order: what the first instructions need comes first (A0, all B, then the other A)
    auto read_frag = [&](int stage, int buf, int r, int s) {
        // with a constant stage the whole offset is an immediate of the read
        auto frag_a = [&](int f) {
            const int off = stage * kAStage + TA::addr_imm(f, s);
            const int k = TA::addr_index(f, s);
            if (kFarA && off >= 32768) return TA::fragment16(lds + xa_far[kFarA ? k : 0] + (off - 32768));
            return TA::fragment16(lds + xa[k] + off);
        };
        auto frag_b = [&](int f) {
            const int off = stage * kBStage + TB::addr_imm(f, s);
            const int k = TB::addr_index(f, s);
            if (kFarB && off >= 32768) return TB::fragment16(lds + xb_far[kFarB ? k : 0] + (off - 32768));
            return TB::fragment16(lds + xb[k] + off);
        };
        if (r == 0)
            fa[buf][0] = frag_a(0);
        else if (r <= NTL)
            fb[buf][r - 1] = frag_b(r - 1);
        else
            fa[buf][r - NTL] = frag_a(r - NTL);
    };

    // One iteration (tile kt in `stage`, an int or a compile-time constant).  HAS_NEXT: tile kt+1
    // exists; DMA_REST: tile kt+STAGES-1 exists (its first loads are in flight, `walk` describes
    // it, the others are issued now); DMA_FIRST: tile kt+STAGES exists (its first loads are issued
    // in the last phase).
    auto iteration = [&](auto stage_v, auto has_next, auto dma_rest, auto dma_first) __attribute__((always_inline)) {
        constexpr bool HAS_NEXT = decltype(has_next)::value, DMA_REST = decltype(dma_rest)::value,
                       DMA_FIRST = decltype(dma_first)::value;
        const int stage = stage_v;
        const int stage1 = stage + 1 == STAGES ? 0 : stage + 1;      // tile kt+1
        const int stage_rest = stage == 0 ? STAGES - 1 : stage - 1;  // tile kt+STAGES-1
        const char *ab = nullptr, *bb = nullptr;
        if (DMA_REST) {
            ab = uniform_ptr(walk.abase);
            bb = uniform_ptr(walk.bbase);
        }
#pragma unroll
        for (int p = 0; p < kPhases; ++p) {
            const int cur = p >> 1, half = p & 1;
            if (p == kPhases - 1) {
                if (DMA_REST) next_tile();  // every load of tile kt+STAGES-1 has been issued
                if (DMA_FIRST) {
                    ab = uniform_ptr(walk.abase);
                    bb = uniform_ptr(walk.bbase);
                }
            }
            if (p == kPhases - 1 && HAS_NEXT) {
                probe.wait_begin();
                if (DMA_REST && STAGES == 3)
                    wait_vmcnt<kPerTile>();
                else
                    wait_vmcnt<0>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                probe.wait_end();
                __builtin_amdgcn_sched_barrier(0);
            }
            // fragment reads of this phase: half of k-step 1's in phases 0 and 1, all of the next
            // tile's k-step 0 in phase 3
            const int r_begin = p == 1 ? kReads / 2 : 0;
            const int r_end = p == 0 ? kReads / 2 : (p == 1 || (p == 3 && HAS_NEXT)) ? kReads : 0;
            const int r_count = r_end - r_begin;
#pragma unroll
            for (int m = 0; m < kMfma; ++m) {
                const int i = half * (MT / 2) + m / NTL, j = m % NTL;
                // the wait state in front of the instruction is needed where the compiler copies
                // accumulators: between the differently scheduled iterations that run on a run-time
                // stage, not in the steady state (4-5 % of its cycles; check_isa.py looks for a
                // copy directly in front of an instruction without one)
                if constexpr (FIXED)
                    mfma_f16_fixed(i * NTL + j, fa[cur][i], fb[cur][j]);
                else
                    mfma_f16_16x16x32<std::is_same<decltype(stage_v), int>::value>(acc[i][j], fa[cur][i], fb[cur][j]);
                __builtin_amdgcn_sched_barrier(0);
                // reads m*r_count/kMfma .. (m+1)*r_count/kMfma of the phase's share go into this slot
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int r = r_begin + m * r_count / kMfma + q;
                    if (r < r_begin + (m + 1) * r_count / kMfma) {
                        if (p < 2)
                            read_frag(stage, 1, r, 1);
                        else
                            read_frag(stage1, 0, r, 0);
                    }
                }
                // load d of a window of n slots goes into slot floor(d * n / count): a pure function
                // of the slot, so that every index is a constant after unrolling
                if (DMA_REST && p < kRestSteps) {
                    const int slot = p * kMfma + m;
#pragma unroll
                    for (int q = 0; q < kRestPerSlot; ++q) {
                        const int d = cdiv(slot * kRest, kRestSlots) + q;
                        if (d < cdiv((slot + 1) * kRest, kRestSlots)) issue_one(stage_rest, ab, bb, kFirst + d);
                    }
                }
                if (DMA_FIRST && p == kPhases - 1) {
#pragma unroll
                    for (int q = 0; q < kFirstPerSlot; ++q) {
                        const int d = cdiv(m * kFirst, kMfma) + q;
                        if (d < cdiv((m + 1) * kFirst, kMfma)) issue_one(stage, ab, bb, d);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Wherever the accumulators may be touched by anything but a matrix instruction -- the
    // epilogue, and the copies the compiler may place between the differently unrolled
    // iterations below -- the matrix pipeline is drained first and every accumulator is tied to
    // a point after the drain.
    auto settle = [&]() __attribute__((always_inline)) {
        if constexpr (FIXED) return;  // nothing but matrix instructions touches the accumulators
        mfma_drain();
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j) pin(acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
    };
    using T = std::true_type;
    using F = std::false_type;

    // Prologue: tiles 0 .. STAGES-2 and the first loads of tile STAGES-1 in flight, tile 0 landed
    // and visible, its first fragments read.
    issue_all(0);
    if (STAGES == 3 && (kAlwaysFull || n_ktiles > 1)) issue_all(1);
    if (kAlwaysFull || n_ktiles > STAGES - 1) {
        const char* ab = uniform_ptr(walk.abase);
        const char* bb = uniform_ptr(walk.bbase);
#pragma unroll
        for (int idx = 0; idx < kFirst; ++idx) issue_one(STAGES - 1, ab, bb, idx);
        wait_vmcnt<(STAGES - 2) * kPerTile + kFirst>();
    } else if (STAGES == 3 && n_ktiles > 1) {
        wait_vmcnt<kPerTile>();
    } else {
        wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < kReads; ++r) read_frag(0, 0, r, 0);

    probe.prologue_done();
    if (kAlwaysFull) {
        // rounds of STAGES iterations whose stages are constants, then the n % STAGES left over
        for (int round = n_ktiles / STAGES; round > 0; --round) {
            iteration(std::integral_constant<int, 0>{}, T{}, T{}, T{});
            iteration(std::integral_constant<int, 1>{}, T{}, T{}, T{});
            if (STAGES == 3) iteration(std::integral_constant<int, 2>{}, T{}, T{}, T{});
        }
        const int left = n_ktiles % STAGES;
        if (left >= 1) iteration(std::integral_constant<int, 0>{}, T{}, T{}, T{});
        if (STAGES == 3 && left >= 2) iteration(std::integral_constant<int, 1>{}, T{}, T{}, T{});
        wait_vmcnt<0>();  // the loads issued past the end
        settle();
        return;
    }
    int kt = 0;
    // steady state: rounds of STAGES iterations whose stages are constants
    for (; kt + 2 * STAGES - 1 < n_ktiles; kt += STAGES) {
        iteration(std::integral_constant<int, 0>{}, T{}, T{}, T{});
        iteration(std::integral_constant<int, 1>{}, T{}, T{}, T{});
        if (STAGES == 3) iteration(std::integral_constant<int, 2>{}, T{}, T{}, T{});
    }
    settle();
    // what is left: up to STAGES-1 full iterations, then the ones that run out of tiles to fetch
    int stage = 0;
    auto next_stage = [&] { stage = stage + 1 == STAGES ? 0 : stage + 1; };
    for (; kt + 1 < n_ktiles; ++kt) {
        if (kt + STAGES < n_ktiles)
            iteration(stage, T{}, T{}, T{});
        else if (kt + STAGES - 1 < n_ktiles)
            iteration(stage, T{}, T{}, F{});
        else
            iteration(stage, T{}, F{}, F{});
        next_stage();
        settle();
    }
    iteration(stage, F{}, F{}, F{});
    settle();
    if constexpr (FIXED) {
        mfma_drain();
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j) acc[i][j] = acc_f16_read(i * NTL + j);
    }
}

}  // namespace f16p
}  // namespace dm
