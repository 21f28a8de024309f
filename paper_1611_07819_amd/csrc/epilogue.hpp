// Epilogue of the specialised GEMM kernels: C <- alpha*acc + beta*C (or the plain accumulators
// into a split-K workspace) from the MFMA result registers of one wavefront.
//
// A full tile stores unmasked.  A ragged last tile goes block by block (one MFMA result tile,
// 32x32 or 16x16): blocks outside the tile's extent are skipped (decided on scalars), blocks
// wholly inside it are stored unmasked, and the blocks across its edge mask every element
// without a branch, through raw buffer accesses whose masked-out lanes get an offset past the
// descriptor's extent (buffer stores with per-lane offsets issue 2.7 times slower than plain
// stores here, hence only for those blocks).  With one branch per masked element the compiler
// waited for all outstanding memory operations, stores included, before every element: the
// epilogue of a ragged 256x256 fp16 tile took 69000 cycles against 8000 for a full one.  The
// beta == 0 and beta != 0 cases are separate code; with beta != 0 the old values of a block are
// loaded together, before its stores.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "tables.hpp"

namespace dm {

template <class TC, class AccT> __device__ __forceinline__ TC epilogue_cast(AccT v) { return static_cast<TC>(v); }

// Raw buffer accesses (no stride, no swizzle): a byte offset at or past the descriptor's extent
// is dropped by the hardware (stores) or reads as zero (loads), so a masked-out lane is given
// the offset 0xFFFFFFFF instead of a branch.
typedef unsigned int epilogue_u2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void buffer_store(float v, __amdgpu_buffer_rsrc_t r, uint32_t off)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r, off, 0, 0);
}
__device__ __forceinline__ void buffer_store(_Float16 v, __amdgpu_buffer_rsrc_t r, uint32_t off)
{
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, v), r, off, 0, 0);
}
__device__ __forceinline__ void buffer_store(double v, __amdgpu_buffer_rsrc_t r, uint32_t off)
{
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(epilogue_u2, v), r, off, 0, 0);
}
template <class TC> __device__ __forceinline__ TC buffer_load(__amdgpu_buffer_rsrc_t r, uint32_t off);
template <> __device__ __forceinline__ float buffer_load<float>(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}
template <> __device__ __forceinline__ _Float16 buffer_load<_Float16>(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(_Float16, __builtin_amdgcn_raw_buffer_load_b16(r, off, 0, 0));
}
template <> __device__ __forceinline__ double buffer_load<double>(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0));
}

// E: edge of an MFMA result tile (32: 16 registers, row 8*(r/4) + 4*(lane/32) + r%4, column
// lane%32; 16: 4 registers, column lane%16, row 4*r + lane/16 (fp64) or, with QUAD, row
// 4*(lane/16) + r (the 16x16 fp32 result of the fp16 instruction)).  row0 / col0: origin of this
// wavefront's part of the tile.  MASKED: the tile is ragged.  BETA: C is read.
// c (the tile's first element), ld and the extents are the same in every lane and the tile spans
// less than 4 GiB (the plan sees to that): addresses are a scalar base plus 32-bit byte offsets.
template <int E, bool MASKED, bool BETA, bool QUAD = false, class TC, class AccT, class Acc, int MT, int NTL>
__device__ __forceinline__ void store_wave_tile(TC* c, int64_t ld, int m_len, int n_len, int row0, int col0, int lane,
                                                const Acc (&acc)[MT][NTL], AccT alpha, AccT beta)
{
    constexpr int REGS = E == 32 ? 16 : 4;
    constexpr uint32_t ES = sizeof(TC);
    typedef __attribute__((address_space(1))) char GChar;
    typedef __attribute__((address_space(1))) TC GTC;
    const uint64_t addr = reinterpret_cast<uint64_t>(c);
    const uint64_t sbase = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(addr >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)addr);
    const uint32_t ldb = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint64_t)ld * ES));  // bytes per row
    m_len = __builtin_amdgcn_readfirstlane(m_len);
    n_len = __builtin_amdgcn_readfirstlane(n_len);
    const int lane_row = E == 32 ? 4 * (lane >> 5) : QUAD ? 4 * (lane >> 4) : (lane >> 4), lane_col = lane & (E - 1);
    const uint32_t lane_off = (uint32_t)(row0 + lane_row) * ldb + (uint32_t)(col0 + lane_col) * ES;
    auto reg_row = [](int r) { return E == 32 ? 8 * (r >> 2) + (r & 3) : QUAD ? r : 4 * r; };  // the register's part of the row
    if constexpr (!MASKED) {
        GChar* base = reinterpret_cast<GChar*>(sbase);
        auto at = [&](uint32_t off) { return reinterpret_cast<GTC*>(base + off); };
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j) {
                const uint32_t blk = lane_off + (uint32_t)(i * E) * ldb + (uint32_t)(j * E) * ES;
                if constexpr (!BETA) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r)
                        *at(blk + (uint32_t)reg_row(r) * ldb) = epilogue_cast<TC>(alpha * acc[i][j][r]);
                } else {
                    AccT v[REGS];
#pragma unroll
                    for (int r = 0; r < REGS; ++r) v[r] = static_cast<AccT>(*at(blk + (uint32_t)reg_row(r) * ldb));
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        const AccT scaled = alpha * acc[i][j][r];
                        *at(blk + (uint32_t)reg_row(r) * ldb) = epilogue_cast<TC>(scaled + beta * v[r]);
                    }
                }
            }
    } else {
        // the descriptor covers the tile's rows up to the end of its last one
        const uint32_t extent = (uint32_t)(m_len - 1) * ldb + (uint32_t)n_len * ES;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(sbase), 0, (int)extent, 0x00020000);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j) {
                const int rows_left = m_len - (row0 + i * E), cols_left = n_len - (col0 + j * E);
                if (rows_left <= 0 || cols_left <= 0) continue;  // the same for the whole wavefront
                const uint32_t blk = lane_off + (uint32_t)(i * E) * ldb + (uint32_t)(j * E) * ES;
                if (rows_left >= E && cols_left >= E) {  // a whole block: plain stores (faster than buffer stores)
                    GChar* base = reinterpret_cast<GChar*>(sbase);
                    auto at = [&](uint32_t o) { return reinterpret_cast<GTC*>(base + o); };
                    if constexpr (!BETA) {
#pragma unroll
                        for (int r = 0; r < REGS; ++r)
                            *at(blk + (uint32_t)reg_row(r) * ldb) = epilogue_cast<TC>(alpha * acc[i][j][r]);
                    } else {
                        AccT v[REGS];
#pragma unroll
                        for (int r = 0; r < REGS; ++r) v[r] = static_cast<AccT>(*at(blk + (uint32_t)reg_row(r) * ldb));
#pragma unroll
                        for (int r = 0; r < REGS; ++r) {
                            const AccT scaled = alpha * acc[i][j][r];
                            *at(blk + (uint32_t)reg_row(r) * ldb) = epilogue_cast<TC>(scaled + beta * v[r]);
                        }
                    }
                    continue;
                }
                uint32_t off[REGS];
#pragma unroll
                for (int r = 0; r < REGS; ++r)
                    off[r] = (lane_col < cols_left && lane_row + reg_row(r) < rows_left) ? blk + (uint32_t)reg_row(r) * ldb
                                                                                        : 0xFFFFFFFFu;
                if constexpr (!BETA) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r) buffer_store(epilogue_cast<TC>(alpha * acc[i][j][r]), rsrc, off[r]);
                } else {
                    AccT v[REGS];
#pragma unroll
                    for (int r = 0; r < REGS; ++r) v[r] = static_cast<AccT>(buffer_load<TC>(rsrc, off[r]));
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        const AccT scaled = alpha * acc[i][j][r];
                        buffer_store(epilogue_cast<TC>(scaled + beta * v[r]), rsrc, off[r]);
                    }
                }
            }
    }
}

// The whole epilogue of a workgroup tile (wavefront part at row0 / col0 of it).
template <int E, int BM, int BN, class TC, bool QUAD = false, class AccT, class Acc, int MT, int NTL>
__device__ __forceinline__ void store_tile(const GemmTables& t, const Tile& tile, int split, int row0, int col0, int lane,
                                           const Acc (&acc)[MT][NTL], AccT alpha, AccT beta)
{
    const bool full = tile.m_len == BM && tile.n_len == BN;
    if (t.split_k > 1) {  // partial sums; the fixed-order reduction kernel finishes the job
        AccT* ws = static_cast<AccT*>(t.workspace) + (int64_t)split * t.M * t.N + (int64_t)tile.m_glob * t.N + tile.n_glob;
        if (full) store_wave_tile<E, false, false, QUAD>(ws, t.N, tile.m_len, tile.n_len, row0, col0, lane, acc, AccT(1), AccT(0));
        else store_wave_tile<E, true, false, QUAD>(ws, t.N, tile.m_len, tile.n_len, row0, col0, lane, acc, AccT(1), AccT(0));
        return;
    }
    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    TC* c = static_cast<TC*>(const_cast<void*>(pc.ptr)) + (int64_t)tile.m_off * pc.ld + tile.n_off;
    if (beta == AccT(0)) {
        if (full) store_wave_tile<E, false, false, QUAD>(c, pc.ld, tile.m_len, tile.n_len, row0, col0, lane, acc, alpha, beta);
        else store_wave_tile<E, true, false, QUAD>(c, pc.ld, tile.m_len, tile.n_len, row0, col0, lane, acc, alpha, beta);
    } else {
        if (full) store_wave_tile<E, false, true, QUAD>(c, pc.ld, tile.m_len, tile.n_len, row0, col0, lane, acc, alpha, beta);
        else store_wave_tile<E, true, true, QUAD>(c, pc.ld, tile.m_len, tile.n_len, row0, col0, lane, acc, alpha, beta);
    }
}

}  // namespace dm
