// Descriptor tables shared by the host scheduler and the kernels (plain structs, device
// memory, built once per plan and cached; paper section 3.3: operation metadata is computed
// once and remembered).
#pragma once
#include <cstdint>

namespace dm {

// Origin of one (segment x segment) panel of an operand, in elements of the operand's dtype.
// Element (mn, k) of the panel sits at ptr[mn * s_mn + k * s_k]; one of the two strides is 1.
struct Panel {
    const void* ptr;
    int64_t ld;  // leading dimension of the block that holds the panel
};

// One C tile: a rectangle inside one (m-segment x n-segment) cell, so it touches exactly one
// block of every operand.
struct Tile {
    int32_t mseg, nseg;      // cell
    int32_t m_off, n_off;    // offset of the tile inside the cell
    int32_t m_len, n_len;    // extent (<= tile size; smaller on ragged edges)
    int32_t m_glob, n_glob;  // position in the whole C (for the split-K workspace)
};

struct GemmTables {
    const Panel* a;       // [n_mseg][n_kseg]  panel origin of op(A)
    const Panel* b;       // [n_kseg][n_nseg]  panel origin of op(B)
    const Panel* c;       // [n_mseg][n_nseg]
    const int32_t* klen;  // [n_kseg] length of each k-segment
    const int32_t* ksplit;  // [split_k + 1] first k-segment of each split
    const Tile* tiles;
    int32_t n_mseg, n_nseg, n_kseg, n_tiles, split_k;
    int32_t a_kcontig, b_kcontig;  // 1: k is the unit-stride axis of the operand
    void* workspace;               // [split_k][M][N] partial sums in the accumulation type
    int64_t M, N;
};

// One rectangle of a re-layout: it lies inside one block of the source and one of the destination.
struct CopyCell {
    const void* src;
    void* dst;
    int64_t src_ld, dst_ld;
    int32_t rows, cols;
};

struct ConvGeom {
    int32_t n, c, h, w, k, r, s, pad_h, pad_w, stride_h, stride_w, oh, ow;
};

// Convolution operands are addressed through per-row pointer tables (row = image or filter),
// so any g x 1 block grid works.
struct ConvTables {
    ConvGeom g;
    const void* const* x_rows;  // [n] image rows of X / dX
    const void* const* f_rows;  // [k] filter rows of F / dF
    const void* const* y_rows;  // [n] image rows of Y / dY
    int32_t split_k;
    void* workspace;  // [split_k][M][N]
    int64_t M, N, K;  // implicit GEMM sizes of the chosen mode
    void* sink;       // 256 bytes nobody reads (the specialised kernels' masked-out lanes store there)
};

}  // namespace dm
