// Re-layout with optional precision change: dst <- src for any two block grids and dtypes
// (paper section 3.3, "Data Reorganization": reshape with a change of layout and/or precision).
// The host cuts rows and columns at every block boundary of both matrices; every resulting
// cell lies in one source block and one destination block and is copied by workgroups of 256
// threads, 16 rows per workgroup, 16 bytes of the wider type per lane where alignment allows.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "context.hpp"

namespace dm {

namespace {

constexpr int kRows = 16;

template <class TD, class TS> __device__ __forceinline__ TD convert(TS v) { return static_cast<TD>(v); }

// double -> half in one rounding: first to float with round-to-odd (truncate, then set the last
// bit if anything was lost), then the float -> half conversion rounds to nearest even exactly.
template <> __device__ __forceinline__ _Float16 convert<_Float16, double>(double v)
{
    float f = static_cast<float>(v);  // round to nearest
    if (static_cast<double>(f) != v && v == v) {
        uint32_t bits = __float_as_uint(f);
        // step back towards zero if the rounding went away from zero
        if (fabs(static_cast<double>(f)) > fabs(v)) bits -= 1;
        bits |= 1u;  // sticky bit: the value is not exactly representable
        f = __uint_as_float(bits);
    }
    return static_cast<_Float16>(f);
}

// VEC elements per lane and step: 16 bytes of the wider of the two types when every cell's
// origin, leading dimensions and width allow it (the host checks), else 1.
template <class TD, class TS, int VEC>
__global__ __launch_bounds__(256) void reblock_kernel(const CopyCell* cells)
{
    const CopyCell c = cells[blockIdx.x];
    // grid.y is capped by the launcher: taller cells are walked in strides of the grid
    for (int r0 = blockIdx.y * kRows; r0 < c.rows; r0 += gridDim.y * kRows) {
        const int rows = min(kRows, c.rows - r0);
        const TS* src = static_cast<const TS*>(c.src);
        TD* dst = static_cast<TD*>(c.dst);
        const int vcols = c.cols / VEC;
        const int count = rows * vcols;
        for (int e = threadIdx.x; e < count; e += 256) {
            const int i = r0 + e / vcols, j = (e % vcols) * VEC;
            const TS* sp = src + (int64_t)i * c.src_ld + j;
            TD* dp = dst + (int64_t)i * c.dst_ld + j;
            if constexpr (VEC == 1) {
                *dp = convert<TD, TS>(*sp);
            } else {
                typedef TS vsrc __attribute__((ext_vector_type(VEC)));
                typedef TD vdst __attribute__((ext_vector_type(VEC)));
                const vsrc v = *reinterpret_cast<const vsrc*>(sp);
                vdst o;
#pragma unroll
                for (int q = 0; q < VEC; ++q) o[q] = convert<TD, TS>(v[q]);
                *reinterpret_cast<vdst*>(dp) = o;
            }
        }
    }
}

template <class TD, class TS>
hipError_t launch_pair(const CopyCell* cells, dim3 grid, bool vectors, hipStream_t st)
{
    constexpr int kVec = 16 / (sizeof(TD) > sizeof(TS) ? sizeof(TD) : sizeof(TS));
    if (vectors)
        reblock_kernel<TD, TS, kVec><<<grid, 256, 0, st>>>(cells);
    else
        reblock_kernel<TD, TS, 1><<<grid, 256, 0, st>>>(cells);
    return hipGetLastError();
}

template <class TS>
hipError_t launch_src(dmath_dtype_t dd, const CopyCell* cells, dim3 grid, bool vectors, hipStream_t st)
{
    if (dd == DMATH_F64) return launch_pair<double, TS>(cells, grid, vectors, st);
    if (dd == DMATH_F32) return launch_pair<float, TS>(cells, grid, vectors, st);
    return launch_pair<_Float16, TS>(cells, grid, vectors, st);
}

}  // namespace

// Elements per lane of the vector path for this pair of types.
int reblock_vector_width(dmath_dtype_t sd, dmath_dtype_t dd)
{
    const size_t w = elem_size(sd) > elem_size(dd) ? elem_size(sd) : elem_size(dd);
    return (int)(16 / w);
}

hipError_t launch_reblock(dmath_dtype_t sd, dmath_dtype_t dd, const CopyCell* cells, int n_cells,
                          int max_rows, bool vectors, hipStream_t st)
{
    dim3 grid(n_cells, std::min((max_rows + kRows - 1) / kRows, 65535));  // grid.y limit of the device
    if (sd == DMATH_F64) return launch_src<double>(dd, cells, grid, vectors, st);
    if (sd == DMATH_F32) return launch_src<float>(dd, cells, grid, vectors, st);
    return launch_src<_Float16>(dd, cells, grid, vectors, st);
}

}  // namespace dm
