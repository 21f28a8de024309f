// Re-layout with optional precision change: dst <- src for any two block grids and dtypes
// (paper section 3.3, "Data Reorganization": reshape with a change of layout and/or precision).
// The host cuts rows and columns at every block boundary of both matrices; every resulting
// cell lies in one source block and one destination block and is copied by workgroups of 256
// threads, 16 rows per workgroup.
#include <hip/hip_runtime.h>

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

template <class TD, class TS>
__global__ __launch_bounds__(256) void reblock_kernel(const CopyCell* cells)
{
    const CopyCell c = cells[blockIdx.x];
    const int r0 = blockIdx.y * kRows;
    if (r0 >= c.rows) return;
    const int rows = min(kRows, c.rows - r0);
    const TS* src = static_cast<const TS*>(c.src);
    TD* dst = static_cast<TD*>(c.dst);
    const int count = rows * c.cols;
    for (int e = threadIdx.x; e < count; e += 256) {
        const int i = r0 + e / c.cols, j = e % c.cols;
        dst[(int64_t)i * c.dst_ld + j] = convert<TD, TS>(src[(int64_t)i * c.src_ld + j]);
    }
}

template <class TS>
hipError_t launch_src(dmath_dtype_t dd, const CopyCell* cells, dim3 grid, hipStream_t st)
{
    if (dd == DMATH_F64) reblock_kernel<double, TS><<<grid, 256, 0, st>>>(cells);
    else if (dd == DMATH_F32) reblock_kernel<float, TS><<<grid, 256, 0, st>>>(cells);
    else reblock_kernel<_Float16, TS><<<grid, 256, 0, st>>>(cells);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_reblock(dmath_dtype_t sd, dmath_dtype_t dd, const CopyCell* cells, int n_cells,
                          int max_rows, hipStream_t st)
{
    dim3 grid(n_cells, (max_rows + kRows - 1) / kRows);
    if (sd == DMATH_F64) return launch_src<double>(dd, cells, grid, st);
    if (sd == DMATH_F32) return launch_src<float>(dd, cells, grid, st);
    return launch_src<_Float16>(dd, cells, grid, st);
}

}  // namespace dm
