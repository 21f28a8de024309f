// Specialised convolution kernels for gfx950, fp16 (fp32 accumulate), fp32 and fp64: forward,
// weight gradient and data gradient as implicit GEMMs on the MFMA pipelines of f16_pipeline.hpp,
// f32_pipeline.hpp and f64_pipeline.hpp (paper abstract: convolutions; section 1: data
// reorganisation to support a series of operations, double / float / half precision).
//
// NCHW keeps pixels, not channels, contiguous, and the 3x3 taps shift the pixel index by +-1,
// which no 16-byte load can follow.  So the activations are first rewritten into a
// zero-bordered channels-last copy in the pool,
//     Xp[n][h + 2*pad_h][w + 2*pad_w][c]          (borders zeroed once, when the copy is allocated)
// after which row (n, oh, ow) of the lowered matrix for tap (r, s) is the contiguous c-vector
// at Xp[n][oh*stride + r][ow*stride + s][:]: a k unit-stride operand whose rows are gathered,
// with K ordered (r, s, c) and no masks.  The filter is permuted to the same K order, Fp[k][(r,s,c)].
//   forward        : Y[m, k]   = sum_K  Xp-rows[m, K] * Fp[k, K]          (N,T)-like, M = n*oh*ow
//   weight gradient: dF[k, K]  = sum_m  Yt[m, k] * Xp-rows[m, K]          (T,N)-like, deep sum over
//                    m, split over workgroups, fixed-order reduction; Yt = dY rewritten
//                    channels-last, [m][k].
//   data gradient  : the forward kernel again (stride 1), over the zero-bordered channels-last
//                    copy of dY (padding r-1-pad, pixels spread out by the stride) with the filter
//                    rotated by 180 degrees and its channel roles swapped, Gp[c][(r',s',k)].
// Channel and filter counts that are not multiples of 64 are rounded up in the copies (the pad
// channels stay zero, as the allocation left them; stores skip the pad filters), and a pixel count
// n*oh*ow that is not a multiple of the pipeline's k-tile (64 pixels fp16, 32 fp32, 16 fp64) reads zeros
// past its end (an extra, never-written image in Xp, extra rows in Yt).
// A rewrite is skipped when the caller says the copy is still current (the context keeps the
// copies and the version of the matrix each was made from); otherwise it is part of the call.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "context.hpp"
#include "f16_pipeline.hpp"
#include "f32_pipeline.hpp"
#include "f64_pipeline.hpp"

namespace dm {

namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
constexpr int NT = 256;

// What the kernels below need to know about a pipeline.
// Accumulators of the 32x32 MFMAs (fp16, fp32): 16 registers, register r of lane l holds row
// 8*(r/4) + 4*(l/32) + r%4 and column l%32, so four consecutive registers are four consecutive rows.
struct Acc32 {
    using AccT = float;
    using Acc = v16f;
    static constexpr int kRegs = 16, kEdge = 32;
    static constexpr bool kRowQuads = true;
    __device__ __forceinline__ static int row(int lane, int r) { return acc32_row(lane, r); }
    __device__ __forceinline__ static int col(int lane) { return acc32_col(lane); }
};
// Accumulators of the 16x16 fp64 MFMA: 4 registers, register r of lane l holds row 4*r + l/16.
struct Acc16d {
    using AccT = double;
    using Acc = v4d;
    static constexpr int kRegs = 4, kEdge = 16;
    static constexpr bool kRowQuads = false;
    __device__ __forceinline__ static int row(int lane, int r) { return acc16d_row(lane, r); }
    __device__ __forceinline__ static int col(int lane) { return acc16d_col(lane); }
};

// Accumulators of the 16x16x32 fp16 MFMA: 4 registers, register r of lane l holds row
// 4*(l/16) + r and column l%16: the four registers are four consecutive rows.
struct Acc16q {
    using AccT = float;
    using Acc = v4f;
    static constexpr int kRegs = 4, kEdge = 16;
    static constexpr bool kRowQuads = true;
    __device__ __forceinline__ static int row(int lane, int r) { return 4 * (lane >> 4) + r; }
    __device__ __forceinline__ static int col(int lane) { return lane & 15; }
};

struct PipeF16 : Acc32 {
    using Elem = _Float16;
    static constexpr int BK = f16p::BK;
    template <int BMN, bool KC> using Tile = f16p::OperandTile<BMN, KC>;
    template <int BM, int BN> using Shape = f16p::TileShape<BM, BN>;
    template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Acc>
    __device__ __forceinline__ static void run(Walk& walk, int n_ktiles, char* smem, Acc& acc)
    {
        f16p::run<BM, BN, STAGES, AKC, BKC>(walk, n_ktiles, smem, acc);
    }
    static constexpr int lds_bytes(int bm, int bn, int stages) { return stages * (bm + bn) * BK * 2; }
};
// fp16 on 16x16x32 fragments (tiles of 128 rows and columns or more)
struct PipeF16Q : Acc16q {
    using Elem = _Float16;
    static constexpr int BK = f16p::BK;
    template <int BMN, bool KC> using Tile = f16p::OperandTile<BMN, KC, 16>;
    template <int BM, int BN> using Shape = f16p::TileShape16<BM, BN>;
    template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Acc>
    __device__ __forceinline__ static void run(Walk& walk, int n_ktiles, char* smem, Acc& acc)
    {
        f16p::NoProbe none;
        f16p::run16<BM, BN, STAGES, AKC, BKC>(walk, n_ktiles, smem, acc, none);
    }
    static constexpr int lds_bytes(int bm, int bn, int stages) { return stages * (bm + bn) * BK * 2; }
};
// ... with the accumulators in fixed registers (the weight gradient)
struct PipeF16QF : PipeF16Q {
    template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Acc>
    __device__ __forceinline__ static void run(Walk& walk, int n_ktiles, char* smem, Acc& acc)
    {
        f16p::NoProbe none;
        f16p::run16<BM, BN, STAGES, AKC, BKC, true>(walk, n_ktiles, smem, acc, none);
    }
};
struct PipeF32 : Acc32 {
    using Elem = float;
    static constexpr int BK = f32p::BK;
    template <int BMN, bool KC> using Tile = f32p::OperandTile<BMN, KC>;
    template <int BM, int BN> struct Shape {  // wavefronts 2 x 2
        static constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 32, NTL = WN / 32;
        __device__ __forceinline__ static int wm(int wave) { return wave / 2; }
        __device__ __forceinline__ static int wn(int wave) { return wave % 2; }
    };
    template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Acc>
    __device__ __forceinline__ static void run(Walk& walk, int n_ktiles, char* smem, Acc& acc)
    {
        static_assert(STAGES == f32p::STAGES, "the fp32 ring has three stages");
        f32p::run<BM, BN, 2, AKC, BKC>(walk, n_ktiles, smem, acc);
    }
    static constexpr int lds_bytes(int bm, int bn, int stages) { return stages * (bm + bn) * BK * 4; }
};

struct PipeF64 : Acc16d {
    using Elem = double;
    static constexpr int BK = f64p::BK;
    template <int BMN, bool KC> using Tile = f64p::OperandTile<BMN, KC>;
    template <int BM, int BN> struct Shape {  // wavefronts 2 x 2, 16 x 16 result tiles
        static constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 16, NTL = WN / 16;
        __device__ __forceinline__ static int wm(int wave) { return wave / 2; }
        __device__ __forceinline__ static int wn(int wave) { return wave % 2; }
    };
    template <int BM, int BN, int STAGES, bool AKC, bool BKC, class Walk, class Acc>
    __device__ __forceinline__ static void run(Walk& walk, int n_ktiles, char* smem, Acc& acc)
    {
        static_assert(STAGES == f64p::STAGES, "the fp64 ring has three stages");
        f64p::run<BM, BN, 2, AKC, BKC>(walk, n_ktiles, smem, acc);
    }
    static constexpr int lds_bytes(int bm, int bn, int stages) { return stages * (bm + bn) * BK * 8; }
};

template <class TC, class A> __device__ __forceinline__ TC to_out(A v) { return (TC)v; }

// ------------------------------------------------------------------------------------------
// layout rewrites
// ------------------------------------------------------------------------------------------

// src rows: image n -> [ch][hw] elements (NCHW inside a row).  dst: [n][HP][WP][chd] with pixel
// (y, x) of the image placed at (ph + y*sy, pw + x*sx); sy = sx = 1 except for the data gradient
// of a strided convolution, which reads dY spread out with zeros between its pixels.  One
// workgroup of 1024 threads moves 64 channels of `chunk` pixels of one image (blockIdx.y: which
// chunk) through LDS: fully coalesced 16-byte reads of the 64 planes, 16-byte writes of
// consecutive channels per lane.  dst has chd >= ch channels per pixel (a multiple of 64);
// channels ch .. chd-1 are written as zeros.
// The chunk is chosen (tcl_chunk) so that two or three workgroups share a CU: a workgroup reads
// all its planes, waits, and then writes, so a lone workgroup per CU leaves the memory system idle
// in one direction at a time (one chunk of 784 pixels per workgroup: 11.9 us for the 55 MB of
// configuration 5; two chunks of 392: see the profile summary).
// LDS banks (64 of 4 bytes): the plane stride (pixels + pad) is 8 bytes mod 32 for 16-bit and 32-bit
// elements.  Writes: a lane's 16 bytes go out as two 8-byte halves, lanes 16 apart hit the same
// banks, so every other group of 16 lanes writes its upper half first.  Reads: a wavefront takes
// 16 (fp16) or 8 (fp32) pixels x half of the channel groups at a time, which puts the channel
// groups 8 rows = 64 bytes apart on four (eight) different bank groups and the pixels of a group
// side by side (with all eight channel groups of 8 pixels in one instruction, groups 0 and 4 met on
// the same banks: the counters showed two turns per access).
constexpr int kTclThreads = 1024;
template <class T> constexpr int tcl_max_pixels() { return 2048 / sizeof(T); }  // 64 planes: 128 KiB of LDS
template <class T> __host__ __device__ inline int tcl_stride(int px)
{
    // 16-bit: stride = 4 mod 16 elements; 32-bit: stride = 2 mod 8
    return sizeof(T) == 2 ? px + ((20 - px % 16) % 16) : px + ((10 - px % 8) % 8);
}
// pixels per workgroup: whole planes where they are small or the grid fills the chip anyway,
// otherwise the fewest parts (of a multiple of 16 pixels) that give every CU two workgroups
template <class T> inline int tcl_chunk(int groups, int hw)
{
    int parts = (hw + tcl_max_pixels<T>() - 1) / tcl_max_pixels<T>();
    while (groups * parts < 512 && hw / (parts + 1) >= 128) ++parts;
    const int chunk = ((hw + parts - 1) / parts + 15) / 16 * 16;
    return std::min(chunk, tcl_max_pixels<T>());
}

// One NCHW -> channels-last rewrite: what a workgroup needs to know.
struct TclJob {
    const void* const* src_rows;
    void* dst;
    int ch, chd, h, w, ph, pw, sy, sx, hp, wp;
    int chunk;   // pixels per workgroup
    int vb;      // bytes per global read: 16 where a plane is a multiple of 16 bytes, 8 where of 8, else one element
    int groups;  // images x groups of 64 channels
    int blocks;  // groups x chunks per plane (0: no such job)
};

// group: which (image, 64 channels); part: which chunk of the plane.  Every thread of the workgroup calls it.
template <class T, int VB> __device__ __forceinline__ void tcl_body(const TclJob& j, int group, int part, char* smem)
{
    const void* const* src_rows = j.src_rows;
    T* const dst = static_cast<T*>(j.dst);
    const int ch = j.ch, chd = j.chd, h = j.h, w = j.w, ph = j.ph, pw = j.pw, sy = j.sy, sx = j.sx, hp = j.hp,
              wp = j.wp, chunk = j.chunk;
    T* planes = reinterpret_cast<T*>(smem);  // [64][stride]
    constexpr int VEC = VB / (int)sizeof(T);
    constexpr int kPerLane = 16 / (int)sizeof(T), kLanesPerPixel = 64 / kPerLane;  // 16-byte writes
    const int hw = h * w;
    const int p0 = part * chunk, pixels = min(chunk, hw - p0);  // this workgroup's pixels
    const int stride = tcl_stride<T>(min(chunk, hw));
    const int chunks_c = chd / 64;
    const int n = group / chunks_c, c0 = (group % chunks_c) * 64;
    const int planes_here = min(64, ch - c0);  // the last group of a padded channel count is short
    const T* src = static_cast<const T*>(src_rows[n]) + (int64_t)c0 * hw + p0;
    const int vec_per_plane = pixels / VEC;
    const int swap = (threadIdx.x >> 4) & 1;  // which half of its 16 bytes this lane writes first
    for (int e = threadIdx.x; e < 64 * vec_per_plane; e += kTclThreads) {
        const int c = e / vec_per_plane, v = e - c * vec_per_plane;
        // planes past the last channel read plane 0 instead (unconditional loads) and store zeros
        const bool real = c < planes_here;
        const T* from = src + (int64_t)(real ? c : 0) * hw + v * VEC;
        if (VEC == 1) {
            const T d = *from;
            planes[c * stride + v] = real ? d : (T)0.f;
            continue;
        }
        v2u* q = reinterpret_cast<v2u*>(planes + c * stride + v * VEC);  // rows are 8-byte aligned
        const uint32_t keep = real ? ~0u : 0u;
        if (VB == 16) {
            const v4u d = *reinterpret_cast<const v4u*>(from);
            const v2u lo = v2u{d[0] & keep, d[1] & keep}, hi = v2u{d[2] & keep, d[3] & keep};
            q[swap] = swap ? hi : lo;
            q[swap ^ 1] = swap ? lo : hi;
        } else {
            const v2u d = *reinterpret_cast<const v2u*>(from);
            q[0] = v2u{d[0] & keep, d[1] & keep};
        }
    }
    __syncthreads();
    T* out = dst + ((int64_t)n * hp * wp) * chd + c0;
    typedef T vout __attribute__((ext_vector_type(kPerLane)));
    // a wavefront's 64 lanes: G channel groups x 64/G pixels (G: all groups for 64-bit elements, half otherwise)
    constexpr int G = sizeof(T) == 8 ? kLanesPerPixel : kLanesPerPixel / 2, H = kLanesPerPixel / G, PW = 64 / G;
    const int items = (pixels + PW - 1) / PW * H * 64;
    for (int e = threadIdx.x; e < items; e += kTclThreads) {
        const int wi = e >> 6, l = e & 63;
        const int pix = (wi / H) * PW + l / G, cg = (wi % H) * G + l % G;
        if (pix >= pixels) continue;
        const int y = (p0 + pix) / w, x = (p0 + pix) - y * w;
        vout v;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) v[i] = planes[(cg * kPerLane + i) * stride + pix];
        *reinterpret_cast<vout*>(out + ((int64_t)(y * sy + ph) * wp + (x * sx + pw)) * chd + cg * kPerLane) = v;
    }
}

// F[k][c][r][s] -> Fp[k][(r,s,cp)], cp >= c channels per tap (the pad channels written as zeros)
template <class T>
__global__ __launch_bounds__(256) void filter_to_rsc_kernel(const void* const* f_rows, int c, int cp, int rs,
                                                            int k, T* fp)
{
    const int64_t total = (int64_t)k * cp * rs;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int kk = (int)(e / (cp * rs)), rem = (int)(e % (cp * rs));
        const int q = rem / cp, cc = rem % cp;  // destination order (rs, cp)
        fp[e] = cc < c ? static_cast<const T*>(f_rows[kk])[cc * rs + q] : (T)0.f;
    }
}

// The same through LDS: workgroup (channel chunk, filter) reads 64 channels x rs taps, which lie
// contiguously in F, and writes rs runs of 64 consecutive channels (both sides coalesced; the
// tile's rows are an odd number of elements apart).
template <class T>
__global__ __launch_bounds__(256) void filter_to_rsc_tiled_kernel(const void* const* f_rows, int c, int cp, int rs,
                                                                  T* fp)
{
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    T* tile = reinterpret_cast<T*>(smem_raw);
    const int rsp = rs | 1, kk = blockIdx.y, c0 = blockIdx.x * 64, nch = min(64, c - c0);
    const int tid = threadIdx.x;
    if (nch > 0) {
        const T* src = static_cast<const T*>(f_rows[kk]) + (int64_t)c0 * rs;
        for (int i = tid; i < nch * rs; i += 256) {
            const int ch = i / rs;
            tile[ch * rsp + (i - ch * rs)] = src[i];
        }
    }
    __syncthreads();
    T* dst = fp + (int64_t)kk * rs * cp + c0;
    for (int i = tid; i < 64 * rs; i += 256) {
        const int q = i >> 6, ch = i & 63;
        dst[(int64_t)q * cp + ch] = ch < nch ? tile[ch * rsp + q] : (T)0.f;
    }
}

template <class T>
void filter_to_rsc(const void* const* f_rows, int c, int cp, int rs, int k, T* fp, hipStream_t st)
{
    const size_t lds = (size_t)64 * (rs | 1) * sizeof(T);
    if (lds <= 64 * 1024)
        filter_to_rsc_tiled_kernel<T><<<dim3(cp / 64, k), 256, lds, st>>>(f_rows, c, cp, rs, fp);
    else
        filter_to_rsc_kernel<T><<<512, 256, 0, st>>>(f_rows, c, cp, rs, k, fp);
}

// F[k][c][r][s] -> Gp[c][(r',s',kp)] with r' = R-1-r, s' = S-1-s: the filter of the forward
// convolution (over dY, channels k) that computes the data gradient; kp >= k filters per tap
// (the pad filters written as zeros).  A tiled transpose of F seen as [k][c*rs]: 64 filters x 64
// columns per workgroup through LDS, the taps of a channel written in reverse order.
template <class T>
__global__ __launch_bounds__(256) void filter_to_rsk_rotated_tiled_kernel(const void* const* f_rows, int c, int rs,
                                                                          int k, int kp, T* gp)
{
    __shared__ T tile[64][65];
    const int crs = c * rs, col0 = blockIdx.x * 64, k0 = blockIdx.y * 64, tid = threadIdx.x;
    {
        // 16 rows per thread: all row pointers first, then all elements, so that the loads overlap
        const int col = tid & 63, row0 = tid >> 6;
        const bool col_ok = col0 + col < crs;
        const T* src[16];
        T v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) src[j] = static_cast<const T*>(f_rows[min(k0 + row0 + 4 * j, k - 1)]);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = col_ok ? src[j][col0 + col] : (T)0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) tile[row0 + 4 * j][col] = k0 + row0 + 4 * j < k ? v[j] : (T)0.f;
    }
    __syncthreads();
    for (int i = tid; i < 64 * 64; i += 256) {
        const int col = i >> 6, row = i & 63, cidx = col0 + col;
        if (cidx >= crs) continue;
        const int cc = cidx / rs, q = cidx - cc * rs;
        gp[((int64_t)cc * rs + (rs - 1 - q)) * kp + k0 + row] = tile[row][col];
    }
}

// The bodies of filter_to_rsc_tiled_kernel and filter_to_rsk_rotated_tiled_kernel for one quarter
// (256 threads, t = its thread index) of a 1024-thread workgroup; every thread of the workgroup
// calls them (`active`: this quarter has work), the barrier inside is the workgroup's.
template <class T>
__device__ __forceinline__ void filter_rsc_quarter(const void* const* f_rows, int c, int cp, int rs, T* fp, int kk,
                                                   int c0, T* tile, int t, bool active)
{
    const int rsp = rs | 1, nch = min(64, c - c0);
    if (active && nch > 0) {
        const T* src = static_cast<const T*>(f_rows[kk]) + (int64_t)c0 * rs;
        for (int i = t; i < nch * rs; i += 256) {
            const int ch = i / rs;
            tile[ch * rsp + (i - ch * rs)] = src[i];
        }
    }
    __syncthreads();
    if (!active) return;
    T* dst = fp + (int64_t)kk * rs * cp + c0;
    for (int i = t; i < 64 * rs; i += 256) {
        const int q = i >> 6, ch = i & 63;
        dst[(int64_t)q * cp + ch] = ch < nch ? tile[ch * rsp + q] : (T)0.f;
    }
}

template <class T>
__device__ __forceinline__ void filter_rotated_quarter(const void* const* f_rows, int c, int rs, int k, int kp, T* gp,
                                                       int col0, int k0, T* tile /* [64][65] */, int t, bool active)
{
    const int crs = c * rs;
    if (active) {
        const int col = t & 63, row0 = t >> 6;
        const bool col_ok = col0 + col < crs;
        const T* src[16];
        T v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) src[j] = static_cast<const T*>(f_rows[min(k0 + row0 + 4 * j, k - 1)]);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = col_ok ? src[j][col0 + col] : (T)0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) tile[(row0 + 4 * j) * 65 + col] = k0 + row0 + 4 * j < k ? v[j] : (T)0.f;
    }
    __syncthreads();
    if (!active) return;
    for (int i = t; i < 64 * 64; i += 256) {
        const int col = i >> 6, row = i & 63, cidx = col0 + col;
        if (cidx >= crs) continue;
        const int cc = cidx / rs, q = cidx - cc * rs;
        gp[((int64_t)cc * rs + (rs - 1 - q)) * kp + k0 + row] = tile[row * 65 + col];
    }
}

// A filter permutation that rides along with the rewrites of the activations.
struct FilterJob {
    int kind;  // 0: none, 1: F -> Fp[k][(r,s,cp)], 2: F -> Gp[c][(r',s',kp)]
    const void* const* f_rows;
    void* out;
    int c, cp, rs, k, kp;
    int tiles_x;  // kind 1: groups of 64 channels; kind 2: tiles of 64 columns of [k][c*rs]
    int tiles;    // kind 1: tiles_x x filters; kind 2: tiles_x x tiles of 64 filters
    int blocks;   // workgroups: four tiles each
};
struct RelayoutJobs {
    TclJob a, b;
    FilterJob f;
};

// Every re-layout a convolution call needs, in one launch: the short filter permutation no longer
// waits for (or delays) the rewrites of the activations behind a launch boundary of its own.
// Workgroups [0, f.blocks) permute the filter, four tiles each (one per 256 threads); the next
// a.blocks rewrite tensor a, the last b.blocks tensor b.
template <class T> __global__ __launch_bounds__(kTclThreads) void relayout_kernel(RelayoutJobs r)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int bid = blockIdx.x;
    if (bid < r.f.blocks) {
        const int quarter = threadIdx.x >> 8, t = threadIdx.x & 255, tile_idx = bid * 4 + quarter;
        const bool active = tile_idx < r.f.tiles;
        const int tx = active ? tile_idx % r.f.tiles_x : 0, ty = active ? tile_idx / r.f.tiles_x : 0;
        if (r.f.kind == 1) {
            T* tile = reinterpret_cast<T*>(smem) + quarter * 64 * (r.f.rs | 1);
            filter_rsc_quarter<T>(r.f.f_rows, r.f.c, r.f.cp, r.f.rs, static_cast<T*>(r.f.out), ty, tx * 64, tile, t, active);
        } else {
            T* tile = reinterpret_cast<T*>(smem) + quarter * 64 * 65;
            filter_rotated_quarter<T>(r.f.f_rows, r.f.c, r.f.rs, r.f.k, r.f.kp, static_cast<T*>(r.f.out), tx * 64, ty * 64,
                                      tile, t, active);
        }
        return;
    }
    bid -= r.f.blocks;
    const bool first = bid < r.a.blocks;
    const TclJob& j = first ? r.a : r.b;
    if (!first) bid -= r.a.blocks;
    const int group = bid % j.groups, part = bid / j.groups;
    if (j.vb == 16)
        tcl_body<T, 16>(j, group, part, smem);
    else if (j.vb == 8)
        tcl_body<T, 8>(j, group, part, smem);
    else
        tcl_body<T, sizeof(T)>(j, group, part, smem);
}

// NCHW rows -> zero-bordered channels-last copy: the job description and the LDS it needs.
template <class T>
static TclJob tcl_job(const void* const* src_rows, int n, int ch, int chd, int h, int w, int ph, int pw, int sy,
                      int sx, int hp, int wp, T* dst, int* lds)
{
    TclJob j{};
    const int hw = h * w, plane_bytes = hw * (int)sizeof(T);
    j.src_rows = src_rows; j.dst = dst;
    j.ch = ch; j.chd = chd; j.h = h; j.w = w; j.ph = ph; j.pw = pw; j.sy = sy; j.sx = sx; j.hp = hp; j.wp = wp;
    j.groups = n * (chd / 64);
    j.chunk = tcl_chunk<T>(j.groups, hw);
    j.vb = plane_bytes % 16 == 0 ? 16 : plane_bytes % 8 == 0 ? 8 : (int)sizeof(T);
    j.blocks = j.groups * ((hw + j.chunk - 1) / j.chunk);
    *lds = std::max(*lds, 64 * tcl_stride<T>(std::min(j.chunk, hw)) * (int)sizeof(T));
    return j;
}
// The filter permutation as a job of the same launch; false: too large for that (the caller
// launches the kernel of its own).
template <class T>
static bool filter_job(int kind, const void* const* f_rows, int c, int cp, int rs, int k, int kp, T* out,
                       FilterJob* f, int* lds)
{
    const size_t tile_bytes = (kind == 1 ? (size_t)64 * (rs | 1) : (size_t)64 * 65) * sizeof(T);
    if (4 * tile_bytes > 64 * 1024) return false;
    f->kind = kind; f->f_rows = f_rows; f->out = out;
    f->c = c; f->cp = cp; f->rs = rs; f->k = k; f->kp = kp;
    f->tiles_x = kind == 1 ? cp / 64 : (c * rs + 63) / 64;
    f->tiles = f->tiles_x * (kind == 1 ? k : kp / 64);
    f->blocks = (f->tiles + 3) / 4;
    *lds = std::max(*lds, (int)(4 * tile_bytes));
    return true;
}
template <class T> static hipError_t launch_relayout(const RelayoutJobs& r, int lds, hipStream_t st)
{
    const int blocks = r.f.blocks + r.a.blocks + r.b.blocks;
    if (blocks == 0) return hipSuccess;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(relayout_kernel<T>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    relayout_kernel<T><<<blocks, kTclThreads, lds, st>>>(r);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------
struct FastConv {
    ConvGeom g;  // c and k rounded up to multiples of 64: the extents of the copies
    int c_real, k_real;  // what the tensors hold (forward, data gradient: k_real = output channels stored)
    int hp, wp;
    const void* const* y_rows;  // forward: output rows (images)
    const void* const* f_rows;  // weight gradient: output rows (filters)
    const void* xp;  // the copies, elements of the pipeline's input type
    const void* fp;
    const void* yt;
    const void* y_src;  // weight gradient reading dY where it lies (NCHW, one block): its first element; else null
    void* ws;  // partial sums in the accumulation type (weight gradient: always; others: when split)
    int split, ktiles, ktiles_per_split;  // parts of the k-loop, its k-tiles in all and per part
    // forward, data gradient: tiles (in launch order) that run the whole k-loop; the tiles after
    // them run it in `split` parts.  tail_only (host side): only the tiles after the last full
    // round of workgroups are split.
    int full_tiles, tail_only;
    void* sink;  // 256 bytes that nobody reads: where lanes with nothing to store store
};

// byte offset of pixel m = (n, oh, ow) in Xp (tap (0,0), channel 0)
template <class T> __device__ __forceinline__ uint32_t pixel_offset(const FastConv& p, int m)
{
    const int sp_out = p.g.oh * p.g.ow;
    const int n = m / sp_out, sp = m % sp_out, oy = sp / p.g.ow, ox = sp % p.g.ow;
    return (uint32_t)((((int64_t)n * p.hp + oy * p.g.stride_h) * p.wp + ox * p.g.stride_w) * p.g.c * sizeof(T));
}

template <class P, int BM, int BN> struct FwdWalk {
    using T = typename P::Elem;
    using TA = typename P::template Tile<BM, true>;
    using TB = typename P::template Tile<BN, true>;
    static constexpr int BK = P::BK;
    const char *abase, *bbase, *xp;
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];
    int c, wp, s_taps, cchunks, r, s, cc;
    int ahead = 0;  // k-tiles after the current one (advance_or_stay only)

    // starts at k-tile kt0 of the (r, s, c) order
    __device__ __forceinline__ FwdWalk(const FastConv& p, int m0, int n0, int wave, int lane, int kt0)
    {
        xp = reinterpret_cast<const char*>(p.xp);
        c = p.g.c; wp = p.wp; s_taps = p.g.s; cchunks = p.g.c / BK;
        cc = kt0 % cchunks;
        r = (kt0 / cchunks) / s_taps;
        s = (kt0 / cchunks) % s_taps;
        abase = xp + ((int64_t)(r * wp + s) * c + cc * BK) * sizeof(T);
        bbase = reinterpret_cast<const char*>(p.fp) + (int64_t)kt0 * BK * sizeof(T);
        // rows past the last pixel (ragged last tile) fetch the last pixel again: in bounds, and
        // what they bring in only reaches accumulators that the epilogue does not store
        const int m_last = p.g.n * p.g.oh * p.g.ow - 1;
#pragma unroll
        for (int q = 0; q < TA::kInstr; ++q) {
            int row, chunk;
            TA::lane_slot(q, wave, lane, row, chunk);
            aoff[q] = pixel_offset<T>(p, min(m0 + row, m_last)) + chunk * 16;
        }
        TB::offsets((int64_t)p.g.c * p.g.r * p.g.s, n0, BN, wave, lane, boff);
    }
    __device__ __forceinline__ void advance()
    {
        bbase += BK * sizeof(T);
        if (++cc == cchunks) {
            cc = 0;
            if (++s == s_taps) {
                s = 0;
                ++r;
            }
        }
        abase = xp + ((int64_t)(r * wp + s) * c + cc * BK) * sizeof(T);
    }
    // for pipelines that issue loads to the end of the k-loop: stays on the last k-tile
    __device__ __forceinline__ void advance_or_stay()
    {
        if (ahead > 0) {
            --ahead;
            advance();
        }
    }
};

// workgroup w of n: XCD w % 8 gets a contiguous run of the logical order
__device__ __forceinline__ int xcd_logical(int w, int n)
{
    const int base = n / 8, rem = n % 8, x = w % 8, j = w / 8;
    if (n < 16) return w;
    return x * base + min(x, rem) + j;
}

template <class P, int BM, int BN, int STAGES, class TC>
__global__ __launch_bounds__(NT) void conv_fwd_kernel(FastConv p, typename P::AccT alpha, typename P::AccT beta)
{
    using TS = typename P::template Shape<BM, BN>;
    using AccT = typename P::AccT;
    constexpr int E = P::kEdge;
    constexpr int WM = TS::WM, WN = TS::WN, MT = TS::MT, NTL = TS::NTL;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tiles_n = p.g.k / BN;
    // whole tiles first; then the split ones, part-major (same k-range, same XCD)
    const bool partial = (int)blockIdx.x >= p.full_tiles;
    const int split_wgs = gridDim.x - p.full_tiles, split_tiles = split_wgs / p.split;
    int part = 0, mn;
    if (!partial) {
        mn = xcd_logical(blockIdx.x, p.full_tiles);
    } else {
        const int lt = xcd_logical(blockIdx.x - p.full_tiles, split_wgs);
        part = lt / split_tiles;
        mn = p.full_tiles + lt % split_tiles;
    }
    const int m0 = (mn / tiles_n) * BM, n0 = (mn % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = TS::wm(wave), wn = TS::wn(wave), lcol = P::col(lane);

    typename P::Acc acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < P::kRegs; ++r) acc[i][j][r] = AccT(0);

    const int kt0 = part * p.ktiles_per_split;
    FwdWalk<P, BM, BN> walk(p, m0, n0, wave, lane, kt0);
    const int n_ktiles = partial ? min(p.ktiles_per_split, p.ktiles - kt0) : p.ktiles;
    walk.ahead = n_ktiles - 1;
    P::template run<BM, BN, STAGES, true, true>(walk, n_ktiles, smem, acc);

    if (partial) {
        // partial sums [part][output channel][pixel], the pixels those of the split tiles (whole
        // rows of tiles: full_tiles is a multiple of tiles_n)
        const int64_t mp = (int64_t)(split_tiles / tiles_n) * BM;
        const int m_first = (p.full_tiles / tiles_n) * BM;
        AccT* ws = static_cast<AccT*>(p.ws) + (int64_t)part * p.g.k * mp;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NTL; ++j) {
                AccT* col = ws + (int64_t)(n0 + wn * WN + j * E + lcol) * mp + (m0 - m_first) + wm * WM + i * E;
                if constexpr (P::kRowQuads) {
                    typedef AccT acc4 __attribute__((ext_vector_type(4)));
#pragma unroll
                    for (int q4 = 0; q4 < P::kRegs / 4; ++q4) {
                        acc4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = acc[i][j][q4 * 4 + e];
                        *reinterpret_cast<acc4*>(col + P::row(lane, 4 * q4)) = o;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < P::kRegs; ++r) col[P::row(lane, r)] = acc[i][j][r];
                }
            }
        return;
    }

    // Epilogue.  No store sits in a branch of its own and no load between two stores: the row
    // pointers (one per image) of a block of rows are loaded together before its stores, and a
    // lane with nothing to store (pixels past the end, pad filters) stores to `sink`, 256 bytes of
    // the plan that nobody reads.  (Loads and stores complete in order, so a pointer loaded
    // between two stores waited for every store before it, and a branch per element made the
    // compiler wait for everything outstanding.)
    typedef __attribute__((address_space(1))) TC GTC;
    const int sp_out = p.g.oh * p.g.ow, m_end = p.g.n * sp_out;
    GTC* const sink = (GTC*)static_cast<TC*>(p.sink);
    const bool read_c = beta != AccT(0);
    if (!P::kRowQuads || sp_out % 4 != 0) {
        // one element at a time, four rows (registers) of a block per round
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int g4 = 0; g4 < P::kRegs / 4; ++g4) {
                GTC* rowp[4];  // &Y[image][0][pixel] of each of these rows; null: no such pixel
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = m0 + wm * WM + i * E + P::row(lane, g4 * 4 + e);
                    const bool ok = m < m_end;
                    const int mm = ok ? m : 0, n_img = mm / sp_out, sp = mm - n_img * sp_out;
                    GTC* y = (GTC*)static_cast<TC*>(const_cast<void*>(p.y_rows[n_img]));
                    rowp[e] = ok ? y + sp : nullptr;
                }
#pragma unroll
                for (int j = 0; j < NTL; ++j) {
                    const int ko = n0 + wn * WN + j * E + lcol;
                    const bool k_ok = ko < p.k_real;
                    const int64_t plane = (int64_t)ko * sp_out;
                    GTC* dst[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[e] = (k_ok && rowp[e]) ? rowp[e] + plane : sink;
                    if (!read_c) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) *dst[e] = to_out<TC>(alpha * acc[i][j][g4 * 4 + e]);
                    } else {
                        AccT old[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) old[e] = (AccT)*dst[e];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            AccT v = alpha * acc[i][j][g4 * 4 + e];
                            v += beta * old[e];
                            *dst[e] = to_out<TC>(v);
                        }
                    }
                }
            }
        return;
    }
    if constexpr (P::kRowQuads) {
        // with the fp16 / fp32 MFMAs four consecutive registers are four consecutive pixels of one
        // output plane: stored together where a plane is a multiple of 4 pixels
        typedef TC out4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(1))) out4 GOut4;
        constexpr int kQuads = P::kRegs / 4;
        // the row pointers of block row i + 1 are loaded before the stores of block row i
        auto row_pointers = [&](int i, GTC* (&rowp)[kQuads]) {
#pragma unroll
            for (int q4 = 0; q4 < kQuads; ++q4) {
                const int m = m0 + wm * WM + i * E + P::row(lane, 4 * q4);
                const bool ok = m < m_end;  // ragged last tile (m_end is a multiple of 4, as sp_out is)
                const int mm = ok ? m : 0, n_img = mm / sp_out, sp = mm - n_img * sp_out;
                GTC* y = (GTC*)static_cast<TC*>(const_cast<void*>(p.y_rows[n_img]));
                rowp[q4] = ok ? y + sp : nullptr;
            }
        };
        GTC* rowp[kQuads];
        row_pointers(0, rowp);
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            GTC* next[kQuads];
#pragma unroll
            for (int q4 = 0; q4 < kQuads; ++q4) next[q4] = nullptr;
            if (i + 1 < MT) row_pointers(i + 1, next);
#pragma unroll
            for (int q4 = 0; q4 < kQuads; ++q4) {
                GOut4* dst[NTL];
#pragma unroll
                for (int j = 0; j < NTL; ++j) {
                    const int ko = n0 + wn * WN + j * E + lcol;
                    GTC* d = (ko < p.k_real && rowp[q4]) ? rowp[q4] + (int64_t)ko * sp_out : sink;  // pad filters
                    dst[j] = reinterpret_cast<GOut4*>(d);
                }
                if (!read_c) {
#pragma unroll
                    for (int j = 0; j < NTL; ++j) {
                        out4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = to_out<TC>(alpha * acc[i][j][q4 * 4 + e]);
                        *dst[j] = o;
                    }
                } else {
                    out4 o[NTL];
#pragma unroll
                    for (int j = 0; j < NTL; ++j) o[j] = *dst[j];
#pragma unroll
                    for (int j = 0; j < NTL; ++j) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float v = alpha * acc[i][j][q4 * 4 + e];
                            v += beta * (float)o[j][e];
                            o[j][e] = to_out<TC>(v);
                        }
                        *dst[j] = o[j];
                    }
                }
            }
#pragma unroll
            for (int q4 = 0; q4 < kQuads; ++q4) rowp[q4] = next[q4];
        }
    }
}

// Y[n][ko][pixel] <- alpha * sum over parts (ascending) + beta * Y from the partial sums
// [part][ko][pixel of the split tiles: mp of them, the first one pixel m_first].
template <class AccT, class TC>
__global__ __launch_bounds__(256) void conv_fwd_reduce_kernel(FastConv p, int64_t mp, int m_first, AccT alpha,
                                                              AccT beta)
{
    const AccT* ws = static_cast<const AccT*>(p.ws);
    const int sp_out = p.g.oh * p.g.ow;
    const int64_t m_end = (int64_t)p.g.n * sp_out, span = m_end - m_first;
    const int64_t total = (int64_t)p.k_real * span, part_elems = (int64_t)p.g.k * mp;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int ko = (int)(e / span);
        const int64_t m = m_first + e % span;
        const AccT* src = ws + (int64_t)ko * mp + (m - m_first);
        AccT sum = AccT(0);
#pragma unroll 8
        for (int s = 0; s < p.split; ++s) sum += src[(int64_t)s * part_elems];
        const int n_img = (int)(m / sp_out), sp = (int)(m % sp_out);
        TC* dst = static_cast<TC*>(const_cast<void*>(p.y_rows[n_img])) + (int64_t)ko * sp_out + sp;
        AccT v = alpha * sum;
        if (beta != AccT(0)) v += beta * (AccT)*dst;
        *dst = to_out<TC>(v);
    }
}

// ------------------------------------------------------------------------------------------
// weight gradient
// ------------------------------------------------------------------------------------------
// IN_PLACE: the A' operand is dY itself.  In NCHW the pixels of one (image, filter) plane are
// unit-stride, so dY is the k unit-stride form of A'[filter][pixel] where it lies: row `filter` of
// a k-tile is 128 bytes of a plane, and a 16-byte chunk never straddles two images when the plane
// is a whole number of chunks.  The k-tile's first pixel is tracked in scalars (its plane and its
// place in it go into the base pointer); a plane holds at least one k-tile, so a lane's chunk is
// either in that plane or in the same filter's plane of the next image: one compare and one
// select between two fixed offsets per segment and k-tile (per-lane pixel counters with their
// wraps cost the matrix instructions a tenth of their issue slots).
// TABLE: the byte offset of every pixel of this workgroup's k-range lies in an LDS table that the
// workgroup filled before the k-loop (wgrad_fill_table); stepping the B rows by a k-tile is then one
// LDS read and one add per segment instead of counters with wraps (a wavefront of the 16x16x32
// pipeline has three issue slots per matrix instruction and this kernel fills nearly all of them).
template <class P, int BM, int BN, bool IN_PLACE = false, bool TABLE = false> struct WgradWalk {
    using T = typename P::Elem;
    using TA = typename P::template Tile<BM, IN_PLACE>;
    using TB = typename P::template Tile<BN, false>;
    static constexpr int BK = P::BK;
    const char *abase, *bbase;
    uint32_t aoff[TA::kInstr], boff[TB::kInstr];
    // IN_PLACE: the lane's chunk of each A segment: its pixel inside the k-tile, its offset from the
    // k-tile's first pixel in the same plane and in the next image's
    int apix[IN_PLACE ? TA::kInstr : 1];
    uint32_t aoff_here[IN_PLACE ? TA::kInstr : 1], aoff_next[IN_PLACE ? TA::kInstr : 1];
    int sp_plane, a_first;  // pixels of a plane; the k-tile's first pixel inside its plane (uniform)
    uint32_t a_next_image_bytes;
    // pixel (oy, ox) of its image fetched by this lane for each B segment; stepping it by one
    // k-tile moves the byte offset by sums of four constants (all arithmetic modulo 2^32: the
    // copy is smaller than 4 GiB, so the true offset is what remains)
    int py[TABLE ? 1 : TB::kInstr], px[TABLE ? 1 : TB::kInstr];
    typedef const __attribute__((address_space(3))) uint32_t LdsU32;
    LdsU32* tab_lane;  // TABLE: entry of this lane's row of segment 0 in the current k-tile
    uint32_t bchunk[TABLE ? TB::kInstr : 1];  // ... and the lane's 16-byte chunk of each segment
    int oh, ow, d_oy, d_ox;
    uint32_t step_bytes, wrap_x_bytes, wrap_y_bytes;
    int64_t astep;

    __device__ __forceinline__ WgradWalk(const FastConv& p, int k0_pixels, int m0_filters, int n0_cols, int wave,
                                         int lane, const char* table = nullptr)
    {
        const int hp = p.hp, wp = p.wp, c = p.g.c;
        oh = p.g.oh; ow = p.g.ow;
        d_oy = BK / ow; d_ox = BK % ow;
        const uint32_t col_bytes = (uint32_t)(p.g.stride_w * c * (int)sizeof(T));   // ox + 1
        const uint32_t row_bytes = (uint32_t)p.g.stride_h * wp * c * sizeof(T);     // oy + 1
        const uint32_t img_bytes = (uint32_t)hp * wp * c * sizeof(T);               // n + 1
        step_bytes = d_oy * row_bytes + d_ox * col_bytes;
        wrap_x_bytes = row_bytes - ow * col_bytes;
        wrap_y_bytes = img_bytes - oh * row_bytes;
        sp_plane = oh * ow;
        a_next_image_bytes = (uint32_t)(p.g.k - 1) * (uint32_t)sp_plane * (uint32_t)sizeof(T);
        if (IN_PLACE) {
            astep = 0;
            const int pn = k0_pixels / sp_plane;
            a_first = k0_pixels - pn * sp_plane;
            abase = reinterpret_cast<const char*>(p.y_src) +
                    (((int64_t)pn * p.g.k + m0_filters) * sp_plane + a_first) * sizeof(T);
#pragma unroll
            for (int q = 0; q < TA::kInstr; ++q) {
                int row, chunk;
                TA::lane_slot(q, wave, lane, row, chunk);
                apix[q] = chunk * (16 / (int)sizeof(T));
                aoff_here[q] = (uint32_t)(((int64_t)row * sp_plane + apix[q]) * sizeof(T));
                aoff_next[q] = aoff_here[q] + a_next_image_bytes;
            }
            select_a();
        } else {
            // A' = Yt[m][k]: dense, m/n (= k_out) unit-stride, filters m0 .. m0+BM of the tile
            TA::offsets(p.g.k, m0_filters, BM, wave, lane, aoff);
            astep = TA::step(p.g.k);
            abase = reinterpret_cast<const char*>(p.yt) + (int64_t)k0_pixels * p.g.k * sizeof(T);
        }
        // B' columns n0 .. n0+BN of (r, s, c): one tap, BN consecutive channels
        const int tap = n0_cols / c, c0 = n0_cols % c, r = tap / p.g.s, s = tap % p.g.s;
        bbase = reinterpret_cast<const char*>(p.xp) + ((int64_t)(r * wp + s) * c + c0) * sizeof(T);
        const int sp_out = oh * ow;
        if constexpr (TABLE) {
            // segment q holds rows q * kRowStep further on (lane_slot: 4 segments of kRowsPerSeg rows per step of q)
            int row0, chunk0;
            TB::lane_slot(0, wave, lane, row0, chunk0);
            tab_lane = (LdsU32*)table + row0;
#pragma unroll
            for (int q = 0; q < TB::kInstr; ++q) {
                int row, chunk;
                TB::lane_slot(q, wave, lane, row, chunk);
                bchunk[q] = chunk * 16;
            }
            select_b();
        } else {
#pragma unroll
            for (int q = 0; q < TB::kInstr; ++q) {
                int row, chunk;
                TB::lane_slot(q, wave, lane, row, chunk);
                const int m = k0_pixels + row;
                const int pn = m / sp_out, sp = m % sp_out;
                py[q] = sp / ow;
                px[q] = sp % ow;
                boff[q] = pn * img_bytes + py[q] * row_bytes + px[q] * col_bytes + chunk * 16;
            }
        }
    }
    static constexpr int kRowStep = 4 * TB::kRowsPerSeg;
    __device__ __forceinline__ void select_b()
    {
        if constexpr (TABLE) {
#pragma unroll
            for (int q = 0; q < TB::kInstr; ++q) boff[q] = tab_lane[q * kRowStep] + bchunk[q];
        }
    }
    __device__ __forceinline__ void select_a()
    {
        const int left = sp_plane - a_first;  // pixels of the k-tile that lie in its first pixel's plane
#pragma unroll
        for (int q = 0; q < (IN_PLACE ? TA::kInstr : 0); ++q) aoff[q] = apix[q] < left ? aoff_here[q] : aoff_next[q];
    }
    __device__ __forceinline__ void advance()
    {
        if (IN_PLACE) {
            a_first += BK;
            abase += BK * sizeof(T);
            if (a_first >= sp_plane) {
                a_first -= sp_plane;
                abase += a_next_image_bytes;
            }
            select_a();
        } else {
            abase += astep;
        }
        if constexpr (TABLE) {
            tab_lane += BK;
            select_b();
        } else {
#pragma unroll
            for (int q = 0; q < TB::kInstr; ++q) {  // pixel index += BK
                px[q] += d_ox;
                py[q] += d_oy;
                boff[q] += step_bytes;
                if (px[q] >= ow) { px[q] -= ow; ++py[q]; boff[q] += wrap_x_bytes; }
                // a k-tile spans at most three image boundaries (conv_fast_ok: BK / ow < 3 * oh); one
                // where dY is read in place (a plane holds at least one k-tile there)
                if (py[q] >= oh) { py[q] -= oh; boff[q] += wrap_y_bytes; }
                if (!IN_PLACE) {
                    if (py[q] >= oh) { py[q] -= oh; boff[q] += wrap_y_bytes; }
                    if (py[q] >= oh) { py[q] -= oh; boff[q] += wrap_y_bytes; }
                }
            }
        }
    }
};

// table[e] = byte offset in Xp (tap (0,0), channel 0) of pixel k0_pixels + e, e < entries; the
// `spare` entries after them (the k-tile that the walk steps onto after its last load) hold 0.
// Each thread takes a run of consecutive pixels: one division at its start, then counters.
template <class T>
__device__ __forceinline__ void wgrad_fill_table(const FastConv& p, int k0_pixels, int entries, int spare, char* table)
{
    uint32_t* tab = reinterpret_cast<uint32_t*>(table);
    const int oh = p.g.oh, ow = p.g.ow, sp_out = oh * ow;
    const uint32_t col_bytes = (uint32_t)(p.g.stride_w * p.g.c * (int)sizeof(T));
    const uint32_t row_bytes = (uint32_t)p.g.stride_h * p.wp * p.g.c * sizeof(T);
    const uint32_t img_bytes = (uint32_t)p.hp * p.wp * p.g.c * sizeof(T);
    const int per = (entries + NT - 1) / NT, e0 = threadIdx.x * per, e1 = min(e0 + per, entries);
    if (e0 < e1) {
        const int m = k0_pixels + e0, pn = m / sp_out, sp = m - pn * sp_out;
        int py = sp / ow, px = sp - py * ow;
        uint32_t off = pn * img_bytes + py * row_bytes + px * col_bytes;
        for (int e = e0; e < e1; ++e) {
            tab[e] = off;
            off += col_bytes;
            if (++px == ow) {
                px = 0;
                off += row_bytes - ow * col_bytes;
                if (++py == oh) {
                    py = 0;
                    off += img_bytes - oh * row_bytes;
                }
            }
        }
    }
    for (int e = entries + threadIdx.x; e < entries + spare; e += NT) tab[e] = 0;
    __syncthreads();
}

template <class P, int BM, int BN, bool IN_PLACE, bool TABLE>
__global__ __launch_bounds__(NT) void conv_wgrad_kernel(FastConv p)
{
    using TS = typename P::template Shape<BM, BN>;
    constexpr int BK = P::BK;
    constexpr int WM = TS::WM, WN = TS::WN, MT = TS::MT, NTL = TS::NTL;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int ncols = p.g.c * p.g.r * p.g.s, tiles_n = ncols / BN, tiles_mn = (p.g.k / BM) * tiles_n;
    const int idx = xcd_logical(blockIdx.x, gridDim.x);
    const int split = idx / tiles_mn, mn = idx % tiles_mn;  // split-major: same pixels, same XCD
    const int m0 = (mn / tiles_n) * BM, n0 = (mn % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = TS::wm(wave), wn = TS::wn(wave);
    using AccT = typename P::AccT;

    typename P::Acc acc[MT][NTL];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < P::kRegs; ++r) acc[i][j][r] = AccT(0);

    // the last part may be shorter; pixels past n*oh*ow (last k-tile) read zeros on both sides
    const int kt0 = split * p.ktiles_per_split;
    const int n_ktiles = min(p.ktiles_per_split, p.ktiles - kt0);
    char* table = smem + P::lds_bytes(BM, BN, 3);  // TABLE: behind the pipeline's stages
    if (TABLE) wgrad_fill_table<typename P::Elem>(p, kt0 * BK, n_ktiles * BK, BK, table);
    WgradWalk<P, BM, BN, IN_PLACE, TABLE> walk(p, kt0 * BK, m0, n0, wave, lane, table);
    P::template run<BM, BN, 3, IN_PLACE, false>(walk, n_ktiles, smem, acc);

    AccT* ws = static_cast<AccT*>(p.ws) + (int64_t)split * p.g.k * ncols;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
#pragma unroll
            for (int r = 0; r < P::kRegs; ++r) {
                const int row = m0 + wm * WM + i * P::kEdge + P::row(lane, r);
                const int col = n0 + wn * WN + j * P::kEdge + P::col(lane);
                ws[(int64_t)row * ncols + col] = acc[i][j][r];
            }
}

// dF[k][c][r][s] <- alpha * sum over splits (ascending) + beta * dF; the partials are
// [k][(r,s,c)], read four channels at a time.
template <class AccT, class TC>
__global__ __launch_bounds__(256) void conv_wgrad_reduce_kernel(FastConv p, AccT alpha, AccT beta)
{
    typedef AccT acc4 __attribute__((ext_vector_type(4)));
    const AccT* ws = static_cast<const AccT*>(p.ws);
    const int rs = p.g.r * p.g.s, c = p.g.c, ncols = rs * c;
    const int64_t total = (int64_t)p.g.k * ncols, quads = total / 4;
    for (int64_t e4 = (int64_t)blockIdx.x * 256 + threadIdx.x; e4 < quads; e4 += (int64_t)gridDim.x * 256) {
        const int64_t e = e4 * 4;
        const int kk = (int)(e / ncols), col = (int)(e % ncols), q = col / c, cc = col % c;
        if (kk >= p.k_real || cc >= p.c_real) continue;  // pad filters, pad channels
        acc4 sum = {AccT(0), AccT(0), AccT(0), AccT(0)};
        for (int s = 0; s < p.split; ++s) sum += *reinterpret_cast<const acc4*>(ws + (int64_t)s * total + e);
        TC* dst = static_cast<TC*>(const_cast<void*>(p.f_rows[kk])) + cc * rs + q;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (cc + i >= p.c_real) break;
            AccT v = alpha * sum[i];
            if (beta != AccT(0)) v += beta * (AccT)dst[i * rs];
            dst[i * rs] = to_out<TC>(v);
        }
    }
}

// The same through LDS: workgroup (channel chunk, filter) sums 64 channels x rs taps (runs of 64
// consecutive channels in the partials), and writes them where they lie contiguously in dF.
// With many parts and few workgroups (64-channel layers) the parts are dealt to `groups` sets of
// threads (part s to set s % groups, each set adding its parts in ascending order) and the sets'
// sums are added in ascending order: still one fixed order.
template <class AccT, class TC>
__global__ __launch_bounds__(256) void conv_wgrad_reduce_tiled_kernel(FastConv p, int groups, AccT alpha, AccT beta)
{
    typedef AccT acc4 __attribute__((ext_vector_type(4)));
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    AccT* tile = reinterpret_cast<AccT*>(smem_raw);  // [groups][64][rsp]
    const int rs = p.g.r * p.g.s, rsp = rs | 1, c = p.g.c, ncols = rs * c;
    const int kk = blockIdx.y, c0 = blockIdx.x * 64, nch = min(64, p.c_real - c0), tid = threadIdx.x;
    if (nch <= 0) return;  // a chunk of pad channels only (the whole workgroup leaves)
    const int64_t total = (int64_t)p.g.k * ncols;
    const AccT* ws = static_cast<const AccT*>(p.ws) + (int64_t)kk * ncols + c0;
    for (int i = tid; i < groups * rs * 16; i += 256) {
        const int grp = i / (rs * 16), rem = i - grp * (rs * 16), q = rem >> 4, c4 = (rem & 15) * 4;
        const AccT* src = ws + (int64_t)q * c + c4;
        acc4 sum = {AccT(0), AccT(0), AccT(0), AccT(0)};
#pragma unroll 8
        for (int s = grp; s < p.split; s += groups) sum += *reinterpret_cast<const acc4*>(src + (int64_t)s * total);
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[(grp * 64 + c4 + e) * rsp + q] = sum[e];
    }
    __syncthreads();
    TC* dst = static_cast<TC*>(const_cast<void*>(p.f_rows[kk])) + (int64_t)c0 * rs;
    for (int i = tid; i < nch * rs; i += 256) {
        const int ch = i / rs, at = ch * rsp + (i - ch * rs);
        AccT sum = tile[at];
        for (int grp = 1; grp < groups; ++grp) sum += tile[grp * 64 * rsp + at];
        AccT v = alpha * sum;
        if (beta != AccT(0)) v += beta * (AccT)dst[i];
        dst[i] = to_out<TC>(v);
    }
}

template <class AccT, class TC>
void wgrad_reduce(const FastConv& p, double alpha, double beta, hipStream_t st)
{
    const size_t lds = (size_t)64 * ((p.g.r * p.g.s) | 1) * sizeof(AccT);
    const int wgs = p.g.c / 64 * p.k_real;
    const int groups = (p.split >= 8 && wgs < 1024 && 4 * lds <= 64 * 1024) ? 4 : 1;
    if (lds <= 64 * 1024)
        conv_wgrad_reduce_tiled_kernel<AccT, TC>
            <<<dim3(p.g.c / 64, p.k_real), 256, groups * lds, st>>>(p, groups, (AccT)alpha, (AccT)beta);
    else
        conv_wgrad_reduce_kernel<AccT, TC><<<1024, 256, 0, st>>>(p, (AccT)alpha, (AccT)beta);
}

template <class K> hipError_t set_lds(K kern, int bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

static int round64(int v) { return (v + 63) / 64 * 64; }
static int elem_bytes(dmath_dtype_t dt) { return dt == DMATH_F16 ? 2 : dt == DMATH_F32 ? 4 : 8; }
// pixels per k-tile of the weight gradient (= the pipeline's k-tile)
static int pixel_tile(dmath_dtype_t dt)
{
    return dt == DMATH_F16 ? PipeF16::BK : dt == DMATH_F32 ? PipeF32::BK : PipeF64::BK;
}

// Sizes of the copies that the specialised kernels read.
ConvFastLayout conv_fast_layout(int mode, const ConvGeom& g, dmath_dtype_t dt)
{
    ConvFastLayout l{};
    l.cp = round64(g.c);
    l.kp = round64(g.k);
    const int64_t m = (int64_t)g.n * g.oh * g.ow, crs_p = (int64_t)g.r * g.s * l.cp;
    const int64_t eb = elem_bytes(dt), pt = pixel_tile(dt);
    // one more (all-zero) image where the weight gradient's last pixel tile is not full
    l.x_images = g.n + (m % pt ? 1 : 0);
    if (mode == CONV_BWD_DATA) {
        l.x_bytes = (int64_t)g.n * (g.h + g.r - 1) * (g.w + g.s - 1) * l.kp * eb;
        l.f_bytes = (int64_t)l.cp * g.r * g.s * l.kp * eb;
    } else {
        l.x_bytes = (int64_t)l.x_images * (g.h + 2 * g.pad_h) * (g.w + 2 * g.pad_w) * l.cp * eb;
        l.f_bytes = mode == CONV_FWD ? (int64_t)l.kp * crs_p * eb : 0;
        l.y_bytes = mode == CONV_BWD_FILTER ? (m + pt - 1) / pt * pt * l.kp * eb : 0;
    }
    return l;
}

// Geometry the specialised kernels accept (everything else runs on the generic kernels): every
// copy below 4 GiB (32-bit lane offsets), at most four times the work from rounding
// the channel and filter counts up to multiples of 64 (the matrix pipeline is more than ten
// times faster than the generic kernel in fp16, two to four times in fp32 and fp64: there the
// limit is twice the work), for the data gradient (a forward convolution of dY with padding r-1-pad)
// a padding that does not exceed the filter, and for the weight gradient output planes that are
// not tiny (4x4 and less in fp16).
bool conv_fast_ok(int mode, const ConvGeom& g, dmath_dtype_t in_dtype)
{
    const ConvFastLayout l = conv_fast_layout(mode, g, in_dtype);
    const int64_t limit = 1ll << 32;
    if (l.x_bytes >= limit || l.f_bytes >= limit || l.y_bytes >= limit) return false;
    if ((int64_t)g.n * g.oh * g.ow >= (1ll << 31) - 256 || (int64_t)g.n * g.h * g.w >= (1ll << 31) - 256) return false;
    if ((int64_t)l.cp * l.kp > (int64_t)g.c * g.k * (in_dtype == DMATH_F16 ? 4 : 2)) return false;
    if (mode == CONV_BWD_DATA) return g.pad_h <= g.r - 1 && g.pad_w <= g.s - 1;
    // the weight gradient steps its pixel index by one k-tile with three conditional wraps
    if (mode == CONV_BWD_FILTER) return pixel_tile(in_dtype) / g.ow < 3 * g.oh;
    return true;
}

// The weight gradient can read dY where it lies (no channels-last copy of it) when a plane of oh*ow
// pixels is a whole number of 16-byte chunks, the pixels of all images are a whole number of
// k-tiles (there are no zero rows to read past the end), no filter row is padding, a plane holds
// at least one k-tile, and 32-bit lane offsets reach all of dY.  The caller checks that dY is one
// block.  DMATH_CONV_DY_COPY=1 keeps the copy (experiments and tests).
bool conv_fast_wgrad_dy_in_place(const ConvGeom& g, dmath_dtype_t in_dtype)
{
    static const bool keep_copy = std::getenv("DMATH_CONV_DY_COPY") != nullptr;
    if (keep_copy) return false;
    const int64_t eb = elem_bytes(in_dtype), pt = pixel_tile(in_dtype), sp = (int64_t)g.oh * g.ow;
    return (sp * eb) % 16 == 0 && ((int64_t)g.n * sp) % pt == 0 && g.k % 64 == 0 && pt <= sp &&
           (int64_t)g.n * g.k * sp * eb < (1ll << 32);
}

// A 1x1 convolution with stride 1 and no padding is, image by image, Y_n[k x hw] = F[k x c] *
// X_n[c x hw] on the tensors as they lie in memory (dX_n = F^T * dY_n; dF = sum over the images
// of dY_n * X_n^T, the images being the k-segments): a block GEMM with one column block per
// image.  No copy is made.  Taken where the rows of a plane and of the filter are 16-byte aligned
// and rounding a plane up to whole 64-element tiles (ragged last column tile; weight gradient:
// padded k-tail) adds at most 35 %: in the timing samples the mapping still wins on 14x14 and
// 12x12 planes (+31 %, +33 %), where it saves the re-layout copies.
bool conv_as_gemm_ok(int mode, const ConvGeom& g, dmath_dtype_t in_dtype)
{
    if (g.r != 1 || g.s != 1 || g.stride_h != 1 || g.stride_w != 1 || g.pad_h != 0 || g.pad_w != 0) return false;
    const int64_t sp = (int64_t)g.h * g.w, eb = elem_bytes(in_dtype);
    if ((sp * eb) % 16 != 0 || ((int64_t)g.c * eb) % 16 != 0) return false;
    return (sp + 63) / 64 * 64 * 100 <= sp * 135;  // planes padded to 64-element tiles: at most 35 % more
}

// C tiles of the weight gradient: 256 (fp16 only), 128 or 64 filters x 128 or 64 columns of
// (r,s,c) (64 where the channel count is not a multiple of 128: a tile's columns are consecutive
// channels of one tap).
static int wgrad_tile_m(const ConvGeom& g, dmath_dtype_t dt)
{
    const int kp = round64(g.k);
    return (kp % 256 == 0 && dt == DMATH_F16) ? 256 : kp % 128 == 0 ? 128 : 64;
}
static int wgrad_tile_n(const ConvGeom& g, dmath_dtype_t dt)
{
    if (round64(g.c) % 128 != 0) return 64;
    // fp64: two 64-wide workgroups per CU are 8-25 % faster than one 128-wide (seven layers);
    // fp32: level, except where there are few tiles (1x1 layers: 50 -> 41 us with 8 -> 16 tiles)
    if (dt == DMATH_F64) return 64;
    if (dt == DMATH_F32) {
        const int64_t tiles128 = (int64_t)(round64(g.k) / wgrad_tile_m(g, dt)) * ((int64_t)round64(g.c) * g.r * g.s / 128);
        return tiles128 < 16 ? 64 : 128;
    }
    return 128;
}
static int64_t wgrad_tiles(const ConvGeom& g, dmath_dtype_t dt)
{
    return (int64_t)(round64(g.k) / wgrad_tile_m(g, dt)) * ((int64_t)round64(g.c) * g.r * g.s / wgrad_tile_n(g, dt));
}
static int64_t wgrad_ktiles(const ConvGeom& g, dmath_dtype_t dt)
{
    const int pt = pixel_tile(dt);
    return ((int64_t)g.n * g.oh * g.ow + pt - 1) / pt;
}

// A split count is usable when no part is empty.
static bool wgrad_split_ok(int64_t ktiles, int s)
{
    const int64_t per = (ktiles + s - 1) / s;
    return (s - 1) * per < ktiles;
}

// Workgroups per CU by the LDS their tile needs (160 KiB per CU).
static int per_cu(int bm, int bn, dmath_dtype_t dt)
{
    // (fp16: the 256x256 and 224x256 forward tiles run two stages, every other tile three)
    if (dt == DMATH_F16) return 160 * 1024 / PipeF16::lds_bytes(bm, bn, bm * bn >= 224 * 256 ? 2 : 3);
    return 160 * 1024 / (dt == DMATH_F32 ? PipeF32::lds_bytes(bm, bn, 3) : PipeF64::lds_bytes(bm, bn, 3));
}

// Split count for the weight gradient: the number of parts s (each of ceil(k-tiles / s) pixel
// tiles, at least 256 pixels, the last one possibly shorter) with at most four rounds of
// workgroups (144 tiles of an fp32 layer leave 112 CUs idle unsplit: 424 us, 332 us in four
// parts) that minimises
// (w x 64-pixel steps of the busiest CU + s): the parts shorten with s, the partial sums written
// and read back grow with it.  w = 1 in fp16 (the balance point sqrt(k-tiles) matches the timing
// samples on 1x1 and 3x3 layers of 14x14 and 28x28 pixels), 4 in fp32 and 8 in fp64, whose steps
// take that many times as long; an fp32 / fp64 CU with a single workgroup runs at 0.87 of the
// rate (as in choose_conv).  Small fp16 tiles leave a CU partly idle unless several workgroups
// share it (64x64: three fit, one alone reaches 0.45 of the rate of three, two 0.8; 128x64 and
// 64x128: two fit, one alone 0.73): measured on 64-channel layers of 56x56 pixels, where 56 parts
// on two workgroups per CU take 37.7 us against 47.0 us for 28 parts on one.
int conv_fast_wgrad_split(const ConvGeom& g, dmath_dtype_t dt)
{
    const int64_t ktiles = wgrad_ktiles(g, dt);
    const int64_t tiles = wgrad_tiles(g, dt);
    const int unit = 64 / pixel_tile(dt);  // k-tiles per 64 pixels
    const int slots = 256 * per_cu(wgrad_tile_m(g, dt), wgrad_tile_n(g, dt), dt);
    const double w = dt == DMATH_F16 ? 1 : dt == DMATH_F32 ? 4 : 8;
    const int fit = slots / 256;
    auto cost = [&](int s) {
        const int64_t per = (ktiles + s - 1) / s, on_cu = (tiles * s + 255) / 256;
        double rate = 1.0;
        if (dt != DMATH_F16)
            rate = on_cu == 1 ? 0.87 : 1.0;
        else if (fit == 3)
            rate = on_cu == 1 ? 0.45 : on_cu == 2 ? 0.8 : 1.0;
        else if (fit == 2)
            rate = on_cu == 1 ? 0.73 : 1.0;
        return on_cu * (double)(per / unit) * w / rate + s;
    };
    int best = 1;
    for (int s = 2; s <= 96; ++s) {
        const int64_t per = (ktiles + s - 1) / s;
        if (wgrad_split_ok(ktiles, s) && tiles * s <= 4 * slots && per >= 4 * unit && cost(s) < cost(best)) best = s;
    }
    return best;
}

// Generic weight gradient: few C tiles and a very deep K.
static int32_t generic_wgrad_split(const ConvGeom& g)
{
    const int64_t M = g.k, N = (int64_t)g.c * g.r * g.s, K = (int64_t)g.n * g.oh * g.ow;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    const int64_t want = std::max<int64_t>(1, 1024 / std::max<int64_t>(1, tiles));
    const int64_t max_by_k = std::max<int64_t>(1, K / 512);
    return (int32_t)std::min<int64_t>({want, max_by_k, 512});  // first layers: 3 tiles, K of 800 thousand
}

// Elements of the partial sums of a forward pass / data gradient whose k-loop is split:
// [part][output channel, padded][pixel of whole tiles].
// Tiles of the forward pass / data gradient (in launch order: row of tiles by row of tiles) that
// fill whole rounds of workgroups, as whole rows of tiles.
static int64_t fwd_full_tiles(int64_t tiles_m, int tiles_n, int bm, int bn, dmath_dtype_t dt)
{
    const int64_t slots = 256 * per_cu(bm, bn, dt);
    return tiles_m * tiles_n / slots * slots / tiles_n * tiles_n;
}

int64_t conv_fast_partial_elems(int mode, const ConvGeom& g, dmath_dtype_t dt, const ConvChoice& c)
{
    const int64_t m = mode == CONV_FWD ? (int64_t)g.n * g.oh * g.ow : (int64_t)g.n * g.h * g.w;
    const int n_out = round64(mode == CONV_FWD ? g.k : g.c), tiles_n = n_out / c.tile_n;
    const int64_t tiles_m = (m + c.tile_m - 1) / c.tile_m;
    const int64_t full = c.tail_only ? fwd_full_tiles(tiles_m, tiles_n, c.tile_m, c.tile_n, dt) : 0;
    return (tiles_m - full / tiles_n) * c.tile_m * n_out;
}

// k-tiles of the forward pass (data gradient: filters take the channels' place)
static int64_t fwd_ktiles(int mode, const ConvGeom& g, dmath_dtype_t dt)
{
    return (int64_t)g.r * g.s * round64(mode == CONV_FWD ? g.c : g.k) / pixel_tile(dt);
}

// Tile shapes of the forward kernel (also the data gradient's), widest first.
struct FwdShape { int bm, bn; };
static std::vector<FwdShape> fwd_shapes(dmath_dtype_t dt, int n_out)
{
    std::vector<FwdShape> all;
    if (dt == DMATH_F16)
        all = {{256, 256}, {224, 256}, {256, 128}, {256, 64}};
    else
        all = {{128, 128}, {128, 64}};
    std::vector<FwdShape> out;
    for (const FwdShape& sh : all)
        if (n_out % sh.bn == 0) out.push_back(sh);
    return out;
}

// The cost model: the specialised kernels wherever their preconditions hold; the tile shape of
// the forward pass and the data gradient from a cycle count per round of workgroups, the split
// of the weight gradient from conv_fast_wgrad_split.
ConvChoice choose_conv(int mode, const ConvGeom& g, dmath_dtype_t in_dtype, int32_t policy)
{
    ConvChoice ch;
    if (policy == 0 && conv_as_gemm_ok(mode, g, in_dtype)) {
        ch.kernel = 2;  // tile shape and split are the GEMM chooser's
        return ch;
    }
    if (policy != 0 || !conv_fast_ok(mode, g, in_dtype)) {
        if (mode == CONV_BWD_FILTER) ch.split_k = generic_wgrad_split(g);
        return ch;
    }
    ch.kernel = 1;
    if (mode == CONV_BWD_FILTER) {
        ch.tile_m = wgrad_tile_m(g, in_dtype);
        ch.tile_n = wgrad_tile_n(g, in_dtype);
        ch.split_k = conv_fast_wgrad_split(g, in_dtype);
        if (const char* e = std::getenv("DMATH_CONV_SPLIT")) {  // experiments and tests
            const int forced = std::atoi(e);
            if (forced >= 1 && forced <= 128 && wgrad_split_ok(wgrad_ktiles(g, in_dtype), forced)) ch.split_k = forced;
        }
        return ch;
    }
    const int64_t m = mode == CONV_FWD ? (int64_t)g.n * g.oh * g.ow : (int64_t)g.n * g.h * g.w;
    const int n_out = round64(mode == CONV_FWD ? g.k : g.c);
    // the tile shape whose longest chain of tiles on one CU takes the fewest cycles: rounds of
    // workgroups over all slots x (k x the slower of the tile's matrix instructions -- fp16: 32.5
    // cycles per 32x32x16 over four SIMDs, fp32: 64 per 32x32x2, fp64: 64 per 16x16x4 -- and its operand loads at 60
    // bytes per cycle and CU, + the tile's stores at 10 bytes per cycle and CU).  fp16, 50176
    // pixels x 256 channels: 224 tiles of 224x256 are one round, against 196 of 256x256 or two
    // rounds of 256x128; 64-wide tiles are load-bound and win only where they save whole
    // rounds.  A narrower tile has to win by 3 %.  fp32: with one workgroup per CU (128x128) the
    // gathers are hidden less well than with two (128x64): 0.87 of the rate in the samples.
    const int64_t k_depth = (int64_t)g.r * g.s * round64(mode == CONV_FWD ? g.c : g.k);
    const int64_t ktiles = fwd_ktiles(mode, g, in_dtype);
    const int eb = elem_bytes(in_dtype);
    // cycles per unit of k and 32x32 block (fp64: four 16x16x4 instructions of 64 cycles per 4 of k)
    const double mfma_per_k = in_dtype == DMATH_F16 ? 32.5 / 16 : in_dtype == DMATH_F32 ? 64.0 / 2 : 64.0;
    // Few tiles and a deep k-loop (small batches, late layers): the loop is cut into parts
    // (powers of two, no part empty, at least four k-tiles each) that different workgroups run,
    // and a second kernel adds the partial sums in a fixed order: + its launch (3 us at 2.4 GHz)
    // and the partial sums written and read back at 3 TB/s.  A split has to win by 3 % as well.
    // Against that absolute cost the cycle count of the tiles is scaled to what small batches
    // take in the timing samples (1.75, 1.15 and 1.4 measured cycles per modelled one).
    const double measured = in_dtype == DMATH_F16 ? 1.75 : in_dtype == DMATH_F32 ? 1.15 : 1.4;
    double best = -1;
    for (const FwdShape& sh : fwd_shapes(in_dtype, n_out)) {
        const int64_t tiles = (m + sh.bm - 1) / sh.bm * (n_out / sh.bn);
        const int slots = per_cu(sh.bm, sh.bn, in_dtype);
        const double area = (double)sh.bm * sh.bn;
        const double per_k = std::max(area / 1024 * mfma_per_k / 4, (sh.bm + sh.bn) * eb / 60.0);
        for (int split = 1; split <= 32; split *= 2) {
            if (split > 1 && (!wgrad_split_ok(ktiles, split) || (ktiles + split - 1) / split < 4)) break;
            const int64_t wgs = tiles * split;
            // tiles the busiest CU runs
            const int64_t chain = wgs <= 256 ? 1 : (wgs + 256 * slots - 1) / (256 * slots) * slots;
            const double rate = (in_dtype != DMATH_F16 && (slots == 1 || chain == 1)) ? 0.87 : 1.0;  // a workgroup alone on its CU
            double cost = measured * (double)chain * ((double)k_depth / split * per_k / rate + 0.4 * area);
            if (split > 1)
                cost += 2.4e9 * (3e-6 + (split + 1.0) * (double)m * n_out * (in_dtype == DMATH_F64 ? 8 : 4) / 3e12);
            if (best < 0 || cost < 0.97 * best) {
                best = cost;
                ch.tile_m = sh.bm;
                ch.tile_n = sh.bn;
                ch.split_k = split;
                ch.tail_only = 0;
            }
        }
        // More than one round of workgroups and a last round that is not full: only the tiles of
        // that round are split, into 2, 4, 8 or 16 parts (which may take several short rounds of
        // their own).
        const int tiles_n = n_out / sh.bn;
        const int64_t full = fwd_full_tiles(tiles / tiles_n, tiles_n, sh.bm, sh.bn, in_dtype), left = tiles - full;
        for (int split = 2; full > 0 && left > 0 && split <= 16; split *= 2) {
            if (!wgrad_split_ok(ktiles, split) || (ktiles + split - 1) / split < 4) break;
            const int64_t wgs = left * split;
            const int64_t chain_left = wgs <= 256 ? 1 : (wgs + 256 * slots - 1) / (256 * slots) * slots;
            const double rate = (in_dtype != DMATH_F16 && (slots == 1 || chain_left == 1)) ? 0.87 : 1.0;
            const double full_rate = (in_dtype != DMATH_F16 && slots == 1) ? 0.87 : 1.0;
            double cost = measured * ((double)(full / 256) * ((double)k_depth * per_k / full_rate + 0.4 * area) +
                                      (double)chain_left * ((double)k_depth / split * per_k / rate + 0.4 * area));
            cost += 2.4e9 * (3e-6 + (split + 1.0) * (double)left / tiles_n * sh.bm * n_out *
                                        (in_dtype == DMATH_F64 ? 8 : 4) / 3e12);
            if (cost < (ch.tail_only ? 1.0 : 0.97) * best) {
                best = cost;
                ch.tile_m = sh.bm;
                ch.tile_n = sh.bn;
                ch.split_k = split;
                ch.tail_only = 1;
            }
        }
    }
    // optional overrides for experiments and tests: DMATH_CONV_TILE=128x64 (one of the shapes
    // above), DMATH_CONV_SPLIT=3 (parts may be uneven) or =8t (only the tiles after the last full
    // round of workgroups)
    if (const char* e = std::getenv("DMATH_CONV_TILE")) {
        int bm = 0, bn = 0;
        if (std::sscanf(e, "%dx%d", &bm, &bn) == 2)
            for (const FwdShape& sh : fwd_shapes(in_dtype, n_out))
                if (sh.bm == bm && sh.bn == bn) {
                    ch.tile_m = bm;
                    ch.tile_n = bn;
                }
    }
    if (const char* e = std::getenv("DMATH_CONV_SPLIT")) {
        const int forced = std::atoi(e);
        if (forced >= 1 && forced <= 64 && wgrad_split_ok(ktiles, forced)) {
            ch.split_k = forced;
            ch.tail_only = std::strchr(e, 't') != nullptr;
        }
    }
    return ch;
}

// Everything worth a timing sample: the generic kernel (weight gradient: unsplit and with its
// own split), and where the specialised kernels apply, every tile shape (forward, data
// gradient) or the cost model's split and every split count that divides the k-tiles evenly,
// keeps at least 4 of them per part and at most 1024 workgroups (weight gradient).
std::vector<ConvChoice> conv_candidates(int mode, const ConvGeom& g, dmath_dtype_t in_dtype, int32_t policy)
{
    std::vector<ConvChoice> out;
    ConvChoice c;
    out.push_back(c);
    if (mode == CONV_BWD_FILTER && generic_wgrad_split(g) > 1) {
        c.split_k = generic_wgrad_split(g);
        out.push_back(c);
    }
    if (policy == 0 && conv_as_gemm_ok(mode, g, in_dtype)) {
        c = ConvChoice{};
        c.kernel = 2;
        out.push_back(c);
    }
    if (policy != 0 || !conv_fast_ok(mode, g, in_dtype)) return out;
    c = ConvChoice{};
    c.kernel = 1;
    if (mode == CONV_BWD_FILTER) {
        const int64_t ktiles = wgrad_ktiles(g, in_dtype), tiles = wgrad_tiles(g, in_dtype);
        const int model = conv_fast_wgrad_split(g, in_dtype);
        c.tile_m = wgrad_tile_m(g, in_dtype);
        c.tile_n = wgrad_tile_n(g, in_dtype);
        for (int s = 1; s <= 96; ++s)
            if (s == model || (ktiles % s == 0 && tiles * s <= 1024 && ktiles / s >= 4)) {
                c.split_k = s;
                out.push_back(c);
            }
        return out;
    }
    const int64_t m = mode == CONV_FWD ? (int64_t)g.n * g.oh * g.ow : (int64_t)g.n * g.h * g.w;
    const int n_out = round64(mode == CONV_FWD ? g.k : g.c);
    const int64_t ktiles = fwd_ktiles(mode, g, in_dtype);
    for (const FwdShape& sh : fwd_shapes(in_dtype, n_out)) {
        const int64_t tiles = (m + sh.bm - 1) / sh.bm * (n_out / sh.bn);
        c.tile_m = sh.bm;
        c.tile_n = sh.bn;
        for (int split = 1; split <= 32; split *= 2) {
            if (split > 1 && (!wgrad_split_ok(ktiles, split) || (ktiles + split - 1) / split < 4 || tiles * split > 512))
                break;
            c.split_k = split;
            out.push_back(c);
        }
        const int tiles_n = n_out / sh.bn;
        const int64_t slots = 256 * per_cu(sh.bm, sh.bn, in_dtype);
        const int64_t left = tiles - fwd_full_tiles(tiles / tiles_n, tiles_n, sh.bm, sh.bn, in_dtype);
        if (left < tiles && left > 0)
            for (int split = 2; split <= 16; split *= 2)
                if (wgrad_split_ok(ktiles, split) && (ktiles + split - 1) / split >= 4) {
                    c.split_k = split;
                    c.tail_only = 1;
                    out.push_back(c);
                }
        c.tail_only = 0;
    }
    const ConvChoice model = choose_conv(mode, g, in_dtype, policy);
    bool listed = false;
    for (const ConvChoice& o : out) listed = listed || o == model;
    if (!listed) out.push_back(model);
    return out;
}

namespace {

// Launches the forward kernel (also the data gradient's) on tiles of BM x BN.
template <class P, int BM, int BN, int STAGES>
hipError_t launch_fwd_shape(const FastConv& geom, dmath_dtype_t out, double alpha, double beta, hipStream_t st)
{
    using AccT = typename P::AccT;
    using Wide = typename std::conditional<std::is_same<P, PipeF64>::value, double, float>::type;  // the wider output type
    FastConv p = geom;
    const int64_t m = (int64_t)p.g.n * p.g.oh * p.g.ow;
    const int tiles_m = (int)((m + BM - 1) / BM), tiles_n = p.g.k / BN;
    if (p.split < 1) p.split = 1;
    p.ktiles = p.g.r * p.g.s * (p.g.c / P::BK);
    p.ktiles_per_split = (p.ktiles + p.split - 1) / p.split;
    if (!wgrad_split_ok(p.ktiles, p.split) || (p.split > 1 && !p.ws)) return hipErrorInvalidValue;
    constexpr bool kHalf = std::is_same<typename P::Elem, _Float16>::value;
    const dmath_dtype_t in = kHalf ? DMATH_F16 : std::is_same<P, PipeF32>::value ? DMATH_F32 : DMATH_F64;
    p.full_tiles = p.split == 1    ? tiles_m * tiles_n
                   : p.tail_only   ? (int)fwd_full_tiles(tiles_m, tiles_n, BM, BN, in)
                                   : 0;
    const int split_tiles = tiles_m * tiles_n - p.full_tiles;
    const int tiles = p.full_tiles + split_tiles * p.split;
    constexpr int lds = P::lds_bytes(BM, BN, STAGES);
    static bool configured = false;  // more than 64 KiB of LDS has to be asked for once per kernel
    if (!configured) {
        hipError_t e = set_lds(conv_fwd_kernel<P, BM, BN, STAGES, Wide>, lds);
        if (e == hipSuccess && kHalf)
            e = set_lds(conv_fwd_kernel<P, BM, BN, STAGES, typename P::Elem>, lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    if (out == DMATH_F16)
        conv_fwd_kernel<P, BM, BN, STAGES, typename P::Elem><<<tiles, NT, lds, st>>>(p, (AccT)alpha, (AccT)beta);
    else
        conv_fwd_kernel<P, BM, BN, STAGES, Wide><<<tiles, NT, lds, st>>>(p, (AccT)alpha, (AccT)beta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split_tiles == 0) return e;
    const int64_t mp = (int64_t)(split_tiles / tiles_n) * BM;
    const int m_first = p.full_tiles / tiles_n * BM;
    const int blocks = (int)std::min<int64_t>(2048, ((int64_t)p.k_real * (m - m_first) + 255) / 256);
    if (out == DMATH_F16)
        conv_fwd_reduce_kernel<AccT, typename P::Elem><<<blocks, 256, 0, st>>>(p, mp, m_first, (AccT)alpha, (AccT)beta);
    else
        conv_fwd_reduce_kernel<AccT, Wide><<<blocks, 256, 0, st>>>(p, mp, m_first, (AccT)alpha, (AccT)beta);
    return hipGetLastError();
}

hipError_t launch_fwd(const FastConv& p, dmath_dtype_t in, int tile_m, int tile_n, dmath_dtype_t out, double alpha,
                      double beta, hipStream_t st)
{
    if (in == DMATH_F64) {
        if (tile_m == 128 && tile_n == 128) return launch_fwd_shape<PipeF64, 128, 128, 3>(p, out, alpha, beta, st);
        if (tile_m == 128 && tile_n == 64) return launch_fwd_shape<PipeF64, 128, 64, 3>(p, out, alpha, beta, st);
        return hipErrorInvalidValue;
    }
    if (in == DMATH_F32) {
        if (tile_m == 128 && tile_n == 128) return launch_fwd_shape<PipeF32, 128, 128, 3>(p, out, alpha, beta, st);
        if (tile_m == 128 && tile_n == 64) return launch_fwd_shape<PipeF32, 128, 64, 3>(p, out, alpha, beta, st);
        return hipErrorInvalidValue;
    }
    // The tiles whose wavefront parts are multiples of 64 on both sides run on 16x16x32 fragments;
    // DMATH_F16_MFMA32=1 switches them back to 32x32x16 (A/B measurements).
    static const bool mf32 = std::getenv("DMATH_F16_MFMA32") != nullptr;
    if (!mf32) {
        if (tile_m == 224 && tile_n == 256) return launch_fwd_shape<PipeF16Q, 224, 256, 2>(p, out, alpha, beta, st);
        if (tile_m == 256 && tile_n == 256) return launch_fwd_shape<PipeF16Q, 256, 256, 2>(p, out, alpha, beta, st);
        if (tile_m == 256 && tile_n == 128) return launch_fwd_shape<PipeF16Q, 256, 128, 3>(p, out, alpha, beta, st);
    }
    if (tile_m == 224 && tile_n == 256) return launch_fwd_shape<PipeF16, 224, 256, 2>(p, out, alpha, beta, st);
    if (tile_m == 256 && tile_n == 256) return launch_fwd_shape<PipeF16, 256, 256, 2>(p, out, alpha, beta, st);
    if (tile_m == 256 && tile_n == 128) return launch_fwd_shape<PipeF16, 256, 128, 3>(p, out, alpha, beta, st);
    if (tile_m == 256 && tile_n == 64) return launch_fwd_shape<PipeF16, 256, 64, 3>(p, out, alpha, beta, st);
    return hipErrorInvalidValue;
}

template <class P, int BM, int BN, bool IN_PLACE, bool TABLE>
hipError_t launch_wgrad_kernel(const FastConv& p, int tiles, hipStream_t st)
{
    // TABLE: one offset per pixel of a part's k-range and of one k-tile more, behind the stages
    const int lds = P::lds_bytes(BM, BN, 3) + (TABLE ? (p.ktiles_per_split + 1) * P::BK * 4 : 0);
    static int configured = 0;
    if (configured < lds) {
        hipError_t e = set_lds(conv_wgrad_kernel<P, BM, BN, IN_PLACE, TABLE>, lds);
        if (e != hipSuccess) return e;
        configured = lds;
    }
    conv_wgrad_kernel<P, BM, BN, IN_PLACE, TABLE><<<tiles, NT, lds, st>>>(p);
    return hipGetLastError();
}
constexpr int kLdsPerCu = 160 * 1024;
template <class P, int BM, int BN> hipError_t launch_wgrad_shape(const FastConv& p, int tiles, hipStream_t st)
{
    // the pixel-offset table where the pipeline has few issue slots to spare (16x16x32 fragments)
    // and the table fits beside its stages
    if constexpr (std::is_same<P, PipeF16QF>::value) {
        if (P::lds_bytes(BM, BN, 3) + (int64_t)(p.ktiles_per_split + 1) * P::BK * 4 <= kLdsPerCu) {
            if (p.y_src) return launch_wgrad_kernel<P, BM, BN, true, true>(p, tiles, st);
            return launch_wgrad_kernel<P, BM, BN, false, true>(p, tiles, st);
        }
    }
    if (p.y_src) return launch_wgrad_kernel<P, BM, BN, true, false>(p, tiles, st);
    return launch_wgrad_kernel<P, BM, BN, false, false>(p, tiles, st);
}

hipError_t launch_wgrad(const FastConv& p, dmath_dtype_t in, int bm, int bn, int tiles, hipStream_t st)
{
    if (in == DMATH_F64) {
        if (bm == 128 && bn == 128) return launch_wgrad_shape<PipeF64, 128, 128>(p, tiles, st);
        if (bm == 128 && bn == 64) return launch_wgrad_shape<PipeF64, 128, 64>(p, tiles, st);
        if (bm == 64 && bn == 128) return launch_wgrad_shape<PipeF64, 64, 128>(p, tiles, st);
        if (bm == 64 && bn == 64) return launch_wgrad_shape<PipeF64, 64, 64>(p, tiles, st);
        return hipErrorInvalidValue;
    }
    if (in == DMATH_F32) {
        if (bm == 128 && bn == 128) return launch_wgrad_shape<PipeF32, 128, 128>(p, tiles, st);
        if (bm == 128 && bn == 64) return launch_wgrad_shape<PipeF32, 128, 64>(p, tiles, st);
        if (bm == 64 && bn == 128) return launch_wgrad_shape<PipeF32, 64, 128>(p, tiles, st);
        if (bm == 64 && bn == 64) return launch_wgrad_shape<PipeF32, 64, 64>(p, tiles, st);
        return hipErrorInvalidValue;
    }
    // Tiles of 128 columns run on 16x16x32 fragments with the accumulators in fixed registers: with
    // tied accumulators the compiler, given this walk's many per-lane values, renamed them between
    // the iterations and read them before the matrix instructions written as assembly had finished
    // (found by check_isa.py); draining the matrix cores at those points was correct and slower
    // than 32x32x16 fragments.  DMATH_F16_MFMA32=1 switches back to those (A/B measurements).
    static const bool mf32 = std::getenv("DMATH_F16_MFMA32") != nullptr;
    if (!mf32 && bm == 256 && bn == 128) return launch_wgrad_shape<PipeF16QF, 256, 128>(p, tiles, st);
    if (!mf32 && bm == 128 && bn == 128) return launch_wgrad_shape<PipeF16QF, 128, 128>(p, tiles, st);
    if (bm == 256 && bn == 128) return launch_wgrad_shape<PipeF16, 256, 128>(p, tiles, st);
    if (bm == 128 && bn == 128) return launch_wgrad_shape<PipeF16, 128, 128>(p, tiles, st);
    if (bm == 64 && bn == 128) return launch_wgrad_shape<PipeF16, 64, 128>(p, tiles, st);
    if (bm == 256 && bn == 64) return launch_wgrad_shape<PipeF16, 256, 64>(p, tiles, st);
    if (bm == 128 && bn == 64) return launch_wgrad_shape<PipeF16, 128, 64>(p, tiles, st);
    if (bm == 64 && bn == 64) return launch_wgrad_shape<PipeF16, 64, 64>(p, tiles, st);
    return hipErrorInvalidValue;
}

// The whole call for input element type T.
template <class T>
hipError_t launch_typed(const ConvPlan& plan, int mode, double alpha, double beta, unsigned rewrite, hipStream_t st)
{
    const ConvTables& t = plan.t;
    const ConvGeom& g = t.g;
    const dmath_dtype_t in = plan.in_dtype;
    const int cp = round64(g.c), kp = round64(g.k);
    FastConv p{};
    p.g = g;
    p.g.c = cp;
    p.g.k = kp;
    p.c_real = g.c;
    p.k_real = g.k;
    p.hp = g.h + 2 * g.pad_h;
    p.wp = g.w + 2 * g.pad_w;
    p.y_rows = t.y_rows;
    p.f_rows = t.f_rows;
    T* const xp = plan.xp ? static_cast<T*>(plan.xp->buf) : nullptr;
    T* const fp = plan.fp ? static_cast<T*>(plan.fp->buf) : nullptr;
    T* const yt = plan.yt ? static_cast<T*>(plan.yt->buf) : nullptr;
    p.xp = xp;
    p.fp = fp;
    p.yt = yt;
    p.y_src = mode == CONV_BWD_FILTER ? plan.dy_in_place : nullptr;
    p.ws = t.workspace;
    p.split = t.split_k;
    p.tail_only = plan.tail_only;
    p.sink = t.sink;
    if (!xp || !p.sink || (mode != CONV_BWD_FILTER && !fp) || (mode == CONV_BWD_FILTER && ((!yt && !p.y_src) || !p.ws)))
        return hipErrorInvalidValue;  // the plan was not made for this path

    RelayoutJobs jobs{};
    int lds = 0;
    if (mode == CONV_BWD_DATA) {
        // forward convolution (stride 1) over dY with its pixels spread out by the stride: input
        // channels k, padding r-1-pad in front, rotated filter, output channels c, output
        // spatial h x w (so the copy has h+r-1 x w+s-1 pixels), output rows = images of dX
        FastConv q = p;
        const int pph = g.r - 1 - g.pad_h, ppw = g.s - 1 - g.pad_w;
        q.g.c = kp; q.g.k = cp;
        q.k_real = g.c;
        q.g.h = g.oh; q.g.w = g.ow; q.g.oh = g.h; q.g.ow = g.w;
        q.g.pad_h = pph; q.g.pad_w = ppw;
        q.g.stride_h = q.g.stride_w = 1;
        q.hp = g.h + g.r - 1;
        q.wp = g.w + g.s - 1;
        q.y_rows = t.x_rows;
        if (rewrite & REWRITE_X)
            jobs.a = tcl_job<T>(t.y_rows, g.n, g.k, kp, g.oh, g.ow, pph, ppw, g.stride_h, g.stride_w, q.hp, q.wp, xp, &lds);
        bool filter_apart = false;
        if (rewrite & REWRITE_F)
            filter_apart = !filter_job<T>(2, t.f_rows, g.c, cp, g.r * g.s, g.k, kp, fp, &jobs.f, &lds);
        if (hipError_t e = launch_relayout<T>(jobs, lds, st); e != hipSuccess) return e;
        if (filter_apart)
            filter_to_rsk_rotated_tiled_kernel<T>
                <<<dim3((g.c * g.r * g.s + 63) / 64, kp / 64), 256, 0, st>>>(t.f_rows, g.c, g.r * g.s, g.k, kp, fp);
        return launch_fwd(q, in, plan.tile_m, plan.tile_n, plan.out_dtype, alpha, beta, st);
    }
    // activations -> zero-bordered channels-last copy (borders were zeroed when the copy was allocated)
    if (rewrite & REWRITE_X)
        jobs.a = tcl_job<T>(t.x_rows, g.n, g.c, cp, g.h, g.w, g.pad_h, g.pad_w, 1, 1, p.hp, p.wp, xp, &lds);
    if (mode == CONV_FWD) {
        bool filter_apart = false;
        if (rewrite & REWRITE_F)
            filter_apart = !filter_job<T>(1, t.f_rows, g.c, cp, g.r * g.s, g.k, kp, fp, &jobs.f, &lds);
        if (hipError_t e = launch_relayout<T>(jobs, lds, st); e != hipSuccess) return e;
        if (filter_apart) filter_to_rsc<T>(t.f_rows, g.c, cp, g.r * g.s, g.k, fp, st);
        return launch_fwd(p, in, plan.tile_m, plan.tile_n, plan.out_dtype, alpha, beta, st);
    }
    // weight gradient: dY -> channels-last [m][k], split GEMM, fixed-order reduction
    if (!p.y_src && (rewrite & REWRITE_Y))
        jobs.b = tcl_job<T>(t.y_rows, g.n, g.k, kp, g.oh, g.ow, 0, 0, 1, 1, g.oh, g.ow, yt, &lds);
    if (hipError_t e = launch_relayout<T>(jobs, lds, st); e != hipSuccess) return e;
    p.ktiles = (int)wgrad_ktiles(g, in);
    p.ktiles_per_split = (p.ktiles + t.split_k - 1) / t.split_k;
    if (!wgrad_split_ok(p.ktiles, t.split_k)) return hipErrorInvalidValue;  // a part without pixels
    const int tiles = (int)wgrad_tiles(g, in) * t.split_k;
    hipError_t e = launch_wgrad(p, in, wgrad_tile_m(g, in), wgrad_tile_n(g, in), tiles, st);
    if (e != hipSuccess) return e;
    if (plan.out_dtype == DMATH_F64)
        wgrad_reduce<double, double>(p, alpha, beta, st);
    else if (plan.out_dtype == DMATH_F16)
        wgrad_reduce<float, _Float16>(p, alpha, beta, st);
    else
        wgrad_reduce<float, float>(p, alpha, beta, st);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv_fast(const ConvPlan& plan, int mode, double alpha, double beta, unsigned rewrite,
                            hipStream_t st)
{
    if (plan.in_dtype == DMATH_F16) return launch_typed<_Float16>(plan, mode, alpha, beta, rewrite, st);
    if (plan.in_dtype == DMATH_F32) return launch_typed<float>(plan, mode, alpha, beta, rewrite, st);
    return launch_typed<double>(plan, mode, alpha, beta, rewrite, st);
}

}  // namespace dm
