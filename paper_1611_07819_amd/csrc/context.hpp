// Host-side objects behind the opaque handles of dmath.h.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <map>
#include <memory>
#include <set>
#include <tuple>
#include <vector>

#include "../../include/dmath.h"
#include "pool.hpp"
#include "tables.hpp"

namespace dm {

inline size_t elem_size(dmath_dtype_t d) { return d == DMATH_F64 ? 8 : d == DMATH_F32 ? 4 : 2; }

// Split rule of a dimension of length n into g parts (see dmath.h).
struct Split {
    int64_t n = 0, step = 0;
    int32_t g = 0;
    Split() = default;
    Split(int64_t n_, int32_t g_) : n(n_), step((n_ + g_ - 1) / g_), g(g_) {}
    bool valid() const { return n > 0 && g > 0 && (int64_t)(g - 1) * step < n; }
    int64_t lo(int32_t p) const { return (int64_t)p * step; }
    int64_t hi(int32_t p) const { return lo(p) + step < n ? lo(p) + step : n; }
    int64_t len(int32_t p) const { return hi(p) - lo(p); }
    int32_t part(int64_t i) const { return (int32_t)(i / step); }
};

}  // namespace dm

struct dmath_matrix_s {
    dmath_ctx_s* ctx = nullptr;
    uint64_t id = 0;
    int64_t rows = 0, cols = 0;
    dm::Split rsplit, csplit;
    dmath_dtype_t dtype = DMATH_F32;
    std::vector<void*> blocks;  // grid row-major
    // Bumped by every call that writes the matrix; re-layout copies remember the value they were
    // made from.  A matrix whose block pointers were handed out can change unseen: never reused.
    uint64_t version = 1;
    bool exposed = false;
    void* block(int32_t bi, int32_t bj) const { return blocks[(size_t)bi * csplit.g + bj]; }
};

namespace dm {

enum KernelId : int32_t {
    KERNEL_GENERIC = 0,
    KERNEL_F32_128 = 1,
    KERNEL_F16_256 = 2,
    KERNEL_F64_128 = 3,
};

struct GemmPlan {
    std::vector<uint64_t> uses;  // matrix ids
    GemmTables t{};
    void* dev_tables = nullptr;
    void* workspace = nullptr;
    dmath_plan_info_t info{};
    dmath_dtype_t in_dtype = DMATH_F32, out_dtype = DMATH_F32;
    // the reduction / beta-only kernel may move 16 bytes per lane: every n-segment a multiple of
    // 4, every C panel and the workspace rows 16-byte aligned
    bool reduce_vectors = false;
    // k-segments that are not multiples of the kernel's k-tile: their last elements are copied
    // into zero-padded scratch panels (which the panel tables point to) before every launch
    const CopyCell* tail_cells = nullptr;
    int32_t n_tail_cells = 0, tail_rows = 0;
    void* tail_scratch = nullptr;
    // > 0: only the tiles from this index on (those after the last full round of workgroups) are
    // split; their m_glob / n_glob address a compact workspace [split][tiles x tile_m][tile_n]
    int32_t full_tiles = 0;
    const int32_t* ksplit_whole = nullptr;  // {0, n_kseg}: the whole k-loop as one part
    bool in_arena = false;  // tables, partial sums and k-tail panels lie in a fixed arena, not in the pool
};

// A fixed range of device memory handed out front to back, 256 bytes at a time (the plan of the
// entry point that allocates nothing lives in one).
struct Arena {
    char* base = nullptr;
    size_t cap = 0, used = 0;
    void* take(size_t bytes)
    {
        const size_t need = ((bytes ? bytes : 1) + 255) / 256 * 256;
        if (need > cap - used) return nullptr;
        void* p = base + used;
        used += need;
        return p;
    }
};

enum ConvMode : int32_t { CONV_FWD = 0, CONV_BWD_FILTER = 1, CONV_BWD_DATA = 2 };

// A re-laid-out copy of one matrix, kept in the pool beside it (paper section 1, the cache of
// objects already seen; section 3.3, reorganised data kept for the operations that follow).  It
// is current while the source's version and the context's epoch are the ones it was written at.
enum RelayoutKind : int32_t {
    RELAYOUT_CHANNELS_LAST = 0,   // [n][h+2ph][w+2pw][ch], zero border; geometry {ch, h, w, ph, pw}
    RELAYOUT_FILTER_RSC = 1,      // [k][(r,s,c)];                       geometry {c, r, s, k}
    RELAYOUT_FILTER_ROTATED = 2,  // [c][(r',s',k)], taps reversed;      geometry {c, r, s, k}
};
struct Relayout {
    void* buf = nullptr;
    size_t bytes = 0;
    uint64_t version = 0;  // of the source when the copy was last written (0: never)
    uint64_t epoch = 0;
};
using RelayoutKey = std::tuple<uint64_t, int32_t, std::vector<int32_t>>;  // matrix id, kind, geometry

struct ConvPlan {
    std::vector<uint64_t> uses;
    ConvTables t{};
    void* dev_tables = nullptr;
    void* workspace = nullptr;
    // specialised (MFMA pipeline) path: the copies it reads (owned by the context's table of re-layouts)
    Relayout* xp = nullptr;  // gathered activations, channels-last with zero border
    Relayout* fp = nullptr;  // permuted filter
    Relayout* yt = nullptr;  // weight gradient: dY channels-last, [n*oh*ow][k] ...
    const void* dy_in_place = nullptr;  // ... or dY itself (its first element) where the kernel can read it as it lies
    // 0 generic, 1 specialised (gathering MFMA kernels over re-layout copies), 2 as a block GEMM
    // (1x1, stride 1, no padding: the images are the column blocks of a k x c by c x n*h*w product)
    int32_t kernel = 0;
    std::unique_ptr<GemmPlan> gemm;  // kernel 2
    int32_t tile_n = 0;  // specialised forward / data gradient: 128 or 256 output channels per tile
    int32_t tile_m = 0;  //   and 256 or 224 pixels
    int32_t tail_only = 0;  //   split_k parts only for the tiles after the last full round
    dmath_dtype_t in_dtype = DMATH_F16, out_dtype = DMATH_F32;
};

// Kernel / tile / split-K decision for a convolution.
struct ConvChoice {
    int32_t kernel = 0, tile_m = 0, tile_n = 0, split_k = 1;
    // specialised forward / data gradient: the split applies only to the tiles left over after
    // the last full round of workgroups
    int32_t tail_only = 0;
    bool operator==(const ConvChoice& o) const
    {
        return kernel == o.kernel && tile_m == o.tile_m && tile_n == o.tile_n && split_k == o.split_k &&
               tail_only == o.tail_only;
    }
};

using GemmKey = std::tuple<uint64_t, uint64_t, uint64_t, int, int>;
using ConvKey = std::tuple<uint64_t, uint64_t, uint64_t, int, std::vector<int32_t>>;

// A recorded sequence and the matrices its kernels read or write (destroying one of them
// destroys the sequence).
struct Pipeline {
    hipGraphExec_t exec = nullptr;
    std::set<uint64_t> uses;
};

// Tile shape / kernel / split-K decision for a GEMM whose segments are known.
struct GemmChoice {
    int32_t kernel = KERNEL_GENERIC;
    int32_t tile_m = 64, tile_n = 64, tile_k = 16;
    int32_t split_k = 1;
    // > 0 (with split_k > 1): the first full_tiles tiles of the launch order, whole rounds of
    // workgroups, run the whole k-loop; only the tiles after them are split
    int32_t full_tiles = 0;
};

}  // namespace dm

struct dmath_ctx_s {
    dm::Pool pool;
    hipStream_t stream;
    uint64_t next_id = 1;
    int32_t policy = 0;
    std::set<dmath_matrix_s*> matrices;
    std::map<dm::GemmKey, std::unique_ptr<dm::GemmPlan>> gemm_plans;
    std::map<dm::ConvKey, std::unique_ptr<dm::ConvPlan>> conv_plans;
    bool recording = false;  // between dmath_pipeline_begin and _end
    std::set<uint64_t> recording_uses;  // matrices touched by the sequence being recorded
    std::map<int32_t, dm::Pipeline> pipelines;  // recorded sequences
    int32_t next_pipeline = 1;
    // re-layout copies: reused while current unless switched off; the epoch moves at every
    // recording boundary and replay, so nothing is reused across them
    std::map<dm::RelayoutKey, dm::Relayout> relayouts;
    // choices found by timing samples (dmath_gemm_tune / dmath_conv_tune), by layout signature
    std::map<std::vector<int64_t>, dm::GemmChoice> tuned_gemm;
    std::map<std::vector<int64_t>, dm::ConvChoice> tuned_conv;
    bool reuse_relayouts = true;
    uint64_t epoch = 1;
    uint64_t relayouts_reused = 0, relayouts_written = 0;
    // dmath_gemm_noalloc: its one plan (in the device's static scratch array), what it was made
    // for, and the token under which this context last wrote the array
    std::unique_ptr<dm::GemmPlan> noalloc_plan;
    dm::GemmKey noalloc_key{};
    uint64_t noalloc_token = 0;
    dmath_ctx_s(void* slab, size_t bytes, hipStream_t s) : pool(slab, bytes), stream(s) {}
};

namespace dm {

// plan.cpp
dmath_status_t get_gemm_plan(dmath_ctx_s* ctx, int transA, int transB, dmath_matrix_s* A,
                             dmath_matrix_s* B, dmath_matrix_s* C, bool upload, GemmPlan** out,
                             bool* was_cached);
dmath_status_t get_conv_plan(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d,
                             dmath_matrix_s* X, dmath_matrix_s* F, dmath_matrix_s* Y,
                             ConvPlan** out);
void drop_plans_using(dmath_ctx_s* ctx, uint64_t matrix_id);
void drop_all_plans(dmath_ctx_s* ctx);
void drop_pipelines_using(dmath_ctx_s* ctx, uint64_t matrix_id);
void drop_all_pipelines(dmath_ctx_s* ctx);
void drop_unused_relayouts(dmath_ctx_s* ctx);

// kernels (launch.hip)
hipError_t launch_gemm(const GemmPlan& p, double alpha, double beta, hipStream_t stream);
// rewrite: bit 0 the gathered activations, bit 1 the filter, bit 2 dY of the weight gradient have
// to be re-laid-out before the multiplication (specialised path only)
enum : unsigned { REWRITE_X = 1, REWRITE_F = 2, REWRITE_Y = 4 };
hipError_t launch_conv(const ConvPlan& p, int mode, double alpha, double beta, unsigned rewrite,
                       hipStream_t stream);
hipError_t launch_reblock(dmath_dtype_t sd, dmath_dtype_t dd, const CopyCell* cells, int n_cells,
                          int max_rows, bool vectors, hipStream_t st);
int reblock_vector_width(dmath_dtype_t sd, dmath_dtype_t dd);
// Extents and sizes of the copies the specialised convolution kernels read: channel and
// filter counts rounded up to multiples of 64, images in the channels-last copy of X (one more,
// all zeros, where n*oh*ow is not a multiple of the pixel tile), bytes of the activation copy (x), the
// permuted filter (f; 0 for the weight gradient) and the channels-last dY (y; weight gradient only).
struct ConvFastLayout {
    int32_t cp, kp;
    int64_t x_images, x_bytes, f_bytes, y_bytes;
};
ConvFastLayout conv_fast_layout(int mode, const ConvGeom& g, dmath_dtype_t in_dtype);
bool conv_fast_ok(int mode, const ConvGeom& g, dmath_dtype_t in_dtype);
// A 1x1 convolution with stride 1 and no padding that is better run as a block GEMM.
bool conv_as_gemm_ok(int mode, const ConvGeom& g, dmath_dtype_t in_dtype);
bool conv_fast_wgrad_dy_in_place(const ConvGeom& g, dmath_dtype_t in_dtype);
int conv_fast_wgrad_split(const ConvGeom& g, dmath_dtype_t in_dtype);
int64_t conv_fast_partial_elems(int mode, const ConvGeom& g, dmath_dtype_t in_dtype, const ConvChoice& c);
hipError_t launch_conv_fast(const ConvPlan& p, int mode, double alpha, double beta, unsigned rewrite,
                           hipStream_t st);
bool read_cycle_probe(uint64_t* out6);  // gemm_f16.hip; false unless built with the cycle probe
hipError_t launch_mfma_peak(dmath_dtype_t dt, int iters, void* scratch, hipStream_t st, double* flops,
                            bool wide_f16 = false);
// Picks kernel, tile shape and split-K; written next to the kernels whose preconditions it checks.
struct SegView {
    int64_t M, N, K;
    const std::vector<int64_t>* mlen;
    const std::vector<int64_t>* nlen;
    const std::vector<int64_t>* klen;
    bool a_kcontig, b_kcontig;
    bool aligned16;  // every panel origin and leading dimension is a multiple of 16 bytes
    bool offsets32;  // every block of A and B is smaller than 4 GiB (the kernels' 32-bit lane offsets)
    dmath_dtype_t in_dtype, out_dtype;
    int32_t policy;
};
GemmChoice choose_gemm(const SegView& v);
std::vector<GemmChoice> gemm_candidates(const SegView& v);
// conv_mfma.hip / launch.hip: the cost model's choice and everything worth a timing sample
ConvChoice choose_conv(int mode, const ConvGeom& g, dmath_dtype_t in_dtype, int32_t policy);
std::vector<ConvChoice> conv_candidates(int mode, const ConvGeom& g, dmath_dtype_t in_dtype, int32_t policy);
// plan.cpp: plans outside the cache, built for one given choice (timing samples)
dmath_status_t make_gemm_plan(dmath_ctx_s* ctx, int transA, int transB, dmath_matrix_s* A, dmath_matrix_s* B,
                              dmath_matrix_s* C, bool upload, const GemmChoice* forced,
                              std::unique_ptr<GemmPlan>* out, std::vector<GemmChoice>* candidates,
                              bool unsplit = false, Arena* arena = nullptr);
void free_gemm_plan(dmath_ctx_s* ctx, GemmPlan& p);
dmath_status_t make_conv_plan(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d, dmath_matrix_s* X,
                              dmath_matrix_s* F, dmath_matrix_s* Y, const ConvChoice* forced,
                              std::unique_ptr<ConvPlan>* out);
void free_conv_plan(dmath_ctx_s* ctx, ConvPlan& p);
std::vector<int64_t> gemm_signature(int transA, int transB, const dmath_matrix_s* A, const dmath_matrix_s* B,
                                    const dmath_matrix_s* C);
std::vector<int64_t> conv_signature(int mode, const dmath_conv_desc_t* d, const dmath_matrix_s* X,
                                    const dmath_matrix_s* F, const dmath_matrix_s* Y);
size_t conv_choice_bytes(int mode, const ConvGeom& g, const ConvChoice& c, dmath_dtype_t in_dtype);

}  // namespace dm
