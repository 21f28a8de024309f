// C ABI of dmath.h: argument checks, handle bookkeeping, host<->device copies.  All arithmetic
// of the method runs in the kernels; nothing here computes on matrix elements.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <new>
#include <stdexcept>
#include <vector>

#include "../../include/dmath_measure.h"
#include "context.hpp"

using namespace dm;

namespace {

bool valid_dtype(int d) { return d == DMATH_F64 || d == DMATH_F32 || d == DMATH_F16; }
bool valid_op(int o) { return o == DMATH_OP_N || o == DMATH_OP_T; }

bool owns(dmath_ctx_s* ctx, dmath_matrix_s* m) { return m && ctx && ctx->matrices.count(m); }

// C may equal the input dtype; F16 inputs may also write F32.
bool dtype_combo_ok(dmath_dtype_t in_a, dmath_dtype_t in_b, dmath_dtype_t out)
{
    if (in_a != in_b) return false;
    if (out == in_a) return true;
    return in_a == DMATH_F16 && out == DMATH_F32;
}

dmath_status_t check_gemm(dmath_ctx_s* ctx, int ta, int tb, dmath_matrix_s* A, dmath_matrix_s* B,
                          dmath_matrix_s* C)
{
    if (!ctx || !A || !B || !C || !valid_op(ta) || !valid_op(tb)) return DMATH_ERR_INVALID_ARG;
    if (!owns(ctx, A) || !owns(ctx, B) || !owns(ctx, C)) return DMATH_ERR_INVALID_ARG;
    if (C == A || C == B) return DMATH_ERR_ALIAS;
    if (!dtype_combo_ok(A->dtype, B->dtype, C->dtype)) return DMATH_ERR_DTYPE;
    int64_t am = ta ? A->cols : A->rows, ak = ta ? A->rows : A->cols;
    int64_t bk = tb ? B->cols : B->rows, bn = tb ? B->rows : B->cols;
    if (ak != bk || am != C->rows || bn != C->cols) return DMATH_ERR_SHAPE;
    return DMATH_OK;
}

// Every path that changes a matrix's elements ends here.
void wrote(dmath_ctx_s*, dmath_matrix_s* m) { ++m->version; }

dmath_status_t copy_blocks(dmath_matrix_s* m, void* host, int64_t ld, bool to_device)
{
    if (!m || !host) return DMATH_ERR_INVALID_ARG;
    if (m->ctx->recording) return DMATH_ERR_UNSUPPORTED;
    if (ld < m->cols) return DMATH_ERR_INVALID_ARG;
    const size_t es = elem_size(m->dtype);
    hipStream_t st = m->ctx->stream;
    for (int32_t bi = 0; bi < m->rsplit.g; ++bi)
        for (int32_t bj = 0; bj < m->csplit.g; ++bj) {
            int64_t r = m->rsplit.len(bi), c = m->csplit.len(bj);
            char* h = static_cast<char*>(host) + (m->rsplit.lo(bi) * ld + m->csplit.lo(bj)) * es;
            void* d = m->block(bi, bj);
            hipError_t e = to_device
                               ? hipMemcpy2DAsync(d, c * es, h, ld * es, c * es, r, hipMemcpyHostToDevice, st)
                               : hipMemcpy2DAsync(h, ld * es, d, c * es, c * es, r, hipMemcpyDeviceToHost, st);
            if (e != hipSuccess) return DMATH_ERR_DEVICE;
        }
    if (to_device) wrote(m->ctx, m);
    return hipStreamSynchronize(st) == hipSuccess ? DMATH_OK : DMATH_ERR_DEVICE;
}

dmath_status_t check_conv_desc(const dmath_conv_desc_t* d, int64_t* oh, int64_t* ow)
{
    if (!d) return DMATH_ERR_INVALID_ARG;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0 ||
        d->pad_h < 0 || d->pad_w < 0 || d->stride_h <= 0 || d->stride_w <= 0)
        return DMATH_ERR_INVALID_ARG;
    int64_t hh = (int64_t)d->h + 2 * d->pad_h - d->r, ww = (int64_t)d->w + 2 * d->pad_w - d->s;
    if (hh < 0 || ww < 0) return DMATH_ERR_SHAPE;
    *oh = hh / d->stride_h + 1;
    *ow = ww / d->stride_w + 1;
    return DMATH_OK;
}

// Argument checks shared by the convolution calls and their tuner.
dmath_status_t check_conv(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d, dmath_matrix_s* X,
                          dmath_matrix_s* F, dmath_matrix_s* Y)
{
    if (!ctx || !X || !F || !Y) return DMATH_ERR_INVALID_ARG;
    int64_t oh, ow;
    dmath_status_t st = check_conv_desc(d, &oh, &ow);
    if (st != DMATH_OK) return st;
    if (!owns(ctx, X) || !owns(ctx, F) || !owns(ctx, Y)) return DMATH_ERR_INVALID_ARG;
    if (X == F || X == Y || F == Y) return DMATH_ERR_ALIAS;
    dmath_matrix_s* res = mode == CONV_FWD ? Y : mode == CONV_BWD_FILTER ? F : X;
    dmath_matrix_s* in1 = mode == CONV_FWD ? X : mode == CONV_BWD_FILTER ? X : Y;
    dmath_matrix_s* in2 = mode == CONV_FWD ? F : mode == CONV_BWD_FILTER ? Y : F;
    if (!dtype_combo_ok(in1->dtype, in2->dtype, res->dtype)) return DMATH_ERR_DTYPE;
    const int64_t chw = (int64_t)d->c * d->h * d->w, crs = (int64_t)d->c * d->r * d->s;
    const int64_t kow = (int64_t)d->k * oh * ow;
    if (X->rows != d->n || X->cols != chw || F->rows != d->k || F->cols != crs ||
        Y->rows != d->n || Y->cols != kow)
        return DMATH_ERR_SHAPE;
    if (X->csplit.g != 1 || F->csplit.g != 1 || Y->csplit.g != 1) return DMATH_ERR_LAYOUT;
    if (chw >= (1ll << 31) || kow >= (1ll << 31) || crs >= (1ll << 31) ||
        (int64_t)d->n * oh * ow >= (1ll << 31) || (int64_t)d->n * d->h * d->w >= (1ll << 31))
        return DMATH_ERR_UNSUPPORTED;
    return DMATH_OK;
}

// in1, in2: the two tensors that are read; res: the tensor that is written.
dmath_status_t conv_call(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d, double alpha,
                         dmath_matrix_s* X, dmath_matrix_s* F, dmath_matrix_s* Y, double beta)
{
    dmath_status_t st = check_conv(ctx, mode, d, X, F, Y);
    if (st != DMATH_OK) return st;
    dmath_matrix_s* res = mode == CONV_FWD ? Y : mode == CONV_BWD_FILTER ? F : X;
    ConvPlan* plan = nullptr;
    st = get_conv_plan(ctx, mode, d, X, F, Y, &plan);
    if (st != DMATH_OK) return st;
    // which re-layout copies are still current (same version of their matrix, same epoch)
    unsigned rewrite = 0;
    struct Use { Relayout* copy; dmath_matrix_s* src; unsigned bit; };
    const Use used[3] = {{plan->xp, mode == CONV_BWD_DATA ? Y : X, REWRITE_X},
                         {plan->fp, F, REWRITE_F},
                         {plan->yt, Y, REWRITE_Y}};
    const bool specialised = plan->kernel == 1 && alpha != 0.0;
    if (specialised)
        for (const Use& u : used) {
            if (!u.copy) continue;
            const bool current = ctx->reuse_relayouts && !u.src->exposed &&
                                 u.copy->version == u.src->version && u.copy->epoch == ctx->epoch;
            if (current) {
                ++ctx->relayouts_reused;
            } else {
                rewrite |= u.bit;
                ++ctx->relayouts_written;
            }
        }
    if (launch_conv(*plan, mode, alpha, beta, rewrite, ctx->stream) != hipSuccess) return DMATH_ERR_DEVICE;
    if (specialised)
        for (const Use& u : used)
            if (u.copy && (rewrite & u.bit)) {
                u.copy->version = u.src->version;
                u.copy->epoch = ctx->epoch;
            }
    wrote(ctx, res);
    if (ctx->recording) ctx->recording_uses.insert({X->id, F->id, Y->id});
    return DMATH_OK;
}

}  // namespace

namespace {

// Time per launch in microseconds (negative: error): one launch alone to learn the scale, then
// `warm_us` of untimed launches so that the clocks have settled (the first sample after a pause
// read 15 % slow with 3 ms), then the average of `trials`.
template <class Launch>
double sample_us(dmath_ctx_s* ctx, hipEvent_t e0, hipEvent_t e1, int trials, double warm_us, Launch&& launch)
{
    auto timed = [&](int n) -> double {
        if (hipEventRecord(e0, ctx->stream) != hipSuccess) return -1;
        for (int i = 0; i < n; ++i)
            if (launch() != hipSuccess) return -1;
        if (hipEventRecord(e1, ctx->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1;
        float ms = 0;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1;
        return (double)ms * 1e3 / n;
    };
    if (launch() != hipSuccess) return -1;
    const double first = timed(1);
    if (first < 0) return -1;
    const int warm = (int)std::min(400.0, std::max(1.0, warm_us / std::max(first, 1.0)));
    if (timed(warm) < 0) return -1;
    return timed(trials);
}

struct Events {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok() { return hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~Events()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace

namespace {

// Nothing may leave the C boundary as an exception: the containers of the host scheduler can
// throw std::bad_alloc, which the caller sees as DMATH_ERR_OOM; anything else is reported as an
// invalid argument.
template <class F> dmath_status_t guarded(F&& body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return DMATH_ERR_OOM;
    } catch (const std::length_error&) {  // a container asked for more than it can ever hold
        return DMATH_ERR_OOM;
    } catch (...) {
        return DMATH_ERR_INVALID_ARG;
    }
}

}  // namespace

extern "C" {

dmath_status_t dmath_init(dmath_ctx_t* ctx, void* slab, size_t slab_bytes, void* hip_stream)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !slab || slab_bytes < Pool::kAlign * 2) return DMATH_ERR_INVALID_ARG;
        dmath_ctx_s* c = new (std::nothrow) dmath_ctx_s(slab, slab_bytes, static_cast<hipStream_t>(hip_stream));
        if (!c) return DMATH_ERR_OOM;
        *ctx = c;
        return DMATH_OK;
    });
}

dmath_status_t dmath_finalize(dmath_ctx_t ctx)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) {
            hipGraph_t g = nullptr;
            (void)hipStreamEndCapture(ctx->stream, &g);
            if (g) (void)hipGraphDestroy(g);
        }
        drop_all_plans(ctx);  // recorded sequences included
        for (dmath_matrix_s* m : ctx->matrices) delete m;
        delete ctx;
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_create(dmath_ctx_t ctx, int64_t rows, int64_t cols, int32_t grid_rows,
                                   int32_t grid_cols, dmath_dtype_t dtype, dmath_matrix_t* out)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !out || rows <= 0 || cols <= 0 || grid_rows <= 0 || grid_cols <= 0 ||
            !valid_dtype(dtype))
            return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        if (rows >= (1ll << 31) || cols >= (1ll << 31)) return DMATH_ERR_UNSUPPORTED;
        Split rs(rows, grid_rows), cs(cols, grid_cols);
        if (!rs.valid() || !cs.valid()) return DMATH_ERR_LAYOUT;
        // the handle and its blocks are given back if anything below fails or throws
        struct Rollback {
            dmath_ctx_s* ctx;
            dmath_matrix_s* m;
            ~Rollback()
            {
                if (!m) return;
                for (void* q : m->blocks) ctx->pool.free(q);
                delete m;
            }
        } guard{ctx, new (std::nothrow) dmath_matrix_s};
        dmath_matrix_s* m = guard.m;
        if (!m) return DMATH_ERR_OOM;
        m->ctx = ctx;
        m->rows = rows;
        m->cols = cols;
        m->rsplit = rs;
        m->csplit = cs;
        m->dtype = dtype;
        const size_t es = elem_size(dtype);
        m->blocks.reserve((size_t)grid_rows * grid_cols);
        for (int32_t bi = 0; bi < grid_rows; ++bi)
            for (int32_t bj = 0; bj < grid_cols; ++bj) {
                void* p = ctx->pool.alloc((size_t)rs.len(bi) * cs.len(bj) * es);
                if (!p) return DMATH_ERR_OOM;
                m->blocks.push_back(p);
            }
        m->id = ctx->next_id;
        ctx->matrices.insert(m);
        ++ctx->next_id;
        guard.m = nullptr;
        *out = m;
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_destroy(dmath_matrix_t m)
{
    return guarded([&]() -> dmath_status_t {
        if (!m || !m->ctx || !m->ctx->matrices.count(m)) return DMATH_ERR_INVALID_ARG;
        dmath_ctx_s* ctx = m->ctx;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        drop_plans_using(ctx, m->id);
        for (void* p : m->blocks) ctx->pool.free(p);
        ctx->matrices.erase(m);
        delete m;
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_set(dmath_matrix_t m, const void* host, int64_t ld_elems)
{
    return guarded([&]() -> dmath_status_t {
        return copy_blocks(m, const_cast<void*>(host), ld_elems, true);
    });
}

dmath_status_t dmath_matrix_get(dmath_matrix_t m, void* host, int64_t ld_elems)
{
    return guarded([&]() -> dmath_status_t {
        return copy_blocks(m, host, ld_elems, false);
    });
}

dmath_status_t dmath_matrix_info(dmath_matrix_t m, int64_t* rows, int64_t* cols, int32_t* grid_rows,
                                 int32_t* grid_cols, dmath_dtype_t* dtype)
{
    return guarded([&]() -> dmath_status_t {
        if (!m) return DMATH_ERR_INVALID_ARG;
        if (rows) *rows = m->rows;
        if (cols) *cols = m->cols;
        if (grid_rows) *grid_rows = m->rsplit.g;
        if (grid_cols) *grid_cols = m->csplit.g;
        if (dtype) *dtype = m->dtype;
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_block(dmath_matrix_t m, int32_t bi, int32_t bj, void** dev_ptr,
                                  int64_t* rows, int64_t* cols, int64_t* ld)
{
    return guarded([&]() -> dmath_status_t {
        if (!m || bi < 0 || bj < 0 || bi >= m->rsplit.g || bj >= m->csplit.g)
            return DMATH_ERR_INVALID_ARG;
        if (dev_ptr) {
            *dev_ptr = m->block(bi, bj);
            m->exposed = true;  // the caller may now write behind the library's back
            wrote(m->ctx, m);
        }
        if (rows) *rows = m->rsplit.len(bi);
        if (cols) *cols = m->csplit.len(bj);
        if (ld) *ld = m->csplit.len(bj);
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_reblock(dmath_ctx_t ctx, dmath_matrix_t src, dmath_matrix_t dst)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !owns(ctx, src) || !owns(ctx, dst)) return DMATH_ERR_INVALID_ARG;
        if (src == dst) return DMATH_ERR_ALIAS;
        if (src->rows != dst->rows || src->cols != dst->cols) return DMATH_ERR_SHAPE;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        // cut rows and columns at every block boundary of either matrix
        auto cuts = [](const Split& a, const Split& b) {
            std::vector<int64_t> c{0, a.n};
            for (int32_t p = 1; p < a.g; ++p) c.push_back(a.lo(p));
            for (int32_t p = 1; p < b.g; ++p) c.push_back(b.lo(p));
            std::sort(c.begin(), c.end());
            c.erase(std::unique(c.begin(), c.end()), c.end());
            return c;
        };
        const std::vector<int64_t> rc = cuts(src->rsplit, dst->rsplit), cc = cuts(src->csplit, dst->csplit);
        const int64_t ses = elem_size(src->dtype), des = elem_size(dst->dtype);
        std::vector<CopyCell> cells;
        int max_rows = 0;
        const int64_t vec = reblock_vector_width(src->dtype, dst->dtype);
        bool vectors = true;  // every cell: origins, leading dimensions and width multiples of the vector
        for (size_t i = 0; i + 1 < rc.size(); ++i)
            for (size_t j = 0; j + 1 < cc.size(); ++j) {
                const int64_t r = rc[i], c = cc[j];
                const int32_t sbi = src->rsplit.part(r), sbj = src->csplit.part(c);
                const int32_t dbi = dst->rsplit.part(r), dbj = dst->csplit.part(c);
                CopyCell cell;
                cell.src_ld = src->csplit.len(sbj);
                cell.dst_ld = dst->csplit.len(dbj);
                cell.src = static_cast<const char*>(src->block(sbi, sbj)) +
                           ((r - src->rsplit.lo(sbi)) * cell.src_ld + (c - src->csplit.lo(sbj))) * ses;
                cell.dst = static_cast<char*>(dst->block(dbi, dbj)) +
                           ((r - dst->rsplit.lo(dbi)) * cell.dst_ld + (c - dst->csplit.lo(dbj))) * des;
                cell.rows = (int32_t)(rc[i + 1] - r);
                cell.cols = (int32_t)(cc[j + 1] - c);
                max_rows = std::max(max_rows, cell.rows);
                vectors = vectors && cell.cols % vec == 0 && cell.src_ld % vec == 0 && cell.dst_ld % vec == 0 &&
                          reinterpret_cast<uintptr_t>(cell.src) % (vec * ses) == 0 &&
                          reinterpret_cast<uintptr_t>(cell.dst) % (vec * des) == 0;
                cells.push_back(cell);
            }
        const size_t bytes = cells.size() * sizeof(CopyCell);
        void* dev = ctx->pool.alloc(bytes);
        if (!dev) return DMATH_ERR_OOM;
        // the table is pageable host memory: copy, wait, then it may go; the kernel itself is asynchronous
        hipError_t e = hipMemcpyAsync(dev, cells.data(), bytes, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e == hipSuccess)
            e = launch_reblock(src->dtype, dst->dtype, static_cast<const CopyCell*>(dev), (int)cells.size(),
                               max_rows, vectors, ctx->stream);
        ctx->pool.free(dev);  // reuse of the table's memory is ordered after the kernel by the stream
        wrote(ctx, dst);
        return e == hipSuccess ? DMATH_OK : DMATH_ERR_DEVICE;
    });
}

dmath_status_t dmath_gemm(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB, double alpha,
                          dmath_matrix_t A, dmath_matrix_t B, double beta, dmath_matrix_t C)
{
    return guarded([&]() -> dmath_status_t {
        dmath_status_t st = check_gemm(ctx, transA, transB, A, B, C);
        if (st != DMATH_OK) return st;
        GemmPlan* plan = nullptr;
        st = get_gemm_plan(ctx, transA, transB, A, B, C, true, &plan, nullptr);
        if (st != DMATH_OK) return st;
        if (launch_gemm(*plan, alpha, beta, ctx->stream) != hipSuccess) return DMATH_ERR_DEVICE;
        wrote(ctx, C);
        if (ctx->recording) ctx->recording_uses.insert({A->id, B->id, C->id});
        return DMATH_OK;
    });
}

dmath_status_t dmath_gemm_plan_info(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB,
                                    dmath_matrix_t A, dmath_matrix_t B, dmath_matrix_t C,
                                    dmath_plan_info_t* info)
{
    return guarded([&]() -> dmath_status_t {
        if (!info) return DMATH_ERR_INVALID_ARG;
        dmath_status_t st = check_gemm(ctx, transA, transB, A, B, C);
        if (st != DMATH_OK) return st;
        GemmPlan* plan = nullptr;
        bool cached = false;
        st = get_gemm_plan(ctx, transA, transB, A, B, C, false, &plan, &cached);
        if (st != DMATH_OK) return st;
        *info = plan->info;
        info->cached = cached ? 1 : 0;
        return DMATH_OK;
    });
}

dmath_status_t dmath_conv_fwd(dmath_ctx_t ctx, const dmath_conv_desc_t* desc, double alpha,
                              dmath_matrix_t X, dmath_matrix_t F, double beta, dmath_matrix_t Y)
{
    return guarded([&]() -> dmath_status_t {
        return conv_call(ctx, CONV_FWD, desc, alpha, X, F, Y, beta);
    });
}

dmath_status_t dmath_conv_bwd_filter(dmath_ctx_t ctx, const dmath_conv_desc_t* desc, double alpha,
                                     dmath_matrix_t X, dmath_matrix_t dY, double beta,
                                     dmath_matrix_t dF)
{
    return guarded([&]() -> dmath_status_t {
        return conv_call(ctx, CONV_BWD_FILTER, desc, alpha, X, dF, dY, beta);
    });
}

dmath_status_t dmath_conv_bwd_data(dmath_ctx_t ctx, const dmath_conv_desc_t* desc, double alpha,
                                   dmath_matrix_t dY, dmath_matrix_t F, double beta,
                                   dmath_matrix_t dX)
{
    return guarded([&]() -> dmath_status_t {
        return conv_call(ctx, CONV_BWD_DATA, desc, alpha, dX, F, dY, beta);
    });
}

dmath_status_t dmath_pipeline_begin(dmath_ctx_t ctx)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || ctx->recording) return DMATH_ERR_INVALID_ARG;
        if (!ctx->stream) return DMATH_ERR_UNSUPPORTED;  // the default stream cannot be captured
        if (hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal) != hipSuccess)
            return DMATH_ERR_DEVICE;
        ctx->recording = true;
        ctx->recording_uses.clear();
        ++ctx->epoch;  // a copy made before the recording is not rewritten by its replays
        return DMATH_OK;
    });
}

dmath_status_t dmath_pipeline_end(dmath_ctx_t ctx, int32_t* pipeline_id)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !pipeline_id || !ctx->recording) return DMATH_ERR_INVALID_ARG;
        ctx->recording = false;
        ++ctx->epoch;
        hipGraph_t graph = nullptr;
        if (hipStreamEndCapture(ctx->stream, &graph) != hipSuccess || !graph) return DMATH_ERR_DEVICE;
        hipGraphExec_t exec = nullptr;
        hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess || !exec) return DMATH_ERR_DEVICE;
        *pipeline_id = ctx->next_pipeline++;
        Pipeline& p = ctx->pipelines[*pipeline_id];
        p.exec = exec;
        p.uses.swap(ctx->recording_uses);
        return DMATH_OK;
    });
}

dmath_status_t dmath_pipeline_replay(dmath_ctx_t ctx, int32_t pipeline_id)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || ctx->recording) return DMATH_ERR_INVALID_ARG;
        auto it = ctx->pipelines.find(pipeline_id);
        if (it == ctx->pipelines.end()) return DMATH_ERR_INVALID_ARG;
        // the replay rewrites matrices and re-layout copies that the host-side versions do not follow
        ++ctx->epoch;
        for (dmath_matrix_s* m : ctx->matrices)
            if (it->second.uses.count(m->id)) wrote(ctx, m);
        return hipGraphLaunch(it->second.exec, ctx->stream) == hipSuccess ? DMATH_OK : DMATH_ERR_DEVICE;
    });
}

dmath_status_t dmath_pipeline_destroy(dmath_ctx_t ctx, int32_t pipeline_id)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        auto it = ctx->pipelines.find(pipeline_id);
        if (it == ctx->pipelines.end()) return DMATH_ERR_INVALID_ARG;
        (void)hipGraphExecDestroy(it->second.exec);
        ctx->pipelines.erase(it);
        return DMATH_OK;
    });
}

dmath_status_t dmath_gemm_tune(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB, dmath_matrix_t A,
                               dmath_matrix_t B, dmath_matrix_t C, size_t workspace_limit, int32_t trials,
                               dmath_tune_result_t* result)
{
    return guarded([&]() -> dmath_status_t {
        if (!result || trials <= 0) return DMATH_ERR_INVALID_ARG;
        dmath_status_t st = check_gemm(ctx, transA, transB, A, B, C);
        if (st != DMATH_OK) return st;
        if (ctx->recording || ctx->policy != 0) return DMATH_ERR_UNSUPPORTED;
        // the cost model's own choice and the list of candidates
        const std::vector<int64_t> sig = gemm_signature(transA, transB, A, B, C);
        ctx->tuned_gemm.erase(sig);
        std::unique_ptr<GemmPlan> described;
        std::vector<GemmChoice> cands;
        st = make_gemm_plan(ctx, transA, transB, A, B, C, false, nullptr, &described, &cands);
        if (st != DMATH_OK) return st;
        const dmath_plan_info_t model = described->info;
        const int32_t model_full_tiles = described->full_tiles;
        Events ev;
        if (!ev.ok()) return DMATH_ERR_DEVICE;
        dmath_tune_result_t found{};  // copied out on success only
        double best = -1;
        GemmChoice best_choice;
        for (const GemmChoice& c : cands) {
            // what this candidate takes from the pool (partial sums, scratch panels of k-tails)
            std::unique_ptr<GemmPlan> sized;
            st = make_gemm_plan(ctx, transA, transB, A, B, C, false, &c, &sized, nullptr);
            if (st != DMATH_OK) return st;
            const size_t need = sized->info.workspace_bytes;
            if (need > workspace_limit) {
                ++found.skipped;
                continue;
            }
            std::unique_ptr<GemmPlan> plan;
            st = make_gemm_plan(ctx, transA, transB, A, B, C, true, &c, &plan, nullptr);
            if (st == DMATH_ERR_OOM) {  // the pool cannot hold it now: as good as over the limit
                ++found.skipped;
                continue;
            }
            if (st != DMATH_OK) return st;
            const double us = sample_us(ctx, ev.e0, ev.e1, trials, found.candidates ? 3e3 : 2e4,
                                        [&] { return launch_gemm(*plan, 1.0, 0.0, ctx->stream); });
            const dmath_plan_info_t info = plan->info;
            const int32_t full_tiles = plan->full_tiles;
            free_gemm_plan(ctx, *plan);  // stream order: the samples have completed (event wait)
            if (us < 0) return DMATH_ERR_DEVICE;
            ++found.candidates;
            const bool is_model = info.kernel == model.kernel && info.tile_m == model.tile_m &&
                                  info.tile_n == model.tile_n && info.split_k == model.split_k &&
                                  full_tiles == model_full_tiles;
            if (is_model) found.default_us = us;
            // a sample has to beat the cost model's choice by more than 2 % (noise) to replace it
            const double handicap = is_model ? 0.98 : 1.0;
            if (best < 0 || us * handicap < best) {
                best = us * handicap;
                best_choice = c;
                found.kernel = info.kernel;
                found.tile_m = info.tile_m;
                found.tile_n = info.tile_n;
                found.split_k = info.split_k;
                found.workspace_bytes = info.workspace_bytes;
                found.chosen_us = us;
            }
        }
        wrote(ctx, C);
        if (best < 0) return DMATH_ERR_OOM;  // nothing fitted
        ctx->tuned_gemm[sig] = best_choice;
        *result = found;
        // plans made before for matrices laid out like these were built on the cost model's choice
        for (auto it = ctx->gemm_plans.begin(); it != ctx->gemm_plans.end();) {
            const auto& u = it->second->uses;
            dmath_matrix_s *a = nullptr, *b = nullptr, *c = nullptr;
            for (dmath_matrix_s* m : ctx->matrices) {
                if (m->id == u[0]) a = m;
                if (m->id == u[1]) b = m;
                if (m->id == u[2]) c = m;
            }
            const bool same = a && b && c &&
                              gemm_signature(std::get<3>(it->first), std::get<4>(it->first), a, b, c) == sig;
            if (same) {
                for (uint64_t id : u) drop_pipelines_using(ctx, id);
                free_gemm_plan(ctx, *it->second);
                it = ctx->gemm_plans.erase(it);
            } else
                ++it;
        }
        return DMATH_OK;
    });
}

dmath_status_t dmath_conv_tune(dmath_ctx_t ctx, int32_t mode, const dmath_conv_desc_t* desc, dmath_matrix_t X,
                               dmath_matrix_t F, dmath_matrix_t Y, size_t workspace_limit, int32_t trials,
                               dmath_tune_result_t* result)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !result || trials <= 0 || mode < CONV_FWD || mode > CONV_BWD_DATA || !X || !F || !Y)
            return DMATH_ERR_INVALID_ARG;
        dmath_status_t st = check_conv(ctx, mode, desc, X, F, Y);
        if (st != DMATH_OK) return st;
        if (ctx->recording || ctx->policy != 0) return DMATH_ERR_UNSUPPORTED;
        const std::vector<int64_t> sig = conv_signature(mode, desc, X, F, Y);
        ctx->tuned_conv.erase(sig);
        // plans of this signature go first: their re-layout copies would otherwise be counted as held
        auto drop_same = [&] {
            for (auto it = ctx->conv_plans.begin(); it != ctx->conv_plans.end();) {
                const auto& u = it->second->uses;
                dmath_matrix_s *x = nullptr, *f = nullptr, *y = nullptr;
                for (dmath_matrix_s* m : ctx->matrices) {
                    if (m->id == u[0]) x = m;
                    if (m->id == u[1]) f = m;
                    if (m->id == u[2]) y = m;
                }
                const std::vector<int32_t>& gv = std::get<4>(it->first);
                dmath_conv_desc_t d{gv[0], gv[1], gv[2], gv[3], gv[4], gv[5], gv[6], gv[7], gv[8], gv[9], gv[10]};
                if (x && f && y && conv_signature(std::get<3>(it->first), &d, x, f, y) == sig) {
                    for (uint64_t id : u) drop_pipelines_using(ctx, id);
                    free_conv_plan(ctx, *it->second);
                    it = ctx->conv_plans.erase(it);
                } else
                    ++it;
            }
        };
        drop_same();
        dmath_matrix_s* res = mode == CONV_FWD ? Y : mode == CONV_BWD_FILTER ? F : X;
        const dmath_dtype_t in_dtype = mode == CONV_FWD ? X->dtype : Y->dtype;
        std::unique_ptr<ConvPlan> probe;
        ConvChoice none;
        st = make_conv_plan(ctx, mode, desc, X, F, Y, &none, &probe);  // generic, unsplit: only for the geometry
        if (st != DMATH_OK) return st;
        const ConvGeom g = probe->t.g;
        free_conv_plan(ctx, *probe);
        const ConvChoice model = choose_conv(mode, g, in_dtype, ctx->policy);
        Events ev;
        if (!ev.ok()) return DMATH_ERR_DEVICE;
        dmath_tune_result_t found{};  // copied out on success only
        double best = -1;
        ConvChoice best_choice;
        for (const ConvChoice& c : conv_candidates(mode, g, in_dtype, ctx->policy)) {
            const size_t need = conv_choice_bytes(mode, g, c, in_dtype);
            if (need > workspace_limit) {
                ++found.skipped;
                continue;
            }
            std::unique_ptr<ConvPlan> plan;
            st = make_conv_plan(ctx, mode, desc, X, F, Y, &c, &plan);
            if (st == DMATH_ERR_OOM) {
                ++found.skipped;
                continue;
            }
            if (st != DMATH_OK) return st;
            // a convolution run as a block GEMM takes what its GEMM plan takes (partial sums, k-tails)
            const size_t taken = plan->gemm ? (size_t)plan->gemm->info.workspace_bytes : need;
            if (taken > workspace_limit) {
                free_conv_plan(ctx, *plan);
                ++found.skipped;
                continue;
            }
            const double us = sample_us(ctx, ev.e0, ev.e1, trials, found.candidates ? 3e3 : 2e4, [&] {
                return launch_conv(*plan, mode, 1.0, 0.0, REWRITE_X | REWRITE_F | REWRITE_Y, ctx->stream);
            });
            for (Relayout* r : {plan->xp, plan->fp, plan->yt})
                if (r) r->version = 0;  // written outside the version bookkeeping: never trusted
            const int32_t gemm_tile_m = plan->gemm ? plan->gemm->info.tile_m : 0;
            const int32_t gemm_tile_n = plan->gemm ? plan->gemm->info.tile_n : 0;
            const int32_t gemm_split = plan->gemm ? plan->gemm->info.split_k : 1;
            free_conv_plan(ctx, *plan);
            if (us < 0) return DMATH_ERR_DEVICE;
            ++found.candidates;
            const bool is_model = c == model;
            if (is_model) found.default_us = us;
            const double handicap = is_model ? 0.98 : 1.0;
            if (best < 0 || us * handicap < best) {
                best = us * handicap;
                best_choice = c;
                found.kernel = c.kernel;
                found.tile_m = c.kernel == 1 ? c.tile_m : c.kernel == 2 ? gemm_tile_m : 64;
                found.tile_n = c.kernel == 1 ? c.tile_n : c.kernel == 2 ? gemm_tile_n : 64;
                found.split_k = c.kernel == 2 ? gemm_split : c.split_k;
                found.workspace_bytes = taken;
                found.chosen_us = us;
            }
        }
        wrote(ctx, res);
        drop_unused_relayouts(ctx);  // what only a rejected candidate needed goes back to the pool
        if (best < 0) return DMATH_ERR_OOM;
        ctx->tuned_conv[sig] = best_choice;
        *result = found;
        return DMATH_OK;
    });
}

dmath_status_t dmath_tune_reset(dmath_ctx_t ctx)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        ctx->tuned_gemm.clear();
        ctx->tuned_conv.clear();
        drop_all_plans(ctx);
        return DMATH_OK;
    });
}

dmath_status_t dmath_set_relayout_reuse(dmath_ctx_t ctx, int32_t enable)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || enable < 0 || enable > 1) return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        ctx->reuse_relayouts = enable != 0;
        return DMATH_OK;
    });
}

dmath_status_t dmath_relayout_stats(dmath_ctx_t ctx, uint64_t* reused, uint64_t* written, size_t* bytes_held)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        if (reused) *reused = ctx->relayouts_reused;
        if (written) *written = ctx->relayouts_written;
        if (bytes_held) {
            size_t b = 0;
            for (const auto& kv : ctx->relayouts) b += kv.second.bytes;
            *bytes_held = b;
        }
        return DMATH_OK;
    });
}

dmath_status_t dmath_matrix_touch(dmath_matrix_t m)
{
    return guarded([&]() -> dmath_status_t {
        if (!m || !m->ctx || !m->ctx->matrices.count(m)) return DMATH_ERR_INVALID_ARG;
        wrote(m->ctx, m);
        return DMATH_OK;
    });
}

dmath_status_t dmath_set_kernel_policy(dmath_ctx_t ctx, int32_t policy)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || policy < 0 || policy > 1) return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        ctx->policy = policy;
        drop_all_plans(ctx);
        return DMATH_OK;
    });
}

static dmath_status_t mfma_peak_probe(dmath_ctx_t ctx, dmath_dtype_t dtype, int32_t iters, double* flops, bool wide_f16)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !flops || !valid_dtype(dtype) || iters <= 0) return DMATH_ERR_INVALID_ARG;
        void* scratch = ctx->pool.alloc(256);
        if (!scratch) return DMATH_ERR_OOM;
        double f = 0;
        hipError_t e = launch_mfma_peak(dtype, iters, scratch, ctx->stream, &f, wide_f16);
        ctx->pool.free(scratch);  // the kernel practically never writes; reuse is stream-ordered anyway
        if (e != hipSuccess) return DMATH_ERR_DEVICE;
        *flops = f;
        return DMATH_OK;
    });
}

dmath_status_t dmath_mfma_peak_probe(dmath_ctx_t ctx, dmath_dtype_t dtype, int32_t iters, double* flops)
{
    return mfma_peak_probe(ctx, dtype, iters, flops, false);
}

dmath_status_t dmath_mfma_peak_probe_f16_32x32x16(dmath_ctx_t ctx, int32_t iters, double* flops)
{
    return mfma_peak_probe(ctx, DMATH_F16, iters, flops, true);
}

dmath_status_t dmath_cycle_probe_read(dmath_ctx_t ctx, uint64_t* out6)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx || !out6) return DMATH_ERR_INVALID_ARG;
        if (ctx->recording) return DMATH_ERR_UNSUPPORTED;
        if (hipStreamSynchronize(ctx->stream) != hipSuccess) return DMATH_ERR_DEVICE;
        return read_cycle_probe(out6) ? DMATH_OK : DMATH_ERR_UNSUPPORTED;
    });
}

dmath_status_t dmath_synchronize(dmath_ctx_t ctx)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        return hipStreamSynchronize(ctx->stream) == hipSuccess ? DMATH_OK : DMATH_ERR_DEVICE;
    });
}

dmath_status_t dmath_pool_stats(dmath_ctx_t ctx, size_t* in_use, size_t* high_water,
                                size_t* capacity)
{
    return guarded([&]() -> dmath_status_t {
        if (!ctx) return DMATH_ERR_INVALID_ARG;
        if (in_use) *in_use = ctx->pool.in_use();
        if (high_water) *high_water = ctx->pool.high_water();
        if (capacity) *capacity = ctx->pool.capacity();
        return DMATH_OK;
    });
}

const char* dmath_status_string(dmath_status_t s)
{
    switch (s) {
    case DMATH_OK: return "DMATH_OK";
    case DMATH_ERR_INVALID_ARG: return "DMATH_ERR_INVALID_ARG";
    case DMATH_ERR_SHAPE: return "DMATH_ERR_SHAPE";
    case DMATH_ERR_LAYOUT: return "DMATH_ERR_LAYOUT";
    case DMATH_ERR_DTYPE: return "DMATH_ERR_DTYPE";
    case DMATH_ERR_ALIAS: return "DMATH_ERR_ALIAS";
    case DMATH_ERR_OOM: return "DMATH_ERR_OOM";
    case DMATH_ERR_UNSUPPORTED: return "DMATH_ERR_UNSUPPORTED";
    case DMATH_ERR_DEVICE: return "DMATH_ERR_DEVICE";
    case DMATH_ERR_SCRATCH_LIMIT: return "DMATH_ERR_SCRATCH_LIMIT";
    }
    return "DMATH_ERR_UNKNOWN";
}

}  // extern "C"
