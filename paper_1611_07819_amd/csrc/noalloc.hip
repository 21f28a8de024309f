// dmath_gemm_noalloc: dmath_gemm for callers that must not allocate (code under HIP graph
// capture, tight serving loops, harnesses that forbid allocation).  Everything the GEMM kernels
// need beyond their operands -- the plan's descriptor tables, the partial sums of a split k-loop,
// the zero-padded panels of k-tails -- lies in one file-scope array of device memory instead of
// the context's pool.  The call takes nothing from the pool and makes no driver allocation.
//
// The array exists once per GPU (each device that loads the library holds its own copy until
// the process ends) and is shared by every call on that GPU: it keeps the last call's plan, a
// call for other operands rewrites it (stream-ordered on the calling context's stream), and calls
// that overlap on one GPU -- two contexts on different streams -- race.
#include <hip/hip_runtime.h>

#include <atomic>

#include "context.hpp"

using namespace dm;

namespace {

constexpr size_t kScratchBytes = (size_t)DMATH_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Host-side view of one device's copy of the array.  In host code the array's name is only a
// stand-in for the symbol; the address kernels and copies may use comes from
// hipGetSymbolAddress, once per device with that device current.
struct DeviceScratch {
    void* ptr = nullptr;
    uint64_t owner = 0;  // token of the plan the array currently holds (0: none)
};
DeviceScratch g_scratch[kMaxDevices];
std::atomic<uint64_t> g_next_token{1};

hipError_t scratch_of_current_device(DeviceScratch** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    DeviceScratch& d = g_scratch[dev];
    if (!d.ptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        d.ptr = p;
    }
    *out = &d;
    return hipSuccess;
}

bool valid_op(int o) { return o == DMATH_OP_N || o == DMATH_OP_T; }

dmath_status_t gemm_noalloc(dmath_ctx_s* ctx, int transA, int transB, double alpha, dmath_matrix_s* A,
                            dmath_matrix_s* B, double beta, dmath_matrix_s* C)
{
    // the argument checks of dmath_gemm
    if (!ctx || !A || !B || !C || !valid_op(transA) || !valid_op(transB)) return DMATH_ERR_INVALID_ARG;
    for (dmath_matrix_s* m : {A, B, C})
        if (!ctx->matrices.count(m)) return DMATH_ERR_INVALID_ARG;
    if (C == A || C == B) return DMATH_ERR_ALIAS;
    if (A->dtype != B->dtype || !(C->dtype == A->dtype || (A->dtype == DMATH_F16 && C->dtype == DMATH_F32)))
        return DMATH_ERR_DTYPE;
    const int64_t am = transA ? A->cols : A->rows, ak = transA ? A->rows : A->cols;
    const int64_t bk = transB ? B->cols : B->rows, bn = transB ? B->rows : B->cols;
    if (ak != bk || am != C->rows || bn != C->cols) return DMATH_ERR_SHAPE;

    // A recorded pipeline would replay against whatever plan the shared array holds by then.
    if (ctx->recording) return DMATH_ERR_UNSUPPORTED;

    const GemmKey key{A->id, B->id, C->id, transA, transB};
    const bool have = ctx->noalloc_plan && ctx->noalloc_key == key;
    DeviceScratch* dev = nullptr;
    if (scratch_of_current_device(&dev) != hipSuccess) return DMATH_ERR_DEVICE;
    if (!have || dev->owner != ctx->noalloc_token) {  // other operands, or another context rewrote the array
        ctx->noalloc_plan.reset();
        dev->owner = 0;
        const GemmChoice* forced = nullptr;
        auto tuned = ctx->tuned_gemm.find(gemm_signature(transA, transB, A, B, C));
        if (tuned != ctx->tuned_gemm.end() && ctx->policy == 0) forced = &tuned->second;
        // as in dmath_gemm, memory decides: if the partial sums of a split k-loop do not fit the
        // array the same kernel runs unsplit, if the k-tail panels do not fit the generic kernel
        // runs; if not even the tables fit, the sizes are beyond this entry point
        std::unique_ptr<GemmPlan> plan;
        dmath_status_t st = DMATH_ERR_OOM;
        for (int attempt = 0; attempt < 3 && st == DMATH_ERR_OOM; ++attempt) {
            Arena arena{static_cast<char*>(dev->ptr), kScratchBytes, 0};
            const GemmChoice frugal;  // generic kernel, unsplit
            st = make_gemm_plan(ctx, transA, transB, A, B, C, true, attempt == 2 ? &frugal : forced, &plan, nullptr,
                                attempt >= 1, &arena);
        }
        if (st == DMATH_ERR_OOM) return DMATH_ERR_SCRATCH_LIMIT;
        if (st != DMATH_OK) return st;
        ctx->noalloc_plan = std::move(plan);
        ctx->noalloc_key = key;
        ctx->noalloc_token = g_next_token.fetch_add(1);
        dev->owner = ctx->noalloc_token;
    }
    if (launch_gemm(*ctx->noalloc_plan, alpha, beta, ctx->stream) != hipSuccess) return DMATH_ERR_DEVICE;
    ++C->version;
    return DMATH_OK;
}

}  // namespace

extern "C" dmath_status_t dmath_gemm_noalloc(dmath_ctx_t ctx, dmath_op_t transA, dmath_op_t transB, double alpha,
                                             dmath_matrix_t A, dmath_matrix_t B, double beta, dmath_matrix_t C)
{
    try {
        return gemm_noalloc(ctx, transA, transB, alpha, A, B, beta, C);
    } catch (const std::bad_alloc&) {  // host bookkeeping only; nothing crosses the C boundary
        return DMATH_ERR_OOM;
    } catch (...) {
        return DMATH_ERR_INVALID_ARG;
    }
}
