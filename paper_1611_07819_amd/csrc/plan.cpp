// The tile scheduler: turns three independent block grids into the tables the kernels walk.
//
// Paper section 2.1: every worker knows the layout of every matrix and works out by itself
// which blocks it needs; section 3.2: results must not depend on the layout.  Here the one
// worker owns every block.  Each dimension (m, n, k) is cut at every block boundary of every
// operand that spans it, so that a (segment x segment) panel lies inside exactly one block of
// each operand; C tiles are laid inside (m-segment x n-segment) cells and the k-loop walks
// the k-segments.  Section 3.3: the result is cached per (A, B, C, ops).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>

#include "context.hpp"

namespace dm {

namespace {

struct Seg {
    int64_t start, len;
};

// Union of the cut points of several partitions of [0, n).
std::vector<Seg> refine(int64_t n, std::initializer_list<const Split*> parts,
                        const std::vector<int64_t>& extra_cuts = {})
{
    std::vector<int64_t> cuts{0, n};
    for (const Split* s : parts)
        for (int32_t p = 1; p < s->g; ++p) cuts.push_back(s->lo(p));
    for (int64_t c : extra_cuts)
        if (c > 0 && c < n) cuts.push_back(c);
    std::sort(cuts.begin(), cuts.end());
    cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
    std::vector<Seg> segs;
    for (size_t i = 0; i + 1 < cuts.size(); ++i) segs.push_back({cuts[i], cuts[i + 1] - cuts[i]});
    return segs;
}

// Address of logical element (i, j) of a matrix and the leading dimension of its block.
Panel locate(const dmath_matrix_s* m, int64_t i, int64_t j)
{
    int32_t bi = m->rsplit.part(i), bj = m->csplit.part(j);
    int64_t ld = m->csplit.len(bj);
    int64_t off = (i - m->rsplit.lo(bi)) * ld + (j - m->csplit.lo(bj));
    const char* base = static_cast<const char*>(m->block(bi, bj));
    return Panel{base + off * (int64_t)elem_size(m->dtype), ld};
}

template <class T>
size_t append(std::vector<char>& buf, const std::vector<T>& v)
{
    size_t off = (buf.size() + 15) / 16 * 16;
    buf.resize(off + v.size() * sizeof(T));
    if (!v.empty()) std::memcpy(buf.data() + off, v.data(), v.size() * sizeof(T));
    return off;
}

// Orders tiles so that consecutive workgroups of one XCD (workgroup w runs on XCD w % 8) work
// on neighbouring tiles: the logical sequence is cut into 8 contiguous runs, one per XCD, and
// the table is written so that hardware workgroup w gets element (w / 8) of run (w % 8).
std::vector<Tile> xcd_interleave(const std::vector<Tile>& logical)
{
    const size_t n = logical.size(), X = 8;
    if (n < 2 * X) return logical;
    // run x has base (+1 if x < rem) tiles, so that position w = j*8 + x exists for every
    // element j of run x and the table has no holes.
    const size_t base = n / X, rem = n % X;
    std::vector<Tile> out(n);
    size_t start = 0;
    for (size_t x = 0; x < X; ++x) {
        size_t len = base + (x < rem ? 1 : 0);
        for (size_t j = 0; j < len; ++j) out[j * X + x] = logical[start + j];
        start += len;
    }
    return out;
}

}  // namespace

void free_conv_plan(dmath_ctx_s* ctx, ConvPlan& p)
{
    for (void** q : {&p.dev_tables, &p.workspace})
        if (*q) {
            ctx->pool.free(*q);
            *q = nullptr;
        }
    p.xp = p.fp = p.yt = nullptr;  // the copies belong to the context's table
    if (p.gemm) {
        free_gemm_plan(ctx, *p.gemm);
        p.gemm.reset();
    }
}

// The copy of matrix `src` in the given layout: found, or allocated (zeroed once: the border of a
// padded copy is never written again).  Null when the pool is full.
static Relayout* get_relayout(dmath_ctx_s* ctx, const dmath_matrix_s* src, int32_t kind,
                              std::vector<int32_t> geom, size_t bytes)
{
    RelayoutKey key{src->id, kind, std::move(geom)};
    auto it = ctx->relayouts.find(key);
    if (it != ctx->relayouts.end()) return &it->second;
    void* buf = ctx->pool.alloc(bytes);
    if (!buf) return nullptr;
    if (hipMemsetAsync(buf, 0, bytes, ctx->stream) != hipSuccess) {
        ctx->pool.free(buf);
        return nullptr;
    }
    Relayout r;
    r.buf = buf;
    r.bytes = bytes;
    return &(ctx->relayouts[key] = r);
}

static void drop_relayouts_of(dmath_ctx_s* ctx, uint64_t id)
{
    for (auto it = ctx->relayouts.begin(); it != ctx->relayouts.end();)
        if (std::get<0>(it->first) == id) {
            ctx->pool.free(it->second.buf);
            it = ctx->relayouts.erase(it);
        } else
            ++it;
}

// Copies that no plan reads any more (their plans were replaced) give their memory back.
void drop_unused_relayouts(dmath_ctx_s* ctx)
{
    std::set<const Relayout*> used;
    for (auto& kv : ctx->conv_plans)
        for (const Relayout* r : {kv.second->xp, kv.second->fp, kv.second->yt})
            if (r) used.insert(r);
    for (auto it = ctx->relayouts.begin(); it != ctx->relayouts.end();)
        if (!used.count(&it->second)) {
            ctx->pool.free(it->second.buf);
            it = ctx->relayouts.erase(it);
        } else
            ++it;
}

void drop_pipelines_using(dmath_ctx_s* ctx, uint64_t id)
{
    for (auto it = ctx->pipelines.begin(); it != ctx->pipelines.end();)
        if (it->second.uses.count(id)) {
            (void)hipGraphExecDestroy(it->second.exec);
            it = ctx->pipelines.erase(it);
        } else
            ++it;
}

void drop_all_pipelines(dmath_ctx_s* ctx)
{
    for (auto& kv : ctx->pipelines) (void)hipGraphExecDestroy(kv.second.exec);
    ctx->pipelines.clear();
}

// Everything derived from matrix `id` goes: recorded sequences first (their kernels hold the
// addresses of the tables and copies freed next).
void drop_plans_using(dmath_ctx_s* ctx, uint64_t id)
{
    drop_pipelines_using(ctx, id);
    if (ctx->noalloc_plan) {
        const auto& u = ctx->noalloc_plan->uses;
        if (std::find(u.begin(), u.end(), id) != u.end()) ctx->noalloc_plan.reset();
    }
    for (auto it = ctx->gemm_plans.begin(); it != ctx->gemm_plans.end();) {
        auto& u = it->second->uses;
        if (std::find(u.begin(), u.end(), id) != u.end()) {
            free_gemm_plan(ctx, *it->second);
            it = ctx->gemm_plans.erase(it);
        } else
            ++it;
    }
    for (auto it = ctx->conv_plans.begin(); it != ctx->conv_plans.end();) {
        auto& u = it->second->uses;
        if (std::find(u.begin(), u.end(), id) != u.end()) {
            free_conv_plan(ctx, *it->second);
            it = ctx->conv_plans.erase(it);
        } else
            ++it;
    }
    drop_relayouts_of(ctx, id);
}

void drop_all_plans(dmath_ctx_s* ctx)
{
    drop_all_pipelines(ctx);
    ctx->noalloc_plan.reset();
    for (auto& kv : ctx->gemm_plans) free_gemm_plan(ctx, *kv.second);
    ctx->gemm_plans.clear();
    for (auto& kv : ctx->conv_plans) free_conv_plan(ctx, *kv.second);
    ctx->conv_plans.clear();
    for (auto& kv : ctx->relayouts) ctx->pool.free(kv.second.buf);
    ctx->relayouts.clear();
}

static hipError_t upload(dmath_ctx_s* ctx, void* dst, const std::vector<char>& buf)
{
    hipError_t e = hipMemcpyAsync(dst, buf.data(), buf.size(), hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(ctx->stream);  // buf is pageable and about to go away
}

// What the choice of kernel depends on besides the device addresses: ops, precisions, shapes
// and block grids.  Choices found by timing samples are stored under this key, so that they
// serve every set of matrices laid out the same way.
std::vector<int64_t> gemm_signature(int transA, int transB, const dmath_matrix_s* A, const dmath_matrix_s* B,
                                    const dmath_matrix_s* C)
{
    std::vector<int64_t> sig{transA, transB};
    for (const dmath_matrix_s* m : {A, B, C})
        for (int64_t x : {(int64_t)m->dtype, m->rows, m->cols, (int64_t)m->rsplit.g, (int64_t)m->csplit.g})
            sig.push_back(x);
    return sig;
}

void free_gemm_plan(dmath_ctx_s* ctx, GemmPlan& p)
{
    if (!p.in_arena) {  // an arena is not given back piece by piece
        if (p.dev_tables) ctx->pool.free(p.dev_tables);
        if (p.workspace) ctx->pool.free(p.workspace);
        if (p.tail_scratch) ctx->pool.free(p.tail_scratch);
    }
    p.dev_tables = p.workspace = p.tail_scratch = nullptr;
    p.n_tail_cells = 0;
}

dmath_status_t get_gemm_plan(dmath_ctx_s* ctx, int transA, int transB, dmath_matrix_s* A,
                             dmath_matrix_s* B, dmath_matrix_s* C, bool do_upload, GemmPlan** out,
                             bool* was_cached)
{
    GemmKey key{A->id, B->id, C->id, transA, transB};
    auto found = ctx->gemm_plans.find(key);
    if (found != ctx->gemm_plans.end() && (found->second->dev_tables || !do_upload)) {
        *out = found->second.get();
        if (was_cached) *was_cached = true;
        return DMATH_OK;
    }
    if (was_cached) *was_cached = false;
    if (do_upload && ctx->recording) return DMATH_ERR_UNSUPPORTED;  // uploading synchronises
    if (found != ctx->gemm_plans.end()) ctx->gemm_plans.erase(found);  // described, never uploaded
    const GemmChoice* forced = nullptr;
    auto tuned = ctx->tuned_gemm.find(gemm_signature(transA, transB, A, B, C));
    if (tuned != ctx->tuned_gemm.end() && ctx->policy == 0) forced = &tuned->second;
    std::unique_ptr<GemmPlan> plan;
    dmath_status_t st = make_gemm_plan(ctx, transA, transB, A, B, C, do_upload, forced, &plan, nullptr);
    // the pool cannot hold the split-K partial sums: same kernel and tiles, unsplit (slower, but
    // memory decides, as in the paper's choice of algorithm under memory constraints, section 4.1)
    if (st == DMATH_ERR_OOM)
        st = make_gemm_plan(ctx, transA, transB, A, B, C, do_upload, forced, &plan, nullptr, true);
    if (st == DMATH_ERR_OOM) {  // nor the scratch panels of the k-tails: the generic kernel needs none
        const GemmChoice frugal;  // generic kernel, unsplit
        st = make_gemm_plan(ctx, transA, transB, A, B, C, do_upload, &frugal, &plan, nullptr, true);
    }
    if (st != DMATH_OK) return st;
    *out = plan.get();
    ctx->gemm_plans[key] = std::move(plan);
    return DMATH_OK;
}

dmath_status_t make_gemm_plan(dmath_ctx_s* ctx, int transA, int transB, dmath_matrix_s* A, dmath_matrix_s* B,
                              dmath_matrix_s* C, bool do_upload, const GemmChoice* forced,
                              std::unique_ptr<GemmPlan>* out, std::vector<GemmChoice>* candidates, bool unsplit,
                              Arena* arena)
{
    // device memory beyond the operands comes from the pool, or from the caller's fixed arena
    auto take = [&](size_t bytes) -> void* { return arena ? arena->take(bytes) : ctx->pool.alloc(bytes); };
    auto give = [&](void* q) {
        if (!arena) ctx->pool.free(q);
    };
    const int64_t M = C->rows, N = C->cols, K = transA ? A->rows : A->cols;
    const Split& a_m = transA ? A->csplit : A->rsplit;
    const Split& a_k = transA ? A->rsplit : A->csplit;
    const Split& b_k = transB ? B->csplit : B->rsplit;
    const Split& b_n = transB ? B->rsplit : B->csplit;

    // first pass without split-K cuts to let the kernel chooser see the natural segments
    std::vector<Seg> ms = refine(M, {&a_m, &C->rsplit});
    std::vector<Seg> ns = refine(N, {&b_n, &C->csplit});
    std::vector<Seg> ks = refine(K, {&a_k, &b_k});

    const size_t es = elem_size(A->dtype);
    auto panel_a = [&](const Seg& m, const Seg& k) {
        return transA ? locate(A, k.start, m.start) : locate(A, m.start, k.start);
    };
    auto panel_b = [&](const Seg& k, const Seg& n) {
        return transB ? locate(B, n.start, k.start) : locate(B, k.start, n.start);
    };
    auto aligned = [&](const Panel& p, size_t esz) {
        return (reinterpret_cast<uintptr_t>(p.ptr) % 16 == 0) && ((p.ld * (int64_t)esz) % 16 == 0);
    };
    bool al = true;
    for (auto& m : ms)
        for (auto& k : ks) al = al && aligned(panel_a(m, k), es);
    for (auto& k : ks)
        for (auto& n : ns) al = al && aligned(panel_b(k, n), es);
    for (auto& m : ms)
        for (auto& n : ns) al = al && aligned(locate(C, m.start, n.start), elem_size(C->dtype));

    // k-segments that are not multiples of the specialised kernels' k-tile: those kernels can
    // still run when the last (len % bk) of such a segment is copied, before every launch, into
    // a zero-padded scratch panel of bk.  The chooser sees the lengths rounded up.
    const int64_t bk = A->dtype == DMATH_F16 ? 64 : A->dtype == DMATH_F32 ? 32 : 16;
    bool k_tails = false;
    for (auto& s : ks) k_tails = k_tails || s.len % bk != 0;
    const bool pad_tails = k_tails && K >= 4 * bk;

    std::vector<int64_t> mlen, nlen, klen;
    for (auto& s : ms) mlen.push_back(s.len);
    for (auto& s : ns) nlen.push_back(s.len);
    for (auto& s : ks) klen.push_back(pad_tails ? (s.len + bk - 1) / bk * bk : s.len);
    bool small = true;  // the specialised kernels address a block through 32-bit byte offsets
    for (const dmath_matrix_s* m : {(const dmath_matrix_s*)A, (const dmath_matrix_s*)B, (const dmath_matrix_s*)C})  // C: the epilogue
        small = small && (uint64_t)m->rsplit.step * (uint64_t)m->csplit.step * elem_size(m->dtype) < (1ull << 32);
    SegView view{M, N, K, &mlen, &nlen, &klen, !transA, (bool)transB, al, small, A->dtype, C->dtype,
                 ctx->policy};
    GemmChoice ch = forced ? *forced : choose_gemm(view);
    if (unsplit) ch.split_k = 1;
    if (candidates) *candidates = gemm_candidates(view);

    // the specialised kernels store a tile's partial sums through 32-bit byte offsets from the
    // tile's first element: rows of the whole-C workspace must allow that
    if (ch.split_k > 1 && ch.kernel != KERNEL_GENERIC && ch.full_tiles == 0 &&
        (uint64_t)N * (uint64_t)ch.tile_m * 8 >= (1ull << 32))
        ch.split_k = 1;
    // split-K: extra cuts of the k axis at multiples of 64 (every kernel's k-step divides 64)
    std::vector<int64_t> split_cuts;
    if (ch.split_k > 1) {
        int64_t per = (K + ch.split_k - 1) / ch.split_k;
        per = (per + 63) / 64 * 64;
        for (int32_t s = 1; s < ch.split_k; ++s)
            if (s * per < K) split_cuts.push_back(s * per);
        ch.split_k = (int32_t)split_cuts.size() + 1;
        ks = refine(K, {&a_k, &b_k}, split_cuts);
    }
    // cut the tails off: afterwards a segment is a multiple of bk or shorter than bk (a tail)
    const bool tails = pad_tails && ch.kernel != KERNEL_GENERIC;
    if (tails) {
        std::vector<int64_t> cuts = split_cuts;
        for (auto& k : ks)
            if (k.len % bk != 0 && k.len > bk) cuts.push_back(k.start + k.len - k.len % bk);
        ks = refine(K, {&a_k, &b_k}, cuts);
    }
    std::vector<int32_t> ksplit{0};
    for (int64_t c : split_cuts)
        for (size_t i = 0; i < ks.size(); ++i)
            if (ks[i].start == c) ksplit.push_back((int32_t)i);
    ksplit.push_back((int32_t)ks.size());

    // scratch panels of the tails, in the operand's own orientation: [M][bk] (k unit-stride) or
    // [bk][M rounded up to 64]; zeroed once here, their first (len) k written before every launch
    const int64_t Mp = (M + 63) / 64 * 64, Np = (N + 63) / 64 * 64;
    const int64_t a_tail = (transA ? Mp : M) * bk, b_tail = (transB ? N : Np) * bk;  // elements per tail
    size_t n_tails = 0;
    for (auto& k : ks) n_tails += tails && k.len % bk != 0;
    char* scratch = nullptr;
    const size_t scratch_bytes = n_tails * (size_t)(a_tail + b_tail) * es;
    if (n_tails && do_upload) {
        const size_t bytes = scratch_bytes;
        scratch = static_cast<char*>(take(bytes));
        if (!scratch) return DMATH_ERR_OOM;
        if (hipMemsetAsync(scratch, 0, bytes, ctx->stream) != hipSuccess) {
            give(scratch);
            return DMATH_ERR_DEVICE;
        }
    }
    std::vector<Panel> pa, pb, pc;
    std::vector<CopyCell> tail_cells;
    int32_t tail_rows = 0;
    {
        std::vector<const char*> as(ks.size(), nullptr), bs(ks.size(), nullptr);
        size_t t = 0;
        for (size_t i = 0; i < ks.size(); ++i)
            if (tails && ks[i].len % bk != 0 && scratch) {
                as[i] = scratch + t * (size_t)(a_tail + b_tail) * es;
                bs[i] = as[i] + a_tail * es;
                ++t;
            }
        // one workgroup copies 16 rows of a cell: wide cells (few k rows x many columns) are cut
        // into runs of 256 columns so that the copy spreads over the chip
        auto cell = [&](const Panel& src, const char* dst, int64_t dst_ld, int64_t rows, int64_t cols) {
            for (int64_t c0 = 0; c0 < cols; c0 += 256)
                tail_cells.push_back({static_cast<const char*>(src.ptr) + c0 * es, const_cast<char*>(dst) + c0 * es,
                                      src.ld, dst_ld, (int32_t)rows, (int32_t)std::min<int64_t>(256, cols - c0)});
            tail_rows = std::max(tail_rows, (int32_t)rows);
        };
        for (auto& m : ms)
            for (size_t i = 0; i < ks.size(); ++i) {
                const Seg& k = ks[i];
                if (!as[i]) {
                    pa.push_back(panel_a(m, k));
                } else if (transA) {  // stored [k][m]
                    pa.push_back({as[i] + m.start * es, Mp});
                    cell(panel_a(m, k), as[i] + m.start * es, Mp, k.len, m.len);
                } else {
                    pa.push_back({as[i] + m.start * bk * es, bk});
                    cell(panel_a(m, k), as[i] + m.start * bk * es, bk, m.len, k.len);
                }
            }
        for (size_t i = 0; i < ks.size(); ++i)
            for (auto& n : ns) {
                const Seg& k = ks[i];
                if (!bs[i]) {
                    pb.push_back(panel_b(k, n));
                } else if (transB) {  // stored [n][k]
                    pb.push_back({bs[i] + n.start * bk * es, bk});
                    cell(panel_b(k, n), bs[i] + n.start * bk * es, bk, n.len, k.len);
                } else {
                    pb.push_back({bs[i] + n.start * es, Np});
                    cell(panel_b(k, n), bs[i] + n.start * es, Np, k.len, n.len);
                }
            }
    }
    for (auto& m : ms)
        for (auto& n : ns) pc.push_back(locate(C, m.start, n.start));
    std::vector<int32_t> kl;
    for (auto& k : ks) kl.push_back((int32_t)(tails ? (k.len + bk - 1) / bk * bk : k.len));

    // Tiles of all cells form one global grid (every cell of a segment row has the same m
    // cuts, every cell of a segment column the same n cuts).  Logical order: super-blocks of
    // SR x SC tiles holding about one XCD's worth of workgroups (32), R/C chosen so that the A row
    // panels and B column panels a super-block touches are as few bytes as possible; xcd_interleave
    // then hands contiguous runs of the order to the XCDs, so the workgroups resident on one XCD
    // at a time share operand panels out of that XCD's L2.
    struct Cut {
        int32_t seg, off, len, glob;
    };
    auto cuts_of = [](const std::vector<Seg>& segs, int32_t tile) {
        std::vector<Cut> v;
        for (size_t si = 0; si < segs.size(); ++si)
            for (int64_t o = 0; o < segs[si].len; o += tile)
                v.push_back({(int32_t)si, (int32_t)o, (int32_t)std::min<int64_t>(tile, segs[si].len - o),
                             (int32_t)(segs[si].start + o)});
        return v;
    };
    const std::vector<Cut> mt = cuts_of(ms, ch.tile_m), nt = cuts_of(ns, ch.tile_n);
    const int64_t Mt = (int64_t)mt.size(), Nt = (int64_t)nt.size();
    int64_t SR = 1;
    {
        const int64_t P = 32;
        int64_t best = -1;
        for (int64_t r = 1; r <= P; r *= 2) {
            int64_t rr = std::min(r, Mt), cc = std::min((P + rr - 1) / rr, Nt);
            int64_t cost = (rr * ch.tile_m + cc * ch.tile_n) * 1024 / (rr * cc);  // bytes per tile
            if (best < 0 || cost < best) {
                best = cost;
                SR = rr;
            }
        }
    }
    const int64_t SC = std::min<int64_t>(std::max<int64_t>(1, (32 + SR - 1) / SR), Nt);
    std::vector<Tile> tiles;
    tiles.reserve((size_t)(Mt * Nt));
    for (int64_t i0 = 0; i0 < Mt; i0 += SR)
        for (int64_t j0 = 0; j0 < Nt; j0 += SC)
            for (int64_t i = i0; i < std::min(Mt, i0 + SR); ++i)
                for (int64_t j = j0; j < std::min(Nt, j0 + SC); ++j) {
                    Tile t;
                    t.mseg = mt[i].seg;
                    t.nseg = nt[j].seg;
                    t.m_off = mt[i].off;
                    t.n_off = nt[j].off;
                    t.m_len = mt[i].len;
                    t.n_len = nt[j].len;
                    t.m_glob = mt[i].glob;
                    t.n_glob = nt[j].glob;
                    tiles.push_back(t);
                }
    tiles = xcd_interleave(tiles);
    // split only the tiles after the last full round: they get a compact workspace of their own,
    // [split][those tiles x tile_m][tile_n]
    int32_t full_tiles = 0;
    if (ch.split_k > 1 && ch.full_tiles > 0 && ch.full_tiles < (int32_t)tiles.size() && ch.kernel != KERNEL_GENERIC) {
        full_tiles = ch.full_tiles;
        for (size_t j = (size_t)full_tiles; j < tiles.size(); ++j) {
            tiles[j].m_glob = (int32_t)(j - (size_t)full_tiles) * ch.tile_m;
            tiles[j].n_glob = 0;
        }
    }

    auto plan = std::make_unique<GemmPlan>();
    plan->in_arena = arena != nullptr;
    plan->full_tiles = full_tiles;
    plan->uses = {A->id, B->id, C->id};
    plan->in_dtype = A->dtype;
    plan->out_dtype = C->dtype;
    plan->reduce_vectors = N % 4 == 0;
    for (auto& n : ns) plan->reduce_vectors = plan->reduce_vectors && n.len % 4 == 0 && n.start % 4 == 0;
    for (auto& m : ms)
        for (auto& n : ns) {
            const Panel pc_ = locate(C, m.start, n.start);
            plan->reduce_vectors = plan->reduce_vectors && reinterpret_cast<uintptr_t>(pc_.ptr) % 16 == 0 &&
                                   pc_.ld % 8 == 0;
        }
    dmath_plan_info_t& info = plan->info;
    info.m = M;
    info.n = N;
    info.k = K;
    info.m_segments = (int32_t)ms.size();
    info.n_segments = (int32_t)ns.size();
    info.k_segments = (int32_t)ks.size();
    info.tile_m = ch.tile_m;
    info.tile_n = ch.tile_n;
    info.tile_k = ch.tile_k;
    info.tiles = (int32_t)tiles.size();
    info.split_k = ch.split_k;
    info.kernel = ch.kernel;
    const size_t acc_size = A->dtype == DMATH_F64 ? 8 : 4;
    // pool memory beyond the operands: split-K partial sums and the scratch panels of k-tails
    const uint64_t split_elems = full_tiles ? (uint64_t)(tiles.size() - (size_t)full_tiles) * ch.tile_m * ch.tile_n
                                            : (uint64_t)M * N;
    const uint64_t partial_bytes = ch.split_k > 1 ? (uint64_t)ch.split_k * split_elems * acc_size : 0;
    info.workspace_bytes = partial_bytes + scratch_bytes;
    info.split_tiles = ch.split_k > 1 ? (int32_t)tiles.size() - full_tiles : 0;

    GemmTables& t = plan->t;
    t.n_mseg = (int32_t)ms.size();
    t.n_nseg = (int32_t)ns.size();
    t.n_kseg = (int32_t)ks.size();
    t.n_tiles = (int32_t)tiles.size();
    t.split_k = ch.split_k;
    t.a_kcontig = !transA;
    t.b_kcontig = transB ? 1 : 0;
    t.M = M;
    t.N = N;

    if (do_upload) {
        std::vector<char> buf;
        size_t oa = append(buf, pa), ob = append(buf, pb), oc = append(buf, pc);
        size_t ok = append(buf, kl), os = append(buf, ksplit), ot = append(buf, tiles);
        size_t ow = append(buf, std::vector<int32_t>{0, (int32_t)ks.size()});
        size_t otc = append(buf, tail_cells);
        plan->tail_scratch = scratch;  // from here on the plan owns it
        void* dev = take(buf.size());
        if (!dev) {
            free_gemm_plan(ctx, *plan);
            return DMATH_ERR_OOM;
        }
        void* ws = nullptr;
        if (partial_bytes) {
            ws = take(partial_bytes);
            if (!ws) {
                give(dev);
                free_gemm_plan(ctx, *plan);
                return DMATH_ERR_OOM;
            }
        }
        if (upload(ctx, dev, buf) != hipSuccess) {
            give(dev);
            if (ws) give(ws);
            free_gemm_plan(ctx, *plan);
            return DMATH_ERR_DEVICE;
        }
        plan->tail_cells = reinterpret_cast<const CopyCell*>(static_cast<char*>(dev) + otc);
        plan->n_tail_cells = (int32_t)tail_cells.size();
        plan->tail_rows = tail_rows;
        char* d = static_cast<char*>(dev);
        t.a = reinterpret_cast<const Panel*>(d + oa);
        t.b = reinterpret_cast<const Panel*>(d + ob);
        t.c = reinterpret_cast<const Panel*>(d + oc);
        t.klen = reinterpret_cast<const int32_t*>(d + ok);
        t.ksplit = reinterpret_cast<const int32_t*>(d + os);
        plan->ksplit_whole = reinterpret_cast<const int32_t*>(d + ow);
        t.tiles = reinterpret_cast<const Tile*>(d + ot);
        t.workspace = ws;
        plan->dev_tables = dev;
        plan->workspace = ws;
    }
    *out = std::move(plan);
    return DMATH_OK;
}

static ConvGeom geometry_of(const dmath_conv_desc_t* d);

dmath_status_t get_conv_plan(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d,
                             dmath_matrix_s* X, dmath_matrix_s* F, dmath_matrix_s* Y,
                             ConvPlan** out)
{
    std::vector<int32_t> geom{d->n, d->c, d->h, d->w, d->k, d->r, d->s,
                              d->pad_h, d->pad_w, d->stride_h, d->stride_w};
    ConvKey key{X->id, F->id, Y->id, mode, geom};
    auto found = ctx->conv_plans.find(key);
    if (found != ctx->conv_plans.end()) {
        *out = found->second.get();
        return DMATH_OK;
    }
    if (ctx->recording) return DMATH_ERR_UNSUPPORTED;  // building a plan synchronises
    const ConvChoice* forced = nullptr;
    auto tuned = ctx->tuned_conv.find(conv_signature(mode, d, X, F, Y));
    if (tuned != ctx->tuned_conv.end() && ctx->policy == 0) forced = &tuned->second;
    std::unique_ptr<ConvPlan> plan;
    dmath_status_t st = make_conv_plan(ctx, mode, d, X, F, Y, forced, &plan);
    if (st == DMATH_ERR_OOM) {
        // no room for the partial sums of a split forward pass / data gradient: the same kernel
        // and tile without the split
        ConvChoice ch = forced ? *forced
                               : choose_conv(mode, geometry_of(d), mode == CONV_FWD ? X->dtype : Y->dtype, ctx->policy);
        if (ch.kernel == 1 && mode != CONV_BWD_FILTER && ch.split_k > 1) {
            ch.split_k = 1;
            ch.tail_only = 0;
            drop_unused_relayouts(ctx);
            st = make_conv_plan(ctx, mode, d, X, F, Y, &ch, &plan);
        }
    }
    if (st == DMATH_ERR_OOM) {
        // no room for the re-layout copies or the partial sums: the generic kernel, unsplit,
        // needs neither (section 4.1: a slower algorithm where memory is the constraint)
        const ConvChoice frugal;
        drop_unused_relayouts(ctx);
        st = make_conv_plan(ctx, mode, d, X, F, Y, &frugal, &plan);
    }
    if (st != DMATH_OK) return st;
    *out = plan.get();
    ctx->conv_plans[key] = std::move(plan);
    return DMATH_OK;
}

std::vector<int64_t> conv_signature(int mode, const dmath_conv_desc_t* d, const dmath_matrix_s* X,
                                    const dmath_matrix_s* F, const dmath_matrix_s* Y)
{
    std::vector<int64_t> sig{mode, d->n, d->c, d->h, d->w, d->k, d->r, d->s,
                             d->pad_h, d->pad_w, d->stride_h, d->stride_w};
    for (const dmath_matrix_s* m : {X, F, Y})
        for (int64_t x : {(int64_t)m->dtype, (int64_t)m->rsplit.g}) sig.push_back(x);
    return sig;
}

static ConvGeom geometry_of(const dmath_conv_desc_t* d)
{
    ConvGeom g;
    g.n = d->n; g.c = d->c; g.h = d->h; g.w = d->w; g.k = d->k; g.r = d->r; g.s = d->s;
    g.pad_h = d->pad_h; g.pad_w = d->pad_w; g.stride_h = d->stride_h; g.stride_w = d->stride_w;
    g.oh = (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
    g.ow = (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
    return g;
}

// Pool memory a choice needs beyond the tensors: split-K partial sums and, for the specialised
// kernels, the re-layout copies they read.
size_t conv_choice_bytes(int mode, const ConvGeom& g, const ConvChoice& c, dmath_dtype_t in_dtype)
{
    const size_t sp_out = (size_t)g.oh * g.ow, crs = (size_t)g.c * g.r * g.s;
    size_t bytes = 0;
    if (c.kernel == 2) return 0;  // no copies; its GEMM plan takes partial sums only for tiny outputs
    if (c.kernel == 1 && mode == CONV_BWD_FILTER) {
        const ConvFastLayout l = conv_fast_layout(mode, g, in_dtype);
        bytes += (size_t)c.split_k * l.kp * l.cp * g.r * g.s * (in_dtype == DMATH_F64 ? 8 : 4);
    } else if (c.kernel == 1 && c.split_k > 1) {
        bytes += (size_t)c.split_k * conv_fast_partial_elems(mode, g, in_dtype, c) * (in_dtype == DMATH_F64 ? 8 : 4);
    } else if (mode == CONV_BWD_FILTER && c.split_k > 1) {
        bytes += (size_t)c.split_k * g.k * crs * (in_dtype == DMATH_F64 ? 8 : 4);
    }
    if (c.kernel == 1) {
        const ConvFastLayout l = conv_fast_layout(mode, g, in_dtype);
        bytes += (size_t)(l.x_bytes + l.f_bytes + l.y_bytes);
    }
    return bytes;
}

dmath_status_t make_conv_plan(dmath_ctx_s* ctx, int mode, const dmath_conv_desc_t* d, dmath_matrix_s* X,
                              dmath_matrix_s* F, dmath_matrix_s* Y, const ConvChoice* forced,
                              std::unique_ptr<ConvPlan>* out)
{
    auto plan = std::make_unique<ConvPlan>();
    plan->uses = {X->id, F->id, Y->id};
    ConvTables& t = plan->t;
    ConvGeom& g = t.g;
    g = geometry_of(d);
    const int64_t sp_out = (int64_t)g.oh * g.ow, sp_in = (int64_t)g.h * g.w;
    const int64_t crs = (int64_t)g.c * g.r * g.s;
    dmath_matrix_s* result = nullptr;
    switch (mode) {
    case CONV_FWD:
        t.M = g.n * sp_out; t.N = g.k; t.K = crs; result = Y;
        break;
    case CONV_BWD_FILTER:
        t.M = g.k; t.N = crs; t.K = g.n * sp_out; result = F;
        break;
    default:
        t.M = g.n * sp_in; t.N = g.c; t.K = (int64_t)g.k * g.r * g.s; result = X;
        break;
    }
    plan->in_dtype = (mode == CONV_FWD) ? X->dtype : Y->dtype;
    plan->out_dtype = result->dtype;

    const ConvChoice ch = forced ? *forced : choose_conv(mode, g, plan->in_dtype, ctx->policy);
    const bool fast = ch.kernel == 1;
    plan->kernel = ch.kernel;
    plan->tile_n = ch.tile_n;
    plan->tile_m = ch.tile_m;
    plan->tail_only = ch.tail_only;
    t.split_k = ch.split_k;  // few C tiles, deep K (generic kernel: weight gradient only)

    auto row_ptrs = [](const dmath_matrix_s* m) {
        std::vector<const void*> v((size_t)m->rows);
        for (int64_t i = 0; i < m->rows; ++i) {
            int32_t bi = m->rsplit.part(i);
            v[(size_t)i] = static_cast<const char*>(m->block(bi, 0)) +
                           (i - m->rsplit.lo(bi)) * m->cols * (int64_t)elem_size(m->dtype);
        }
        return v;
    };
    std::vector<char> buf;
    size_t ox = append(buf, row_ptrs(X)), of = append(buf, row_ptrs(F)), oy = append(buf, row_ptrs(Y));
    const size_t osink = (buf.size() + 255) / 256 * 256;
    buf.resize(osink + 256);
    void* dev = ctx->pool.alloc(buf.size());
    if (!dev) return DMATH_ERR_OOM;
    void* ws = nullptr;
    // the specialised weight-gradient kernel always goes through the partial-sum workspace,
    // also with a single split
    const ConvFastLayout lay = fast ? conv_fast_layout(mode, g, plan->in_dtype) : ConvFastLayout{};
    if (t.split_k > 1 || (fast && mode == CONV_BWD_FILTER)) {
        size_t acc = plan->in_dtype == DMATH_F64 ? 8 : 4;
        // the specialised kernel's partial sums have the padded extents of its copies
        const size_t elems = !fast                     ? (size_t)(t.M * t.N)
                             : mode == CONV_BWD_FILTER ? (size_t)lay.kp * lay.cp * g.r * g.s
                                                       : (size_t)conv_fast_partial_elems(mode, g, plan->in_dtype, ch);
        ws = ctx->pool.alloc((size_t)t.split_k * elems * acc);
        if (!ws) {
            ctx->pool.free(dev);
            return DMATH_ERR_OOM;
        }
    }
    if (fast) {
        // copies this plan reads; a copy is shared by every plan that wants the same layout of
        // the same matrix (the activations of the forward pass serve the weight gradient too)
        plan->dev_tables = dev;
        plan->workspace = ws;
        const int32_t pph = g.r - 1 - g.pad_h, ppw = g.s - 1 - g.pad_w;
        if (mode == CONV_BWD_DATA) {
            // dY gathered with padding r-1-pad and its pixels spread out by the stride (the zeros
            // between them are those of the allocation), filter rotated with its channel roles swapped
            plan->xp = get_relayout(ctx, Y, RELAYOUT_CHANNELS_LAST,
                                    {g.k, g.oh, g.ow, pph, ppw, g.stride_h, g.stride_w, g.h + g.r - 1, g.w + g.s - 1},
                                    (size_t)lay.x_bytes);
            plan->fp = get_relayout(ctx, F, RELAYOUT_FILTER_ROTATED, {g.c, g.r, g.s, g.k}, (size_t)lay.f_bytes);
        } else {
            plan->xp = get_relayout(ctx, X, RELAYOUT_CHANNELS_LAST,
                                    {g.c, g.h, g.w, g.pad_h, g.pad_w, (int32_t)lay.x_images}, (size_t)lay.x_bytes);
            if (mode == CONV_FWD)
                plan->fp = get_relayout(ctx, F, RELAYOUT_FILTER_RSC, {g.c, g.r, g.s, g.k}, (size_t)lay.f_bytes);
            else if (Y->rsplit.g == 1 && conv_fast_wgrad_dy_in_place(g, plan->in_dtype))
                plan->dy_in_place = Y->block(0, 0);
            else
                plan->yt = get_relayout(ctx, Y, RELAYOUT_CHANNELS_LAST, {g.k, g.oh, g.ow, 0, 0}, (size_t)lay.y_bytes);
        }
        const bool ok = plan->xp && (mode == CONV_BWD_FILTER ? (plan->yt || plan->dy_in_place) : plan->fp != nullptr);
        if (!ok) {
            free_conv_plan(ctx, *plan);
            return DMATH_ERR_OOM;
        }
    }
    if (upload(ctx, dev, buf) != hipSuccess) {
        plan->dev_tables = dev;
        plan->workspace = ws;
        free_conv_plan(ctx, *plan);
        return DMATH_ERR_DEVICE;
    }
    char* dp = static_cast<char*>(dev);
    t.x_rows = reinterpret_cast<const void* const*>(dp + ox);
    t.f_rows = reinterpret_cast<const void* const*>(dp + of);
    t.y_rows = reinterpret_cast<const void* const*>(dp + oy);
    t.sink = dp + osink;
    t.workspace = ws;
    plan->dev_tables = dev;
    plan->workspace = ws;
    if (ch.kernel == 2) {
        // 1x1, stride 1, no padding: image i of a tensor with `channels` channels is a dense
        // [channels x h*w] matrix where it lies, so the tensor is a [channels x n*h*w] block matrix
        // with one column block per image, and F is [k x c] as stored:
        //   forward:         Y (k x n*hw) = F * X (c x n*hw)
        //   data gradient:  dX (c x n*hw) = F^T * dY (k x n*hw)
        //   weight gradient: dF (k x c)   = dY (k x n*hw) * X^T (n*hw x c), one k-segment per image
        auto images_as_blocks = [&](const dmath_matrix_s* m, int64_t channels) {
            dmath_matrix_s v;
            v.ctx = ctx;
            v.id = m->id;
            v.rows = channels;
            v.cols = g.n * sp_in;
            v.rsplit = Split(channels, 1);
            v.csplit = Split(g.n * sp_in, g.n);
            v.dtype = m->dtype;
            for (const void* row : row_ptrs(m)) v.blocks.push_back(const_cast<void*>(row));
            return v;
        };
        dmath_matrix_s xs = images_as_blocks(X, g.c), ys = images_as_blocks(Y, g.k);
        std::unique_ptr<GemmPlan> gp;
        auto make = [&](bool unsplit) {
            if (mode == CONV_FWD) return make_gemm_plan(ctx, 0, 0, F, &xs, &ys, true, nullptr, &gp, nullptr, unsplit);
            if (mode == CONV_BWD_DATA) return make_gemm_plan(ctx, 1, 0, F, &ys, &xs, true, nullptr, &gp, nullptr, unsplit);
            return make_gemm_plan(ctx, 0, 1, &ys, &xs, F, true, nullptr, &gp, nullptr, unsplit);
        };
        dmath_status_t st = make(false);
        if (st == DMATH_ERR_OOM) st = make(true);
        if (st != DMATH_OK) {
            free_conv_plan(ctx, *plan);
            return st;
        }
        plan->gemm = std::move(gp);
    }
    *out = std::move(plan);
    return DMATH_OK;
}

}  // namespace dm
