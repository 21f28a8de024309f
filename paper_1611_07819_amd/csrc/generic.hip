// Guarded generic kernels: every precision, every transpose combination, ragged tiles, any
// alignment, every convolution geometry.  They are the fallback of the specialised kernels
// and the reference inside the library for them: element-wise guarded loads into LDS, MFMA on
// 64x64x16 workgroup tiles (4 wavefronts, 32x32 each), fused alpha/beta epilogue.
//
// Operation: C <- alpha * op(A) * op(B) + beta * C over block grids (paper abstract and
// section 2.1), and the convolutions as implicit GEMMs whose A or B operand is gathered from
// the NCHW tensor on the fly.
#include <hip/hip_runtime.h>

#include "context.hpp"
#include "mfma.hpp"

namespace dm {

hipError_t launch_gemm_reduce(const GemmPlan& p, const GemmTables& t, int n_partials, double alpha, double beta,
                              hipStream_t st);

namespace {

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // k-step
constexpr int GTHREADS = 256;

template <class T> struct Traits;
template <> struct Traits<float> {
    using acc_t = float;
    static constexpr int kStride = GK + 1;
    static constexpr int kAccRegs = 16;
};
template <> struct Traits<_Float16> {
    using acc_t = float;
    static constexpr int kStride = GK + 8;  // rows stay 16-byte aligned
    static constexpr int kAccRegs = 16;
};
template <> struct Traits<double> {
    using acc_t = double;
    static constexpr int kStride = GK + 1;
    static constexpr int kAccRegs = 16;  // 2x2 tiles of 16x16, 4 registers each
};

template <class T> struct Acc { typename Traits<T>::acc_t v[16]; };

// One k-step of the workgroup tile out of LDS.  As/Bs: [64][kStride], k contiguous.
__device__ __forceinline__ void mma_step(const float* As, const float* Bs, int wm, int wn, int lane,
                                         Acc<float>& acc)
{
    v16f c;
#pragma unroll
    for (int r = 0; r < 16; ++r) c[r] = acc.v[r];
    const float* ap = As + (wm * 32 + (lane & 31)) * Traits<float>::kStride + (lane >> 5);
    const float* bp = Bs + (wn * 32 + (lane & 31)) * Traits<float>::kStride + (lane >> 5);
#pragma unroll
    for (int s = 0; s < GK / 2; ++s) c = mfma_f32_32x32x2(ap[2 * s], bp[2 * s], c);
#pragma unroll
    for (int r = 0; r < 16; ++r) acc.v[r] = c[r];
}

__device__ __forceinline__ void mma_step(const _Float16* As, const _Float16* Bs, int wm, int wn,
                                         int lane, Acc<_Float16>& acc)
{
    v16f c;
#pragma unroll
    for (int r = 0; r < 16; ++r) c[r] = acc.v[r];
    const _Float16* ap = As + (wm * 32 + (lane & 31)) * Traits<_Float16>::kStride + 8 * (lane >> 5);
    const _Float16* bp = Bs + (wn * 32 + (lane & 31)) * Traits<_Float16>::kStride + 8 * (lane >> 5);
    v8h a = *reinterpret_cast<const v8h*>(ap);
    v8h b = *reinterpret_cast<const v8h*>(bp);
    c = mfma_f16_32x32x16(a, b, c);
#pragma unroll
    for (int r = 0; r < 16; ++r) acc.v[r] = c[r];
}

__device__ __forceinline__ void mma_step(const double* As, const double* Bs, int wm, int wn, int lane,
                                         Acc<double>& acc)
{
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int tj = 0; tj < 2; ++tj) {
            v4d c;
#pragma unroll
            for (int r = 0; r < 4; ++r) c[r] = acc.v[(ti * 2 + tj) * 4 + r];
            const double* ap = As + (wm * 32 + ti * 16 + (lane & 15)) * Traits<double>::kStride + (lane >> 4);
            const double* bp = Bs + (wn * 32 + tj * 16 + (lane & 15)) * Traits<double>::kStride + (lane >> 4);
#pragma unroll
            for (int s = 0; s < GK / 4; ++s) c = mfma_f64_16x16x4(ap[4 * s], bp[4 * s], c);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc.v[(ti * 2 + tj) * 4 + r] = c[r];
        }
}

// (row, column) inside the wavefront's 32x32 tile of accumulator register r.
template <class T> __device__ __forceinline__ void acc_pos(int lane, int r, int& i, int& j)
{
    i = acc32_row(lane, r);
    j = acc32_col(lane);
}
template <> __device__ __forceinline__ void acc_pos<double>(int lane, int r, int& i, int& j)
{
    int t = r >> 2, ti = t >> 1, tj = t & 1;
    i = ti * 16 + acc16d_row(lane, r & 3);
    j = tj * 16 + acc16d_col(lane);
}

template <class TC, class AccT>
__device__ __forceinline__ void epilogue_store(TC* p, AccT acc, AccT alpha, AccT beta)
{
    AccT v = alpha * acc;
    if (beta != AccT(0)) v += beta * static_cast<AccT>(*p);
    *p = static_cast<TC>(v);
}

// ---------------------------------------------------------------------------------------
// GEMM over the segment tables
// ---------------------------------------------------------------------------------------
template <class T, class TC>
__global__ __launch_bounds__(GTHREADS) void gemm_generic_kernel(GemmTables t, double alpha_d,
                                                                double beta_d)
{
    using AccT = typename Traits<T>::acc_t;
    constexpr int S = Traits<T>::kStride;
    __shared__ __attribute__((aligned(16))) T As[GT * S];
    __shared__ __attribute__((aligned(16))) T Bs[GT * S];

    const Tile tile = t.tiles[blockIdx.x];
    const int split = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    Acc<T> acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc.v[r] = AccT(0);

    if constexpr (sizeof(T) == 2) {
        // 16-bit elements: fetched where they are stored (fetching ahead was measured slower)
        const int ks0 = t.ksplit[split], ks1 = t.ksplit[split + 1];
        for (int ks = ks0; ks < ks1; ++ks) {
            const Panel pa = t.a[tile.mseg * t.n_kseg + ks];
            const Panel pb = t.b[ks * t.n_nseg + tile.nseg];
            const T* a = static_cast<const T*>(pa.ptr);
            const T* b = static_cast<const T*>(pb.ptr);
            const int64_t a_smn = t.a_kcontig ? pa.ld : 1, a_sk = t.a_kcontig ? 1 : pa.ld;
            const int64_t b_smn = t.b_kcontig ? pb.ld : 1, b_sk = t.b_kcontig ? 1 : pb.ld;
            const int kl = t.klen[ks];
            for (int k0 = 0; k0 < kl; k0 += GK) {
#pragma unroll
                for (int q = 0; q < GT * GK / GTHREADS; ++q) {
                    int e = q * GTHREADS + tid;
                    int row, kk;
                    if (t.a_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                    T v = T(0);
                    if (row < tile.m_len && k0 + kk < kl)
                        v = a[(int64_t)(tile.m_off + row) * a_smn + (int64_t)(k0 + kk) * a_sk];
                    As[row * S + kk] = v;
                    if (t.b_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                    v = T(0);
                    if (row < tile.n_len && k0 + kk < kl)
                        v = b[(int64_t)(tile.n_off + row) * b_smn + (int64_t)(k0 + kk) * b_sk];
                    Bs[row * S + kk] = v;
                }
                __syncthreads();
                mma_step(As, Bs, wm, wn, lane, acc);
                __syncthreads();
            }
        }

    } else {
        // The k-steps of all k-segments of this split form one sequence; the elements of step i+1
        // are fetched into registers while step i is multiplied out of LDS (fp32, fp64).
        constexpr int Q = GT * GK / GTHREADS;
        const int ks1 = t.ksplit[split + 1];
        int ks = t.ksplit[split], k0 = 0;  // the step that is fetched next
        const T *a = nullptr, *b = nullptr;  // its k-segment's panels
        int64_t a_smn = 0, a_sk = 0, b_smn = 0, b_sk = 0;
        int kl = 0;
        auto enter = [&]() {
            if (ks >= ks1) return;
            const Panel pa = t.a[tile.mseg * t.n_kseg + ks];
            const Panel pb = t.b[ks * t.n_nseg + tile.nseg];
            a = static_cast<const T*>(pa.ptr);
            b = static_cast<const T*>(pb.ptr);
            a_smn = t.a_kcontig ? pa.ld : 1; a_sk = t.a_kcontig ? 1 : pa.ld;
            b_smn = t.b_kcontig ? pb.ld : 1; b_sk = t.b_kcontig ? 1 : pb.ld;
            kl = t.klen[ks];
        };
        enter();
        auto fetch = [&](T (&ra)[Q], T (&rb)[Q]) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int e = q * GTHREADS + tid;
                int row, kk;
                if (t.a_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                ra[q] = T(0);
                if (row < tile.m_len && k0 + kk < kl)
                    ra[q] = a[(int64_t)(tile.m_off + row) * a_smn + (int64_t)(k0 + kk) * a_sk];
                if (t.b_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                rb[q] = T(0);
                if (row < tile.n_len && k0 + kk < kl)
                    rb[q] = b[(int64_t)(tile.n_off + row) * b_smn + (int64_t)(k0 + kk) * b_sk];
            }
            k0 += GK;
            if (k0 >= kl) {
                k0 = 0;
                ++ks;
                enter();
            }
        };
        auto stash = [&](const T (&ra)[Q], const T (&rb)[Q]) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int e = q * GTHREADS + tid;
                int row, kk;
                if (t.a_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                As[row * S + kk] = ra[q];
                if (t.b_kcontig) { kk = e % GK; row = e / GK; } else { row = e % GT; kk = e / GT; }
                Bs[row * S + kk] = rb[q];
            }
        };
        T ra[Q], rb[Q];
        bool more = ks < ks1;  // a fetched step is waiting in ra, rb
        if (more) fetch(ra, rb);
        while (more) {
            stash(ra, rb);
            __syncthreads();
            more = ks < ks1;
            if (more) fetch(ra, rb);
            mma_step(As, Bs, wm, wn, lane, acc);
            __syncthreads();
        }

    }
    if (t.split_k > 1) {
        AccT* ws = static_cast<AccT*>(t.workspace) + (int64_t)split * t.M * t.N;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int i, j;
            acc_pos<T>(lane, r, i, j);
            i += wm * 32;
            j += wn * 32;
            if (i < tile.m_len && j < tile.n_len)
                ws[(int64_t)(tile.m_glob + i) * t.N + tile.n_glob + j] = acc.v[r];
        }
        return;
    }
    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    TC* c = static_cast<TC*>(const_cast<void*>(pc.ptr));
    const AccT alpha = static_cast<AccT>(alpha_d), beta = static_cast<AccT>(beta_d);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int i, j;
        acc_pos<T>(lane, r, i, j);
        i += wm * 32;
        j += wn * 32;
        if (i < tile.m_len && j < tile.n_len)
            epilogue_store(c + (int64_t)(tile.m_off + i) * pc.ld + tile.n_off + j, acc.v[r], alpha, beta);
    }
}

// Fixed-order sum of the split-K partials followed by the epilogue; with n_partials == 0 it is
// the alpha == 0 path (C <- beta * C) that never touches A or B.  Grid: (tiles, row chunks of
// kReduceRows rows), so that few large tiles still fill the chip.
template <class T, int N> struct VecOf {
    typedef T type __attribute__((ext_vector_type(N)));
};

// VEC consecutive columns per lane (16 bytes of the accumulation type) where the plan says that
// every tile's width, origin and the leading dimensions allow it: the loads of all partials of
// a lane's columns are then in flight together.
constexpr int kReduceRows = 8;
template <class AccT, class TC, int VEC>
__global__ __launch_bounds__(GTHREADS) void gemm_reduce_kernel(GemmTables t, int n_partials,
                                                               double alpha_d, double beta_d)
{
    typedef typename VecOf<AccT, VEC>::type vacc;
    typedef typename VecOf<TC, VEC>::type vout;
    const Tile tile = t.tiles[blockIdx.x];
    const int r0 = blockIdx.y * kReduceRows;
    if (r0 >= tile.m_len) return;
    const int rows = min(kReduceRows, tile.m_len - r0);
    const Panel pc = t.c[tile.mseg * t.n_nseg + tile.nseg];
    TC* c = static_cast<TC*>(const_cast<void*>(pc.ptr));
    const AccT* ws = static_cast<const AccT*>(t.workspace);
    const AccT alpha = static_cast<AccT>(alpha_d), beta = static_cast<AccT>(beta_d);
    const int64_t slice = t.M * t.N;
    const int vcols = tile.n_len / VEC;
    const int count = rows * vcols;
    for (int e = threadIdx.x; e < count; e += GTHREADS) {
        const int i = r0 + e / vcols, j = (e % vcols) * VEC;
        const AccT* p = ws + (int64_t)(tile.m_glob + i) * t.N + tile.n_glob + j;
        vacc sum;
#pragma unroll
        for (int q = 0; q < VEC; ++q) sum[q] = AccT(0);
        int s = 0;
        for (; s + 4 <= n_partials; s += 4) {  // four loads in flight, added in ascending order
            const vacc p0 = *reinterpret_cast<const vacc*>(p + (int64_t)s * slice);
            const vacc p1 = *reinterpret_cast<const vacc*>(p + (int64_t)(s + 1) * slice);
            const vacc p2 = *reinterpret_cast<const vacc*>(p + (int64_t)(s + 2) * slice);
            const vacc p3 = *reinterpret_cast<const vacc*>(p + (int64_t)(s + 3) * slice);
            sum = (((sum + p0) + p1) + p2) + p3;
        }
        for (; s < n_partials; ++s) sum += *reinterpret_cast<const vacc*>(p + (int64_t)s * slice);
        TC* dst = c + (int64_t)(tile.m_off + i) * pc.ld + tile.n_off + j;
        vout o;
        if (beta != AccT(0)) o = *reinterpret_cast<const vout*>(dst);
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            AccT v = alpha * sum[q];
            if (beta != AccT(0)) v += beta * static_cast<AccT>(o[q]);
            o[q] = static_cast<TC>(v);
        }
        *reinterpret_cast<vout*>(dst) = o;
    }
}

// ---------------------------------------------------------------------------------------
// Convolutions as implicit GEMMs (gathered operands)
// ---------------------------------------------------------------------------------------
template <class T> __device__ __forceinline__ T conv_im2col(const ConvTables& t, int m, int kk)
{
    // row m = (image, oh, ow), column kk = (c, r, s): X[n, c, oh*sh + r - ph, ow*sw + s - pw]
    const ConvGeom& g = t.g;
    int sp_out = g.oh * g.ow;
    int n = m / sp_out, sp = m % sp_out, oy = sp / g.ow, ox = sp % g.ow;
    int rs = g.r * g.s;
    int c = kk / rs, q = kk % rs, fr = q / g.s, fs = q % g.s;
    int ih = oy * g.stride_h + fr - g.pad_h, iw = ox * g.stride_w + fs - g.pad_w;
    if (ih < 0 || ih >= g.h || iw < 0 || iw >= g.w) return T(0);
    return static_cast<const T*>(t.x_rows[n])[(c * g.h + ih) * g.w + iw];
}

template <class T, int MODE> __device__ __forceinline__ T conv_a(const ConvTables& t, int m, int kk)
{
    const ConvGeom& g = t.g;
    if (MODE == CONV_FWD) return conv_im2col<T>(t, m, kk);
    if (MODE == CONV_BWD_FILTER) {
        // A = dY viewed as [k x (n, oh, ow)]
        int sp_out = g.oh * g.ow;
        int n = kk / sp_out, sp = kk % sp_out;
        return static_cast<const T*>(t.y_rows[n])[m * sp_out + sp];
    }
    // data gradient: row m = (image, ih, iw), column kk = (k, r, s)
    int sp_in = g.h * g.w;
    int n = m / sp_in, sp = m % sp_in, ih = sp / g.w, iw = sp % g.w;
    int rs = g.r * g.s;
    int ko = kk / rs, q = kk % rs, fr = q / g.s, fs = q % g.s;
    int th = ih + g.pad_h - fr, tw = iw + g.pad_w - fs;
    if (th < 0 || tw < 0 || th % g.stride_h || tw % g.stride_w) return T(0);
    int oy = th / g.stride_h, ox = tw / g.stride_w;
    if (oy >= g.oh || ox >= g.ow) return T(0);
    return static_cast<const T*>(t.y_rows[n])[(ko * g.oh + oy) * g.ow + ox];
}

template <class T, int MODE> __device__ __forceinline__ T conv_b(const ConvTables& t, int kk, int j)
{
    const ConvGeom& g = t.g;
    if (MODE == CONV_FWD) return static_cast<const T*>(t.f_rows[j])[kk];
    if (MODE == CONV_BWD_FILTER) return conv_im2col<T>(t, kk, j);
    int rs = g.r * g.s;
    int ko = kk / rs, q = kk % rs;
    return static_cast<const T*>(t.f_rows[ko])[j * rs + q];
}

template <class TC, int MODE> __device__ __forceinline__ TC* conv_c(const ConvTables& t, int m, int j)
{
    const ConvGeom& g = t.g;
    if (MODE == CONV_FWD) {
        int sp_out = g.oh * g.ow;
        int n = m / sp_out, sp = m % sp_out;
        return static_cast<TC*>(const_cast<void*>(t.y_rows[n])) + j * sp_out + sp;
    }
    if (MODE == CONV_BWD_FILTER) return static_cast<TC*>(const_cast<void*>(t.f_rows[m])) + j;
    int sp_in = g.h * g.w;
    int n = m / sp_in, sp = m % sp_in;
    return static_cast<TC*>(const_cast<void*>(t.x_rows[n])) + j * sp_in + sp;
}

// The gathers of one thread.  Every k-step the workgroup shares a table with the decomposition of
// its 16 k indices (computed by 16 threads instead of by every thread for every element), and a
// thread's own row or column of the lowered matrices is decomposed once.
//   forward        : k = (c, r, s) -> table (c, r, s); A row = pixel (n, oh, ow) of this thread
//   weight gradient: k = pixel     -> table (n, oh, ow); B columns (c, r, s) of this thread's slots
//   data gradient  : k = (ko, r, s) -> table (ko, r, s); A row = input pixel (n, ih, iw)
// Thread -> element maps: the unit-stride axis of the gathered tensor goes across lanes.
// Decomposition of one k index, with the row pointers that go with it (weight gradient: the
// image's rows of dY and X; data gradient: the filter's row).
struct KEntry {
    const void *p0, *p1;
    int d0, d1, d2, pad;
};

template <class T, int MODE> struct ConvGather {
    static constexpr int Q = GT * GK / GTHREADS;
    static constexpr bool a_kfast = (MODE == CONV_BWD_FILTER);
    static constexpr bool b_kfast = (MODE != CONV_BWD_DATA);
    const ConvTables& t;
    const KEntry (*kd)[GK];  // [2][GK] in LDS
    int tid, kend;
    // forward / data gradient: this thread's A row
    const T* a_ptr;
    int a0, a1;  // forward: ih0, iw0; data gradient: ih + pad_h, iw + pad_w
    bool a_ok;
    // per slot: forward B = filter row; weight gradient A = filter index, B = column (c, r, s);
    // data gradient B = channel
    const T* b_ptr[Q];
    int row_q[Q], bc[Q], br[Q], bs[Q];
    bool b_ok[Q], a_okq[Q];

    __device__ __forceinline__ ConvGather(const ConvTables& t_, const KEntry (*kd_)[GK], int m0, int n0, int tid_,
                                          int kend_)
        : t(t_), kd(kd_), tid(tid_), kend(kend_)
    {
        const ConvGeom& g = t.g;
        const int M = (int)t.M, N = (int)t.N;
        a_ptr = nullptr;
        a0 = a1 = 0;
        a_ok = false;
        if (MODE == CONV_FWD) {
            const int m = m0 + tid % GT, sp_out = g.oh * g.ow;
            a_ok = m < M;
            if (a_ok) {
                const int n = m / sp_out, sp = m % sp_out;
                a_ptr = static_cast<const T*>(t.x_rows[n]);
                a0 = (sp / g.ow) * g.stride_h - g.pad_h;
                a1 = (sp % g.ow) * g.stride_w - g.pad_w;
            }
        } else if (MODE == CONV_BWD_DATA) {
            const int m = m0 + tid % GT, sp_in = g.h * g.w;
            a_ok = m < M;
            if (a_ok) {
                const int n = m / sp_in, sp = m % sp_in;
                a_ptr = static_cast<const T*>(t.y_rows[n]);
                a0 = sp / g.w + g.pad_h;
                a1 = sp % g.w + g.pad_w;
            }
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int e = q * GTHREADS + tid;
            b_ptr[q] = nullptr;
            row_q[q] = bc[q] = br[q] = bs[q] = 0;
            a_okq[q] = false;
            if (MODE == CONV_FWD) {
                const int j = n0 + e / GK;
                b_ok[q] = j < N;
                if (b_ok[q]) b_ptr[q] = static_cast<const T*>(t.f_rows[j]);
            } else if (MODE == CONV_BWD_FILTER) {
                row_q[q] = m0 + e / GK;  // filter index of the A element
                a_okq[q] = row_q[q] < M;
                const int j = n0 + e / GK, rs = g.r * g.s;
                b_ok[q] = j < N;
                if (b_ok[q]) {
                    bc[q] = j / rs;
                    br[q] = (j % rs) / g.s - g.pad_h;
                    bs[q] = (j % rs) % g.s - g.pad_w;
                }
            } else {
                row_q[q] = n0 + tid % GT;  // channel of the B element
                b_ok[q] = row_q[q] < N;
            }
        }
    }

    // the shared decomposition of k-step k0, written into table `buf` by the first GK threads
    __device__ __forceinline__ static void fill_table(const ConvTables& t, KEntry (*kd)[GK], int buf, int k0, int tid,
                                                      int kend)
    {
        if (tid >= GK) return;
        const ConvGeom& g = t.g;
        const int kk = k0 + tid;
        if (kk >= kend) return;  // never read
        KEntry e{};
        if (MODE == CONV_BWD_FILTER) {
            const int sp_out = g.oh * g.ow, sp = kk % sp_out;
            e.d0 = kk / sp_out;
            e.d1 = sp / g.ow;
            e.d2 = sp % g.ow;
            e.p0 = t.y_rows[e.d0];
            e.p1 = t.x_rows[e.d0];
        } else {
            const int rs = g.r * g.s, q = kk % rs;
            e.d0 = kk / rs;
            e.d1 = q / g.s;
            e.d2 = q % g.s;
            if (MODE == CONV_BWD_DATA) e.p0 = t.f_rows[e.d0];
        }
        kd[buf][tid] = e;
    }

    __device__ __forceinline__ T a(int q, int k0, int buf) const
    {
        const ConvGeom& g = t.g;
        const int e = q * GTHREADS + tid;
        const int kl = a_kfast ? e % GK : e / GT;
        if (k0 + kl >= kend) return T(0);
        const KEntry& k = kd[buf][kl];
        const int d0 = k.d0, d1 = k.d1, d2 = k.d2;
        if (MODE == CONV_FWD) {
            if (!a_ok) return T(0);
            const int ih = a0 + d1, iw = a1 + d2;
            if (ih < 0 || ih >= g.h || iw < 0 || iw >= g.w) return T(0);
            return a_ptr[(d0 * g.h + ih) * g.w + iw];
        }
        if (MODE == CONV_BWD_FILTER) {
            // dY viewed as [k x (n, oh, ow)]
            if (!a_okq[q]) return T(0);
            return static_cast<const T*>(k.p0)[row_q[q] * (g.oh * g.ow) + d1 * g.ow + d2];
        }
        if (!a_ok) return T(0);
        const int th = a0 - d1, tw = a1 - d2;
        if (th < 0 || tw < 0 || th % g.stride_h || tw % g.stride_w) return T(0);
        const int oy = th / g.stride_h, ox = tw / g.stride_w;
        if (oy >= g.oh || ox >= g.ow) return T(0);
        return a_ptr[(d0 * g.oh + oy) * g.ow + ox];
    }

    __device__ __forceinline__ T b(int q, int k0, int buf) const
    {
        const ConvGeom& g = t.g;
        const int e = q * GTHREADS + tid;
        const int kl = b_kfast ? e % GK : e / GT;
        if (k0 + kl >= kend || !b_ok[q]) return T(0);
        if (MODE == CONV_FWD) return b_ptr[q][k0 + kl];
        const KEntry& k = kd[buf][kl];
        const int d1 = k.d1, d2 = k.d2;
        if (MODE == CONV_BWD_FILTER) {
            const int ih = d1 * g.stride_h + br[q], iw = d2 * g.stride_w + bs[q];
            if (ih < 0 || ih >= g.h || iw < 0 || iw >= g.w) return T(0);
            return static_cast<const T*>(k.p1)[(bc[q] * g.h + ih) * g.w + iw];
        }
        return static_cast<const T*>(k.p0)[row_q[q] * (g.r * g.s) + d1 * g.s + d2];
    }
};

template <class T, class TC, int MODE>
__global__ __launch_bounds__(GTHREADS) void conv_generic_kernel(ConvTables t, int k_per_split,
                                                                double alpha_d, double beta_d)
{
    using AccT = typename Traits<T>::acc_t;
    using Gather = ConvGather<T, MODE>;
    constexpr int S = Traits<T>::kStride;
    constexpr int Q = Gather::Q;
    __shared__ __attribute__((aligned(16))) T As[GT * S];
    __shared__ __attribute__((aligned(16))) T Bs[GT * S];
    __shared__ KEntry kd[2][GK];
    const int tiles_n = (int)((t.N + GT - 1) / GT);
    const int m0 = (blockIdx.x / tiles_n) * GT, n0 = (blockIdx.x % tiles_n) * GT;
    const int split = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const int M = (int)t.M, N = (int)t.N, K = (int)t.K;
    Acc<T> acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc.v[r] = AccT(0);
    const int kbeg = split * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const Gather gather(t, kd, m0, n0, tid, kend);
    auto stash = [&](const T (&ra)[Q], const T (&rb)[Q]) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int e = q * GTHREADS + tid;
            if (Gather::a_kfast) As[(e / GK) * S + e % GK] = ra[q]; else As[(e % GT) * S + e / GT] = ra[q];
            if (Gather::b_kfast) Bs[(e / GK) * S + e % GK] = rb[q]; else Bs[(e % GT) * S + e / GT] = rb[q];
        }
    };
    auto fetch = [&](int k0, int buf, T (&ra)[Q], T (&rb)[Q]) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            ra[q] = gather.a(q, k0, buf);
            rb[q] = gather.b(q, k0, buf);
        }
    };
    T ra[Q], rb[Q];
    Gather::fill_table(t, kd, 0, kbeg, tid, kend);
    if constexpr (sizeof(T) == 2) {
        // 16-bit elements: gathered where they are stored (gathering ahead was measured slower)
        __syncthreads();
        int buf = 0;
        for (int k0 = kbeg; k0 < kend; k0 += GK, buf ^= 1) {
            fetch(k0, buf, ra, rb);
            stash(ra, rb);
            Gather::fill_table(t, kd, buf ^ 1, k0 + GK, tid, kend);  // last read before the barrier below, one step ago
            __syncthreads();
            mma_step(As, Bs, wm, wn, lane, acc);
            __syncthreads();
        }
    } else {
        // the elements of k-step i+1 are gathered into registers while step i is multiplied out of
        // LDS (fp32, fp64); the table of step i+2 is written meanwhile
        Gather::fill_table(t, kd, 1, kbeg + GK, tid, kend);
        __syncthreads();
        if (kbeg < kend) fetch(kbeg, 0, ra, rb);
        __syncthreads();  // table 0 is rewritten in the first iteration
        int buf = 0;      // table of the step held in ra, rb
        for (int k0 = kbeg; k0 < kend; k0 += GK, buf ^= 1) {
            stash(ra, rb);
            Gather::fill_table(t, kd, buf, k0 + 2 * GK, tid, kend);
            __syncthreads();
            if (k0 + GK < kend) fetch(k0 + GK, buf ^ 1, ra, rb);
            mma_step(As, Bs, wm, wn, lane, acc);
            __syncthreads();
        }
    }
    const AccT alpha = static_cast<AccT>(alpha_d), beta = static_cast<AccT>(beta_d);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int i, j;
        acc_pos<T>(lane, r, i, j);
        i += m0 + wm * 32;
        j += n0 + wn * 32;
        if (i < M && j < N) {
            if (t.split_k > 1)
                static_cast<AccT*>(t.workspace)[((int64_t)split * M + i) * N + j] = acc.v[r];
            else
                epilogue_store(conv_c<TC, MODE>(t, i, j), acc.v[r], alpha, beta);
        }
    }
}

template <class AccT, class TC, int MODE>
__global__ __launch_bounds__(GTHREADS) void conv_reduce_kernel(ConvTables t, int n_partials,
                                                               double alpha_d, double beta_d)
{
    const int64_t total = t.M * t.N;
    const AccT alpha = static_cast<AccT>(alpha_d), beta = static_cast<AccT>(beta_d);
    const AccT* ws = static_cast<const AccT*>(t.workspace);
    for (int64_t e = (int64_t)blockIdx.x * GTHREADS + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * GTHREADS) {
        AccT sum = AccT(0);
        for (int s = 0; s < n_partials; ++s) sum += ws[(int64_t)s * total + e];
        epilogue_store(conv_c<TC, MODE>(t, (int)(e / t.N), (int)(e % t.N)), sum, alpha, beta);
    }
}

dim3 reduce_grid(const GemmPlan& p, const GemmTables& t)
{
    return dim3(t.n_tiles, (p.info.tile_m + kReduceRows - 1) / kReduceRows);
}

template <class T, class TC>
hipError_t run_gemm_generic(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    using AccT = typename Traits<T>::acc_t;
    const GemmTables& t = p.t;
    if (alpha == 0.0) {
        return launch_gemm_reduce(p, t, 0, 0.0, beta, st);
    }
    gemm_generic_kernel<T, TC><<<dim3(t.n_tiles, t.split_k), GTHREADS, 0, st>>>(t, alpha, beta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || t.split_k == 1) return e;
    return launch_gemm_reduce(p, t, t.split_k, alpha, beta, st);
}

template <class T, class TC, int MODE>
hipError_t run_conv_generic(const ConvPlan& p, double alpha, double beta, hipStream_t st)
{
    using AccT = typename Traits<T>::acc_t;
    const ConvTables& t = p.t;
    const int64_t total = t.M * t.N;
    const int rblocks = (int)std::min<int64_t>((total + GTHREADS - 1) / GTHREADS, 4096);
    if (alpha == 0.0) {
        conv_reduce_kernel<AccT, TC, MODE><<<rblocks, GTHREADS, 0, st>>>(t, 0, 0.0, beta);
        return hipGetLastError();
    }
    const int tiles = (int)(((t.M + GT - 1) / GT) * ((t.N + GT - 1) / GT));
    int per = (int)((t.K + t.split_k - 1) / t.split_k);
    per = (per + GK - 1) / GK * GK;
    conv_generic_kernel<T, TC, MODE><<<dim3(tiles, t.split_k), GTHREADS, 0, st>>>(t, per, alpha, beta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || t.split_k == 1) return e;
    conv_reduce_kernel<AccT, TC, MODE><<<rblocks, GTHREADS, 0, st>>>(t, t.split_k, alpha, beta);
    return hipGetLastError();
}

template <int MODE>
hipError_t conv_dispatch(const ConvPlan& p, double alpha, double beta, hipStream_t st)
{
    if (p.in_dtype == DMATH_F64) return run_conv_generic<double, double, MODE>(p, alpha, beta, st);
    if (p.in_dtype == DMATH_F32) return run_conv_generic<float, float, MODE>(p, alpha, beta, st);
    if (p.out_dtype == DMATH_F16) return run_conv_generic<_Float16, _Float16, MODE>(p, alpha, beta, st);
    return run_conv_generic<_Float16, float, MODE>(p, alpha, beta, st);
}

}  // namespace

hipError_t launch_gemm_generic(const GemmPlan& p, double alpha, double beta, hipStream_t st)
{
    if (p.in_dtype == DMATH_F64) return run_gemm_generic<double, double>(p, alpha, beta, st);
    if (p.in_dtype == DMATH_F32) return run_gemm_generic<float, float>(p, alpha, beta, st);
    if (p.out_dtype == DMATH_F16) return run_gemm_generic<_Float16, _Float16>(p, alpha, beta, st);
    return run_gemm_generic<_Float16, float>(p, alpha, beta, st);
}

// C <- alpha * (sum of the first n_partials split-K partials, ascending) + beta * C, for any
// tile shape.  n_partials == 0 is the alpha == 0 path: A and B are never read.
template <class AccT, class TC>
static void reduce_launch(const GemmPlan& p, const GemmTables& t, int n_partials, double alpha, double beta,
                          hipStream_t st)
{
    constexpr int kVec = 16 / sizeof(AccT);
    if (p.reduce_vectors)
        gemm_reduce_kernel<AccT, TC, kVec><<<reduce_grid(p, t), GTHREADS, 0, st>>>(t, n_partials, alpha, beta);
    else
        gemm_reduce_kernel<AccT, TC, 1><<<reduce_grid(p, t), GTHREADS, 0, st>>>(t, n_partials, alpha, beta);
}

// t: the plan's tables, or a view of them (some of the tiles, their own workspace extents)
hipError_t launch_gemm_reduce(const GemmPlan& p, const GemmTables& t, int n_partials, double alpha, double beta,
                              hipStream_t st)
{
    if (p.in_dtype == DMATH_F64)
        reduce_launch<double, double>(p, t, n_partials, alpha, beta, st);
    else if (p.out_dtype == DMATH_F32)
        reduce_launch<float, float>(p, t, n_partials, alpha, beta, st);
    else
        reduce_launch<float, _Float16>(p, t, n_partials, alpha, beta, st);
    return hipGetLastError();
}

hipError_t launch_conv_generic(const ConvPlan& p, int mode, double alpha, double beta, hipStream_t st)
{
    switch (mode) {
    case CONV_FWD: return conv_dispatch<CONV_FWD>(p, alpha, beta, st);
    case CONV_BWD_FILTER: return conv_dispatch<CONV_BWD_FILTER>(p, alpha, beta, st);
    default: return conv_dispatch<CONV_BWD_DATA>(p, alpha, beta, st);
    }
}

}  // namespace dm
