/*
 * CPU oracle for the block-matrix multiply and the convolutions of the dMath hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what the GPU
 * library must compute.  It shares no code, header, table or helper with the HIP library and
 * must never be called from the product path: only the tests, the smoke check and the
 * "cpu_baseline" leg of the benchmark use it.
 *
 * What it follows:
 *   - a matrix is a grid of non-overlapping dense blocks (paper section 2.1, "Managing
 *     Persistent Data in the GPUs"); results do not depend on how a matrix is cut into blocks
 *     (section 3.2, "Data Distribution Independence");
 *   - storage precisions double, float and half (section 1, feature d); half values are
 *     widened before any arithmetic (section 4.2, "Accuracy & Half-Precision");
 *   - matrix multiplication and convolution are the two kernels named in the abstract.  The
 *     paper prints no formula for either, so the textbook definitions are written out:
 *         C <- alpha * op(A) * op(B) + beta * C                               (BLAS xGEMM)
 *         Y[n,k,oh,ow] = sum_{c,r,s} X[n,c,oh*sh+r-ph,ow*sw+s-pw] * F[k,c,r,s]  (cross-correlation,
 *     the Caffe convention: the paper's framework is a Caffe fork, section 4).
 *
 * Every input element is first widened exactly to fp64 through block_index(); all products and
 * sums are fp64, ascending in the summation index; the result is NOT rounded back to the
 * storage type.  beta == 0 means the old C is not read, alpha == 0 means A and B are not read
 * (BLAS convention), so NaNs there do not propagate.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { O_F64 = 0, O_F32 = 1, O_F16 = 2 };

/* A matrix as the oracle sees it: logical size, grid of blocks, one pointer per block
 * (row-major over the grid), each block dense row-major with ld == its own column count. */
typedef struct {
    int64_t rows, cols;
    int32_t grid_r, grid_c;
    int32_t dtype;
    int32_t pad_;
    const void *const *blocks;
} omat_t;

/* IEEE binary16 -> double, written from the format definition: 1 sign, 5 exponent (bias 15),
 * 10 fraction bits; exponent 0 = zero/subnormal (fraction * 2^-24), exponent 31 = inf/NaN. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* Split rule for one dimension of length n cut into g parts: part p covers
 * [p*ceil(n/g), min(n,(p+1)*ceil(n/g))).  Returns the part holding index i and its local
 * offset and length. */
static void part_of(int64_t n, int32_t g, int64_t i, int32_t *p, int64_t *local, int64_t *len)
{
    int64_t step = (n + g - 1) / g;
    int32_t q = (int32_t)(i / step);
    int64_t lo = (int64_t)q * step;
    int64_t hi = lo + step < n ? lo + step : n;
    *p = q;
    *local = i - lo;
    *len = hi - lo;
}

/* block_index: logical (i,j) -> (block row, block col, local row, local col, local ld). */
static double mat_get(const omat_t *m, int64_t i, int64_t j)
{
    int32_t bi, bj;
    int64_t li, lj, rlen, clen;
    part_of(m->rows, m->grid_r, i, &bi, &li, &rlen);
    part_of(m->cols, m->grid_c, j, &bj, &lj, &clen);
    const void *blk = m->blocks[(int64_t)bi * m->grid_c + bj];
    int64_t off = li * clen + lj;
    switch (m->dtype) {
    case O_F64: return ((const double *)blk)[off];
    case O_F32: return (double)((const float *)blk)[off];
    default:    return half_bits_to_double(((const uint16_t *)blk)[off]);
    }
}

int oracle_part_valid(int64_t n, int32_t g)
{
    if (n <= 0 || g <= 0) return 0;
    int64_t step = (n + g - 1) / g;
    /* the last part must not be empty */
    return (int64_t)(g - 1) * step < n;
}

double oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Widen rows [sel[0..nsel)] (or all rows when sel == NULL) of op(m) into a dense fp64 array
 * out[r][c], r over the selected rows of op(m), c over all columns of op(m). */
static void widen_op_rows(const omat_t *m, int trans, int64_t nsel, const int64_t *sel,
                          int64_t ncols, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nsel; ++r) {
        int64_t i = sel ? sel[r] : r;
        for (int64_t c = 0; c < ncols; ++c)
            out[r * ncols + c] = trans ? mat_get(m, c, i) : mat_get(m, i, c);
    }
}

/*
 * out[r][j] = alpha * sum_k op(A)[i_r,k] * op(B)[k,j] + beta * C[i_r,j]   for the selected rows.
 * sel == NULL selects all M rows (nsel must then equal M).  out is nsel x N, dense, fp64.
 * C may be NULL only when beta == 0.  Returns 0, or a negative number for a shape/layout error.
 */
int oracle_gemm(int transA, int transB, double alpha, const omat_t *A, const omat_t *B,
                double beta, const omat_t *C, int64_t M, int64_t N, int64_t K, int64_t nsel,
                const int64_t *sel, double *out)
{
    int64_t am = transA ? A->cols : A->rows, ak = transA ? A->rows : A->cols;
    int64_t bk = transB ? B->cols : B->rows, bn = transB ? B->rows : B->cols;
    if (am != M || ak != K || bk != K || bn != N) return -1;
    if (C && (C->rows != M || C->cols != N)) return -1;
    if (!C && beta != 0.0) return -2;
    if (!oracle_part_valid(A->rows, A->grid_r) || !oracle_part_valid(A->cols, A->grid_c) ||
        !oracle_part_valid(B->rows, B->grid_r) || !oracle_part_valid(B->cols, B->grid_c))
        return -3;
    if (C && (!oracle_part_valid(C->rows, C->grid_r) || !oracle_part_valid(C->cols, C->grid_c)))
        return -3;
    if (!sel && nsel != M) return -4;
    for (int64_t r = 0; sel && r < nsel; ++r)
        if (sel[r] < 0 || sel[r] >= M) return -4;

    double *a = NULL, *b = NULL;
    if (alpha != 0.0) {
        a = (double *)malloc(sizeof(double) * (size_t)(nsel > 0 ? nsel : 1) * (size_t)K);
        b = (double *)malloc(sizeof(double) * (size_t)K * (size_t)N);
        if (!a || !b) { free(a); free(b); return -5; }
        widen_op_rows(A, transA, nsel, sel, K, a);
        widen_op_rows(B, transB, K, NULL, N, b);
    }

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nsel; ++r) {
        double *row = out + r * N;
        for (int64_t j = 0; j < N; ++j) row[j] = 0.0;
        if (alpha != 0.0) {
            for (int64_t k = 0; k < K; ++k) {
                double aik = a[r * K + k];
                const double *bk_ = b + k * N;
                for (int64_t j = 0; j < N; ++j) row[j] += aik * bk_[j];
            }
            for (int64_t j = 0; j < N; ++j) row[j] *= alpha;
        }
        if (beta != 0.0) {
            int64_t i = sel ? sel[r] : r;
            for (int64_t j = 0; j < N; ++j) row[j] += beta * mat_get(C, i, j);
        }
    }
    free(a);
    free(b);
    return 0;
}

/* Convolution geometry.  Tensors are matrices in the blob view: X = [N x C*H*W],
 * F = [K x C*R*S], Y = [N x K*OH*OW], each row one image / one filter, NCHW inside a row. */
typedef struct {
    int32_t n, c, h, w, k, r, s, pad_h, pad_w, stride_h, stride_w;
} oconv_t;

static int conv_out_dims(const oconv_t *d, int64_t *oh, int64_t *ow)
{
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 ||
        d->s <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->stride_h <= 0 || d->stride_w <= 0)
        return -1;
    int64_t hh = (int64_t)d->h + 2 * d->pad_h - d->r, ww = (int64_t)d->w + 2 * d->pad_w - d->s;
    if (hh < 0 || ww < 0) return -1;
    *oh = hh / d->stride_h + 1;
    *ow = ww / d->stride_w + 1;
    return 0;
}

int oracle_conv_out_dims(const oconv_t *d, int64_t *oh, int64_t *ow)
{
    return conv_out_dims(d, oh, ow);
}

static double *widen_all(const omat_t *m)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)m->rows * (size_t)m->cols);
    if (p) widen_op_rows(m, 0, m->rows, NULL, m->cols, p);
    return p;
}

/*
 * Forward: out[n][k][oh][ow] = alpha * sum_c sum_r sum_s X[n,c,oh*sh+r-ph,ow*sw+s-pw]*F[k,c,r,s]
 *                              + beta * Y[n,k,oh,ow]; out-of-range input coordinates add 0.
 * Only the images sel[0..nsel) are computed (sel == NULL: all, nsel == n); out is
 * nsel x (K*OH*OW) fp64.
 */
int oracle_conv_fwd(const oconv_t *d, double alpha, const omat_t *X, const omat_t *F, double beta,
                    const omat_t *Y, int64_t nsel, const int64_t *sel, double *out)
{
    int64_t OH, OW;
    if (conv_out_dims(d, &OH, &OW)) return -1;
    int64_t chw = (int64_t)d->c * d->h * d->w, crs = (int64_t)d->c * d->r * d->s;
    int64_t kow = (int64_t)d->k * OH * OW;
    if (X->rows != d->n || X->cols != chw || F->rows != d->k || F->cols != crs) return -1;
    if (Y && (Y->rows != d->n || Y->cols != kow)) return -1;
    if (!Y && beta != 0.0) return -2;
    if (!sel && nsel != d->n) return -4;
    double *x = NULL, *f = NULL;
    if (alpha != 0.0) {
        x = widen_all(X);
        f = widen_all(F);
        if (!x || !f) { free(x); free(f); return -5; }
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t q = 0; q < nsel; ++q) {
        for (int64_t k = 0; k < d->k; ++k) {
            int64_t n = sel ? sel[q] : q;
            double *plane = out + (q * d->k + k) * OH * OW;
            for (int64_t t = 0; t < OH * OW; ++t) plane[t] = 0.0;
            if (alpha != 0.0) {
                for (int64_t c = 0; c < d->c; ++c)
                    for (int64_t r = 0; r < d->r; ++r)
                        for (int64_t s = 0; s < d->s; ++s) {
                            double w = f[k * crs + (c * d->r + r) * d->s + s];
                            for (int64_t oh = 0; oh < OH; ++oh) {
                                int64_t ih = oh * d->stride_h + r - d->pad_h;
                                if (ih < 0 || ih >= d->h) continue;
                                const double *xrow = x + n * chw + (c * d->h + ih) * d->w;
                                for (int64_t ow = 0; ow < OW; ++ow) {
                                    int64_t iw = ow * d->stride_w + s - d->pad_w;
                                    if (iw < 0 || iw >= d->w) continue;
                                    plane[oh * OW + ow] += xrow[iw] * w;
                                }
                            }
                        }
                for (int64_t t = 0; t < OH * OW; ++t) plane[t] *= alpha;
            }
            if (beta != 0.0)
                for (int64_t t = 0; t < OH * OW; ++t)
                    plane[t] += beta * mat_get(Y, n, k * OH * OW + t);
        }
    }
    free(x);
    free(f);
    return 0;
}

/*
 * Weight gradient: out[k][c][r][s] = alpha * sum_n sum_oh sum_ow dY[n,k,oh,ow] *
 *                  X[n,c,oh*sh+r-ph,ow*sw+s-pw] + beta * dF[k,c,r,s].
 * Only the filters sel[0..nsel) (values of k) are computed; out is nsel x (C*R*S) fp64.
 */
int oracle_conv_bwd_filter(const oconv_t *d, double alpha, const omat_t *X, const omat_t *dY,
                           double beta, const omat_t *dF, int64_t nsel, const int64_t *sel,
                           double *out)
{
    int64_t OH, OW;
    if (conv_out_dims(d, &OH, &OW)) return -1;
    int64_t chw = (int64_t)d->c * d->h * d->w, crs = (int64_t)d->c * d->r * d->s;
    int64_t kow = (int64_t)d->k * OH * OW;
    if (X->rows != d->n || X->cols != chw || dY->rows != d->n || dY->cols != kow) return -1;
    if (dF && (dF->rows != d->k || dF->cols != crs)) return -1;
    if (!dF && beta != 0.0) return -2;
    if (!sel && nsel != d->k) return -4;
    double *x = NULL, *g = NULL;
    if (alpha != 0.0) {
        x = widen_all(X);
        g = widen_all(dY);
        if (!x || !g) { free(x); free(g); return -5; }
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t q = 0; q < nsel; ++q) {
        for (int64_t c = 0; c < d->c; ++c) {
            int64_t k = sel ? sel[q] : q;
            for (int64_t r = 0; r < d->r; ++r)
                for (int64_t s = 0; s < d->s; ++s) {
                    double acc = 0.0;
                    if (alpha != 0.0) {
                        for (int64_t n = 0; n < d->n; ++n)
                            for (int64_t oh = 0; oh < OH; ++oh) {
                                int64_t ih = oh * d->stride_h + r - d->pad_h;
                                if (ih < 0 || ih >= d->h) continue;
                                const double *xrow = x + n * chw + (c * d->h + ih) * d->w;
                                const double *grow = g + n * kow + (k * OH + oh) * OW;
                                for (int64_t ow = 0; ow < OW; ++ow) {
                                    int64_t iw = ow * d->stride_w + s - d->pad_w;
                                    if (iw < 0 || iw >= d->w) continue;
                                    acc += grow[ow] * xrow[iw];
                                }
                            }
                        acc *= alpha;
                    }
                    int64_t col = (c * d->r + r) * d->s + s;
                    if (beta != 0.0) acc += beta * mat_get(dF, k, col);
                    out[q * crs + col] = acc;
                }
        }
    }
    free(x);
    free(g);
    return 0;
}

/*
 * Data gradient: out[n][c][h][w] = alpha * sum_k sum_r sum_s dY[n,k,oh,ow] * F[k,c,r,s]
 *                over those (oh,ow) with oh*sh + r - ph == h and ow*sw + s - pw == w,
 *                + beta * dX[n,c,h,w].
 * Written as the scatter that is the adjoint of the forward loops.  Only images sel[0..nsel).
 */
int oracle_conv_bwd_data(const oconv_t *d, double alpha, const omat_t *dY, const omat_t *F,
                         double beta, const omat_t *dX, int64_t nsel, const int64_t *sel,
                         double *out)
{
    int64_t OH, OW;
    if (conv_out_dims(d, &OH, &OW)) return -1;
    int64_t chw = (int64_t)d->c * d->h * d->w, crs = (int64_t)d->c * d->r * d->s;
    int64_t kow = (int64_t)d->k * OH * OW;
    if (dY->rows != d->n || dY->cols != kow || F->rows != d->k || F->cols != crs) return -1;
    if (dX && (dX->rows != d->n || dX->cols != chw)) return -1;
    if (!dX && beta != 0.0) return -2;
    if (!sel && nsel != d->n) return -4;
    double *g = NULL, *f = NULL;
    if (alpha != 0.0) {
        g = widen_all(dY);
        f = widen_all(F);
        if (!g || !f) { free(g); free(f); return -5; }
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t q = 0; q < nsel; ++q) {
        for (int64_t c = 0; c < d->c; ++c) {
            int64_t n = sel ? sel[q] : q;
            double *plane = out + q * chw + c * d->h * d->w;
            for (int64_t t = 0; t < (int64_t)d->h * d->w; ++t) plane[t] = 0.0;
            if (alpha != 0.0) {
                for (int64_t k = 0; k < d->k; ++k)
                    for (int64_t r = 0; r < d->r; ++r)
                        for (int64_t s = 0; s < d->s; ++s) {
                            double w = f[k * crs + (c * d->r + r) * d->s + s];
                            for (int64_t oh = 0; oh < OH; ++oh) {
                                int64_t ih = oh * d->stride_h + r - d->pad_h;
                                if (ih < 0 || ih >= d->h) continue;
                                const double *grow = g + n * kow + (k * OH + oh) * OW;
                                for (int64_t ow = 0; ow < OW; ++ow) {
                                    int64_t iw = ow * d->stride_w + s - d->pad_w;
                                    if (iw < 0 || iw >= d->w) continue;
                                    plane[ih * d->w + iw] += grow[ow] * w;
                                }
                            }
                        }
                for (int64_t t = 0; t < (int64_t)d->h * d->w; ++t) plane[t] *= alpha;
            }
            if (beta != 0.0)
                for (int64_t t = 0; t < (int64_t)d->h * d->w; ++t)
                    plane[t] += beta * mat_get(dX, n, c * d->h * d->w + t);
        }
    }
    free(g);
    free(f);
    return 0;
}
