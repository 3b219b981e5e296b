/*
 * CPU oracle for the SpMM / sparse 3x3 convolution hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or
 * import this file; it exists so the HIP kernels can be checked against a
 * plain, slow, obviously correct statement of what they must compute.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * What is computed is the exact product: the method reaches it by leaving out
 * the terms of the zero elements of A and changes nothing else (the
 * definition of Section 3.2, with Section 3.5's restriction to the nonzeros
 * of A), so the oracle is that definition written out, in double precision,
 * with no blocking, fusion or reordering.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * SpMM, Section 3.2 (Terminology): C[M,N] = A[M,K] * B[K,N], row-major, A
 * sparse and given as CSR.  For every output row, walk the row's nonzeros in
 * stored order and add val * B[col, :] into a double accumulator row.
 *   C[m,n] = sum_p vals[p] * B[col_idx[p], n],  p in [row_ptr[m], row_ptr[m+1])
 *   S[m,n] = sum_p |vals[p]| * |B[col_idx[p], n]|   (scale for error bounds)
 * An empty row gives +0.0.  S may be NULL.  threads <= 0: leave OpenMP default.
 * Rows are independent, so the OpenMP split over m does not change any sum.
 */
void oracle_spmm(int32_t M, int32_t K, int32_t N,
                 const int32_t *row_ptr, const int32_t *col_idx,
                 const double *vals, const double *B,
                 double *C, double *S, int32_t threads)
{
    (void)K;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 8)
    for (int32_t m = 0; m < M; ++m) {
        double *c = C + (size_t)m * N;
        double *s = S ? S + (size_t)m * N : NULL;
        for (int32_t n = 0; n < N; ++n) c[n] = 0.0;
        if (s) for (int32_t n = 0; n < N; ++n) s[n] = 0.0;
        for (int32_t p = row_ptr[m]; p < row_ptr[m + 1]; ++p) {
            const double a = vals[p];
            const double *b = B + (size_t)col_idx[p] * N;
            for (int32_t n = 0; n < N; ++n) c[n] += a * b[n];
            if (s) for (int32_t n = 0; n < N; ++n) s[n] += fabs(a) * fabs(b[n]);
        }
    }
}

/*
 * Sparse 3x3 convolution, Section 3.6: filter size 3x3, padding 1, stride 1,
 * cross-correlation (no filter flip), zero outside the image.  Written as the
 * direct loop nest over the DENSE zero-filled weight tensor, not through
 * im2col, so that it is independent of the lowering under test.
 *   Y[b,m,oh,ow] = sum_c sum_r sum_s W[m,c,r,s] * X[b,c,oh+r-1,ow+s-1]
 * W is [Cout,Cin,3,3], X is [batch,Cin,H,W], Y is [batch,Cout,H,W], all C order.
 */
void oracle_conv3x3(int32_t batch, int32_t Cin, int32_t Cout, int32_t H, int32_t Wd,
                    const double *W, const double *X, double *Y, double *S,
                    int32_t threads)
{
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
    for (int32_t b = 0; b < batch; ++b) {
#pragma omp parallel for schedule(dynamic, 4)
        for (int32_t m = 0; m < Cout; ++m) {
            for (int32_t oh = 0; oh < H; ++oh) {
                for (int32_t ow = 0; ow < Wd; ++ow) {
                    double acc = 0.0, sc = 0.0;
                    for (int32_t c = 0; c < Cin; ++c) {
                        for (int32_t r = 0; r < 3; ++r) {
                            for (int32_t s = 0; s < 3; ++s) {
                                const int32_t ih = oh + r - 1, iw = ow + s - 1;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                                const double w = W[(((size_t)m * Cin + c) * 3 + r) * 3 + s];
                                const double x = X[(((size_t)b * Cin + c) * H + ih) * Wd + iw];
                                acc += w * x;
                                sc += fabs(w) * fabs(x);
                            }
                        }
                    }
                    const size_t o = (((size_t)b * Cout + m) * H + oh) * Wd + ow;
                    Y[o] = acc;
                    if (S) S[o] = sc;
                }
            }
        }
    }
}

/*
 * Explicit im2col of Section 3.6: every receptive field becomes a column of
 * B, every filter a row of A.  Row index k = c*9 + r*3 + s (C-order
 * flattening of [Cin,3,3]); column index n = oh*W + ow.  Used only to
 * cross-check oracle_conv3x3 against oracle_spmm; the HIP path never builds it.
 * X is [Cin,H,W] (batch 1), Bcol is [9*Cin, H*W].
 */
void oracle_im2col3x3(int32_t Cin, int32_t H, int32_t Wd, const double *X, double *Bcol)
{
    const int32_t N = H * Wd;
    for (int32_t c = 0; c < Cin; ++c)
        for (int32_t r = 0; r < 3; ++r)
            for (int32_t s = 0; s < 3; ++s) {
                double *row = Bcol + (size_t)(c * 9 + r * 3 + s) * N;
                for (int32_t oh = 0; oh < H; ++oh)
                    for (int32_t ow = 0; ow < Wd; ++ow) {
                        const int32_t ih = oh + r - 1, iw = ow + s - 1;
                        const int inside = ih >= 0 && ih < H && iw >= 0 && iw < Wd;
                        row[oh * Wd + ow] = inside ? X[((size_t)c * H + ih) * Wd + iw] : 0.0;
                    }
            }
}

int32_t oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
