/*
 * Direct spatial-domain oracle for the three passes of one convolutional layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that
 * the GPU library is checked against.  It shares no code with the GPU path, is
 * never called by it, and contains no Fourier transform: the method under test
 * reaches exactly (up to rounding) the result of the direct sums below, so the
 * oracle is those sums written out.
 *
 * Notation (paper Sec. 2.1): S minibatch size, f input maps, fo (= f') output
 * maps, n input width, k kernel width, no = n - k + 1 output width.  The paper's
 * "*" is read as the cross-correlation used by neural-network layers (stride 1,
 * no spatial padding); bprop is then the adjoint of fprop with respect to x and
 * accGrad the adjoint with respect to w.
 *
 * Layouts (row-major, contiguous, double):
 *   x [S][f ][n ][n ]     w [fo][f][k][k]
 *   y [S][fo][no][no]     g = dL/dy like y,  dx like x,  dw like w
 *
 * Every routine can be restricted to a list of independent output units
 * (whole output maps) so that large layers can be spot-checked; units == NULL
 * means all of them.  Unit numbering: fprop (s*fo + j), bprop (s*f + i),
 * accGrad (j*f + i).  A restricted call writes only the listed maps, packed in
 * list order into `out` (nunits maps), so the caller needs no full-size buffer.
 *
 * OpenMP parallelises over output maps only; each map is summed by one thread
 * in a fixed order, so results do not depend on the thread count.
 */
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(a, A, b, B, c, C, d, D) ((((size_t)(a) * (B) + (b)) * (C) + (c)) * (D) + (d))

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. (1):  y[s,j,p,q] = sum_i sum_{a,b<k} x[s,i,p+a,q+b] * w[j,i,a,b],  0 <= p,q < no. */
void oracle_fprop(const double *x, const double *w, double *out,
                  int S, int f, int fo, int n, int k,
                  const long *units, long nunits)
{
    const int no = n - k + 1;
    const long total = units ? nunits : (long)S * fo;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int s = (int)(unit / fo), j = (int)(unit % fo);
        double *ymap = out + (size_t)u * no * no;
        memset(ymap, 0, sizeof(double) * (size_t)no * no);
        for (int i = 0; i < f; ++i)
            for (int a = 0; a < k; ++a)
                for (int b = 0; b < k; ++b) {
                    const double wv = w[IDX4(j, fo, i, f, a, k, b, k)];
                    for (int p = 0; p < no; ++p) {
                        const double *xrow = x + IDX4(s, S, i, f, p + a, n, b, n);
                        double *yrow = ymap + (size_t)p * no;
                        for (int q = 0; q < no; ++q)
                            yrow[q] += xrow[q] * wv;
                    }
                }
    }
}

/* Eq. (2) with the sum over output maps written out:
 *   dx[s,i,p,q] = sum_j sum_{a,b<k} g[s,j,p-a,q-b] * w[j,i,a,b],  0 <= p,q < n,
 * where g is taken as zero outside [0,no)^2. */
void oracle_bprop(const double *g, const double *w, double *out,
                  int S, int f, int fo, int n, int k,
                  const long *units, long nunits)
{
    const int no = n - k + 1;
    const long total = units ? nunits : (long)S * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int s = (int)(unit / f), i = (int)(unit % f);
        double *dmap = out + (size_t)u * n * n;
        memset(dmap, 0, sizeof(double) * (size_t)n * n);
        for (int j = 0; j < fo; ++j)
            for (int a = 0; a < k; ++a)
                for (int b = 0; b < k; ++b) {
                    const double wv = w[IDX4(j, fo, i, f, a, k, b, k)];
                    /* p - a in [0,no)  <=>  p in [a, a+no) */
                    for (int p = a; p < a + no; ++p) {
                        const double *grow = g + IDX4(s, S, j, fo, p - a, no, 0, no);
                        double *drow = dmap + (size_t)p * n + b;
                        for (int q = 0; q < no; ++q)      /* q here is (q_out - b) */
                            drow[q] += grow[q] * wv;
                    }
                }
    }
}

/* Eq. (3) with the sums over the minibatch and over positions written out:
 *   dw[j,i,a,b] = sum_s sum_{p,q<no} g[s,j,p,q] * x[s,i,p+a,q+b],  0 <= a,b < k. */
void oracle_accgrad(const double *g, const double *x, double *out,
                    int S, int f, int fo, int n, int k,
                    const long *units, long nunits)
{
    const int no = n - k + 1;
    const long total = units ? nunits : (long)fo * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int j = (int)(unit / f), i = (int)(unit % f);
        double *kmap = out + (size_t)u * k * k;
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b) {
                double acc = 0.0;
                for (int s = 0; s < S; ++s)
                    for (int p = 0; p < no; ++p) {
                        const double *grow = g + IDX4(s, S, j, fo, p, no, 0, no);
                        const double *xrow = x + IDX4(s, S, i, f, p + a, n, b, n);
                        for (int q = 0; q < no; ++q)
                            acc += grow[q] * xrow[q];
                    }
                kmap[a * k + b] = acc;
            }
    }
}
