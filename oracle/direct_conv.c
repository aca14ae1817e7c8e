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
 * maps, n input width, k kernel width, no = n - k + 1 output width.  The paper
 * writes square maps and kernels only to keep its notation short; the sums below
 * carry a height and a width (nh x nw inputs, kh x kw kernels,
 * noh = nh - kh + 1, now = nw - kw + 1), which is the same definition per axis.  The paper's
 * "*" is read as the cross-correlation used by neural-network layers (stride 1,
 * no spatial padding); bprop is then the adjoint of fprop with respect to x and
 * accGrad the adjoint with respect to w.
 *
 * Layouts (row-major, contiguous, double):
 *   x [S][f ][nh ][nw ]     w [fo][f][kh][kw]
 *   y [S][fo][noh][now]     g = dL/dy like y,  dx like x,  dw like w
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

/* Eq. (1):  y[s,j,p,q] = sum_i sum_{a<kh,b<kw} x[s,i,p+a,q+b] * w[j,i,a,b],  0 <= p < noh, 0 <= q < now. */
void oracle_fprop(const double *x, const double *w, double *out,
                  int S, int f, int fo, int nh, int nw, int kh, int kw,
                  const long *units, long nunits)
{
    const int noh = nh - kh + 1, now = nw - kw + 1;
    const long total = units ? nunits : (long)S * fo;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int s = (int)(unit / fo), j = (int)(unit % fo);
        double *ymap = out + (size_t)u * noh * now;
        memset(ymap, 0, sizeof(double) * (size_t)noh * now);
        for (int i = 0; i < f; ++i)
            for (int a = 0; a < kh; ++a)
                for (int b = 0; b < kw; ++b) {
                    const double wv = w[IDX4(j, fo, i, f, a, kh, b, kw)];
                    for (int p = 0; p < noh; ++p) {
                        const double *xrow = x + IDX4(s, S, i, f, p + a, nh, b, nw);
                        double *yrow = ymap + (size_t)p * now;
                        for (int q = 0; q < now; ++q)
                            yrow[q] += xrow[q] * wv;
                    }
                }
    }
}

/* Eq. (2) with the sum over output maps written out:
 *   dx[s,i,p,q] = sum_j sum_{a<kh,b<kw} g[s,j,p-a,q-b] * w[j,i,a,b],  0 <= p < nh, 0 <= q < nw,
 * where g is taken as zero outside [0,noh) x [0,now). */
void oracle_bprop(const double *g, const double *w, double *out,
                  int S, int f, int fo, int nh, int nw, int kh, int kw,
                  const long *units, long nunits)
{
    const int noh = nh - kh + 1, now = nw - kw + 1;
    const long total = units ? nunits : (long)S * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int s = (int)(unit / f), i = (int)(unit % f);
        double *dmap = out + (size_t)u * nh * nw;
        memset(dmap, 0, sizeof(double) * (size_t)nh * nw);
        for (int j = 0; j < fo; ++j)
            for (int a = 0; a < kh; ++a)
                for (int b = 0; b < kw; ++b) {
                    const double wv = w[IDX4(j, fo, i, f, a, kh, b, kw)];
                    /* p - a in [0,noh)  <=>  p in [a, a+noh) */
                    for (int p = a; p < a + noh; ++p) {
                        const double *grow = g + IDX4(s, S, j, fo, p - a, noh, 0, now);
                        double *drow = dmap + (size_t)p * nw + b;
                        for (int q = 0; q < now; ++q)      /* q here is (q_out - b) */
                            drow[q] += grow[q] * wv;
                    }
                }
    }
}

/* Eq. (3) with the sums over the minibatch and over positions written out:
 *   dw[j,i,a,b] = sum_s sum_{p<noh,q<now} g[s,j,p,q] * x[s,i,p+a,q+b],  0 <= a < kh, 0 <= b < kw. */
void oracle_accgrad(const double *g, const double *x, double *out,
                    int S, int f, int fo, int nh, int nw, int kh, int kw,
                    const long *units, long nunits)
{
    const int noh = nh - kh + 1, now = nw - kw + 1;
    const long total = units ? nunits : (long)fo * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < total; ++u) {
        const long unit = units ? units[u] : u;
        const int j = (int)(unit / f), i = (int)(unit % f);
        double *kmap = out + (size_t)u * kh * kw;
        for (int a = 0; a < kh; ++a)
            for (int b = 0; b < kw; ++b) {
                double acc = 0.0;
                for (int s = 0; s < S; ++s)
                    for (int p = 0; p < noh; ++p) {
                        const double *grow = g + IDX4(s, S, j, fo, p, noh, 0, now);
                        const double *xrow = x + IDX4(s, S, i, f, p + a, nh, b, nw);
                        for (int q = 0; q < now; ++q)
                            acc += grow[q] * xrow[q];
                    }
                kmap[a * kw + b] = acc;
            }
    }
}
