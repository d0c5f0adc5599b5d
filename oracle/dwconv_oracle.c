/*
 * CPU oracle for the three passes of a depthwise convolution layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct checker
 * that the GPU library is compared against.  It shares no code with the HIP
 * path and must never be called from it: only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load it.
 *
 * What is computed (paper Section II "depthwise convolution": one K x K filter
 * per input channel, an M-channel input giving an M-channel output; Section
 * III-A: the per-channel product w(i) . C(i) of a filter vector with the
 * im2col matrix of the same channel; Eq. 3 forward, Eq. 4 weight gradient that
 * keeps only the block-diagonal entries).  The refactorised dense convolution
 * of the paper reaches exactly this result (the off-diagonal zeros contribute
 * nothing), so the oracle is the plain definition written as loop nests:
 *
 *   fwd        y[n,o,oh,ow]  = sum_{kh,kw} w[o,kh,kw] * x[n,o/m,oh*s-p+kh,ow*s-p+kw]
 *   bwd_data   dx[n,c,ih,iw] = sum over every (q,oh,ow,kh,kw) whose tap lands on (ih,iw)
 *                              of w[c*m+q,kh,kw] * dy[n,c*m+q,oh,ow]
 *   bwd_filter dw[o,kh,kw]   = sum_{n,oh,ow} dy[n,o,oh,ow] * x[n,o/m,oh*s-p+kh,ow*s-p+kw]
 *
 * with x read as zero outside [0,H) x [0,W), cross-correlation (no filter
 * flip: the paper computes W . im2col(X)), symmetric zero padding p, output
 * size floor((H+2p-K)/s)+1, batch gradient summed without 1/N, no bias.
 * All arithmetic is fp64.  Callers pass fp64 arrays (fp32 / bf16 test inputs
 * are widened exactly by the caller).
 *
 * Layouts: layout 0 = NCHW (x [N,C,H,W], y [N,O,Ho,Wo], w [O,K,K]);
 *          layout 1 = NHWC (x [N,H,W,C], y [N,Ho,Wo,O], w [K,K,O]).
 *
 * nthreads > 1 splits the outermost loop (images, or output channels for
 * bwd_filter) over OpenMP threads; the loop nest itself is unchanged and no
 * two threads write the same element.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t N, C, H, W;
    int32_t K, stride, pad, mult;
    int32_t layout; /* 0 NCHW, 1 NHWC */
} oracle_desc;

static int out_dim(int in, int K, int s, int p)
{
    int span = in + 2 * p - K;
    if (span < 0) return 0;
    return span / s + 1;
}

/* element offset of (n, ch, h, w) in a tensor of CH channels and HH x WW pixels */
static size_t at(int layout, int CH, int HH, int WW, int n, int ch, int h, int w)
{
    if (layout == 0)
        return (((size_t)n * CH + ch) * HH + h) * WW + w;
    return (((size_t)n * HH + h) * WW + w) * CH + ch;
}

/* element offset of filter tap (o, kh, kw) */
static size_t wat(int layout, int O, int K, int o, int kh, int kw)
{
    if (layout == 0)
        return ((size_t)o * K + kh) * K + kw;
    return ((size_t)kh * K + kw) * O + o;
}

int oracle_out_dims(const oracle_desc *d, int32_t *Ho, int32_t *Wo)
{
    if (!d || d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 ||
        d->stride < 1 || d->pad < 0 || d->mult < 1 || d->layout < 0 || d->layout > 1)
        return -1;
    int ho = out_dim(d->H, d->K, d->stride, d->pad);
    int wo = out_dim(d->W, d->K, d->stride, d->pad);
    if (ho < 1 || wo < 1) return -1;
    if (Ho) *Ho = ho;
    if (Wo) *Wo = wo;
    return 0;
}

static void set_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
}

int oracle_threads_available(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* Forward (Section III-A, z(i) = w(i) . C(i); Eq. 3). */
int oracle_dwconv_fwd(const oracle_desc *d, const double *x, const double *w, double *y,
                      int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_out_dims(d, &Ho, &Wo) || !x || !w || !y) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              m = d->mult, L = d->layout, O = C * m;
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int kh = 0; kh < K; ++kh)
                        for (int kw = 0; kw < K; ++kw) {
                            int ih = oh * s - p + kh, iw = ow * s - p + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += w[wat(L, O, K, o, kh, kw)] * x[at(L, C, H, W, n, o / m, ih, iw)];
                        }
                    y[at(L, O, Ho, Wo, n, o, oh, ow)] = acc;
                }
    return 0;
}

/* Backward-data: the input gradient of the forward pass above (Section III-A,
 * "during backward propagation"); written as the scatter that transposes the
 * forward gather, image by image. */
int oracle_dwconv_bwd_data(const oracle_desc *d, const double *dy, const double *w, double *dx,
                           int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_out_dims(d, &Ho, &Wo) || !dy || !w || !dx) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              m = d->mult, L = d->layout, O = C * m;
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double g = dy[at(L, O, Ho, Wo, n, o, oh, ow)];
                    for (int kh = 0; kh < K; ++kh)
                        for (int kw = 0; kw < K; ++kw) {
                            int ih = oh * s - p + kh, iw = ow * s - p + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            dx[at(L, C, H, W, n, o / m, ih, iw)] += w[wat(L, O, K, o, kh, kw)] * g;
                        }
                }
    return 0;
}

/* Backward-filter: per-channel weight gradient, the diagonal blocks that Eq. 4
 * keeps; a sum over the batch and every output pixel. */
int oracle_dwconv_bwd_filter(const oracle_desc *d, const double *x, const double *dy, double *dw,
                             int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_out_dims(d, &Ho, &Wo) || !x || !dy || !dw) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              m = d->mult, L = d->layout, O = C * m;
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; ++o)
        for (int kh = 0; kh < K; ++kh)
            for (int kw = 0; kw < K; ++kw) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int oh = 0; oh < Ho; ++oh)
                        for (int ow = 0; ow < Wo; ++ow) {
                            int ih = oh * s - p + kh, iw = ow * s - p + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += dy[at(L, O, Ho, Wo, n, o, oh, ow)] *
                                   x[at(L, C, H, W, n, o / m, ih, iw)];
                        }
                dw[wat(L, O, K, o, kh, kw)] = acc;
            }
    return 0;
}
