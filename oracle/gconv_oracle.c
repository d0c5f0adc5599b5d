/*
 * CPU oracle for the three passes of a group convolution layer (more than one
 * channel per group).
 *
 * TEST INFRASTRUCTURE ONLY.  The slow, obviously-correct checker that the GPU
 * library's group-convolution entry points are compared against.  It shares no
 * code with the HIP path and must never be called from it: only tests, the
 * smoke check and the cpu_baseline leg of the benchmark may load it.
 *
 * What is computed (paper Section V-B, extensibility: a depthwise convolution
 * is the group convolution whose number of groups equals the number of
 * channels; in the general case the 0/1 mask of Section III-A, Eq. 2 keeps,
 * for every output channel, the K x K blocks of all input channels of its own
 * group instead of the one block on the diagonal).  The C input channels and
 * the O output channels are split into G groups of Cg = C/G and Og = O/G
 * consecutive channels; output channel o belongs to group o / Og and sees the
 * input channels (o / Og) * Cg + ci, ci < Cg, only:
 *
 *   fwd        y[n,o,oh,ow]     = sum_{ci,kh,kw} w[o,ci,kh,kw] * x[n,(o/Og)*Cg+ci,oh*s-p+kh,ow*s-p+kw]
 *   bwd_data   dx[n,c,ih,iw]    = sum over every (o,oh,ow,kh,kw) of the group of c whose tap lands
 *                                 on (ih,iw) of w[o,c%Cg,kh,kw] * dy[n,o,oh,ow]
 *   bwd_filter dw[o,ci,kh,kw]   = sum_{n,oh,ow} dy[n,o,oh,ow] * x[n,(o/Og)*Cg+ci,oh*s-p+kh,ow*s-p+kw]
 *
 * with the conventions of the depthwise oracle: x is zero outside the image,
 * cross-correlation, symmetric padding, output size floor((H+2p-K)/s)+1, the
 * batch gradient a plain sum, no bias, fp64 throughout.
 *
 * Layouts: layout 0 = NCHW (x [N,C,H,W], y [N,O,Ho,Wo], w [O,Cg,K,K]);
 *          layout 1 = NHWC (x [N,H,W,C], y [N,Ho,Wo,O], w [K,K,Cg,O]).
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t N, C, H, W;
    int32_t K, stride, pad;
    int32_t groups, O;
    int32_t layout; /* 0 NCHW, 1 NHWC */
} oracle_gdesc;

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

/* element offset of filter entry (o, ci, kh, kw) */
static size_t wat(int layout, int O, int Cg, int K, int o, int ci, int kh, int kw)
{
    if (layout == 0)
        return (((size_t)o * Cg + ci) * K + kh) * K + kw;
    return (((size_t)kh * K + kw) * Cg + ci) * O + o;
}

int oracle_gconv_out_dims(const oracle_gdesc *d, int32_t *Ho, int32_t *Wo)
{
    if (!d || d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->stride < 1 ||
        d->pad < 0 || d->groups < 1 || d->O < 1 || d->layout < 0 || d->layout > 1)
        return -1;
    if (d->C % d->groups != 0 || d->O % d->groups != 0) return -1;
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

/* Forward: every output channel gathers from the Cg input channels of its group. */
int oracle_gconv_fwd(const oracle_gdesc *d, const double *x, const double *w, double *y, int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_gconv_out_dims(d, &Ho, &Wo) || !x || !w || !y) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              L = d->layout, O = d->O, Cg = C / d->groups, Og = O / d->groups;
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            const int c0 = (o / Og) * Cg; /* first input channel of the group of o */
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int ci = 0; ci < Cg; ++ci)
                        for (int kh = 0; kh < K; ++kh)
                            for (int kw = 0; kw < K; ++kw) {
                                int ih = oh * s - p + kh, iw = ow * s - p + kw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += w[wat(L, O, Cg, K, o, ci, kh, kw)] * x[at(L, C, H, W, n, c0 + ci, ih, iw)];
                            }
                    y[at(L, O, Ho, Wo, n, o, oh, ow)] = acc;
                }
        }
    return 0;
}

/* Backward-data: the scatter that transposes the forward gather, image by image. */
int oracle_gconv_bwd_data(const oracle_gdesc *d, const double *dy, const double *w, double *dx, int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_gconv_out_dims(d, &Ho, &Wo) || !dy || !w || !dx) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              L = d->layout, O = d->O, Cg = C / d->groups, Og = O / d->groups;
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            const int c0 = (o / Og) * Cg;
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double g = dy[at(L, O, Ho, Wo, n, o, oh, ow)];
                    for (int ci = 0; ci < Cg; ++ci)
                        for (int kh = 0; kh < K; ++kh)
                            for (int kw = 0; kw < K; ++kw) {
                                int ih = oh * s - p + kh, iw = ow * s - p + kw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                dx[at(L, C, H, W, n, c0 + ci, ih, iw)] += w[wat(L, O, Cg, K, o, ci, kh, kw)] * g;
                            }
                }
        }
    return 0;
}

/* Backward-filter: the entries of the dense weight gradient that the group mask keeps. */
int oracle_gconv_bwd_filter(const oracle_gdesc *d, const double *x, const double *dy, double *dw, int nthreads)
{
    int32_t Ho, Wo;
    if (oracle_gconv_out_dims(d, &Ho, &Wo) || !x || !dy || !dw) return -1;
    const int N = d->N, C = d->C, H = d->H, W = d->W, K = d->K, s = d->stride, p = d->pad,
              L = d->layout, O = d->O, Cg = C / d->groups, Og = O / d->groups;
    set_threads(nthreads);
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; ++o) {
        const int c0 = (o / Og) * Cg;
        for (int ci = 0; ci < Cg; ++ci)
            for (int kh = 0; kh < K; ++kh)
                for (int kw = 0; kw < K; ++kw) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int oh = 0; oh < Ho; ++oh)
                            for (int ow = 0; ow < Wo; ++ow) {
                                int ih = oh * s - p + kh, iw = ow * s - p + kw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += dy[at(L, O, Ho, Wo, n, o, oh, ow)] * x[at(L, C, H, W, n, c0 + ci, ih, iw)];
                            }
                    dw[wat(L, O, Cg, K, o, ci, kh, kw)] = acc;
                }
    }
    return 0;
}
