// Generic fallback kernels: correct for any K, stride, pad and channel multiplier, both layouts,
// both storage types.  One thread per output element; not tuned.  Also holds the second stage of
// the filter-gradient reduction, which every bwd_filter variant shares.
#include "kernels.hpp"

namespace dwc {

template <int LAYOUT>
__device__ __forceinline__ int at(int CH, int HH, int WW, int n, int ch, int h, int w)
{
    if (LAYOUT == LAYOUT_NCHW) return ((n * CH + ch) * HH + h) * WW + w;
    return ((n * HH + h) * WW + w) * CH + ch;
}
template <int LAYOUT>
__device__ __forceinline__ int wat(int O, int K, int o, int kh, int kw)
{
    if (LAYOUT == LAYOUT_NCHW) return (o * K + kh) * K + kw;
    return (kh * K + kw) * O + o;
}
// Decompose a flat element index of a [N,CH,HH,WW] / [N,HH,WW,CH] tensor.
template <int LAYOUT>
__device__ __forceinline__ void unflat(int idx, int CH, int HH, int WW, int &n, int &ch, int &h, int &w)
{
    if (LAYOUT == LAYOUT_NCHW) {
        w = idx % WW; idx /= WW; h = idx % HH; idx /= HH; ch = idx % CH; n = idx / CH;
    } else {
        ch = idx % CH; idx /= CH; w = idx % WW; idx /= WW; h = idx % HH; n = idx / HH;
    }
}

template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void k_generic_fwd(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                     T *__restrict__ y, int total)
{
    const unsigned uidx = blockIdx.x * 256u + threadIdx.x;   // the last block may reach past 2^31
    if (uidx >= (unsigned)total) return;
    int idx = (int)uidx;
    int n, o, oh, ow;
    unflat<LAYOUT>(idx, g.O, g.Ho, g.Wo, n, o, oh, ow);
    const int c = o / g.m;
    float acc = 0.f;
    for (int kh = 0; kh < g.K; ++kh) {
        int ih = oh * g.s - g.p + kh;
        if (ih < 0 || ih >= g.H) continue;
        for (int kw = 0; kw < g.K; ++kw) {
            int iw = ow * g.s - g.p + kw;
            if (iw < 0 || iw >= g.W) continue;
            acc = fmaf(ldf(w + wat<LAYOUT>(g.O, g.K, o, kh, kw)), ldf(x + at<LAYOUT>(g.C, g.H, g.W, n, c, ih, iw)), acc);
        }
    }
    stf(y + idx, acc);
}

template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void k_generic_bwd_data(Geom g, const T *__restrict__ dy, const T *__restrict__ w,
                                                          T *__restrict__ dx, int total)
{
    const unsigned uidx = blockIdx.x * 256u + threadIdx.x;   // the last block may reach past 2^31
    if (uidx >= (unsigned)total) return;
    int idx = (int)uidx;
    int n, c, ih, iw;
    unflat<LAYOUT>(idx, g.C, g.H, g.W, n, c, ih, iw);
    float acc = 0.f;
    for (int q = 0; q < g.m; ++q) {
        const int o = c * g.m + q;
        for (int kh = 0; kh < g.K; ++kh) {
            int th = ih + g.p - kh;
            if (th < 0 || th % g.s != 0) continue;
            int oh = th / g.s;
            if (oh >= g.Ho) continue;
            for (int kw = 0; kw < g.K; ++kw) {
                int tw = iw + g.p - kw;
                if (tw < 0 || tw % g.s != 0) continue;
                int ow = tw / g.s;
                if (ow >= g.Wo) continue;
                acc = fmaf(ldf(w + wat<LAYOUT>(g.O, g.K, o, kh, kw)),
                           ldf(dy + at<LAYOUT>(g.O, g.Ho, g.Wo, n, o, oh, ow)), acc);
            }
        }
    }
    stf(dx + idx, acc);
}

// Stage 1, NCHW: block (tap j = (o*K+kh)*K+kw, part).  Threads stride over the pixels
// (n, oh, ow) of the part with ow fastest; wavefront butterfly, then LDS across the 4 waves.
template <typename T>
__global__ __launch_bounds__(256) void k_generic_bwd_filter_nchw(Geom g, const T *__restrict__ x,
                                                                 const T *__restrict__ dy, float *__restrict__ ws,
                                                                 int parts, int per_part)
{
    __shared__ float red[4];
    const int j = blockIdx.x, part = blockIdx.y;
    const int kw = j % g.K, kh = (j / g.K) % g.K, o = j / (g.K * g.K);
    const int c = o / g.m;
    const int npix = g.N * g.Ho * g.Wo;
    const int lo = part * per_part, hi = min(npix, lo + per_part);
    float acc = 0.f;
    for (int pix = lo + (int)threadIdx.x; pix < hi; pix += 256) {
        int ow = pix % g.Wo, t = pix / g.Wo, oh = t % g.Ho, n = t / g.Ho;
        int ih = oh * g.s - g.p + kh, iw = ow * g.s - g.p + kw;
        if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
        acc = fmaf(ldf(dy + at<LAYOUT_NCHW>(g.O, g.Ho, g.Wo, n, o, oh, ow)),
                   ldf(x + at<LAYOUT_NCHW>(g.C, g.H, g.W, n, c, ih, iw)), acc);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) ws[(size_t)part * (g.O * g.K * g.K) + j] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Stage 1, NHWC: block (tile of 64 output channels, tap (kh,kw), part).  Lane = channel, the 4
// waves stride over pixels; LDS across the waves.
template <typename T>
__global__ __launch_bounds__(256) void k_generic_bwd_filter_nhwc(Geom g, const T *__restrict__ x,
                                                                 const T *__restrict__ dy, float *__restrict__ ws,
                                                                 int parts, int per_part)
{
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int o = blockIdx.x * 64 + lane;
    const int tap = blockIdx.y, part = blockIdx.z;
    const int kw = tap % g.K, kh = tap / g.K;
    const int npix = g.N * g.Ho * g.Wo;
    const int lo = part * per_part, hi = min(npix, lo + per_part);
    float acc = 0.f;
    if (o < g.O) {
        const int c = o / g.m;
        for (int pix = lo + wv; pix < hi; pix += 4) {
            int ow = pix % g.Wo, t = pix / g.Wo, oh = t % g.Ho, n = t / g.Ho;
            int ih = oh * g.s - g.p + kh, iw = ow * g.s - g.p + kw;
            if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
            acc = fmaf(ldf(dy + (size_t)pix * g.O + o), ldf(x + at<LAYOUT_NHWC>(g.C, g.H, g.W, n, c, ih, iw)), acc);
        }
    }
    red[wv][lane] = acc;
    __syncthreads();
    if (wv == 0 && o < g.O)
        ws[(size_t)part * (g.O * g.K * g.K) + tap * g.O + o] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

// Stage 2: dw[j] = sum_p ws[p*J + j].  A block owns JT consecutive j; PT = 256/JT threads per j
// take the partials p = r, r+PT, r+2PT, ... eight at a time.  All eight loads of a batch are issued
// before the first is used, also in the last, partly filled batch (clamped index, value dropped):
// the kernel is a few microseconds of pure load latency, so one latency per batch is what counts.
// The batch is added in a fixed tree, then the PT sub-sums in a fixed tree through LDS.
template <int JT>
__global__ __launch_bounds__(256) void k_reduce_partials(const float *__restrict__ ws, int parts, int J,
                                                         float *__restrict__ dw)
{
    constexpr int PT = 256 / JT;
    __shared__ float red[PT][JT + 1];
    const int jj = threadIdx.x % JT, r = threadIdx.x / JT;
    const int j = blockIdx.x * JT + jj;
    float acc = 0.f;
    if (j < J) {
        const float *p0 = ws + j;
        for (int p = r; p < parts; p += 8 * PT) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int q = p + i * PT;
                const float t = p0[(size_t)min(q, parts - 1) * J];
                v[i] = q < parts ? t : 0.f;
            }
            acc += ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        }
    }
    red[r][jj] = acc;
    __syncthreads();
    // tree over the PT sub-sums: thread (r, jj) adds red[r + half]
    for (int half = PT / 2; half >= 1; half >>= 1) {
        if (r < half) red[r][jj] += red[r + half][jj];
        __syncthreads();
    }
    if (r == 0 && j < J) dw[j] = red[0][jj];
}

// ---- host side --------------------------------------------------------------------------------

hipError_t generic_fwd(const Geom &g, int layout, int dtype, const void *x, const void *w, void *y, hipStream_t st)
{
    const int total = g.N * g.O * g.Ho * g.Wo;
    dim3 grid((unsigned)(((long long)total + 255) / 256)), block(256);
#define LAUNCH(T, L) hipLaunchKernelGGL((k_generic_fwd<T, L>), grid, block, 0, st, g, (const T *)x, (const T *)w, (T *)y, total)
    if (dtype == DT_F32) { if (layout == LAYOUT_NCHW) LAUNCH(float, LAYOUT_NCHW); else LAUNCH(float, LAYOUT_NHWC); }
    else                 { if (layout == LAYOUT_NCHW) LAUNCH(bf16_t, LAYOUT_NCHW); else LAUNCH(bf16_t, LAYOUT_NHWC); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t generic_bwd_data(const Geom &g, int layout, int dtype, const void *dy, const void *w, void *dx, hipStream_t st)
{
    const int total = g.N * g.C * g.H * g.W;
    dim3 grid((unsigned)(((long long)total + 255) / 256)), block(256);
#define LAUNCH(T, L) hipLaunchKernelGGL((k_generic_bwd_data<T, L>), grid, block, 0, st, g, (const T *)dy, (const T *)w, (T *)dx, total)
    if (dtype == DT_F32) { if (layout == LAYOUT_NCHW) LAUNCH(float, LAYOUT_NCHW); else LAUNCH(float, LAYOUT_NHWC); }
    else                 { if (layout == LAYOUT_NCHW) LAUNCH(bf16_t, LAYOUT_NCHW); else LAUNCH(bf16_t, LAYOUT_NHWC); }
#undef LAUNCH
    return hipGetLastError();
}

int generic_bwd_filter_parts(const Geom &g)
{
    // about 8192 pixels per part, at most 64 parts, and never more than 32 MiB of partials
    long long npix = (long long)g.N * g.Ho * g.Wo;
    long long parts = (npix + 8191) / 8192;
    if (parts > 64) parts = 64;
    long long J = (long long)g.O * g.K * g.K;
    while (parts > 1 && parts * J * 4 > (32ll << 20)) parts >>= 1;
    if (parts < 1) parts = 1;
    return (int)parts;
}

hipError_t generic_bwd_filter(const Geom &g, int layout, int dtype, const void *x, const void *dy, float *ws,
                              int parts, hipStream_t st)
{
    const int npix = g.N * g.Ho * g.Wo;
    const int per_part = (npix + parts - 1) / parts;
    if (layout == LAYOUT_NCHW) {
        dim3 grid(g.O * g.K * g.K, parts), block(256);
        if (dtype == DT_F32)
            hipLaunchKernelGGL(k_generic_bwd_filter_nchw<float>, grid, block, 0, st, g, (const float *)x, (const float *)dy, ws, parts, per_part);
        else
            hipLaunchKernelGGL(k_generic_bwd_filter_nchw<bf16_t>, grid, block, 0, st, g, (const bf16_t *)x, (const bf16_t *)dy, ws, parts, per_part);
    } else {
        dim3 grid((g.O + 63) / 64, g.K * g.K, parts), block(256);
        if (dtype == DT_F32)
            hipLaunchKernelGGL(k_generic_bwd_filter_nhwc<float>, grid, block, 0, st, g, (const float *)x, (const float *)dy, ws, parts, per_part);
        else
            hipLaunchKernelGGL(k_generic_bwd_filter_nhwc<bf16_t>, grid, block, 0, st, g, (const bf16_t *)x, (const bf16_t *)dy, ws, parts, per_part);
    }
    return hipGetLastError();
}

hipError_t reduce_partials(const float *ws, int parts, int J, float *dw, hipStream_t st)
{
    // threads per output chosen so that one batch of eight loads per thread covers the partials
    // (PT = 256/JT about parts/8), but enough blocks to spread small J over the chip
    int jt = 4;
    while (jt < 64 && (256 / jt) * 8 > parts && (J + 2 * jt - 1) / (2 * jt) >= 8) jt *= 2;
#define GO(JT) hipLaunchKernelGGL(k_reduce_partials<JT>, dim3((J + JT - 1) / JT), dim3(256), 0, st, ws, parts, J, dw)
    switch (jt) {
    case 4: GO(4); break;
    case 8: GO(8); break;
    case 16: GO(16); break;
    case 32: GO(32); break;
    default: GO(64); break;
    }
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
