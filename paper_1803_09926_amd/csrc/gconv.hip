// Group convolution behind the C ABI (gconv_* in include/dwconv.h): argument validation, variant
// selection, and the generic kernels that are correct for any K, stride, pad and group size in both
// layouts and storage types (one thread per output element; not tuned).  Groups of one input channel
// are the depthwise layer and run on its kernels.
#include "../../include/dwconv.h"
#include "gconv.hpp"

namespace dwc {

template <int LAYOUT>
__device__ __forceinline__ int gat(int CH, int HH, int WW, int n, int ch, int h, int w)
{
    if (LAYOUT == LAYOUT_NCHW) return ((n * CH + ch) * HH + h) * WW + w;
    return ((n * HH + h) * WW + w) * CH + ch;
}
// filter entry (o, ci, kh, kw): [O,Cg,K,K] or [K,K,Cg,O]
template <int LAYOUT>
__device__ __forceinline__ int gwat(const GGeom &g, int o, int ci, int kh, int kw)
{
    if (LAYOUT == LAYOUT_NCHW) return ((o * g.Cg + ci) * g.K + kh) * g.K + kw;
    return ((kh * g.K + kw) * g.Cg + ci) * g.O + o;
}
template <int LAYOUT>
__device__ __forceinline__ void gunflat(int idx, int CH, int HH, int WW, int &n, int &ch, int &h, int &w)
{
    if (LAYOUT == LAYOUT_NCHW) {
        w = idx % WW; idx /= WW; h = idx % HH; idx /= HH; ch = idx % CH; n = idx / CH;
    } else {
        ch = idx % CH; idx /= CH; w = idx % WW; idx /= WW; h = idx % HH; n = idx / HH;
    }
}

template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void k_gconv_generic_fwd(GGeom g, const T *__restrict__ x, const T *__restrict__ w,
                                                           T *__restrict__ y, int total)
{
    const unsigned uidx = blockIdx.x * 256u + threadIdx.x;   // the last block may reach past 2^31
    if (uidx >= (unsigned)total) return;
    int idx = (int)uidx;
    int n, o, oh, ow;
    gunflat<LAYOUT>(idx, g.O, g.Ho, g.Wo, n, o, oh, ow);
    const int c0 = (o / g.Og) * g.Cg;
    float acc = 0.f;
    for (int ci = 0; ci < g.Cg; ++ci)
        for (int kh = 0; kh < g.K; ++kh) {
            const int ih = oh * g.s - g.p + kh;
            if (ih < 0 || ih >= g.H) continue;
            for (int kw = 0; kw < g.K; ++kw) {
                const int iw = ow * g.s - g.p + kw;
                if (iw < 0 || iw >= g.W) continue;
                acc = fmaf(ldf(w + gwat<LAYOUT>(g, o, ci, kh, kw)), ldf(x + gat<LAYOUT>(g.C, g.H, g.W, n, c0 + ci, ih, iw)), acc);
            }
        }
    stf(y + idx, acc);
}

template <typename T, int LAYOUT>
__global__ __launch_bounds__(256) void k_gconv_generic_bwd_data(GGeom g, const T *__restrict__ dy,
                                                                const T *__restrict__ w, T *__restrict__ dx, int total)
{
    const unsigned uidx = blockIdx.x * 256u + threadIdx.x;   // the last block may reach past 2^31
    if (uidx >= (unsigned)total) return;
    int idx = (int)uidx;
    int n, c, ih, iw;
    gunflat<LAYOUT>(idx, g.C, g.H, g.W, n, c, ih, iw);
    const int o0 = (c / g.Cg) * g.Og, ci = c % g.Cg;
    float acc = 0.f;
    for (int oi = 0; oi < g.Og; ++oi) {
        const int o = o0 + oi;
        for (int kh = 0; kh < g.K; ++kh) {
            const int th = ih + g.p - kh;
            if (th < 0 || th % g.s != 0) continue;
            const int oh = th / g.s;
            if (oh >= g.Ho) continue;
            for (int kw = 0; kw < g.K; ++kw) {
                const int tw = iw + g.p - kw;
                if (tw < 0 || tw % g.s != 0) continue;
                const int ow = tw / g.s;
                if (ow >= g.Wo) continue;
                acc = fmaf(ldf(w + gwat<LAYOUT>(g, o, ci, kh, kw)), ldf(dy + gat<LAYOUT>(g.O, g.Ho, g.Wo, n, o, oh, ow)), acc);
            }
        }
    }
    stf(dx + idx, acc);
}

// Stage 1, NCHW: block (weight entry j = ((o*Cg+ci)*K+kh)*K+kw, part); threads stride over the pixels of
// the part; wavefront butterfly, then LDS across the 4 waves.
template <typename T>
__global__ __launch_bounds__(256) void k_gconv_generic_bwd_filter_nchw(GGeom g, const T *__restrict__ x,
                                                                       const T *__restrict__ dy, float *__restrict__ ws,
                                                                       int per_part, int J)
{
    __shared__ float red[4];
    const int j = blockIdx.x, part = blockIdx.y;
    const int kw = j % g.K, kh = (j / g.K) % g.K, ci = (j / (g.K * g.K)) % g.Cg, o = j / (g.K * g.K * g.Cg);
    const int c = (o / g.Og) * g.Cg + ci;
    const int npix = g.N * g.Ho * g.Wo;
    const int lo = part * per_part, hi = min(npix, lo + per_part);
    float acc = 0.f;
    for (int pix = lo + (int)threadIdx.x; pix < hi; pix += 256) {
        const int ow = pix % g.Wo, t = pix / g.Wo, oh = t % g.Ho, n = t / g.Ho;
        const int ih = oh * g.s - g.p + kh, iw = ow * g.s - g.p + kw;
        if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
        acc = fmaf(ldf(dy + gat<LAYOUT_NCHW>(g.O, g.Ho, g.Wo, n, o, oh, ow)),
                   ldf(x + gat<LAYOUT_NCHW>(g.C, g.H, g.W, n, c, ih, iw)), acc);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) ws[(size_t)part * J + j] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Stage 1, NHWC: block (tile of 64 output channels x one (kh,kw,ci), part); lane = channel, the 4 waves
// stride over pixels; LDS across the waves.
template <typename T>
__global__ __launch_bounds__(256) void k_gconv_generic_bwd_filter_nhwc(GGeom g, const T *__restrict__ x,
                                                                       const T *__restrict__ dy, float *__restrict__ ws,
                                                                       int per_part, int J, int notiles)
{
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int otile = blockIdx.x % notiles, e = blockIdx.x / notiles;     // e = (kh*K + kw)*Cg + ci
    const int part = blockIdx.y;
    const int ci = e % g.Cg, kw = (e / g.Cg) % g.K, kh = e / (g.Cg * g.K);
    const int o = otile * 64 + lane;
    const int npix = g.N * g.Ho * g.Wo;
    const int lo = part * per_part, hi = min(npix, lo + per_part);
    float acc = 0.f;
    if (o < g.O) {
        const int c = (o / g.Og) * g.Cg + ci;
        for (int pix = lo + wv; pix < hi; pix += 4) {
            const int ow = pix % g.Wo, t = pix / g.Wo, oh = t % g.Ho, n = t / g.Ho;
            const int ih = oh * g.s - g.p + kh, iw = ow * g.s - g.p + kw;
            if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
            acc = fmaf(ldf(dy + (size_t)pix * g.O + o), ldf(x + gat<LAYOUT_NHWC>(g.C, g.H, g.W, n, c, ih, iw)), acc);
        }
    }
    red[wv][lane] = acc;
    __syncthreads();
    if (wv == 0 && o < g.O)
        ws[(size_t)part * J + (size_t)e * g.O + o] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

hipError_t gconv_generic_fwd(const GGeom &g, int layout, int dtype, const void *x, const void *w, void *y, hipStream_t st)
{
    const int total = g.N * g.O * g.Ho * g.Wo;
    dim3 grid((unsigned)(((long long)total + 255) / 256)), block(256);
#define LAUNCH(T, L) hipLaunchKernelGGL((k_gconv_generic_fwd<T, L>), grid, block, 0, st, g, (const T *)x, (const T *)w, (T *)y, total)
    if (dtype == DT_F32) { if (layout == LAYOUT_NCHW) LAUNCH(float, LAYOUT_NCHW); else LAUNCH(float, LAYOUT_NHWC); }
    else                 { if (layout == LAYOUT_NCHW) LAUNCH(bf16_t, LAYOUT_NCHW); else LAUNCH(bf16_t, LAYOUT_NHWC); }
#undef LAUNCH
    return hipGetLastError();
}

hipError_t gconv_generic_bwd_data(const GGeom &g, int layout, int dtype, const void *dy, const void *w, void *dx,
                                  hipStream_t st)
{
    const int total = g.N * g.C * g.H * g.W;
    dim3 grid((unsigned)(((long long)total + 255) / 256)), block(256);
#define LAUNCH(T, L) hipLaunchKernelGGL((k_gconv_generic_bwd_data<T, L>), grid, block, 0, st, g, (const T *)dy, (const T *)w, (T *)dx, total)
    if (dtype == DT_F32) { if (layout == LAYOUT_NCHW) LAUNCH(float, LAYOUT_NCHW); else LAUNCH(float, LAYOUT_NHWC); }
    else                 { if (layout == LAYOUT_NCHW) LAUNCH(bf16_t, LAYOUT_NCHW); else LAUNCH(bf16_t, LAYOUT_NHWC); }
#undef LAUNCH
    return hipGetLastError();
}

int gconv_generic_bwd_filter_parts(const GGeom &g)
{
    // about 8192 pixels per part, at most 64 parts (the launch's second grid dimension), and never more
    // than 32 MiB of partials
    const long long npix = (long long)g.N * g.Ho * g.Wo;
    long long parts = (npix + 8191) / 8192;
    if (parts > 64) parts = 64;
    const long long J = (long long)g.O * g.Cg * g.K * g.K;
    while (parts > 1 && parts * J * 4 > (32ll << 20)) parts >>= 1;
    if (parts < 1) parts = 1;
    return (int)parts;
}

hipError_t gconv_generic_bwd_filter(const GGeom &g, int layout, int dtype, const void *x, const void *dy, float *ws,
                                    int parts, hipStream_t st)
{
    const int npix = g.N * g.Ho * g.Wo;
    const int per_part = (npix + parts - 1) / parts;
    const int J = g.O * g.Cg * g.K * g.K;
    if (layout == LAYOUT_NCHW) {
        dim3 grid(J, parts), block(256);
        if (dtype == DT_F32)
            hipLaunchKernelGGL(k_gconv_generic_bwd_filter_nchw<float>, grid, block, 0, st, g, (const float *)x, (const float *)dy, ws, per_part, J);
        else
            hipLaunchKernelGGL(k_gconv_generic_bwd_filter_nchw<bf16_t>, grid, block, 0, st, g, (const bf16_t *)x, (const bf16_t *)dy, ws, per_part, J);
    } else {
        const int notiles = (g.O + 63) / 64;
        dim3 grid(notiles * g.K * g.K * g.Cg, parts), block(256);
        if (dtype == DT_F32)
            hipLaunchKernelGGL(k_gconv_generic_bwd_filter_nhwc<float>, grid, block, 0, st, g, (const float *)x, (const float *)dy, ws, per_part, J, notiles);
        else
            hipLaunchKernelGGL(k_gconv_generic_bwd_filter_nhwc<bf16_t>, grid, block, 0, st, g, (const bf16_t *)x, (const bf16_t *)dy, ws, per_part, J, notiles);
    }
    return hipGetLastError();
}

// ---- variant selection -------------------------------------------------------------------------------

// the same tensor shapes as a depthwise geometry (for the kernels shared with the depthwise layer; C == O)
static Geom as_geom(const GGeom &g)
{
    Geom q;
    q.N = g.N; q.C = g.C; q.H = g.H; q.W = g.W; q.K = g.K; q.s = g.s; q.p = g.p; q.m = 1; q.O = g.O; q.Ho = g.Ho; q.Wo = g.Wo;
    return q;
}

static GPlan gplan(const GGeom &g, int layout, int dtype, int pass)
{
    GPlan pl = {GV_GENERIC, pass == 2 ? gconv_generic_bwd_filter_parts(g) : 0, 0, 0, 0, "group_generic"};
    if (tune_env("DWCONV_TUNE_GROUP_GENERIC")) return pl;
    // The filter gradient takes the small-plane form for groups of up to 4 on rows of up to 14, and on 28-wide rows in
    // bf16 (fp32 batch 128: 14x14 groups of 4 37 against 55 us, 28x28 groups of 4 83 against 85, groups of 8 122 against
    // 103; bf16 batch 256: 48 against 95, 83 against 107, 166 against 160)
    // Rows the row-walk kernels cannot take (7 elements) always go to the small-plane form instead of the generic one.
    const bool small_ok = pass < 2 || (g.Cg <= 4 && (g.W <= 14 || dtype == DT_BF16)) || !gconv_nchw_supported(g);      // (stride 2: always)
    if (layout == LAYOUT_NCHW && pass < 2 && gconv_nchws_mfma_fwd_supported(g)) {
        pl.variant = GV_NCHWS_MFMA_FWD;
        pl.name = pass == 0 ? "group_nchw_smallplane_mfma_k3s1" : "group_nchw_smallplane_mfma_k3s1_flip";
    } else if (layout == LAYOUT_NCHW && pass == 2 && gconv_nchws_mfma_bwd_filter_supported(g, dtype, false)) {
        pl.variant = GV_NCHWS_MFMA_BWD_FILTER;
        pl.name = "group_nchw_smallplane_mfma_bwd_filter_k3s1";
        pl.parts = gconv_nchws_mfma_bwd_filter_parts(g, dtype);
    } else if (layout == LAYOUT_NCHW && g.Cg == g.Og && small_ok && nchws_group_supported(as_geom(g), g.Cg) &&
        !tune_env("DWCONV_TUNE_GNOSMALL")) {
        // small planes (rows of 7, 14 or 28): whole groups staged in LDS through flat 16-byte accesses
        pl.variant = GV_NCHWS_K3S1;
        if (g.s == 1)
            pl.name = pass == 0 ? "group_nchw_smallplane_k3s1" : pass == 1 ? "group_nchw_smallplane_k3s1_flip"
                                                                            : "group_nchw_smallplane_bwd_filter_k3s1";
        else
            pl.name = pass == 0 ? "group_nchw_smallplane_fwd_k3s2" : pass == 1 ? "group_nchw_smallplane_bwd_data_k3s2"
                                                                               : "group_nchw_smallplane_bwd_filter_k3s2";
        if (pass == 2) nchws_bwd_filter_tiling(as_geom(g), dtype, &pl.a, &pl.c, &pl.parts, g.Cg);
    } else if (layout == LAYOUT_NCHW && gconv_nchw_supported(g)) {
        pl.variant = GV_NCHW_K3S1;
        pl.name = pass == 0 ? "group_nchw_rowwalk_k3s1" : pass == 1 ? "group_nchw_rowwalk_k3s1_flip" : "group_nchw_bwd_filter_k3s1";
        if (pass == 2) pl.parts = gconv_nchw_bwd_filter_parts(g);
    } else if (layout == LAYOUT_NHWC && pass == 2 && gconv_nchws_mfma_bwd_filter_supported(g, dtype, true)) {
        pl.variant = GV_NHWC_LDS_MFMA_BWD_FILTER;
        pl.name = "group_nhwc_lds_mfma_bwd_filter_k3s1";
        pl.parts = gconv_nchws_mfma_bwd_filter_parts(g, dtype);
    } else if (layout == LAYOUT_NHWC && pass == 2 && gconv_nhwc_tr_bwd_filter_supported(g, dtype)) {
        pl.variant = GV_NHWC_TR_BWD_FILTER;
        pl.name = "group_nhwc_mfma_bwd_filter_k3s1";
        pl.parts = gconv_nhwc_tr_bwd_filter_parts(g, dtype);
    } else if (layout == LAYOUT_NHWC && pass < 2 && gconv_nhwc_mfma_s2_supported(g, dtype, pass)) {
        pl.variant = GV_NHWC_MFMA_S2;
        pl.name = pass == 0 ? "group_nhwc_mfma_fwd_k3s2" : "group_nhwc_mfma_bwd_data_k3s2";
    } else if (layout == LAYOUT_NHWC && pass == 2 && gconv_nhwc_bwd_filter_s2_supported(g)) {
        pl.variant = GV_NHWC_BWD_FILTER_S2;
        pl.name = "group_nhwc_bwd_filter_k3s2";
        pl.parts = gconv_nhwc_bwd_filter_s2_parts(g);
    } else if (layout == LAYOUT_NHWC && gconv_nhwc_supported(g)) {
        pl.variant = GV_NHWC_K3S1;
        const bool mm = pass < 2 && gconv_nhwc_mfma_supported(g, dtype);      // forward and backward-data on the matrix cores
        pl.name = pass == 0 ? (mm ? "group_nhwc_mfma_k3s1" : "group_nhwc_rowwalk_k3s1")
                : pass == 1 ? (mm ? "group_nhwc_mfma_k3s1_flip" : "group_nhwc_rowwalk_k3s1_flip") : "group_nhwc_bwd_filter_k3s1";
        if (pass == 2) pl.parts = gconv_nhwc_bwd_filter_parts(g, dtype);
    }
    // a tuned filter gradient whose partial sums would not fit in 64 MiB (very wide rows): the generic kernels
    if (pass == 2 && pl.variant != GV_GENERIC && (long long)pl.parts * g.O * g.Cg * g.K * g.K * 4 > (64ll << 20)) {
        const GPlan gen = {GV_GENERIC, gconv_generic_bwd_filter_parts(g), 0, 0, 0, "group_generic"};
        return gen;
    }
    return pl;
}

}  // namespace dwc

using namespace dwc;

static int gvalidate(const dwconv_group_desc *d, GGeom *g)
{
    if (!d) return DWCONV_ERR_NULL;
    if (d->layout != DWCONV_NCHW && d->layout != DWCONV_NHWC) return DWCONV_ERR_BAD_ENUM;
    if (d->dtype != DWCONV_F32 && d->dtype != DWCONV_BF16) return DWCONV_ERR_BAD_ENUM;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->stride < 1 || d->pad < 0 || d->groups < 1 ||
        d->O < 1)
        return DWCONV_ERR_BAD_DIM;
    if (d->C % d->groups != 0 || d->O % d->groups != 0) return DWCONV_ERR_BAD_DIM;
    if (d->K > DWCONV_MAX_K) return DWCONV_ERR_UNSUPPORTED;
    const long long sh = (long long)d->H + 2ll * d->pad - d->K, sw = (long long)d->W + 2ll * d->pad - d->K;
    if (sh < 0 || sw < 0) return DWCONV_ERR_BAD_DIM;
    const long long Ho = sh / d->stride + 1, Wo = sw / d->stride + 1;
    const long long lim = 1ll << 31;
    const long long Cg = d->C / d->groups;
    if ((long long)d->pad >= (1 << 20) || (long long)d->N * d->C * d->H * d->W >= lim ||
        (long long)d->N * d->O * Ho * Wo >= lim || (long long)d->O * Cg * d->K * d->K >= lim)
        return DWCONV_ERR_TOO_LARGE;
    if (g) {
        g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W;
        g->K = d->K; g->s = d->stride; g->p = d->pad;
        g->G = d->groups; g->O = d->O; g->Cg = (int)Cg; g->Og = d->O / d->groups;
        g->Ho = (int)Ho; g->Wo = (int)Wo;
    }
    return DWCONV_OK;
}

// one input channel per group: the depthwise layer with multiplier O/C
static inline dwconv_desc as_depthwise(const dwconv_group_desc *d)
{
    dwconv_desc q = {d->N, d->C, d->H, d->W, d->K, d->stride, d->pad, d->O / d->C, d->layout, d->dtype};
    return q;
}

static inline bool gmisaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

extern "C" {

int gconv_out_dims(const dwconv_group_desc *desc, int32_t *Ho, int32_t *Wo)
{
    GGeom g;
    const int rc = gvalidate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (Ho) *Ho = g.Ho;
    if (Wo) *Wo = g.Wo;
    return DWCONV_OK;
}

size_t gconv_bwd_filter_workspace_bytes(const dwconv_group_desc *desc)
{
    GGeom g;
    if (gvalidate(desc, &g) != DWCONV_OK) return 0;
    if (g.Cg == 1) {
        const dwconv_desc q = as_depthwise(desc);
        return dwconv_bwd_filter_workspace_bytes(&q);
    }
    const GPlan pl = gplan(g, desc->layout, desc->dtype, 2);
    return (size_t)pl.parts * (size_t)g.O * g.Cg * g.K * g.K * sizeof(float);
}

int gconv_fwd(const dwconv_group_desc *desc, const void *x, const void *w, void *y, void *stream)
{
    GGeom g;
    const int rc = gvalidate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (g.Cg == 1) {
        const dwconv_desc q = as_depthwise(desc);
        return dwconv_fwd(&q, x, w, y, stream);
    }
    if (!x || !w || !y) return DWCONV_ERR_NULL;
    if (gmisaligned(x) || gmisaligned(w) || gmisaligned(y)) return DWCONV_ERR_ALIGN;
    const GPlan pl = gplan(g, desc->layout, desc->dtype, 0);
    hipError_t e;
    if (pl.variant == GV_NCHWS_MFMA_FWD) e = gconv_nchws_mfma_fwd(g, desc->dtype, x, w, y, false, (hipStream_t)stream);
    else if (pl.variant == GV_NCHWS_K3S1) e = nchws_group_fwd(as_geom(g), g.Cg, desc->dtype, x, w, y, false, (hipStream_t)stream);
    else if (pl.variant == GV_NCHW_K3S1) e = gconv_nchw_s1(g, desc->dtype, x, w, y, false, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_K3S1) e = gconv_nhwc_s1(g, desc->dtype, x, w, y, false, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_MFMA_S2) e = gconv_nhwc_mfma_s2(g, desc->dtype, x, w, y, false, (hipStream_t)stream);
    else e = gconv_generic_fwd(g, desc->layout, desc->dtype, x, w, y, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

int gconv_bwd_data(const dwconv_group_desc *desc, const void *dy, const void *w, void *dx, void *stream)
{
    GGeom g;
    const int rc = gvalidate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (g.Cg == 1) {
        const dwconv_desc q = as_depthwise(desc);
        return dwconv_bwd_data(&q, dy, w, dx, stream);
    }
    if (!dy || !w || !dx) return DWCONV_ERR_NULL;
    if (gmisaligned(dy) || gmisaligned(w) || gmisaligned(dx)) return DWCONV_ERR_ALIGN;
    const GPlan pl = gplan(g, desc->layout, desc->dtype, 1);
    hipError_t e;
    if (pl.variant == GV_NCHWS_MFMA_FWD) e = gconv_nchws_mfma_fwd(g, desc->dtype, dy, w, dx, true, (hipStream_t)stream);
    else if (pl.variant == GV_NCHWS_K3S1 && g.s == 2) e = nchws_group_bwd_data_s2(as_geom(g), g.Cg, desc->dtype, dy, w, dx, (hipStream_t)stream);
    else if (pl.variant == GV_NCHWS_K3S1) e = nchws_group_fwd(as_geom(g), g.Cg, desc->dtype, dy, w, dx, true, (hipStream_t)stream);
    else if (pl.variant == GV_NCHW_K3S1) e = gconv_nchw_s1(g, desc->dtype, dy, w, dx, true, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_K3S1) e = gconv_nhwc_s1(g, desc->dtype, dy, w, dx, true, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_MFMA_S2) e = gconv_nhwc_mfma_s2(g, desc->dtype, dy, w, dx, true, (hipStream_t)stream);
    else e = gconv_generic_bwd_data(g, desc->layout, desc->dtype, dy, w, dx, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

int gconv_bwd_filter(const dwconv_group_desc *desc, const void *x, const void *dy, void *dw, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    GGeom g;
    const int rc = gvalidate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (g.Cg == 1) {
        const dwconv_desc q = as_depthwise(desc);
        return dwconv_bwd_filter(&q, x, dy, dw, workspace, workspace_bytes, stream);
    }
    if (!x || !dy || !dw) return DWCONV_ERR_NULL;
    if (gmisaligned(x) || gmisaligned(dy) || gmisaligned(dw)) return DWCONV_ERR_ALIGN;
    const GPlan pl = gplan(g, desc->layout, desc->dtype, 2);
    const int J = g.O * g.Cg * g.K * g.K;
    const size_t need = (size_t)pl.parts * (size_t)J * sizeof(float);
    if (!workspace || workspace_bytes < need) return DWCONV_ERR_WORKSPACE;
    if (gmisaligned(workspace)) return DWCONV_ERR_ALIGN;
    hipError_t e;
    if (pl.variant == GV_NCHWS_K3S1) e = nchws_group_bwd_filter(as_geom(g), g.Cg, desc->dtype, x, dy, (float *)workspace, pl.a, pl.c, (hipStream_t)stream);
    else if (pl.variant == GV_NCHWS_MFMA_BWD_FILTER) e = gconv_nchws_mfma_bwd_filter(g, desc->dtype, false, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_TR_BWD_FILTER) e = gconv_nhwc_tr_bwd_filter(g, desc->dtype, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_LDS_MFMA_BWD_FILTER) e = gconv_nchws_mfma_bwd_filter(g, desc->dtype, true, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_BWD_FILTER_S2) e = gconv_nhwc_bwd_filter_s2(g, desc->dtype, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else if (pl.variant == GV_NCHW_K3S1) e = gconv_nchw_bwd_filter(g, desc->dtype, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else if (pl.variant == GV_NHWC_K3S1) e = gconv_nhwc_bwd_filter(g, desc->dtype, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    else e = gconv_generic_bwd_filter(g, desc->layout, desc->dtype, x, dy, (float *)workspace, pl.parts, (hipStream_t)stream);
    if (e != hipSuccess) return DWCONV_ERR_LAUNCH;
    e = reduce_partials((const float *)workspace, pl.parts, J, (float *)dw, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

const char *gconv_variant_name(const dwconv_group_desc *desc, int pass)
{
    GGeom g;
    if (gvalidate(desc, &g) != DWCONV_OK || pass < 0 || pass > 2) return "invalid";
    if (g.Cg == 1) {
        const dwconv_desc q = as_depthwise(desc);
        return dwconv_variant_name(&q, pass);
    }
    return gplan(g, desc->layout, desc->dtype, pass).name;
}

}  // extern "C"
