// Fused backward pass for NHWC, 3x3, stride 1, pad 1, multiplier 1 or 2: the input gradient dx and the
// stage-1 partial sums of the filter gradient dw from ONE walk over dy and x.  Run separately the
// two passes read dy twice; fused, the backward pass moves 2|x| + |y| elements instead of
// 2(|x| + |y|) and is one launch less.
//
// Mapping as in the filter-gradient kernel (nhwc.hip): a block is CT channel-vectors x 256/CT
// columns, walks a strip of rows of NI images; a lane owns V channels of one column.  Step t of
// the walk takes dy row t (three columns) and x row t+1 (the lane's own column only):
//   input gradient:  dx[r][ow] = sum_{kh,kw} w[kh][kw] dy[r+1-kh][ow+1-kw]; dy row t is tap row
//     kh = 0, 1, 2 of dx rows t-1, t, t+1, so two rotating accumulators finish dx row t-1 here;
//   filter gradient: dw[kh][kw] = sum dy[oh][ow] x[oh-1+kh][ow-1+kw] is summed per x column c instead
//     of per dy column: the lane's x column meets dy[t][c+1-kw] at tap column kw, and x rows t-1, t, t+1
//     (a three-row window of the lane's own column) at tap rows 0, 1, 2.  The three dy columns are there
//     for the input gradient anyway, so the walk loads four vectors per step instead of six and keeps
//     a third fewer rows in its prefetch ring.  Only dy rows inside the block's own strip count (uniform
//     branch), while the input gradient needs the true halo rows.
// Loads go through buffer views of the image (scalar row offsets; a column outside the image is read
// outside the view and returns the zero of the padding, for both gradients), rows are clamped, stay as
// loaded (packed for bf16) until used, and every condition inside the walk is uniform over the block.
#include "kernels.hpp"

namespace dwc {

// M = 2 (channel multiplier 2): the lane's V output channels sit on V/2 input channels, so x and dx are
// vectors of V/2 channels, an element of dx adds up the terms of its two outputs, and an element of x
// meets the dy of both.
template <typename T, int V, int PF, int M = 1>
__global__ __launch_bounds__(256) void k_nhwc_bwd_fused_k3s1(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                             const T *__restrict__ w, T *__restrict__ dx,
                                                             float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                             int TH, int nstrips, int NI, unsigned nblocks, int nt)
{
    constexpr int K = 3, R = PF + 1;
    __shared__ float red[ReduceLds<K, V>::FLOATS];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    constexpr int VX = V / M;      // input channels behind the lane's V output channels
    const int Q = g.O / V;
    const int cq = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = cq < Q && ow < g.W;

    float acc[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[kh][kw][v] = 0.f;

    if (active) {
        // byte offsets of dy columns ow-1, ow, ow+1 inside an image row; a column outside the image is read at an
        // offset outside the buffer view and comes back as the zero of the padding, for both gradients
        uint32_t coloff[K];
        float wd[K][K][V];      // wd[kh][j]: weight of dy column ow-1+j in tap row kh of the input gradient (= w[kh][2-j])
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int iw = ow - 1 + j;
            coloff[j] = (iw >= 0 && iw < g.W) ? (uint32_t)(iw * g.O + cq * V) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
#pragma unroll
            for (int kh = 0; kh < K; ++kh) Vec<T, V>::load(w + (kh * K + (2 - j)) * g.O + cq * V, wd[kh][j]);
        }
        const uint32_t xcol = (uint32_t)(ow * g.C + cq * VX) * (uint32_t)sizeof(T);     // the lane's x / dx column
        const int rowlen = g.W * g.O, xrowlen = g.W * g.C;
        const uint32_t rowbytes = (uint32_t)rowlen * (uint32_t)sizeof(T), imgbytes = (uint32_t)g.H * rowbytes;   // at most 2 GiB
        const uint32_t xrowbytes = (uint32_t)xrowlen * (uint32_t)sizeof(T), ximgbytes = (uint32_t)g.H * xrowbytes;
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        for (int n = n0; n < n1; ++n) {
            const BufView xin(x + (size_t)n * g.H * xrowlen, ximgbytes), dyin(dy + (size_t)n * g.H * rowlen, imgbytes);
            const BufView dxout(dx + (size_t)n * g.H * xrowlen, ximgbytes);

            // step t brings dy row t (three columns) and x row t+1 (the lane's own column)
            RawVec<T, V> dr[R][K];
            RawVec<T, VX> xr[R];
            auto load_rows = [&](int t, RawVec<T, V> (&dd)[K], RawVec<T, VX> &xd) {
                const uint32_t dro = (uint32_t)min(max(t, 0), g.H - 1) * rowbytes;
#pragma unroll
                for (int j = 0; j < K; ++j) dd[j].load_buf(dyin, coloff[j], dro);
                xd.load_buf(xin, xcol, (uint32_t)min(max(t + 1, 0), g.H - 1) * xrowbytes);
            };

            // xw[kh] = x row t-1+kh at the lane's column (zero outside the image); A0, A1: the two unfinished dx rows
            float A0[VX], A1[VX], xw[K][VX];
#pragma unroll
            for (int v = 0; v < VX; ++v) { A0[v] = 0.f; A1[v] = 0.f; }
            const int t0 = oh0 - 1, nsteps = (oh1 - oh0) + 2;       // t = oh0-1 .. oh1: the dy rows a strip's dx needs
            {
                // x row t0 enters the window ahead of the first step (it becomes row t-1 of the strip's first dy row)
                RawVec<T, VX> first;
                first.load_buf(xin, xcol, (uint32_t)max(t0, 0) * xrowbytes);
                float f[VX];
                first.get(f);
#pragma unroll
                for (int v = 0; v < VX; ++v) { xw[0][v] = 0.f; xw[1][v] = 0.f; xw[2][v] = t0 >= 0 ? f[v] : 0.f; }
            }

            auto consume = [&](int t, const RawVec<T, V> (&dd)[K], const RawVec<T, VX> &xd) {
                const bool dyok = t >= 0 && t < g.H;                 // dy row t exists
                const bool mine = t >= oh0 && t < oh1;               // ... and belongs to this block's strip
                float d[K][V];
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    dd[j].get(d[j]);
#pragma unroll
                    for (int v = 0; v < V; ++v) d[j][v] = dyok ? d[j][v] : 0.f;
                }
                // input gradient: dy row t is tap row 0 of dx row t-1, tap row 1 of dx row t, tap row 2 of dx row t+1
                float out[VX];
#pragma unroll
                for (int c = 0; c < VX; ++c) {
                    float s0 = A0[c], s1 = A1[c], s2 = 0.f;
#pragma unroll
                    for (int mm = 0; mm < M; ++mm) {
                        const int v = c * M + mm;
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            s0 = fmaf(wd[0][j][v], d[j][v], s0);
                            s1 = fmaf(wd[1][j][v], d[j][v], s1);
                            s2 = fmaf(wd[2][j][v], d[j][v], s2);
                        }
                    }
                    out[c] = s0; A0[c] = s1; A1[c] = s2;
                }
                if (t - 1 >= oh0 && t - 1 < oh1) store_buf<T, VX>(dxout, xcol, (uint32_t)(t - 1) * xrowbytes, out, nt != 0);
                // filter gradient, summed per x column: the lane's x column c meets dy[t][c+1-kw] at tap column kw, and x
                // rows t-1, t, t+1 at tap rows 0, 1, 2 (the sum over all columns is the same as per dy column)
                {
                    float xv[VX];
                    xd.get(xv);
                    const bool xok = t + 1 < g.H;                    // t + 1 >= 0 always (t >= -1)
#pragma unroll
                    for (int v = 0; v < VX; ++v) { xw[0][v] = xw[1][v]; xw[1][v] = xw[2][v]; xw[2][v] = xok ? xv[v] : 0.f; }
                }
                if (mine) {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw)
#pragma unroll
                        for (int v = 0; v < V; ++v) {
                            const float dd1 = d[2 - kw][v];
#pragma unroll
                            for (int kh = 0; kh < K; ++kh) acc[kh][kw][v] = fmaf(dd1, xw[kh][v / M], acc[kh][kw][v]);
                        }
                }
            };

#pragma unroll
            for (int j = 0; j < PF; ++j) load_rows(t0 + j, dr[j], xr[j]);
            int i = 0;
#pragma unroll 1
            for (; i + R <= nsteps; i += R) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    load_rows(t0 + i + j + PF, dr[(j + PF) % R], xr[(j + PF) % R]);
                    consume(t0 + i + j, dr[j], xr[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < R - 1; ++j)
                if (i + j < nsteps) consume(t0 + i + j, dr[j], xr[j]);
        }
    }

    // ---- fixed-order block reduction (as in the filter-gradient kernel) ----
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * (K * K * g.O);
    block_reduce_taps<K, V>(acc, CT, red, [&](int kh, int kw, int v, float total) {
        if (cq < Q) wsp[(kh * K + kw) * g.O + cq * V + v] = total;
    });
}


// ---------------------------------------------------------------------------------------------
// Fused backward pass, 3x3, stride 2, pad 1, multiplier 1, even H and W.  Mapping and tiling of the
// stride-2 filter gradient (nhwc.hip): a lane owns V channels of dy column b and walks the dy rows a
// of its strip.  Step a holds dy rows a and a+1 (columns b and b+1) and x rows 2a-1, 2a, 2a+1
// (columns 2b and 2b+1):
//   input gradient: the 2x2 block dx[2a..2a+1][2b..2b+1] from dy[a..a+1][b..b+1], as in
//     k_nhwc_bwd_data_k3s2 (a missing column b+1 is read outside the buffer view and is zero, a missing
//     row a+1 is a block-uniform condition);
//   filter gradient, summed per x column: x column 2b meets dy[a][b] at tap column 1, x column 2b+1
//     meets dy[a][b] at tap column 2 and dy[a][b+1] at tap column 0 (every x element is then loaded by
//     exactly one lane: two x vectors per row instead of three); x row 2a+1 is kept as the top row of
//     step a+1.
// dy row a+1 and x rows 2a+2, 2a+3 of the next step are loaded while the current one is computed and
// stay as loaded (packed for bf16) until then.  dy is read once: the pass moves 2|x| + |y| elements.
// ---------------------------------------------------------------------------------------------
template <typename T, int V>
__global__ __launch_bounds__(256) void k_nhwc_bwd_fused_k3s2(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                             const T *__restrict__ w, T *__restrict__ dx,
                                                             float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                             int TH, int nstrips, int NI, unsigned nblocks, int nt)
{
    constexpr int K = 3;
    __shared__ float red[ReduceLds<K, V>::FLOATS];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int Q = g.C / V;
    const int cq = ctile * CT + tx, b = owtile * OWT + ty;
    const bool active = cq < Q && b < g.Wo;

    float acc[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[kh][kw][v] = 0.f;

    if (active) {
        float wr[K][K][V];
#pragma unroll
        for (int kh = 0; kh < K; ++kh)
#pragma unroll
            for (int kw = 0; kw < K; ++kw) Vec<T, V>::load(w + (kh * K + kw) * g.C + cq * V, wr[kh][kw]);
        // buffer views of the image: dy column b+1 of the last lane of a row is read outside the view and comes
        // back as zero, for both gradients
        const uint32_t es = (uint32_t)sizeof(T);
        const uint32_t dyrowb = (uint32_t)(g.Wo * g.C) * es, xrowb = (uint32_t)(g.W * g.C) * es, cb = (uint32_t)g.C * es;
        const uint32_t dyoff0 = (uint32_t)(b * g.C + cq * V) * es;
        const uint32_t dyoff1 = b + 1 < g.Wo ? dyoff0 + cb : BufView::OUTSIDE;
        const uint32_t xoff = (uint32_t)(2 * b * g.C + cq * V) * es;       // x / dx column 2b; column 2b+1 is one pixel on
        const int a0 = strip * TH, a1 = min(g.Ho, a0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        for (int n = n0; n < n1; ++n) {
            const BufView dyin(dy + (size_t)n * g.Ho * g.Wo * g.C, (uint32_t)g.Ho * dyrowb);
            const BufView xin(x + (size_t)n * g.H * g.W * g.C, (uint32_t)g.H * xrowb);
            const BufView dxout(dx + (size_t)n * g.H * g.W * g.C, (uint32_t)g.H * xrowb);
            auto load_dy = [&](int a, RawVec<T, V> (&d)[2]) {
                const uint32_t ro = (uint32_t)min(a, g.Ho - 1) * dyrowb;
                d[0].load_buf(dyin, dyoff0, ro); d[1].load_buf(dyin, dyoff1, ro);
            };
            // the lane's two x columns 2b and 2b+1 (the filter gradient is summed per x column)
            auto load_x = [&](int r, RawVec<T, V> (&xd)[2]) {
                const uint32_t ro = (uint32_t)min(max(r, 0), g.H - 1) * xrowb;
                xd[0].load_buf(xin, xoff, ro); xd[1].load_buf(xin, xoff + cb, ro);
            };
            RawVec<T, V> dcur[2], dnext[2][2], xa[2], xb[2][2], xc[2][2];
            load_dy(a0, dcur);
            if (a0 > 0) load_x(2 * a0 - 1, xa);
            else { xa[0].zero(); xa[1].zero(); }
            load_dy(a0 + 1, dnext[0]); load_x(2 * a0, xb[0]); load_x(2 * a0 + 1, xc[0]);
            auto step = [&](int a, int j) {
                const bool below = a + 1 < g.Ho;
                float A0[V], A1[V], B0[V], B1[V];
                dcur[0].get(A0); dcur[1].get(A1); dnext[j][0].get(B0); dnext[j][1].get(B1);
                float o00[V], o01[V], o10[V], o11[V];
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    o00[v] = wr[1][1][v] * A0[v];
                    o01[v] = fmaf(wr[1][0][v], A1[v], wr[1][2][v] * A0[v]);
                    o10[v] = wr[2][1][v] * A0[v];
                    o11[v] = fmaf(wr[2][0][v], A1[v], wr[2][2][v] * A0[v]);
                }
                if (below) {
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        o10[v] = fmaf(wr[0][1][v], B0[v], o10[v]);
                        o11[v] = fmaf(wr[0][0][v], B1[v], fmaf(wr[0][2][v], B0[v], o11[v]));
                    }
                }
                const uint32_t r0 = (uint32_t)(2 * a) * xrowb;
                store_buf<T, V>(dxout, xoff, r0, o00, nt != 0);
                store_buf<T, V>(dxout, xoff + cb, r0, o01, nt != 0);
                store_buf<T, V>(dxout, xoff, r0 + xrowb, o10, nt != 0);
                store_buf<T, V>(dxout, xoff + cb, r0 + xrowb, o11, nt != 0);
                // filter gradient per x column: x rows 2a-1, 2a, 2a+1 are tap rows 0, 1, 2; x column 2b meets dy[a][b] at
                // tap column 1, x column 2b+1 meets dy[a][b] at tap column 2 and dy[a][b+1] at tap column 0
                {
                    float e0[V], e1[V], e2[V], f0[V], f1[V], f2[V];
                    xa[0].get(e0); xb[j][0].get(e1); xc[j][0].get(e2);
                    xa[1].get(f0); xb[j][1].get(f1); xc[j][1].get(f2);
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        acc[0][1][v] = fmaf(A0[v], e0[v], acc[0][1][v]);
                        acc[1][1][v] = fmaf(A0[v], e1[v], acc[1][1][v]);
                        acc[2][1][v] = fmaf(A0[v], e2[v], acc[2][1][v]);
                        acc[0][2][v] = fmaf(A0[v], f0[v], acc[0][2][v]);
                        acc[1][2][v] = fmaf(A0[v], f1[v], acc[1][2][v]);
                        acc[2][2][v] = fmaf(A0[v], f2[v], acc[2][2][v]);
                        acc[0][0][v] = fmaf(A1[v], f0[v], acc[0][0][v]);
                        acc[1][0][v] = fmaf(A1[v], f1[v], acc[1][0][v]);
                        acc[2][0][v] = fmaf(A1[v], f2[v], acc[2][0][v]);
                    }
                }
                dcur[0] = dnext[j][0]; dcur[1] = dnext[j][1];
                xa[0] = xc[j][0]; xa[1] = xc[j][1];
            };
            int a = a0;
#pragma unroll 1
            for (; a + 2 <= a1; a += 2) {
                load_dy(a + 2, dnext[1]); load_x(2 * a + 2, xb[1]); load_x(2 * a + 3, xc[1]);
                step(a, 0);
                load_dy(a + 3, dnext[0]); load_x(2 * a + 4, xb[0]); load_x(2 * a + 5, xc[0]);
                step(a + 1, 1);
            }
            if (a < a1) step(a, 0);
        }
    }

    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * (K * K * g.C);
    block_reduce_taps<K, V>(acc, CT, red, [&](int kh, int kw, int v, float total) {
        if (cq < Q) wsp[(kh * K + kw) * g.C + cq * V + v] = total;
    });
}

bool nhwc_bwd_fused_supported(const Geom &g, int dtype, int V)
{
    if (!(g.K == 3 && g.p == 1 && (g.m == 1 || (g.m == 2 && g.s == 1)))) return false;
    // stride 2 (even maps): 12 % faster than the two passes on 112x112 maps, equal within 2 % on smaller ones
    if (g.s == 2) {
        const char *e = tune_env("DWCONV_TUNE_FUSE_S2H");        // tuning: smallest map height that takes the fused kernel
        if (g.H % 2 != 0 || g.W % 2 != 0 || g.H < (e ? atoi(e) : 2)) return false;
    }
    else if (g.s != 1) return false;
    // bf16 with 8 channels per lane would need more than 256 registers
    return (dtype == DT_F32 && V == 4) || (dtype == DT_BF16 && V == 4);
}

// Same tiling function as the filter gradient (nhwc_bwd_filter_tiling); partial sums at [part][kh][kw][c].
hipError_t nhwc_bwd_fused(const Geom &g, int dtype, int V, const void *x, const void *dy, const void *w, void *dx,
                          float *ws, int TH, int NI, hipStream_t st)
{
    if (!nhwc_bwd_fused_supported(g, dtype, V)) return hipErrorInvalidValue;
    int CT, nctiles, nowtiles, nstrips, ngroups;
    nhwc_bwd_filter_tiling(g, V, TH, NI, &CT, &nctiles, &nowtiles, &nstrips, &ngroups);
    const unsigned nblocks = (unsigned)nctiles * nowtiles * nstrips * ngroups;
    const int esz = dtype == DT_F32 ? 4 : 2;
    const int nt = stream_stores("NHWC_FUSED_BWD", (long long)g.N * g.H * g.W * g.C * esz, 0);
#define GO(T, VV, PP) hipLaunchKernelGGL((k_nhwc_bwd_fused_k3s1<T, VV, PP>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                     (const T *)dy, (const T *)w, (T *)dx, ws, CT, nctiles, nowtiles, TH, nstrips, NI, \
                                     nblocks, nt)
#define GOM2(T) hipLaunchKernelGGL((k_nhwc_bwd_fused_k3s1<T, 4, 2, 2>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                   (const T *)dy, (const T *)w, (T *)dx, ws, CT, nctiles, nowtiles, TH, nstrips, NI, \
                                   nblocks, nt)
#define GO2(T, VV) hipLaunchKernelGGL((k_nhwc_bwd_fused_k3s2<T, VV>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                      (const T *)dy, (const T *)w, (T *)dx, ws, CT, nctiles, nowtiles, TH, nstrips, NI, \
                                      nblocks, nt)
    const char *fpf = tune_env("DWCONV_TUNE_FPF");
    const int pf = fpf ? atoi(fpf) : 2;       // two rows ahead: 2 % faster than one although it leaves two wavefronts per SIMD in fp32
    if (g.m == 2) { if (dtype == DT_F32) GOM2(float); else GOM2(bf16_t); }
    else if (g.s == 2) { if (dtype == DT_F32) GO2(float, 4); else GO2(bf16_t, 4); }
    else if (dtype == DT_F32) { if (pf == 2) GO(float, 4, 2); else GO(float, 4, 1); }
    else { if (pf == 2) GO(bf16_t, 4, 2); else GO(bf16_t, 4, 1); }
#undef GO
#undef GOM2
#undef GO2
    return hipGetLastError();
}

}  // namespace dwc
