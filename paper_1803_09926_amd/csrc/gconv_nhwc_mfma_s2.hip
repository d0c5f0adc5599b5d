// Group convolution, NHWC, 3x3 stride 2 pad 1, groups of 4 or 8 channels on both sides, on the matrix cores:
// forward and backward-data.  Lane and block layout of gconv_nhwc_mfma.hip: a block = one quad of channels, its
// four lanes = four neighbouring pixel columns; of the output in the forward pass, of dy in backward-data, where
// each lane owns the 2x2 block of dx under its dy pixel.
//
// Forward: output row oh reads input rows 2oh-1, 2oh, 2oh+1 at columns 2ow-1, 2ow, 2ow+1.  Row 2oh+1 is also
// the top row of output row oh+1, so the walk loads two input rows per output row and keeps two accumulators
// (the current output row and the next one's first tap row).  A row or column outside the image is read at an
// offset outside the buffer view and comes back as the zero of the padding.
//
// Backward-data (even H and W): dx[2a..2a+1][2b..2b+1] gets, from dy[a..a+1][b..b+1],
//   dx[2a  ][2b  ] = W11' dy[a][b]
//   dx[2a  ][2b+1] = W10' dy[a][b+1] + W12' dy[a][b]
//   dx[2a+1][2b  ] = W01' dy[a+1][b] + W21' dy[a][b]
//   dx[2a+1][2b+1] = W00' dy[a+1][b+1] + W02' dy[a+1][b] + W20' dy[a][b+1] + W22' dy[a][b]
// (Wkh,kw' = the tap's Cg x Og block transposed: the taps (kh, kw) of Eq. 3 that land on each of the four
// positions), nine matrix products per dy pixel and quad, one new dy row per step.
#include "gconv_mfma.hpp"

namespace dwc {

namespace {

// everything a wavefront derives from its index
struct WaveItem { int cs, cq, strip, ngroup; bool live; };
__device__ __forceinline__ WaveItem wave_item(unsigned nblocks, unsigned nwaves, int ncs, int ncq, int nstrips)
{
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    unsigned gw = (unsigned)__builtin_amdgcn_readfirstlane((int)(lb * 4 + (threadIdx.x >> 6)));
    WaveItem it;
    it.live = gw < nwaves;
    it.cs = gw % ncs; gw /= ncs;
    it.cq = gw % ncq; gw /= ncq;
    it.strip = gw % nstrips; it.ngroup = gw / nstrips;
    return it;
}

// d[oq] += (tap's filter block) * (the input quads of oq's group), for every output quad of the lane
template <typename T, int CG>
__device__ __forceinline__ void tap_mma(v4f_t (&d)[LaneIn<T>::LQ], const QuadW<T> (&wt)[LaneIn<T>::LQ][9][CG / 4], int tap,
                                        const LaneIn<T> &own)
{
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG / 4;
    constexpr bool SIB = NQ == 2 && LQ == 1;
    LaneIn<T> sib;
    if constexpr (SIB) sib = own.sibling();
#pragma unroll
    for (int oq = 0; oq < LQ; ++oq)
#pragma unroll
        for (int iq = 0; iq < NQ; ++iq) {
            const LaneIn<T> &b = (SIB && iq == 1) ? sib : own;
            const int q = NQ == 1 ? oq : (SIB ? 0 : iq);
            quad_mma1(d[oq], wt[oq][tap][iq], b, q);
        }
}

template <typename T>
__device__ __forceinline__ void store_quads(const BufView &v, uint32_t voff, uint32_t soff, const v4f_t (&d)[LaneIn<T>::LQ], bool stream)
{
    constexpr int LQ = LaneIn<T>::LQ;
    float o[4 * LQ];
#pragma unroll
    for (int oq = 0; oq < LQ; ++oq)
#pragma unroll
        for (int i = 0; i < 4; ++i) o[4 * oq + i] = d[oq][i];
    store_buf<T, 4 * LQ>(v, voff, soff, o, stream);
}

}  // namespace

template <typename T, int CG>
__global__ __launch_bounds__(256) void k_gconv_nhwc_mfma_fwd_s2(GGeom g, const T *__restrict__ x, const T *__restrict__ w,
                                                                T *__restrict__ y, int TH, int nstrips, int ncq, int ncs,
                                                                int NI, unsigned nwaves, unsigned nblocks, int nt)
{
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG / 4;
    const WaveItem it = wave_item(nblocks, nwaves, ncs, ncq, nstrips);
    if (!it.live) return;                                   // uniform over the wavefront; the kernel has no barrier
    const int lane = threadIdx.x & 63, blk = lane >> 2, j = lane & 3;
    const int cbase = (it.cs * 16 + blk) * 4 * LQ;
    const int ow = it.cq * 4 + j;
    const int C = g.C;

    QuadW<T> wq[LQ][9][NQ];
    load_group_filter<T, CG, 0>(w, C, cbase, j, wq);

    uint32_t coloff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = 2 * ow - 1 + kw;
        coloff[kw] = (ow < g.Wo && iw >= 0 && iw < g.W) ? (uint32_t)(iw * C + cbase) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    }
    const bool colok = ow < g.Wo;
    const uint32_t ocol = (uint32_t)(min(ow, g.Wo - 1) * C + cbase) * (uint32_t)sizeof(T);
    const uint32_t irow = (uint32_t)g.W * (uint32_t)C * (uint32_t)sizeof(T), iimg = (uint32_t)g.H * irow;
    const uint32_t orow = (uint32_t)g.Wo * (uint32_t)C * (uint32_t)sizeof(T), oimg = (uint32_t)g.Ho * orow;
    const int oh0 = it.strip * TH, oh1 = min(g.Ho, oh0 + TH);
    const int n0 = it.ngroup * NI, n1 = min(g.N, n0 + NI);

    for (int n = n0; n < n1; ++n) {
        const BufView vin(x + (size_t)n * g.H * g.W * C, iimg), vout(y + (size_t)n * g.Ho * g.Wo * C, oimg);
        // one input row at the lane's three columns; a row outside the image reads as zero
        auto load_row = [&](int ih, LaneIn<T> (&dst)[3]) {
            const bool ok = ih >= 0 && ih < g.H;                         // uniform
            const uint32_t ro = (uint32_t)min(max(ih, 0), g.H - 1) * irow;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) dst[kw].load(vin, ok ? coloff[kw] : BufView::OUTSIDE, ro);
        };
        v4f_t cur[LQ], nxt[LQ];
#pragma unroll
        for (int oq = 0; oq < LQ; ++oq) { cur[oq] = v4f_t{0.f, 0.f, 0.f, 0.f}; nxt[oq] = cur[oq]; }
        // the rows of output row oh: even = 2oh (tap row 1), odd = 2oh+1 (tap row 2, and tap row 0 of output row oh+1)
        struct Pair { LaneIn<T> even[3], odd[3]; };
        auto load_pair = [&](int oh, Pair &p) { load_row(2 * oh, p.even); load_row(2 * oh + 1, p.odd); };
        auto consume = [&](int oh, const Pair &p) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                tap_mma<T, CG>(cur, wq, 3 + kw, p.even[kw]);
                tap_mma<T, CG>(cur, wq, 6 + kw, p.odd[kw]);
                tap_mma<T, CG>(nxt, wq, kw, p.odd[kw]);
            }
            if (colok) store_quads<T>(vout, ocol, (uint32_t)oh * orow, cur, nt != 0);
#pragma unroll
            for (int oq = 0; oq < LQ; ++oq) { cur[oq] = nxt[oq]; nxt[oq] = v4f_t{0.f, 0.f, 0.f, 0.f}; }
        };
        {
            LaneIn<T> top[3];                               // row 2*oh0 - 1: tap row 0 of the strip's first output row
            load_row(2 * oh0 - 1, top);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) tap_mma<T, CG>(cur, wq, kw, top[kw]);
        }
        Pair pa, pb;
        load_pair(oh0, pa);
        int oh = oh0;
#pragma unroll 1
        for (; oh + 2 <= oh1; oh += 2) {
            load_pair(oh + 1, pb);
            consume(oh, pa);
            load_pair(oh + 2, pa);
            consume(oh + 1, pb);
        }
        if (oh < oh1) consume(oh, pa);
    }
}

template <typename T, int CG>
__global__ __launch_bounds__(256) void k_gconv_nhwc_mfma_bwd_s2(GGeom g, const T *__restrict__ dy, const T *__restrict__ w,
                                                                T *__restrict__ dx, int TH, int nstrips, int ncq, int ncs,
                                                                int NI, unsigned nwaves, unsigned nblocks, int nt)
{
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG / 4;
    const WaveItem it = wave_item(nblocks, nwaves, ncs, ncq, nstrips);
    if (!it.live) return;
    const int lane = threadIdx.x & 63, blk = lane >> 2, j = lane & 3;
    const int cbase = (it.cs * 16 + blk) * 4 * LQ;
    const int b = it.cq * 4 + j;                            // dy column
    const int C = g.C;

    QuadW<T> wq[LQ][9][NQ];
    load_group_filter<T, CG, 2>(w, C, cbase, j, wq);

    const bool colok = b < g.Wo;
    uint32_t dcol[2], xcol[2];
    dcol[0] = colok ? (uint32_t)(b * C + cbase) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    dcol[1] = (b + 1 < g.Wo) ? (uint32_t)((b + 1) * C + cbase) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    const int bc = min(b, g.Wo - 1);
    xcol[0] = (uint32_t)(2 * bc * C + cbase) * (uint32_t)sizeof(T);
    xcol[1] = (uint32_t)((2 * bc + 1) * C + cbase) * (uint32_t)sizeof(T);
    const uint32_t drow = (uint32_t)g.Wo * (uint32_t)C * (uint32_t)sizeof(T), dimg = (uint32_t)g.Ho * drow;
    const uint32_t xrow = (uint32_t)g.W * (uint32_t)C * (uint32_t)sizeof(T), ximg = (uint32_t)g.H * xrow;
    const int a0 = it.strip * TH, a1 = min(g.Ho, a0 + TH);
    const int n0 = it.ngroup * NI, n1 = min(g.N, n0 + NI);

    for (int n = n0; n < n1; ++n) {
        const BufView vin(dy + (size_t)n * g.Ho * g.Wo * C, dimg), vout(dx + (size_t)n * g.H * g.W * C, ximg);
        auto load_row = [&](int a, LaneIn<T> (&dst)[2]) {
            const bool ok = a < g.Ho;                                    // uniform
            const uint32_t ro = (uint32_t)min(a, g.Ho - 1) * drow;
#pragma unroll
            for (int s = 0; s < 2; ++s) dst[s].load(vin, ok ? dcol[s] : BufView::OUTSIDE, ro);
        };
        auto step = [&](int a, const LaneIn<T> (&A)[2], const LaneIn<T> (&B)[2]) {      // dy rows a and a+1
            v4f_t x00[LQ], x01[LQ], x10[LQ], x11[LQ];
#pragma unroll
            for (int oq = 0; oq < LQ; ++oq) { x00[oq] = v4f_t{0.f, 0.f, 0.f, 0.f}; x01[oq] = x00[oq]; x10[oq] = x00[oq]; x11[oq] = x00[oq]; }
            tap_mma<T, CG>(x00, wq, 4, A[0]);
            tap_mma<T, CG>(x01, wq, 3, A[1]); tap_mma<T, CG>(x01, wq, 5, A[0]);
            tap_mma<T, CG>(x10, wq, 1, B[0]); tap_mma<T, CG>(x10, wq, 7, A[0]);
            tap_mma<T, CG>(x11, wq, 0, B[1]); tap_mma<T, CG>(x11, wq, 2, B[0]); tap_mma<T, CG>(x11, wq, 6, A[1]); tap_mma<T, CG>(x11, wq, 8, A[0]);
            if (colok) {
                store_quads<T>(vout, xcol[0], (uint32_t)(2 * a) * xrow, x00, nt != 0);
                store_quads<T>(vout, xcol[1], (uint32_t)(2 * a) * xrow, x01, nt != 0);
                store_quads<T>(vout, xcol[0], (uint32_t)(2 * a + 1) * xrow, x10, nt != 0);
                store_quads<T>(vout, xcol[1], (uint32_t)(2 * a + 1) * xrow, x11, nt != 0);
            }
        };
        LaneIn<T> r0[2], r1[2], r2[2];
        load_row(a0, r0); load_row(a0 + 1, r1);
        int a = a0;
#pragma unroll 1
        for (; a + 2 <= a1; a += 2) {
            load_row(a + 2, r2);
            step(a, r0, r1);
            load_row(a + 3, r0);
            step(a + 1, r1, r2);
            // r2 holds row a+2 and r0 row a+3: back in order for the next trip
#pragma unroll
            for (int s = 0; s < 2; ++s) { r1[s] = r0[s]; r0[s] = r2[s]; }
        }
        if (a < a1) step(a, r0, r1);
    }
}

bool gconv_nhwc_mfma_s2_supported(const GGeom &g, int dtype, int pass)
{
    if (const char *e = tune_env("DWCONV_TUNE_GMFMA")) { if (atoi(e) == 0) return false; }
    if (!(g.K == 3 && g.s == 2 && g.p == 1 && g.Cg == g.Og && (g.Cg == 4 || g.Cg == 8))) return false;
    if (g.C % (dtype == DT_F32 ? 64 : 128) != 0) return false;
    if (pass == 1 && (g.H % 2 != 0 || g.W % 2 != 0)) return false;        // backward-data: whole 2x2 blocks
    if (pass > 1) return false;
    return (long long)g.H * g.W * g.C * 4 <= (1ll << 31);
}

template <typename T, int CG>
static hipError_t launch_s2(const GGeom &g, const void *in, const void *w, void *out, bool bwd, hipStream_t st)
{
    int target = 14;
    if (const char *e = tune_env("DWCONV_TUNE_GMTH")) target = atoi(e) > 0 ? atoi(e) : target;
    int nstrips = (g.Ho + target / 2) / target;
    if (nstrips < 1) nstrips = 1;
    const int TH = (g.Ho + nstrips - 1) / nstrips;
    nstrips = (g.Ho + TH - 1) / TH;
    const int ncq = (g.Wo + 3) / 4, ncs = g.C / (64 * LaneIn<T>::LQ);
    const long long per_image = (long long)nstrips * ncq * ncs;
    int NI = (int)((long long)g.N * per_image / 8192);
    if (const char *e = tune_env("DWCONV_TUNE_GMNI")) NI = atoi(e);
    if (NI < 1) NI = 1;
    if (NI > g.N) NI = g.N;
    const long long nw = (long long)((g.N + NI - 1) / NI) * per_image;
    if (nw >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nwaves = (unsigned)nw, nblocks = (unsigned)((nw + 3) / 4);
    const long long out_elems = bwd ? (long long)g.N * g.H * g.W * g.C : (long long)g.N * g.Ho * g.Wo * g.C;
    const int nt = stream_stores("GROUP_NHWC_MFMA", out_elems * (long long)sizeof(T), 0);
    if (bwd)
        hipLaunchKernelGGL((k_gconv_nhwc_mfma_bwd_s2<T, CG>), dim3(nblocks), dim3(256), 0, st, g, (const T *)in, (const T *)w,
                           (T *)out, TH, nstrips, ncq, ncs, NI, nwaves, nblocks, nt);
    else
        hipLaunchKernelGGL((k_gconv_nhwc_mfma_fwd_s2<T, CG>), dim3(nblocks), dim3(256), 0, st, g, (const T *)in, (const T *)w,
                           (T *)out, TH, nstrips, ncq, ncs, NI, nwaves, nblocks, nt);
    return hipGetLastError();
}

hipError_t gconv_nhwc_mfma_s2(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool bwd, hipStream_t st)
{
    if (!gconv_nhwc_mfma_s2_supported(g, dtype, bwd ? 1 : 0)) return hipErrorInvalidValue;
    if (dtype == DT_F32) return g.Cg == 4 ? launch_s2<float, 4>(g, in, w, out, bwd, st) : launch_s2<float, 8>(g, in, w, out, bwd, st);
    return g.Cg == 4 ? launch_s2<bf16_t, 4>(g, in, w, out, bwd, st) : launch_s2<bf16_t, 8>(g, in, w, out, bwd, st);
}

}  // namespace dwc
