// Group convolution, NHWC, 3x3 stride 1 pad 1, groups of 4 or 8 channels on both sides: forward and
// backward-data on the matrix cores.
//
// With more than one channel per group the layer is a (small) dense contraction over the group's input
// channels (Section V-B: the depthwise layer as the one-channel case of the group convolution), and at 4 or 8
// channels per group the plain multiply-add form is bound by the vector ALU, not by memory: 9*CG
// multiply-adds per output element.  The 4x4 matrix instructions with 16 independent blocks fit it exactly:
//   D[i][j] += sum_k A[i][k] * B[k][j]   per block,   i = output channel of a quad, j = pixel, k = input channel.
// A wavefront is 16 blocks x 4 lanes: block b = one quad of channels (16 consecutive quads = 64 channels,
// contiguous in NHWC), lane j of the block = one of four neighbouring pixel columns.  The lane loads its
// pixel's quad of input channels as one vector, and that vector IS the B operand (bf16: the 4x4x4
// instruction takes the four packed channels as loaded, no unpacking; fp32: the 4x4x1 instruction takes one
// channel at a time).  A holds the filter: lane i of a block keeps the entries of output channel i.
// D comes out as four registers = the four output channels of the lane's pixel: one vector store.
// Groups of 8: the other quad of the group sits in the neighbouring block; its input vector comes through a
// wavefront shuffle and is multiplied with the filter's other 4x4 sub-block.
//
// The lane walks down the rows of a strip: step t loads input row t at the three columns around its pixel
// (buffer views: a column outside the image reads as the zero of the padding) and feeds tap row kh of output
// row t+1-kh, three rotating accumulators.  Rows outside the image or the strip are skipped under
// wavefront-uniform conditions.  Backward-data is the same walk over dy with the filter transposed inside
// the group and rotated by 180 degrees.
#include "gconv_mfma.hpp"

namespace dwc {

// A wavefront takes 16 blocks x LQ quads of channels (64 channels in fp32, 128 in bf16), four pixel columns, one strip
// of rows of NI consecutive images; its filter entries are loaded once.
template <typename T, int CG, bool FLIP, int PF>
__global__ __launch_bounds__(256) void k_gconv_nhwc_mfma(GGeom g, const T *__restrict__ in, const T *__restrict__ w,
                                                         T *__restrict__ out, int TH, int nstrips, int ncq, int ncs, int NI,
                                                         unsigned nwaves, unsigned nblocks, int nt, int CB)
{
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG <= 4 ? 1 : CG / 4, R = PF + 1;
    constexpr bool SIB = NQ == 2 && LQ == 1;                // the group's other quad lives in the neighbouring block
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    // the wavefront's index, as a scalar: everything derived from it (strip, rows, images) then sits in scalar registers
    // and every condition of the walk is a scalar branch
    unsigned gw = (unsigned)__builtin_amdgcn_readfirstlane((int)(lb * 4 + (threadIdx.x >> 6)));
    if (gw >= nwaves) return;                               // the kernel has no barrier
    const int cs = gw % ncs; gw /= ncs;
    const int cq = gw % ncq; gw /= ncq;
    const int strip = gw % nstrips; const int ngroup = gw / nstrips;

    // CB: blocks that hold one pixel's channels.  16 when the tensor has at least a wavefront's worth of channels; with
    // fewer, the remaining blocks take the next four pixel columns (the wavefront's accesses stay one contiguous range)
    const int lane = threadIdx.x & 63, blk = lane >> 2, j = lane & 3;
    const int cbase = (cs * 16 + blk % CB) * 4 * LQ;        // the lane's channels (read and written): LQ quads from here
    const int col = (cq * (16 / CB) + blk / CB) * 4 + j;
    const int C = g.C;                                      // = g.O

    QuadW<T> wq[LQ][9][NQ];
    load_group_filter<T, CG, FLIP ? 1 : 0>(w, C, cbase, j, wq);

    uint32_t coloff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = col - 1 + kw;
        coloff[kw] = (iw >= 0 && iw < g.W) ? (uint32_t)(iw * C + cbase) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    }
    const bool colok = col < g.W;
    const uint32_t rowbytes = (uint32_t)g.W * (uint32_t)C * (uint32_t)sizeof(T), imgbytes = (uint32_t)g.H * rowbytes;
    const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
    const int t0 = max(oh0 - 1, 0), t1 = min(oh1 + 1, g.H);     // input rows [t0, t1)
    const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);

    for (int n = n0; n < n1; ++n) {
        const BufView vin(in + (size_t)n * g.H * g.W * C, imgbytes), vout(out + (size_t)n * g.H * g.W * C, imgbytes);
        LaneIn<T> ring[R][3];
        auto load_row = [&](int t, LaneIn<T> (&dst)[3]) {
            const uint32_t ro = (uint32_t)min(t, g.H - 1) * rowbytes;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) dst[kw].load(vin, coloff[kw], ro);
        };
        v4f_t D0[LQ], D1[LQ], D2[LQ];                       // output rows t-1, t, t+1
#pragma unroll
        for (int oq = 0; oq < LQ; ++oq) { D0[oq] = v4f_t{0.f, 0.f, 0.f, 0.f}; D1[oq] = D0[oq]; D2[oq] = D0[oq]; }
        auto emit = [&](int row) {
            float o[4 * LQ];
#pragma unroll
            for (int oq = 0; oq < LQ; ++oq)
#pragma unroll
                for (int i = 0; i < 4; ++i) o[4 * oq + i] = D0[oq][i];
            if (colok) store_buf<T, 4 * LQ>(vout, coloff[1], (uint32_t)row * rowbytes, o, nt != 0);
        };
        auto consume = [&](int t, const LaneIn<T> (&src)[3]) {
            // input row t is tap row 2 of output row t-1, tap row 1 of row t, tap row 0 of row t+1.  All three are
            // always computed: at the ends of a strip one or two of these rows lie outside it, and their sums are
            // simply never written (straight-line code; the matrix cores are not what bounds the walk).
            const bool up = t - 1 >= oh0;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                LaneIn<T> sib;
                if constexpr (SIB) sib = src[kw].sibling();
#pragma unroll
                for (int oq = 0; oq < LQ; ++oq)
#pragma unroll
                    for (int iq = 0; iq < NQ; ++iq) {
                        // the registers that hold this input quad, and which quad of them it is
                        const LaneIn<T> &b = (SIB && iq == 1) ? sib : src[kw];
                        const int q = NQ == 1 ? oq : (SIB ? 0 : iq);
                        quad_mma3(D0[oq], D1[oq], D2[oq], wq[oq][6 + kw][iq], wq[oq][3 + kw][iq], wq[oq][kw][iq], b, q);
                    }
            }
            if (up) emit(t - 1);
#pragma unroll
            for (int oq = 0; oq < LQ; ++oq) { D0[oq] = D1[oq]; D1[oq] = D2[oq]; D2[oq] = v4f_t{0.f, 0.f, 0.f, 0.f}; }
        };

#pragma unroll
        for (int p = 0; p < PF; ++p) load_row(t0 + p, ring[p]);
        int t = t0;
#pragma unroll 1
        for (; t + R <= t1; t += R) {
#pragma unroll
            for (int p = 0; p < R; ++p) {
                load_row(t + p + PF, ring[(p + PF) % R]);
                consume(t + p, ring[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < R - 1; ++p)
            if (t + p < t1) consume(t + p, ring[p]);
        // the strip's last row when the image ends with it (no input row below it closes it)
        if (oh1 == g.H) emit(oh1 - 1);
    }
}

bool gconv_nhwc_mfma_supported(const GGeom &g, int dtype)
{
    if (const char *e = tune_env("DWCONV_TUNE_GMFMA")) { if (atoi(e) == 0) return false; }
    if (!(g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && (g.Cg == 2 || g.Cg == 4 || g.Cg == 8))) return false;
    // groups of 2 (a quad = two groups, block-diagonal filter tiles): bf16 only, where the row walk is bound by its
    // arithmetic (112x112, batch 256: 230 us); in fp32 the row walk is the faster one
    if (g.Cg == 2 && !(dtype == DT_BF16 || tune_env("DWCONV_TUNE_GMFMA2F32"))) return false;
    // a wavefront takes 16 lanes' worth of channels at every pixel, 64 channels in fp32 and 128 in bf16, or, of a
    // tensor with fewer channels (a power-of-two fraction of that), several groups of four pixel columns
    const int wc = dtype == DT_F32 ? 64 : 128;
    if (g.C % wc != 0 && !(wc % g.C == 0 && g.C % (wc / 16) == 0)) return false;
    return (long long)g.H * g.W * g.C * 4 <= (1ll << 31);              // an image through a buffer view: at most 2 GiB
}

static inline int cdivm(int a, int b) { return (a + b - 1) / b; }

template <typename T, int CG>
static hipError_t launch_m(const GGeom &g, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    int target = 28;
    if (const char *e = tune_env("DWCONV_TUNE_GMTH")) target = atoi(e) > 0 ? atoi(e) : target;
    int nstrips = (g.H + target / 2) / target;
    if (nstrips < 1) nstrips = 1;
    const int TH = cdivm(g.H, nstrips);
    nstrips = cdivm(g.H, TH);
    const int wc = 64 * LaneIn<T>::LQ;                      // channels of a full wavefront
    const int CB = g.C >= wc ? 16 : g.C / (4 * LaneIn<T>::LQ);
    const int ncq = cdivm(g.W, 4 * (16 / CB)), ncs = g.C >= wc ? g.C / wc : 1;
    // images per wavefront: the filter entries (9*CG registers) are loaded once per wavefront, so as few wavefronts as
    // still fill the chip about twice
    const long long per_image = (long long)nstrips * ncq * ncs;
    int NI = (int)((long long)g.N * per_image / 8192);
    if (const char *e = tune_env("DWCONV_TUNE_GMNI")) NI = atoi(e);
    if (NI < 1) NI = 1;
    if (NI > g.N) NI = g.N;
    const long long nw = (long long)cdivm(g.N, NI) * per_image;
    if (nw >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nwaves = (unsigned)nw, nblocks = (unsigned)((nw + 3) / 4);
    const int nt = stream_stores("GROUP_NHWC_MFMA", (long long)g.N * g.H * g.W * g.C * sizeof(T), 0);
#define GO(FL, PP) hipLaunchKernelGGL((k_gconv_nhwc_mfma<T, CG, FL, PP>), dim3(nblocks), dim3(256), 0, st, g, (const T *)in, \
                                      (const T *)w, (T *)out, TH, nstrips, ncq, ncs, NI, nwaves, nblocks, nt, CB)
    int pf = 2;
    if (const char *e = tune_env("DWCONV_TUNE_GMPF")) pf = atoi(e);
    if (pf == 3) { if (flip) GO(true, 3); else GO(false, 3); }
    else if (pf == 1) { if (flip) GO(true, 1); else GO(false, 1); }
    else { if (flip) GO(true, 2); else GO(false, 2); }
#undef GO
    return hipGetLastError();
}

hipError_t gconv_nhwc_mfma_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    if (!gconv_nhwc_mfma_supported(g, dtype)) return hipErrorInvalidValue;
    if (dtype == DT_F32)
        return g.Cg == 2 ? launch_m<float, 2>(g, in, w, out, flip, st)
                         : g.Cg == 4 ? launch_m<float, 4>(g, in, w, out, flip, st) : launch_m<float, 8>(g, in, w, out, flip, st);
    return g.Cg == 2 ? launch_m<bf16_t, 2>(g, in, w, out, flip, st)
                     : g.Cg == 4 ? launch_m<bf16_t, 4>(g, in, w, out, flip, st) : launch_m<bf16_t, 8>(g, in, w, out, flip, st);
}

}  // namespace dwc
