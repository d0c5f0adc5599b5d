// Group convolution, NHWC, 3x3 stride 1 pad 1, groups of 2, 4 or 8 channels on the side that is read.
//
// The channels of a group are contiguous in a pixel, so the depthwise row-walk carries over: a lane owns OB
// consecutive channels of the tensor that is written, at one pixel column, and walks down the rows of its
// strip.  Per input row it loads, for each of the three columns it needs, the CG channels of its group (one or
// two 16-byte vectors; the lanes of a group load the same addresses, which the memory pipeline merges), and
// updates two rotating rows of accumulators plus the finished output row: 9*CG*OB multiply-adds.  The lane's
// 9*CG*OB filter entries stay in registers for the whole walk (OB is chosen so that they are at most 72).
// Columns outside the image get zeroed weights; rows outside the image are handled as in the depthwise
// kernel (the walk starts at the first valid row, rows below the image only flush the accumulators).
// Backward-data is the same walk over dy with the channel roles swapped and the taps reversed.
//
// Filter gradient: same lane mapping (OB output channels of one column), 9*CG*OB sums per lane.  Step r of
// the walk takes x row r (three columns, CG channels) and dy row r+1 (own column, OB channels); x row r meets
// dy rows r+1, r, r-1 at tap rows 0, 1, 2, so a window of three dy rows rotates.  Sums are added over the
// columns of the block (wavefront butterfly, then LDS across the wavefronts) in a fixed order; one partial
// per block and weight entry goes to the workspace for the shared second stage.
#include "gconv.hpp"

namespace dwc {

// CG consecutive channels as loaded (bf16 stays packed until used)
template <typename T, int CG> struct InVec {
    static constexpr int VW = CG <= 4 ? CG : 4, NV = CG / VW;
    RawVec<T, VW> v[NV];
    __device__ __forceinline__ void load(const T *p)
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) v[i].load(p + i * VW);
    }
    __device__ __forceinline__ void get(float (&r)[CG]) const
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            float t[VW];
            v[i].get(t);
#pragma unroll
            for (int j = 0; j < VW; ++j) r[i * VW + j] = t[j];
        }
    }
};

// filter entry (kh, kw, ci, o) of the NHWC layout [3][3][Cg][O]
__device__ __forceinline__ int wat_nhwc(const GGeom &g, int kh, int kw, int ci, int o) { return ((kh * 3 + kw) * g.Cg + ci) * g.O + o; }

// GPL = groups per lane: with two channels per group a lane takes two adjacent groups (then OB is the whole
// group), so that its loads and stores are 16 bytes wide.
template <typename T, int CG, int OB, int GPL, int PF, bool FLIP>
__global__ __launch_bounds__(256) void k_gconv_nhwc_s1(GGeom g, const T *__restrict__ in, const T *__restrict__ w,
                                                       T *__restrict__ out, int TH, int nstrips, int nchunks,
                                                       unsigned nblocks, int nt)
{
    constexpr int R = PF + 1;
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int chunk = lb % nchunks; const int n = lb / nchunks;

    const int CIT = FLIP ? g.O : g.C, COT = FLIP ? g.C : g.O;     // channels per pixel: read, written
    const int CGW = FLIP ? g.Cg : g.Og;                           // channels per group in the tensor written
    constexpr int OL = OB * GPL, IL = CG * GPL;                   // channels written / read per lane
    const int Q = COT / OL;
    const int f = chunk * blockDim.x + threadIdx.x;
    if (f >= g.W * Q) return;
    const int cq = f % Q, ow = f / Q;
    const int o0 = cq * OL, grp = o0 / CGW, sub = o0 % CGW;      // GPL > 1: sub == 0 and OB == CGW

    int coloff[3];
    float wr[3][3][GPL][CG][OB];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = ow - 1 + kw;
        const bool ok = iw >= 0 && iw < g.W;
        coloff[kw] = (ok ? iw - ow : 0) * CIT;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int gi = 0; gi < GPL; ++gi)
#pragma unroll
                for (int b = 0; b < CG; ++b)
#pragma unroll
                    for (int a = 0; a < OB; ++a) {
                        // forward: output o0+gi*OB+a from input b of its group; backward-data: dx channel sub+a of
                        // group grp+gi from dy channel b of that group, taps reversed
                        const int idx = FLIP ? wat_nhwc(g, 2 - kh, 2 - kw, sub + a, (grp + gi) * g.Og + b)
                                             : wat_nhwc(g, kh, kw, b, o0 + gi * OB + a);
                        const float wv = ldf(w + idx);     // unconditional: a select, not a branch per entry
                        wr[kh][kw][gi][b][a] = ok ? wv : 0.f;
                    }
    }

    const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
    const int rowstride = g.W * CIT, orowstride = g.W * COT;
    const T *xin = in + (size_t)n * g.H * rowstride + (size_t)ow * CIT + grp * CG;
    T *yout = out + (size_t)n * g.H * orowstride + (size_t)ow * COT + o0;

    float acc[2][OL];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int a = 0; a < OL; ++a) acc[j][a] = 0.f;

    const int r0 = oh0 - 1, r1 = oh1 + 1;
    const int ra = max(r0, 0), rb = min(r1, g.H);
    InVec<T, IL> ring[R][3];
    auto load_row = [&](int r, InVec<T, IL> (&dst)[3]) {
        const T *rp = xin + (size_t)min(r, rb - 1) * rowstride;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) dst[kw].load(rp + coloff[kw]);
    };
    auto consume = [&](int r, const InVec<T, IL> (&raw)[3]) {
        // input row r is tap row kh of output row r + 1 - kh
        float cur[3][IL];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) raw[kw].get(cur[kw]);
        float o[OL];
#pragma unroll
        for (int gi = 0; gi < GPL; ++gi)
#pragma unroll
            for (int a = 0; a < OB; ++a) {
                float s2 = acc[0][gi * OB + a], s1 = acc[1][gi * OB + a], s0 = 0.f;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                    for (int b = 0; b < CG; ++b) {
                        s2 = fmaf(wr[2][kw][gi][b][a], cur[kw][gi * CG + b], s2);
                        s1 = fmaf(wr[1][kw][gi][b][a], cur[kw][gi * CG + b], s1);
                        s0 = fmaf(wr[0][kw][gi][b][a], cur[kw][gi * CG + b], s0);
                    }
                o[gi * OB + a] = s2; acc[0][gi * OB + a] = s1; acc[1][gi * OB + a] = s0;
            }
        const int oh = r - 1;
        if (oh >= oh0) store_vec<T, OL>(yout + (size_t)oh * orowstride, o, nt != 0);
    };

#pragma unroll
    for (int j = 0; j < PF; ++j) load_row(ra + j, ring[j]);
    int base = ra;
#pragma unroll 1
    for (; base + R <= rb; base += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            load_row(base + j + PF, ring[(j + PF) % R]);
            consume(base + j, ring[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < R - 1; ++j)
        if (base + j < rb) consume(base + j, ring[j]);
    // rows below the image: zero rows, each completes one more output row
    for (int r = rb; r < r1; ++r) {
        float o[OL];
#pragma unroll
        for (int a = 0; a < OL; ++a) { o[a] = acc[0][a]; acc[0][a] = acc[1][a]; acc[1][a] = 0.f; }
        const int oh = r - 1;
        if (oh >= oh0) store_vec<T, OL>(yout + (size_t)oh * orowstride, o, nt != 0);
    }
}

// Filter gradient, stage 1.  Block: CT lanes over the OB-channel sub-vectors x 256/CT columns, one strip of
// NI images.  ws[part][kh][kw][ci][o].
template <typename T, int CG, int OB>
__global__ __launch_bounds__(256) void k_gconv_nhwc_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                               float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                               int TH, int nstrips, int NI, unsigned nblocks, int J)
{
    __shared__ float red[4][CG * OB][64];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int Q = g.O / OB;
    const int cq = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = cq < Q && ow < g.W;
    const int o0 = cq * OB, grp = o0 / g.Og;

    float acc[3][3][CG][OB];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
#pragma unroll
            for (int b = 0; b < CG; ++b)
#pragma unroll
                for (int a = 0; a < OB; ++a) acc[kh][kw][b][a] = 0.f;

    if (active) {
        bool colok[3];
        int coloff[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int iw = ow - 1 + kw;
            colok[kw] = iw >= 0 && iw < g.W;
            coloff[kw] = (colok[kw] ? iw : ow) * g.C;
        }
        const int xrow = g.W * g.C, drow = g.W * g.O;
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        for (int n = n0; n < n1; ++n) {
            const T *xin = x + (size_t)n * g.H * xrow + grp * CG;
            const T *dyin = dy + ((size_t)n * g.H * g.W + ow) * g.O + o0;
            float dyw[3][OB];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int a = 0; a < OB; ++a) dyw[kh][a] = 0.f;
            // step r: x row r and dy row r+1; one step ahead in registers
            InVec<T, CG> xr[2][3];
            RawVec<T, OB> dr[2];
            auto load_step = [&](int r, InVec<T, CG> (&xd)[3], RawVec<T, OB> &dd) {
                const T *xp = xin + (size_t)min(max(r, 0), g.H - 1) * xrow;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) xd[kw].load(xp + coloff[kw]);
                dd.load(dyin + (size_t)min(max(r + 1, 0), g.H - 1) * drow);
            };
            auto consume = [&](int r, const InVec<T, CG> (&xd)[3], const RawVec<T, OB> &dd) {
                const bool xok = r >= 0 && r < g.H;
                const bool dok = r + 1 >= oh0 && r + 1 < oh1;       // only dy rows of this block's strip count
                float d[OB];
                dd.get(d);
#pragma unroll
                for (int a = 0; a < OB; ++a) { dyw[2][a] = dyw[1][a]; dyw[1][a] = dyw[0][a]; dyw[0][a] = dok ? d[a] : 0.f; }
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    float xv[CG];
                    xd[kw].get(xv);
#pragma unroll
                    for (int b = 0; b < CG; ++b) {
                        const float xx = xok ? xv[b] : 0.f;
#pragma unroll
                        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                            for (int a = 0; a < OB; ++a) acc[kh][kw][b][a] = fmaf(dyw[kh][a], xx, acc[kh][kw][b][a]);
                    }
                }
            };
            // x rows oh0-1 .. oh1: TH + 2 steps
            const int r0 = oh0 - 1, nsteps = (oh1 - oh0) + 2;
            load_step(r0, xr[0], dr[0]);
            int i = 0;
#pragma unroll 1
            for (; i + 2 <= nsteps; i += 2) {
                load_step(r0 + i + 1, xr[1], dr[1]);
                consume(r0 + i, xr[0], dr[0]);
                load_step(r0 + i + 2, xr[0], dr[0]);
                consume(r0 + i + 1, xr[1], dr[1]);
            }
            if (i < nsteps) consume(r0 + i, xr[0], dr[0]);
        }
        // taps on columns outside the image accumulated clamped data: drop them
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
            if (!colok[kw]) {
#pragma unroll
                for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                    for (int b = 0; b < CG; ++b)
#pragma unroll
                        for (int a = 0; a < OB; ++a) acc[kh][kw][b][a] = 0.f;
            }
    }

    // fixed-order block reduction, one tap at a time
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int b = 0; b < CG; ++b)
#pragma unroll
                for (int a = 0; a < OB; ++a) red[wv][b * OB + a][lane] = wave_sum_strided(acc[kh][kw][b][a], CT);
            __syncthreads();
            if (wv == 0 && lane < CT && cq < Q) {
#pragma unroll
                for (int b = 0; b < CG; ++b)
#pragma unroll
                    for (int a = 0; a < OB; ++a) {
                        const int e = b * OB + a;
                        wsp[((kh * 3 + kw) * g.Cg + b) * g.O + o0 + a] =
                            (red[0][e][lane] + red[1][e][lane]) + (red[2][e][lane] + red[3][e][lane]);
                    }
            }
            __syncthreads();
        }
}

// The same filter gradient in bf16 with packed dot products (see nhwc_dot2.hip): the sum runs over output positions, so two
// consecutive ROWS of one channel form the two elements of v_dot2c_f32_bf16 after one byte permute per loaded word;
// the walk takes the strip's x rows two at a time against a window of three dy row pairs, and every (tap, input
// channel, output channel) sum costs one instruction per row pair with nothing widened.  Mapping, tiling, workspace
// layout and block reduction of k_gconv_nhwc_bwd_filter; loads go through buffer views (a column outside the image
// reads as zero).
__device__ __forceinline__ uint32_t gpair_even(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x05040100u); }
__device__ __forceinline__ uint32_t gpair_odd(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

template <int CG, int OB>
__global__ __launch_bounds__(256) void k_gconv_nhwc_bwd_filter_dot2(GGeom g, const bf16_t *__restrict__ x,
                                                                    const bf16_t *__restrict__ dy, float *__restrict__ ws, int CT,
                                                                    int nctiles, int nowtiles, int TH, int nstrips, int NI,
                                                                    unsigned nblocks, int J)
{
    static_assert(CG % 2 == 0 && OB % 2 == 0, "whole 32-bit words of channels");
    constexpr int XD = CG / 2, DD = OB / 2;
    __shared__ float red[4][CG * OB][64];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int Q = g.O / OB;
    const int cq = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = cq < Q && ow < g.W;
    const int o0 = cq * OB, grp = o0 / g.Og;

    float acc[3][3][CG][OB];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
#pragma unroll
            for (int b = 0; b < CG; ++b)
#pragma unroll
                for (int a = 0; a < OB; ++a) acc[kh][kw][b][a] = 0.f;

    if (active) {
        uint32_t xoff[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int iw = ow - 1 + kw;
            xoff[kw] = (iw >= 0 && iw < g.W) ? (uint32_t)(iw * g.C + grp * CG) * 2u : BufView::OUTSIDE;
        }
        const uint32_t doff = (uint32_t)(ow * g.O + o0) * 2u;
        const uint32_t xrow = (uint32_t)g.W * (uint32_t)g.C * 2u, drow = (uint32_t)g.W * (uint32_t)g.O * 2u;
        const uint32_t ximg = (uint32_t)g.H * xrow, dimg = (uint32_t)g.H * drow;             // at most 2 GiB each
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        const int ra = max(oh0 - 1, 0), rb = min(oh1 + 1, g.H);       // the x rows this strip's sums need
        const int nsteps = (rb - ra + 1) / 2;

        struct Step { uint32_t x[2][3][XD], d[2][DD]; };              // x rows r, r+1 (three columns), dy rows r+1, r+2
        for (int n = n0; n < n1; ++n) {
            const BufView xin(x + (size_t)n * g.H * g.W * g.C, ximg), dyin(dy + (size_t)n * g.H * g.W * g.O, dimg);
            auto load_x = [&](uint32_t voff, int row, uint32_t (&dst)[XD]) {
                const uint32_t so = (uint32_t)min(max(row, 0), g.H - 1) * xrow;
                if constexpr (XD == 1) dst[0] = xin.b32(voff, so);
                else if constexpr (XD == 2) { const u2raw_t q = xin.b64(voff, so); dst[0] = q.x; dst[1] = q.y; }
                else { static_assert(XD == 4, "2, 4 or 8 channels per group"); const u4raw_t q = xin.b128(voff, so); dst[0] = q.x; dst[1] = q.y; dst[2] = q.z; dst[3] = q.w; }
            };
            auto load_d = [&](int row, uint32_t (&dst)[DD]) {
                const uint32_t so = (uint32_t)min(max(row, 0), g.H - 1) * drow;
                if constexpr (DD == 1) dst[0] = dyin.b32(doff, so);
                else { static_assert(DD == 2, "2 or 4 output channels per lane"); const u2raw_t q = dyin.b64(doff, so); dst[0] = q.x; dst[1] = q.y; }
            };
            auto load_step = [&](int r, Step &s) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) load_x(xoff[kw], r + h, s.x[h][kw]);
                    load_d(r + 1 + h, s.d[h]);
                }
            };
            // dp[kh][a]: dy rows (r+1-kh, r+2-kh) of output channel a; last = the words of dy row r
            uint32_t dp[3][OB], last[DD];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int a = 0; a < OB; ++a) dp[kh][a] = 0u;
#pragma unroll
            for (int j = 0; j < DD; ++j) last[j] = 0u;

            auto consume = [&](int r, const Step &s) {
                // the window moves by two rows: pairs (r, r+1) and (r+1, r+2) enter
                const bool ok0 = r + 1 >= oh0 && r + 1 < oh1, ok1 = r + 2 >= oh0 && r + 2 < oh1;
#pragma unroll
                for (int a = 0; a < OB; ++a) dp[2][a] = dp[0][a];
#pragma unroll
                for (int j = 0; j < DD; ++j) {
                    const uint32_t d0 = ok0 ? s.d[0][j] : 0u, d1 = ok1 ? s.d[1][j] : 0u;
                    dp[1][2 * j] = gpair_even(last[j], d0); dp[1][2 * j + 1] = gpair_odd(last[j], d0);
                    dp[0][2 * j] = gpair_even(d0, d1);      dp[0][2 * j + 1] = gpair_odd(d0, d1);
                    last[j] = d1;
                }
                const bool xok0 = r >= 0 && r < g.H, xok1 = r + 1 < g.H;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                    for (int j = 0; j < XD; ++j) {
                        const uint32_t x0 = xok0 ? s.x[0][kw][j] : 0u, x1 = xok1 ? s.x[1][kw][j] : 0u;
                        const uint32_t xe = gpair_even(x0, x1), xo = gpair_odd(x0, x1);
#pragma unroll
                        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                            for (int a = 0; a < OB; ++a) {
                                acc[kh][kw][2 * j][a] = dot2_bf16(dp[kh][a], xe, acc[kh][kw][2 * j][a]);
                                acc[kh][kw][2 * j + 1][a] = dot2_bf16(dp[kh][a], xo, acc[kh][kw][2 * j + 1][a]);
                            }
                    }
            };

            Step sa, sb;
            load_step(ra, sa);
            if (oh0 < 1) {
                // the first strip of an image (ra = 0): dy row 0 belongs to the strip but lies above the rows the first step
                // brings (1, 2); it enters the window as the pair (row -1 = zero, row 0)
                uint32_t top[DD];
                load_d(0, top);
#pragma unroll
                for (int a = 0; a < OB; ++a) { dp[2][a] = dp[1][a]; dp[1][a] = dp[0][a]; }
#pragma unroll
                for (int j = 0; j < DD; ++j) {
                    const uint32_t cur = oh1 > 0 ? top[j] : 0u;
                    dp[0][2 * j] = gpair_even(last[j], cur); dp[0][2 * j + 1] = gpair_odd(last[j], cur);
                    last[j] = cur;
                }
            }
            int i = 0;
#pragma unroll 1
            for (; i + 2 <= nsteps; i += 2) {
                load_step(ra + 2 * i + 2, sb);
                consume(ra + 2 * i, sa);
                load_step(ra + 2 * i + 4, sa);
                consume(ra + 2 * i + 2, sb);
            }
            if (i < nsteps) consume(ra + 2 * i, sa);
        }
    }

    // fixed-order block reduction, one tap at a time
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int b = 0; b < CG; ++b)
#pragma unroll
                for (int a = 0; a < OB; ++a) red[wv][b * OB + a][lane] = wave_sum_strided(acc[kh][kw][b][a], CT);
            __syncthreads();
            if (wv == 0 && lane < CT && cq < Q) {
#pragma unroll
                for (int b = 0; b < CG; ++b)
#pragma unroll
                    for (int a = 0; a < OB; ++a) {
                        const int e = b * OB + a;
                        wsp[((kh * 3 + kw) * g.Cg + b) * g.O + o0 + a] =
                            (red[0][e][lane] + red[1][e][lane]) + (red[2][e][lane] + red[3][e][lane]);
                    }
            }
            __syncthreads();
        }
}

// ---- host side ---------------------------------------------------------------------------------------------

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// channels written per lane: as many as keep the lane's 9*CG*OB filter entries within 72 registers
static int nhwc_ob(int CG, int CGW)
{
    int ob = 72 / (9 * CG);
    if (ob > 4) ob = 4;
    while (ob > 1 && (CGW % ob != 0 || (ob & (ob - 1)) != 0)) --ob;
    return ob < 1 ? 1 : ob;
}

bool gconv_nhwc_supported(const GGeom &g)
{
    if (!(g.K == 3 && g.s == 1 && g.p == 1)) return false;
    // both directions: the channels read per group are 2, 4 or 8 (forward reads Cg, backward-data reads Og)
    const bool cg_ok = g.Cg == 2 || g.Cg == 4 || g.Cg == 8, og_ok = g.Og == 2 || g.Og == 4 || g.Og == 8;
    return cg_ok && og_ok;
}

static int nhwc_pick_th(int rows)
{
    const int target = 28;
    int ns = (rows + target / 2) / target;
    if (ns < 1) ns = 1;
    return cdiv(rows, ns);
}

template <typename T, int CG, int OB, int GPL, int PF>
static hipError_t launch_gs1(const GGeom &g, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    const int COT = flip ? g.C : g.O;
    const int lanes = g.W * (COT / (OB * GPL));
    const int bs = 256;
    const char *eth = tune_env("DWCONV_TUNE_GHTH");
    const int TH = eth && atoi(eth) > 0 ? atoi(eth) : nhwc_pick_th(g.H);
    const int nchunks = cdiv(lanes, bs), nstrips = cdiv(g.H, TH);
    const long long nb = (long long)g.N * nchunks * nstrips;
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int nt = stream_stores(flip ? "GROUP_NHWC_BWD" : "GROUP_NHWC_FWD", (long long)g.N * g.H * g.W * COT * sizeof(T), 0);
    if (flip)
        hipLaunchKernelGGL((k_gconv_nhwc_s1<T, CG, OB, GPL, PF, true>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)in,
                           (const T *)w, (T *)out, TH, nstrips, nchunks, nblocks, nt);
    else
        hipLaunchKernelGGL((k_gconv_nhwc_s1<T, CG, OB, GPL, PF, false>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)in,
                           (const T *)w, (T *)out, TH, nstrips, nchunks, nblocks, nt);
    return hipGetLastError();
}

hipError_t gconv_nhwc_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    if (!gconv_nhwc_supported(g)) return hipErrorInvalidValue;
    if (gconv_nhwc_mfma_supported(g, dtype)) return gconv_nhwc_mfma_s1(g, dtype, in, w, out, flip, st);
    if (gconv_nhwc_xchg_supported(g)) return gconv_nhwc_xchg_s1(g, dtype, in, w, out, flip, st);
    const int CG = flip ? g.Og : g.Cg, CGW = flip ? g.Cg : g.Og;
    const int OB = nhwc_ob(CG, CGW);
    // two channels per group on both sides and an even number of groups: two groups per lane
    const int GPL = (CG == 2 && CGW == 2 && g.G % 2 == 0 && !tune_env("DWCONV_TUNE_GGPL1")) ? 2 : 1;
#define TRY(T, CGG, OBB, GG, PPF) if (CG == CGG && OB == OBB && GPL == GG) return launch_gs1<T, CGG, OBB, GG, PPF>(g, in, w, out, flip, st)
    if (dtype == DT_F32) {
        TRY(float, 2, 4, 1, 2); TRY(float, 2, 2, 1, 2); TRY(float, 2, 2, 2, 2); TRY(float, 4, 2, 1, 2); TRY(float, 4, 1, 1, 2); TRY(float, 8, 1, 1, 1);
    } else {
        TRY(bf16_t, 2, 4, 1, 2); TRY(bf16_t, 2, 2, 1, 2); TRY(bf16_t, 2, 2, 2, 2); TRY(bf16_t, 4, 2, 1, 2); TRY(bf16_t, 4, 1, 1, 2); TRY(bf16_t, 8, 1, 1, 1);
    }
#undef TRY
    return hipErrorInvalidValue;
}

// Which filter-gradient kernel: the lane-exchange one where it applies, except for bf16 groups of 4, where its
// 2-byte loads per lane measured slower than the 8-byte ones of the first form (groups of 8: the other way round).
static bool nhwc_bwd_filter_xchg(const GGeom &g, int dtype)
{
    if (!gconv_nhwc_xchg_supported(g) || tune_env("DWCONV_TUNE_GNOXCHGW")) return false;
    return !(dtype == DT_BF16 && g.Cg == 4) || tune_env("DWCONV_TUNE_GXCHGW");
}

// Filter-gradient tiling.  CT: lanes over sub-vectors (a power of two up to 64), 256/CT columns per block.
static void gconv_nhwc_bwd_filter_tiling(const GGeom &g, int dtype, int *OBp, int *CT, int *nctiles, int *nowtiles, int *TH,
                                         int *nstrips, int *NI, int *ngroups)
{
    // the lane-exchange kernel takes one channel per lane
    const int OB = nhwc_bwd_filter_xchg(g, dtype) ? 1 : nhwc_ob(g.Cg, g.Og);
    const int Q = g.O / OB;
    int ct = 1;
    while (ct < 64 && ct < Q) ct *= 2;
    const int nct = cdiv(Q, ct), nowt = cdiv(g.W, 256 / ct);
    // whole columns unless the launch would have too few blocks; then about two blocks per compute unit,
    // a block walking several images when there are plenty
    int th = g.H;
    const long long per_strip = (long long)nct * nowt * g.N;
    while (th > 7 && per_strip * cdiv(g.H, th) < 384) th = (th + 1) / 2;
    int ni = 1;
    while (ni < g.N && per_strip * cdiv(g.H, th) / (ni * 2) >= 384) ni *= 2;
    if (const char *e = tune_env("DWCONV_TUNE_GHWTH")) if (atoi(e) > 0) th = atoi(e);
    if (const char *e = tune_env("DWCONV_TUNE_GHWNI")) if (atoi(e) > 0) ni = atoi(e);
    const long long J = (long long)g.O * g.Cg * 9;
    while ((long long)nowt * cdiv(g.H, th) * cdiv(g.N, ni) * J * 4 > (64ll << 20)) {
        if (ni < g.N) ni *= 2; else if (th < g.H) th *= 2; else break;
    }
    *OBp = OB; *CT = ct; *nctiles = nct; *nowtiles = nowt; *TH = th; *nstrips = cdiv(g.H, th); *NI = ni;
    *ngroups = cdiv(g.N, ni);
}

int gconv_nhwc_bwd_filter_parts(const GGeom &g, int dtype)
{
    int OB, CT, nct, nowt, TH, nst, NI, ngr;
    gconv_nhwc_bwd_filter_tiling(g, dtype, &OB, &CT, &nct, &nowt, &TH, &nst, &NI, &ngr);
    return nowt * nst * ngr;
}

hipError_t gconv_nhwc_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts,
                                 hipStream_t st)
{
    if (!gconv_nhwc_supported(g)) return hipErrorInvalidValue;
    int OB, CT, nct, nowt, TH, nst, NI, ngr;
    gconv_nhwc_bwd_filter_tiling(g, dtype, &OB, &CT, &nct, &nowt, &TH, &nst, &NI, &ngr);
    if (parts != nowt * nst * ngr) return hipErrorInvalidValue;
    const long long nb = (long long)nct * nowt * nst * ngr;
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int J = g.O * g.Cg * 9;
    if (nhwc_bwd_filter_xchg(g, dtype))
        return gconv_nhwc_xchg_bwd_filter(g, dtype, x, dy, ws, CT, nct, nowt, TH, nst, NI, nblocks, J, st);
    // bf16 with an even number of channels on both sides of the lane: the dot-product form (image sizes within a buffer view)
    const bool d2 = dtype == DT_BF16 && !tune_env("DWCONV_TUNE_GNODOT2") && (long long)g.H * g.W * g.C * 2 <= (1ll << 31) &&
                    (long long)g.H * g.W * g.O * 2 <= (1ll << 31);
#define TRYD(CGG, OBB) if (d2 && g.Cg == CGG && OB == OBB) { hipLaunchKernelGGL((k_gconv_nhwc_bwd_filter_dot2<CGG, OBB>), dim3(nblocks), dim3(256), 0, st, g, (const bf16_t *)x, (const bf16_t *)dy, ws, CT, nct, nowt, TH, nst, NI, nblocks, J); return hipGetLastError(); }
    TRYD(2, 4); TRYD(2, 2); TRYD(4, 2);
#undef TRYD
#define TRY(T, CGG, OBB) if (g.Cg == CGG && OB == OBB) { hipLaunchKernelGGL((k_gconv_nhwc_bwd_filter<T, CGG, OBB>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, (const T *)dy, ws, CT, nct, nowt, TH, nst, NI, nblocks, J); return hipGetLastError(); }
    if (dtype == DT_F32) {
        TRY(float, 2, 4); TRY(float, 2, 2); TRY(float, 4, 2); TRY(float, 4, 1); TRY(float, 8, 1);
    } else {
        TRY(bf16_t, 2, 4); TRY(bf16_t, 2, 2); TRY(bf16_t, 4, 2); TRY(bf16_t, 4, 1); TRY(bf16_t, 8, 1);
    }
#undef TRY
    return hipErrorInvalidValue;
}

}  // namespace dwc
