// Filter gradient (Eq. 4), NHWC, bf16 storage, stride 1, "same" padding: stage 1 with packed dot products.
//
// In bf16 the multiply-add form of this pass is bound by the vector ALU: every loaded element is widened to
// fp32 (one operation) and then takes K*K multiply-adds.  gfx950 has a two-element bf16 dot product with an
// fp32 accumulator (v_dot2c_f32_bf16: d += a.lo*b.lo + a.hi*b.hi).  The sum of Eq. 4 runs over the output
// positions, so the two elements of a dot product are two ROWS of the same channel and column:
//   dw[kh][kw] += dy[oh][ow]*x[oh-P+kh][ow-P+kw] + dy[oh+1][ow]*x[oh+1-P+kh][ow-P+kw].
// NHWC packs two CHANNELS per 32-bit word, so the loaded words of two consecutive rows are re-paired with one
// byte permute per word ({c0,c1}@r, {c0,c1}@r+1 -> {c0@r,c0@r+1}, {c1@r,c1@r+1}); after that a tap costs one
// instruction per channel and row PAIR, with nothing widened: per pair of rows K*K*V dot products and (K+2)*V
// permutes instead of 2*K*K*V multiply-adds and 2*(K+1)*V widenings.
//
// Mapping, tiling and block reduction as k_nhwc_bwd_filter (nhwc.hip): a block is CT channel-vectors x 256/CT
// columns and owns one strip of output rows of NI images; a lane keeps K*K*V fp32 sums.  The walk takes the x
// rows of the strip two at a time; step r (x rows r, r+1) meets, at tap row kh, the dy rows r+P-kh and
// r+P-kh+1.  A window holds those K row pairs of dy; it moves by two rows per step, i.e. two new pairs.
// dy rows outside the block's strip and x rows outside the image are zeroed as loaded (uniform conditions);
// columns outside the image are read outside the buffer view and come back as zero.
#include "kernels.hpp"

namespace dwc {

// words of rows r (lo) and r+1 (hi), each {channel 2j, channel 2j+1} -> {2j@r, 2j@r+1} and {2j+1@r, 2j+1@r+1}
__device__ __forceinline__ uint32_t pair_even(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x05040100u); }
__device__ __forceinline__ uint32_t pair_odd(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

template <int V, int K>
__global__ __launch_bounds__(256) void k_nhwc_bwd_filter_dot2(Geom g, const bf16_t *__restrict__ x,
                                                              const bf16_t *__restrict__ dy, float *__restrict__ ws,
                                                              int CT, int nctiles, int nowtiles, int TH, int nstrips,
                                                              int NI, unsigned nblocks)
{
    static_assert(V % 2 == 0 && K % 2 == 1, "whole 32-bit words of channels, odd filters");
    constexpr int P = (K - 1) / 2, VD = V / 2;
    __shared__ float red[ReduceLds<K, V>::FLOATS];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int Q = g.C / V;
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
        uint32_t coloff[K];
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const int iw = ow - P + kw;
            coloff[kw] = (iw >= 0 && iw < g.W) ? (uint32_t)(iw * g.C + cq * V) * 2u : BufView::OUTSIDE;
        }
        const uint32_t rowbytes = (uint32_t)g.W * (uint32_t)g.C * 2u, imgbytes = (uint32_t)g.H * rowbytes;   // at most 2 GiB
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        const int ra = max(oh0 - P, 0), rb = min(oh1 + P, g.H);       // the x rows this strip's sums need
        const int nsteps = (rb - ra + 1) / 2;

        struct Step { uint32_t x[2][K][VD], d[2][VD]; };              // as loaded: x rows r, r+1 (K columns), dy rows r+P, r+P+1
        for (int n = n0; n < n1; ++n) {
            const BufView xin(x + (size_t)n * g.H * g.W * g.C, imgbytes), dyin(dy + (size_t)n * g.H * g.W * g.C, imgbytes);
            auto load_words = [&](const BufView &b, uint32_t voff, int row, uint32_t (&dst)[VD]) {
                const uint32_t so = (uint32_t)min(max(row, 0), g.H - 1) * rowbytes;
                if constexpr (VD == 1) dst[0] = b.b32(voff, so);
                else if constexpr (VD == 2) { const u2raw_t q = b.b64(voff, so); dst[0] = q.x; dst[1] = q.y; }
                else { static_assert(VD == 4, "2, 4 or 8 channels per lane"); const u4raw_t q = b.b128(voff, so); dst[0] = q.x; dst[1] = q.y; dst[2] = q.z; dst[3] = q.w; }
            };
            auto load_step = [&](int r, Step &s) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) load_words(xin, coloff[kw], r + h, s.x[h][kw]);
                    load_words(dyin, coloff[P], r + P + h, s.d[h]);
                }
            };
            // dp[kh][v]: dy rows (r+P-kh, r+P-kh+1) of channel v; last = the words of dy row r+P-1
            uint32_t dp[K][V], last[VD];
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int v = 0; v < V; ++v) dp[kh][v] = 0u;
#pragma unroll
            for (int j = 0; j < VD; ++j) last[j] = 0u;
            auto consume = [&](int r, const Step &s) {
                // the window moves by two rows: pairs (r+P-1, r+P) and (r+P, r+P+1) enter
                const bool ok0 = r + P >= oh0 && r + P < oh1, ok1 = r + P + 1 >= oh0 && r + P + 1 < oh1;
#pragma unroll
                for (int kh = K - 1; kh > 1; --kh)
#pragma unroll
                    for (int v = 0; v < V; ++v) dp[kh][v] = dp[kh - 2][v];
#pragma unroll
                for (int j = 0; j < VD; ++j) {
                    const uint32_t d0 = ok0 ? s.d[0][j] : 0u, d1 = ok1 ? s.d[1][j] : 0u;
                    dp[1][2 * j] = pair_even(last[j], d0); dp[1][2 * j + 1] = pair_odd(last[j], d0);
                    dp[0][2 * j] = pair_even(d0, d1);      dp[0][2 * j + 1] = pair_odd(d0, d1);
                    last[j] = d1;
                }
                const bool xok0 = r >= 0 && r < g.H, xok1 = r + 1 < g.H;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
#pragma unroll
                    for (int j = 0; j < VD; ++j) {
                        const uint32_t x0 = xok0 ? s.x[0][kw][j] : 0u, x1 = xok1 ? s.x[1][kw][j] : 0u;
                        const uint32_t xe = pair_even(x0, x1), xo = pair_odd(x0, x1);
#pragma unroll
                        for (int kh = 0; kh < K; ++kh) {
                            acc[kh][kw][2 * j] = dot2_bf16(dp[kh][2 * j], xe, acc[kh][kw][2 * j]);
                            acc[kh][kw][2 * j + 1] = dot2_bf16(dp[kh][2 * j + 1], xo, acc[kh][kw][2 * j + 1]);
                        }
                    }
                }
            };

            // the loads of the next step are in flight while this one is accumulated
            Step sa, sb;
            load_step(ra, sa);
            if (oh0 < P) {
                // the first strip of an image (ra = 0): the dy rows 0 .. P-1 belong to the strip but lie above the rows the
                // first step brings (P, P+1).  They enter the window one row at a time; everything above them is zero.
                uint32_t top[P][VD];
#pragma unroll
                for (int t = 0; t < P; ++t) load_words(dyin, coloff[P], t, top[t]);
#pragma unroll
                for (int t = 0; t < P; ++t) {
                    const bool ok = t >= oh0 && t < oh1;
#pragma unroll
                    for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                        for (int v = 0; v < V; ++v) dp[kh][v] = dp[kh - 1][v];
#pragma unroll
                    for (int j = 0; j < VD; ++j) {
                        const uint32_t cur = ok ? top[t][j] : 0u;
                        dp[0][2 * j] = pair_even(last[j], cur); dp[0][2 * j + 1] = pair_odd(last[j], cur);
                        last[j] = cur;
                    }
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

    // ---- fixed-order block reduction (as in k_nhwc_bwd_filter) ----
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * (K * K * g.O);
    block_reduce_taps<K, V>(acc, CT, red, [&](int kh, int kw, int v, float total) {
        if (cq < Q) wsp[(kh * K + kw) * g.O + cq * V + v] = total;
    });
}

bool nhwc_bwd_filter_dot2_supported(const Geom &g, int V)
{
    if (const char *e = tune_env("DWCONV_TUNE_DOT2")) { if (atoi(e) == 0) return false; }
    if (!(g.s == 1 && g.m == 1 && (g.K == 3 || g.K == 5) && g.p == (g.K - 1) / 2)) return false;
    if ((long long)g.H * g.W * g.C * 2 > (1ll << 31)) return false;               // one image through a buffer view
    // 5x5 with two channels per lane (four measured 30 % slower: 100 sums per lane), 3x3 with four or eight
    return (g.K == 5 && V == 2) || (g.K == 3 && (V == 8 || V == 4));
}

hipError_t nhwc_bwd_filter_dot2(const Geom &g, int V, const void *x, const void *dy, float *ws, int CT, int nctiles,
                                int nowtiles, int TH, int nstrips, int NI, unsigned nblocks, hipStream_t st)
{
    if (!nhwc_bwd_filter_dot2_supported(g, V)) return hipErrorInvalidValue;
#define GO(VV, KK) hipLaunchKernelGGL((k_nhwc_bwd_filter_dot2<VV, KK>), dim3(nblocks), dim3(256), 0, st, g, (const bf16_t *)x, \
                                      (const bf16_t *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks)
    if (g.K == 5) GO(2, 5);
    else if (V == 8) GO(8, 3);
    else GO(4, 3);
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
