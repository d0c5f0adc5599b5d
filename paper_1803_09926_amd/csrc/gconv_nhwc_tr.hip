// Group convolution, NHWC, 3x3 stride 1 pad 1, groups of 4 or 8 channels on both sides: filter gradient (Eq. 4 with the
// sum over a group's channel pairs) on the matrix cores, with the tensors read as in the forward walk.
//
// The sum over pixels is the contraction: dW[o][b][tap] = sum_p dy[o][p] * x[b][p + tap].  A 4x4 matrix instruction
// wants, from lane i of a block, output channel i at a few pixels (A) and, from lane j, input channel j at the same
// pixels shifted by the tap (B); then D[i][j] (register i of lane j) is the sum for the channel pair (i, j).  In NHWC
// a 16-byte load brings the opposite: one pixel, several channels.  So a block of four lanes is one quad of channels
// at four neighbouring pixel columns exactly as in the forward walk (gconv_nhwc_mfma.hip: the wavefront's loads are
// whole contiguous ranges), and the 4x4 tile (4 pixels x 4 channels) is transposed inside the block with cross-lane
// moves: afterwards lane i holds channel i at the four pixels.  bf16: those four values are the packed inner
// dimension of the 4x4x4 instruction; fp32: four 4x4x1 instructions, one per pixel.
//
// A wavefront walks down the rows of NI images at its four pixel columns: step t loads x row t at the three tap
// columns and dy row t+1, transposes the four tiles and adds, for tap row kh, dy row t+1-kh against x row t (a window
// of three transposed dy rows).  The four wavefronts of a thread block take four neighbouring column quads; their
// sums are added through LDS at the end and the block writes one partial per filter entry; the shared second stage
// adds the partials in a fixed order.
#include "gconv_mfma.hpp"

namespace dwc {

__device__ __forceinline__ uint32_t quad_swap1(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false); }   // lane ^ 1
__device__ __forceinline__ uint32_t quad_swap2(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false); }   // lane ^ 2

// One quad of channels at the block's four pixels, transposed: the lane's channel (lane & 3) at pixels 0..3.
template <typename T> struct QuadT;
template <> struct QuadT<float> {
    float p[4];
    __device__ __forceinline__ void zero() { p[0] = p[1] = p[2] = p[3] = 0.f; }
    // c[0..3]: the lane's pixel, channels 0..3 of the quad
    __device__ __forceinline__ void from(const float *c, bool odd, bool hi2)
    {
        float t[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {           // lanes j, j^1 trade: even keeps channel 2h, odd channel 2h+1, at both pixels
            const float send = odd ? c[2 * h] : c[2 * h + 1];
            const float rc = __uint_as_float(quad_swap1(__float_as_uint(send)));
            t[2 * h] = odd ? rc : c[2 * h];
            t[2 * h + 1] = odd ? c[2 * h + 1] : rc;
        }
        // lanes j, j^2 trade pixel pairs: lanes 0, 1 keep channels 0, 1 (t[0..1]), lanes 2, 3 channels 2, 3 (t[2..3])
        const float s0 = hi2 ? t[0] : t[2], s1 = hi2 ? t[1] : t[3];
        const float r0 = __uint_as_float(quad_swap2(__float_as_uint(s0))), r1 = __uint_as_float(quad_swap2(__float_as_uint(s1)));
        p[0] = hi2 ? r0 : t[0]; p[1] = hi2 ? r1 : t[1];
        p[2] = hi2 ? t[2] : r0; p[3] = hi2 ? t[3] : r1;
    }
};
template <> struct QuadT<bf16_t> {
    uint32_t w[2];                              // pixels (0, 1), (2, 3)
    __device__ __forceinline__ void zero() { w[0] = w[1] = 0u; }
    // a0 = channels (0, 1), a1 = channels (2, 3) of the lane's pixel
    __device__ __forceinline__ void from(uint32_t a0, uint32_t a1, bool odd, bool hi2)
    {
        // lanes j, j^1: even lanes take the low halves of both (channels 0 and 2 at pixels j, j+1), odd lanes the high ones
        const uint32_t sel = odd ? 0x03020706u : 0x05040100u;
        const uint32_t w0 = __builtin_amdgcn_perm(quad_swap1(a0), a0, sel), w1 = __builtin_amdgcn_perm(quad_swap1(a1), a1, sel);
        const uint32_t p0 = quad_swap2(w0), p1 = quad_swap2(w1);
        w[0] = hi2 ? p1 : w0;
        w[1] = hi2 ? w1 : p0;
    }
};

template <typename T, int CG, int PF>
__global__ __launch_bounds__(256) void k_gconv_nhwc_tr_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                  float *__restrict__ ws, int ncqb, int ncs, int NI, unsigned nblocks, int J)
{
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG / 4, R = PF + 1;
    constexpr bool SIB = NQ == 2 && LQ == 1;        // fp32 groups of 8: the group's other quad lives in the neighbouring block
    constexpr int NA = NQ == 1 ? LQ : 2 * LQ;       // accumulator sets of a lane: (its dy quad, an x quad of that quad's group)
    __shared__ __align__(16) float red[4][NA][64][4];

    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int cs = lb % ncs; lb /= ncs;
    const int cqb = lb % ncqb; const int ngroup = lb / ncqb;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63, blk = lane >> 2, j = lane & 3;
    const bool odd = j & 1, hi2 = j & 2;
    const int cbase = (cs * 16 + blk) * 4 * LQ;     // the lane's channels: LQ quads from here
    const int col = (cqb * 4 + wv) * 4 + j;         // past the last column: every load reads zero
    const int C = g.C;                              // = g.O

    uint32_t coloff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = col - 1 + kw;
        coloff[kw] = (iw >= 0 && iw < g.W && col < g.W) ? (uint32_t)(iw * C + cbase) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    }
    const uint32_t rowbytes = (uint32_t)g.W * (uint32_t)C * (uint32_t)sizeof(T), imgbytes = (uint32_t)g.H * rowbytes;

    v4f_t acc[NA][3][3];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) acc[a][kh][kw] = v4f_t{0.f, 0.f, 0.f, 0.f};

    auto transpose = [&](const LaneIn<T> &v, QuadT<T> (&q)[LQ]) {
        if constexpr (F32) q[0].from(v.c, odd, hi2);
        else {
            q[0].from(v.w[0], v.w[1], odd, hi2);
            q[1].from(v.w[2], v.w[3], odd, hi2);
        }
    };
    // acc += (dy quad, transposed) x (x quad, transposed), the contraction over the block's four pixels
    auto mma = [&](v4f_t &d, const QuadT<T> &a, const QuadT<T> &b) {
        if constexpr (F32) {
#pragma unroll
            for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f32_4x4x1f32(a.p[k], b.p[k], d, 0, 0, 0);
        } else {
            d = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4s_t, u2w_t{a.w[0], a.w[1]}),
                                                       __builtin_bit_cast(v4s_t, u2w_t{b.w[0], b.w[1]}), d, 0, 0, 0);
        }
    };

    const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
    for (int n = n0; n < n1; ++n) {
        const BufView vx(x + (size_t)n * g.H * g.W * C, imgbytes), vd(dy + (size_t)n * g.H * g.W * C, imgbytes);
        struct Step { LaneIn<T> x[3], d; };             // x row t at the three tap columns, dy row t+1
        Step ring[R];
        auto load_step = [&](int t, Step &s) {
            const uint32_t ro = (uint32_t)min(t, g.H - 1) * rowbytes, rd = (uint32_t)min(t + 1, g.H - 1) * rowbytes;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) s.x[kw].load(vx, coloff[kw], ro);
            s.d.load(vd, coloff[1], rd);
        };
        // the window of transposed dy rows: D[0] = row t+1, D[1] = row t, D[2] = row t-1
        QuadT<T> D[3][LQ];
        {
            LaneIn<T> first;
            first.load(vd, coloff[1], 0u);
            transpose(first, D[1]);
#pragma unroll
            for (int q = 0; q < LQ; ++q) D[2][q].zero();
        }
        auto consume = [&](int t, const Step &s) {
            if (t + 1 < g.H) transpose(s.d, D[0]);
            else {
#pragma unroll
                for (int q = 0; q < LQ; ++q) D[0][q].zero();
            }
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                QuadT<T> X[LQ];
                transpose(s.x[kw], X);
                QuadT<T> S;                             // fp32 groups of 8: the group's other quad of x, from the neighbouring block
                if constexpr (SIB) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) S.p[k] = __shfl_xor(X[0].p[k], 4, 64);
                }
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    if constexpr (NQ == 1) {
#pragma unroll
                        for (int q = 0; q < LQ; ++q) mma(acc[q][kh][kw], D[kh][q], X[q]);
                    } else if constexpr (SIB) {
                        mma(acc[0][kh][kw], D[kh][0], X[0]);
                        mma(acc[1][kh][kw], D[kh][0], S);
                    } else {
#pragma unroll
                        for (int oq = 0; oq < 2; ++oq)
#pragma unroll
                            for (int iq = 0; iq < 2; ++iq) mma(acc[oq * 2 + iq][kh][kw], D[kh][oq], X[iq]);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < LQ; ++q) { D[2][q] = D[1][q]; D[1][q] = D[0][q]; }
        };

#pragma unroll
        for (int p = 0; p < PF; ++p) load_step(p, ring[p]);
        int t = 0;
#pragma unroll 1
        for (; t + R <= g.H; t += R) {
#pragma unroll
            for (int p = 0; p < R; ++p) {
                load_step(t + p + PF, ring[(p + PF) % R]);
                consume(t + p, ring[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < R - 1; ++p)
            if (t + p < g.H) consume(t + p, ring[p]);
    }

    // the block's four wavefronts (four column quads) hold partial sums of the same entries: add them through LDS, one
    // tap at a time, and write the block's partial
    const int part = ngroup * ncqb + cqb;
    float *wsp = ws + (size_t)part * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int i = 0; i < 4; ++i) red[wv][a][lane][i] = acc[a][kh][kw][i];
            __syncthreads();
            if (wv == 0) {
#pragma unroll
                for (int a = 0; a < NA; ++a) {
                    float s[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) s[i] = (red[0][a][lane][i] + red[1][a][lane][i]) + (red[2][a][lane][i] + red[3][a][lane][i]);
                    // set a: the lane's dy quad oq (output channels cbase + 4 oq + i) against input channel b of the group
                    int oq, b;
                    if constexpr (NQ == 1) { oq = a; b = j; }
                    else if constexpr (SIB) { oq = 0; b = ((((cbase >> 2) & 1) ^ a) << 2) + j; }
                    else { oq = a >> 1; b = ((a & 1) << 2) + j; }
                    float *dst = wsp + ((size_t)(kh * 3 + kw) * CG + b) * g.O + cbase + 4 * oq;
                    *reinterpret_cast<float4 *>(dst) = float4{s[0], s[1], s[2], s[3]};
                }
            }
            __syncthreads();
        }
}

// ---- host side ---------------------------------------------------------------------------------------------

bool gconv_nhwc_tr_bwd_filter_supported(const GGeom &g, int dtype)
{
    if (tune_env("DWCONV_TUNE_GNOTR")) return false;
    // bf16 only: there the earlier kernels are bound by their arithmetic (batch 256, groups of 4: 56x56 134 -> 109 us, 28x28
    // 76 -> 58, 14x14 41 -> 28); in fp32 the lane-exchange kernels measured the same or slightly faster (groups of 4: 211
    // against 217 us for the three layers; groups of 8: 82 against 85) and stay
    if (dtype == DT_F32 && !tune_env("DWCONV_TUNE_GTRALL")) return false;
    if (!(g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && (g.Cg == 4 || g.Cg == 8))) return false;
    if (g.C % (dtype == DT_F32 ? 64 : 128) != 0) return false;          // whole wavefronts of channels
    return (long long)g.H * g.W * g.C * 4 <= (1ll << 31);                // an image through a buffer view
}

// blocks = channel slices x column-quad blocks x image groups: about 512, the partial sums within 16 MiB
static void nhwc_tr_tiling(const GGeom &g, int dtype, int *ncqb, int *ncs, int *NI, int *ngroups)
{
    const int wc = dtype == DT_F32 ? 64 : 128;
    *ncs = g.C / wc;
    *ncqb = ((g.W + 3) / 4 + 3) / 4;
    int target = 512;
    if (const char *e = tune_env("DWCONV_TUNE_GTRBLOCKS")) if (atoi(e) > 0) target = atoi(e);
    long long ng = target / ((long long)*ncs * *ncqb);
    const long long J4 = (long long)g.O * g.Cg * 9 * 4;
    const long long cap = (16ll << 20) / (J4 * *ncqb);
    if (ng > cap) ng = cap;
    if (ng > g.N) ng = g.N;
    if (ng < 1) ng = 1;
    *NI = (int)((g.N + ng - 1) / ng);
    if (const char *e = tune_env("DWCONV_TUNE_GTRNI")) if (atoi(e) > 0) *NI = atoi(e) < g.N ? atoi(e) : g.N;
    *ngroups = (g.N + *NI - 1) / *NI;
}

int gconv_nhwc_tr_bwd_filter_parts(const GGeom &g, int dtype)
{
    int ncqb, ncs, NI, ng;
    nhwc_tr_tiling(g, dtype, &ncqb, &ncs, &NI, &ng);
    return ng * ncqb;
}

hipError_t gconv_nhwc_tr_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts, hipStream_t st)
{
    if (!gconv_nhwc_tr_bwd_filter_supported(g, dtype)) return hipErrorInvalidValue;
    int ncqb, ncs, NI, ng;
    nhwc_tr_tiling(g, dtype, &ncqb, &ncs, &NI, &ng);
    if (parts != ng * ncqb) return hipErrorInvalidValue;
    const long long nb = (long long)ncs * ncqb * ng;
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int J = g.O * g.Cg * 9;
#define GO(T, CGG) hipLaunchKernelGGL((k_gconv_nhwc_tr_bwd_filter<T, CGG, 2>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, (const T *)dy, ws, \
                                      ncqb, ncs, NI, nblocks, J)
    if (dtype == DT_F32) { if (g.Cg == 8) GO(float, 8); else GO(float, 4); }
    else                 { if (g.Cg == 8) GO(bf16_t, 8); else GO(bf16_t, 4); }
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
