// Group convolution, NHWC, 3x3 stride 1 pad 1, groups of 4 or 8 channels on both sides: lane-exchange walk.
//
// In NHWC the channels of a group are neighbours in memory, so the lanes that own them are neighbours in the
// wavefront.  A lane owns V consecutive channels (of the tensor read AND of the tensor written: both have the
// same channels per group here) at one pixel column and walks down the rows.  Per input row it loads only its
// own V channels at the three columns it needs; the channels of the other CG/V - 1 lanes of its group come
// through the cross-lane operand path of the vector ALU (DPP: quad permutes and the half-row mirror reach
// lane l^j for every j < 8), folded into the multiply-add that uses them.  Every input element is therefore
// loaded by exactly one lane per column tap (the first kernel of this family loaded each 8-channel group eight
// times), and loads, stores and arithmetic stay at 9*CG*V multiply-adds per four memory instructions.
// The lane's 9*CG*V filter entries stay in registers; a block walks NI images so that loading them is paid
// once per NI*TH rows.  Backward-data is the same walk over dy with the channel roles swapped and taps reversed.
#include "gconv.hpp"

namespace dwc {

template <int CTRL> __device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// half-row mirror: lane l of every 8 reads lane l^7
__device__ __forceinline__ float half_mirror(float v) { return dpp_f<0x141>(v); }

// s[kh] += w[j][kh] * (v of lane l^j), j < NP (2 or 4), kh < 3: quad permutes [1,0,3,2], [2,3,0,1], [3,2,1,0]
// are l^1, l^2, l^3.  The cross-lane read is the DPP operand of the multiply-add itself; the compiler folds a
// DPP move into a multiply but not into a multiply-add, so the instructions are written out.  A DPP operand
// must not have been written by one of the two preceding vector-ALU instructions: the block starts with the
// three plain multiply-adds, so whatever produced v is at least three instructions back.
#define DWC_FMAC "v_fmac_f32_e32 "
#define DWC_DPP(perm) " quad_perm:[" perm "] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
template <int NP>
__device__ __forceinline__ void fma_quad(float &s0, float &s1, float &s2, float v, const float (&w)[4][3])
{
    if constexpr (NP == 4) {
        asm(DWC_FMAC "%0, %3, %4\n" DWC_FMAC "%1, %3, %5\n" DWC_FMAC "%2, %3, %6\n"
            "v_fmac_f32_dpp %0, %3, %7" DWC_DPP("1,0,3,2") "v_fmac_f32_dpp %1, %3, %8" DWC_DPP("1,0,3,2")
            "v_fmac_f32_dpp %2, %3, %9" DWC_DPP("1,0,3,2")
            "v_fmac_f32_dpp %0, %3, %10" DWC_DPP("2,3,0,1") "v_fmac_f32_dpp %1, %3, %11" DWC_DPP("2,3,0,1")
            "v_fmac_f32_dpp %2, %3, %12" DWC_DPP("2,3,0,1")
            "v_fmac_f32_dpp %0, %3, %13" DWC_DPP("3,2,1,0") "v_fmac_f32_dpp %1, %3, %14" DWC_DPP("3,2,1,0")
            "v_fmac_f32_dpp %2, %3, %15" DWC_DPP("3,2,1,0")
            : "+v"(s0), "+v"(s1), "+v"(s2)
            : "v"(v), "v"(w[0][0]), "v"(w[0][1]), "v"(w[0][2]), "v"(w[1][0]), "v"(w[1][1]), "v"(w[1][2]),
              "v"(w[2][0]), "v"(w[2][1]), "v"(w[2][2]), "v"(w[3][0]), "v"(w[3][1]), "v"(w[3][2]));
    } else {
        asm(DWC_FMAC "%0, %3, %4\n" DWC_FMAC "%1, %3, %5\n" DWC_FMAC "%2, %3, %6\n"
            "v_fmac_f32_dpp %0, %3, %7" DWC_DPP("1,0,3,2") "v_fmac_f32_dpp %1, %3, %8" DWC_DPP("1,0,3,2")
            "v_fmac_f32_dpp %2, %3, %9" DWC_DPP("1,0,3,2")
            : "+v"(s0), "+v"(s1), "+v"(s2)
            : "v"(v), "v"(w[0][0]), "v"(w[0][1]), "v"(w[0][2]), "v"(w[1][0]), "v"(w[1][1]), "v"(w[1][2]));
    }
}
#undef DWC_FMAC
#undef DWC_DPP

template <typename T, int V> __device__ __forceinline__ void store_small(T *p, const float (&r)[V], bool stream)
{
    if constexpr (sizeof(T) == 4 && V == 1) {
        if (stream) __builtin_nontemporal_store(r[0], p); else *p = r[0];
    } else if constexpr (sizeof(T) == 4 && V == 2) {
        typedef float f2v_t __attribute__((ext_vector_type(2)));
        f2v_t v = {r[0], r[1]};
        if (stream) __builtin_nontemporal_store(v, reinterpret_cast<f2v_t *>(p)); else *reinterpret_cast<f2v_t *>(p) = v;
    } else {
        Vec<T, V>::store(p, r);
    }
}

__device__ __forceinline__ int wat_nhwc_x(const GGeom &g, int kh, int kw, int ci, int o) { return ((kh * 3 + kw) * g.Cg + ci) * g.O + o; }

template <typename T, int CG, int V, int PF, bool FLIP>
__global__ __launch_bounds__(256) void k_gconv_nhwc_xchg(GGeom g, const T *__restrict__ in, const T *__restrict__ w,
                                                         T *__restrict__ out, int TH, int nstrips, int nchunks, int NI,
                                                         unsigned nblocks, int nt)
{
    constexpr int LG = CG / V, R = PF + 1;       // lanes per group, ring depth
    static_assert(LG == 2 || LG == 4 || LG == 8, "a group spans 2, 4 or 8 lanes");
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int chunk = lb % nchunks; const int ngrp = lb / nchunks;

    const int CT = g.C;                          // channels per pixel, read and written (C == O)
    const int Q = CT / V;
    const int f = chunk * blockDim.x + threadIdx.x;
    if (f >= g.W * Q) return;                    // whole groups drop out together: W*Q is a multiple of LG
    const int cq = f % Q, ow = f / Q;
    const int c0 = cq * V, grp = c0 / CG, sub = (c0 % CG) / V;     // sub == lane number mod LG

    // Partner p of a lane: the lane whose number differs by p < LG in the low bits.  For p < 4 the value comes
    // through a quad permute of the lane's own register; for p >= 4 through a quad permute (by 7 - p) of the
    // half-row mirror (lane l^7) of that register.  wr[kw][t][a][h][q][kh]: h = 0 own / 1 mirrored register,
    // q = quad permute, t = channel in the partner's V, a = own channel.
    constexpr int NH = LG == 8 ? 2 : 1, NP = LG >= 4 ? 4 : 2;
    int coloff[3];
    float wr[3][V][V][NH][4][3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = ow - 1 + kw;
        const bool ok = iw >= 0 && iw < g.W;
        coloff[kw] = (ok ? iw - ow : 0) * CT;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int q = 0; q < NP; ++q)
#pragma unroll
                    for (int t = 0; t < V; ++t)
#pragma unroll
                        for (int a = 0; a < V; ++a) {
                            const int j = h ? 7 - q : q;                           // partner = lane ^ j
                            const int rd = (sub ^ j) * V + t, wrt = sub * V + a;   // positions in the group: read, written
                            const int idx = FLIP ? wat_nhwc_x(g, 2 - kh, 2 - kw, wrt, grp * CG + rd)
                                                 : wat_nhwc_x(g, kh, kw, rd, grp * CG + wrt);
                            const float wv = ldf(w + idx);     // unconditional: a select, not a branch per entry
                            wr[kw][t][a][h][q][kh] = ok ? wv : 0.f;
                        }
    }

    const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
    const int rowstride = g.W * CT;
    const int r0 = oh0 - 1, r1 = oh1 + 1;
    const int ra = max(r0, 0), rb = min(r1, g.H);
    const int n0 = ngrp * NI, n1 = min(g.N, n0 + NI);

#pragma unroll 1
    for (int n = n0; n < n1; ++n) {
        const T *xin = in + (size_t)n * g.H * rowstride + (size_t)ow * CT + c0;
        T *yout = out + (size_t)n * g.H * rowstride + (size_t)ow * CT + c0;
        float acc[2][V];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int a = 0; a < V; ++a) acc[j][a] = 0.f;

        RawVec<T, V> ring[R][3];
        auto load_row = [&](int r, RawVec<T, V> (&dst)[3]) {
            const T *rp = xin + (size_t)min(r, rb - 1) * rowstride;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) dst[kw].load(rp + coloff[kw]);
        };
        auto consume = [&](int r, const RawVec<T, V> (&raw)[3]) {
            // input row r is tap row kh of output row r + 1 - kh
            float cur[3][V];
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) raw[kw].get(cur[kw]);
            float s2[V], s1[V], s0[V];
#pragma unroll
            for (int a = 0; a < V; ++a) { s2[a] = acc[0][a]; s1[a] = acc[1][a]; s0[a] = 0.f; }
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int t = 0; t < V; ++t) {
#pragma unroll
                    for (int a = 0; a < V; ++a) fma_quad<NP>(s0[a], s1[a], s2[a], cur[kw][t], wr[kw][t][a][0]);
                    if constexpr (NH == 2) {
                        const float m = half_mirror(cur[kw][t]);
#pragma unroll
                        for (int a = 0; a < V; ++a) fma_quad<NP>(s0[a], s1[a], s2[a], m, wr[kw][t][a][1]);
                    }
                }
#pragma unroll
            for (int a = 0; a < V; ++a) { acc[0][a] = s1[a]; acc[1][a] = s0[a]; }
            const int oh = r - 1;
            if (oh >= oh0) store_small<T, V>(yout + (size_t)oh * rowstride, s2, nt != 0);
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
            float o[V];
#pragma unroll
            for (int a = 0; a < V; ++a) { o[a] = acc[0][a]; acc[0][a] = acc[1][a]; acc[1][a] = 0.f; }
            const int oh = r - 1;
            if (oh >= oh0) store_small<T, V>(yout + (size_t)oh * rowstride, o, nt != 0);
        }
    }
}

// acc[q][kh] += (v of lane l^q) * d[kh], q < 4, kh < 3: the filter-gradient counterpart of fma_quad (the
// cross-lane operand is x, the own operand dy).  Same ordering rule: the plain multiply-adds come first.
#define DWC_DPP(perm) " quad_perm:[" perm "] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
__device__ __forceinline__ void fma_quad_acc(float (&a)[4][3], float v, const float (&d)[3])
{
    asm("v_fmac_f32_e32 %0, %12, %13\n v_fmac_f32_e32 %1, %12, %14\n v_fmac_f32_e32 %2, %12, %15\n"
        "v_fmac_f32_dpp %3, %12, %13" DWC_DPP("1,0,3,2") "v_fmac_f32_dpp %4, %12, %14" DWC_DPP("1,0,3,2")
        "v_fmac_f32_dpp %5, %12, %15" DWC_DPP("1,0,3,2")
        "v_fmac_f32_dpp %6, %12, %13" DWC_DPP("2,3,0,1") "v_fmac_f32_dpp %7, %12, %14" DWC_DPP("2,3,0,1")
        "v_fmac_f32_dpp %8, %12, %15" DWC_DPP("2,3,0,1")
        "v_fmac_f32_dpp %9, %12, %13" DWC_DPP("3,2,1,0") "v_fmac_f32_dpp %10, %12, %14" DWC_DPP("3,2,1,0")
        "v_fmac_f32_dpp %11, %12, %15" DWC_DPP("3,2,1,0")
        : "+v"(a[0][0]), "+v"(a[0][1]), "+v"(a[0][2]), "+v"(a[1][0]), "+v"(a[1][1]), "+v"(a[1][2]),
          "+v"(a[2][0]), "+v"(a[2][1]), "+v"(a[2][2]), "+v"(a[3][0]), "+v"(a[3][1]), "+v"(a[3][2])
        : "v"(v), "v"(d[0]), "v"(d[1]), "v"(d[2]));
}
#undef DWC_DPP

// Filter gradient, stage 1, lane-exchange form.  A lane owns one channel (of x and of dy: C == O) at one column;
// block = CT lanes over channels x 256/CT columns, one strip of NI images.  Step r of the walk takes x row r
// (own channel, three columns) and dy row r+1 (own channel, own column); x row r meets dy rows r+1, r, r-1 at tap
// rows 0, 1, 2.  The lane accumulates dw[kh][kw][ci][own o] for the CG input channels ci of its group, whose x
// values it reads from the other lanes of the group.  ws[part][kh][kw][ci][o].
// MM: the sums on the matrix cores.  The four lanes of a quad are four channels of one group at one pixel, so a
// 4x4x1 matrix instruction with A = the lanes' x values and B = their dy values adds the outer product
// x[ci] * dy[o] of the quad in one instruction (D: register i of lane j = input channel i of the quad against the lane's
// own output channel): one instruction per tap instead of four multiply-adds with cross-lane operands.  Groups of 8
// add the mirrored x value (the group's other quad) the same way.  The matrix instructions run on every lane whatever
// the execution mask, so lanes outside the tensor walk along on clamped addresses with their dy forced to zero.
typedef float v4fx_t __attribute__((ext_vector_type(4)));
template <typename T, int CG, int PF, bool MM>
__global__ __launch_bounds__(256) void k_gconv_nhwc_xchg_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                    float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                                    int TH, int nstrips, int NI, unsigned nblocks, int J)
{
    constexpr int NH = CG == 8 ? 2 : 1, R = PF + 1;
    static_assert(CG == 4 || CG == 8, "groups of 4 or 8 lanes");
    __shared__ float red[4][CG][64];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int c = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = c < g.C && ow < g.W;       // the lanes of a group are active together (CT, C multiples of CG)
    const int sub = c % CG;

    float acc[3][NH][4][3];                        // [kw][own / mirrored register][quad permute][kh]
    v4fx_t accm[3][NH][3];                         // MM: [kw][own / mirrored register][kh], element i = lane i of the quad
#pragma unroll
    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int h = 0; h < NH; ++h) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) acc[kw][h][q][kh] = 0.f;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) accm[kw][h][kh] = v4fx_t{0.f, 0.f, 0.f, 0.f};
        }

    if (active || MM) {
        // MM: lanes outside the tensor take the addresses of the last channel / column and contribute zeros
        const int c = min(ctile * CT + tx, g.C - 1), ow = min(owtile * OWT + ty, g.W - 1);
        bool colok[3];
        int coloff[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int iw = ow - 1 + kw;
            colok[kw] = iw >= 0 && iw < g.W;
            coloff[kw] = (colok[kw] ? iw : ow) * g.C;
        }
        const int row = g.W * g.C;
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
#pragma unroll 1
        for (int n = n0; n < n1; ++n) {
            const T *xin = x + (size_t)n * g.H * row + c;
            const T *dyin = dy + (size_t)n * g.H * row + (size_t)ow * g.C + c;
            float dyw[3] = {0.f, 0.f, 0.f};
            RawVec<T, 1> xr[R][3], dr[R];
            auto load_step = [&](int r, RawVec<T, 1> (&xd)[3], RawVec<T, 1> &dd) {
                const T *xp = xin + (size_t)min(max(r, 0), g.H - 1) * row;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) xd[kw].load(xp + coloff[kw]);
                dd.load(dyin + (size_t)min(max(r + 1, 0), g.H - 1) * row);
            };
            auto consume = [&](int r, const RawVec<T, 1> (&xd)[3], const RawVec<T, 1> &dd) {
                const bool xok = r >= 0 && r < g.H;
                const bool dok = r + 1 >= oh0 && r + 1 < oh1 && active;       // only dy rows of this block's strip count
                float d[1];
                dd.get(d);
                dyw[2] = dyw[1]; dyw[1] = dyw[0]; dyw[0] = dok ? d[0] : 0.f;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    float xv[1];
                    xd[kw].get(xv);
                    const float xx = xok ? xv[0] : 0.f;
                    if constexpr (MM) {
#pragma unroll
                        for (int kh = 0; kh < 3; ++kh)
                            accm[kw][0][kh] = __builtin_amdgcn_mfma_f32_4x4x1f32(xx, dyw[kh], accm[kw][0][kh], 0, 0, 0);
                        if constexpr (NH == 2) {
                            const float m = half_mirror(xx);
#pragma unroll
                            for (int kh = 0; kh < 3; ++kh)
                                accm[kw][1][kh] = __builtin_amdgcn_mfma_f32_4x4x1f32(m, dyw[kh], accm[kw][1][kh], 0, 0, 0);
                        }
                    } else {
                        fma_quad_acc(acc[kw][0], xx, dyw);
                        if constexpr (NH == 2) {
                            const float m = half_mirror(xx);
                            fma_quad_acc(acc[kw][1], m, dyw);
                        }
                    }
                }
            };
            // x rows oh0-1 .. oh1: TH + 2 steps
            const int r0 = oh0 - 1, nsteps = (oh1 - oh0) + 2;
#pragma unroll
            for (int j = 0; j < PF; ++j) load_step(r0 + j, xr[j], dr[j]);
            int i = 0;
#pragma unroll 1
            for (; i + R <= nsteps; i += R) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    load_step(r0 + i + j + PF, xr[(j + PF) % R], dr[(j + PF) % R]);
                    consume(r0 + i + j, xr[j], dr[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < R - 1; ++j)
                if (i + j < nsteps) consume(r0 + i + j, xr[j], dr[j]);
        }
        // taps on columns outside the image accumulated clamped data: drop them
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
            if (!colok[kw]) {
#pragma unroll
                for (int h = 0; h < NH; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int kh = 0; kh < 3; ++kh) { acc[kw][h][q][kh] = 0.f; accm[kw][h][kh][q] = 0.f; }
            }
    }

    // fixed-order block reduction, one tap at a time: over the columns of a wavefront, then over the wavefronts
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) red[wv][h * 4 + q][lane] = wave_sum_strided(MM ? accm[kw][h][kh][q] : acc[kw][h][q][kh], CT);
            __syncthreads();
            if (wv == 0 && lane < CT && c < g.C) {
#pragma unroll
                for (int h = 0; h < NH; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // the partner's channel in the group (MM: q is the partner's lane number in the quad; mirrored: of lane^7's quad)
                        const int e = h * 4 + q, ci = MM ? (((sub & ~3) + q) ^ (h ? 7 : 0)) : (sub ^ (h ? 7 - q : q));
                        wsp[((kh * 3 + kw) * g.Cg + ci) * g.O + c] =
                            (red[0][e][lane] + red[1][e][lane]) + (red[2][e][lane] + red[3][e][lane]);
                    }
            }
            __syncthreads();
        }
}

// Filter gradient, stage 1, 3x3 stride 2 pad 1, on the matrix cores: lane and block mapping of the kernel above with the
// lane's column counted in dy (a lane owns one channel at dy column ow); dy row oh meets x rows 2oh-1, 2oh, 2oh+1 at
// columns 2ow-1, 2ow, 2ow+1, and row 2oh+1 is kept as the top row of the next step.  Per step and tap one 4x4x1
// matrix instruction adds the quad's outer product x[ci] * dy[o].  Lanes outside the tensor walk along on clamped
// addresses with their dy forced to zero (the matrix instructions run on every lane).
template <typename T, int CG>
__global__ __launch_bounds__(256) void k_gconv_nhwc_xchg_bwd_filter_s2(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                       float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                                       int TH, int nstrips, int NI, unsigned nblocks, int J)
{
    constexpr int NH = CG == 8 ? 2 : 1;
    static_assert(CG == 4 || CG == 8, "groups of 4 or 8 lanes");
    __shared__ float red[4][CG][64];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int c = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = c < g.C && ow < g.Wo;
    const int sub = c % CG;

    v4fx_t accm[3][NH][3];                         // [kw][own / mirrored register][kh], element i = lane i of the quad
#pragma unroll
    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) accm[kw][h][kh] = v4fx_t{0.f, 0.f, 0.f, 0.f};

    bool colok[3];
    {
        const int cc = min(c, g.C - 1), oc = min(ow, g.Wo - 1);
        int coloff[3];
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int iw = 2 * oc - 1 + kw;
            colok[kw] = iw >= 0 && iw < g.W;
            coloff[kw] = (colok[kw] ? iw : 2 * oc) * g.C;
        }
        const int xrow = g.W * g.C, drow = g.Wo * g.C;
        const int oh0 = strip * TH, oh1 = min(g.Ho, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        struct Step { RawVec<T, 1> e[3], o[3], d; };            // x rows 2oh and 2oh+1 at the three columns, dy row oh
#pragma unroll 1
        for (int n = n0; n < n1; ++n) {
            const T *xin = x + (size_t)n * g.H * xrow + cc;
            const T *dyin = dy + (size_t)n * g.Ho * drow + (size_t)oc * g.C + cc;
            auto load_x = [&](int r, RawVec<T, 1> (&dst)[3]) {
                const T *xp = xin + (size_t)min(max(r, 0), g.H - 1) * xrow;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) dst[kw].load(xp + coloff[kw]);
            };
            auto load_step = [&](int oh, Step &s) {
                load_x(2 * oh, s.e); load_x(2 * oh + 1, s.o);
                s.d.load(dyin + (size_t)min(oh, g.Ho - 1) * drow);
            };
            auto tap_row = [&](int kh, const RawVec<T, 1> (&xr)[3], bool rowok, float dv) {
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    float xv[1];
                    xr[kw].get(xv);
                    const float xx = rowok ? xv[0] : 0.f;
                    accm[kw][0][kh] = __builtin_amdgcn_mfma_f32_4x4x1f32(xx, dv, accm[kw][0][kh], 0, 0, 0);
                    if constexpr (NH == 2) {
                        const float m = half_mirror(xx);
                        accm[kw][1][kh] = __builtin_amdgcn_mfma_f32_4x4x1f32(m, dv, accm[kw][1][kh], 0, 0, 0);
                    }
                }
            };
            RawVec<T, 1> top[3];
            load_x(2 * oh0 - 1, top);
            bool topok = 2 * oh0 - 1 >= 0;
            auto consume = [&](int oh, const Step &s) {
                float d[1];
                s.d.get(d);
                const float dv = active ? d[0] : 0.f;
                tap_row(0, top, topok, dv);
                tap_row(1, s.e, true, dv);                       // 2oh <= H - 1 always
                const bool ook = 2 * oh + 1 < g.H;
                tap_row(2, s.o, ook, dv);
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) top[kw] = s.o[kw];
                topok = ook;
            };
            Step sa, sb;
            load_step(oh0, sa);
            int oh = oh0;
#pragma unroll 1
            for (; oh + 2 <= oh1; oh += 2) {
                load_step(oh + 1, sb);
                consume(oh, sa);
                load_step(oh + 2, sa);
                consume(oh + 1, sb);
            }
            if (oh < oh1) consume(oh, sa);
        }
        // taps on columns outside the image accumulated clamped data: drop them
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
            if (!colok[kw]) {
#pragma unroll
                for (int h = 0; h < NH; ++h)
#pragma unroll
                    for (int kh = 0; kh < 3; ++kh) accm[kw][h][kh] = v4fx_t{0.f, 0.f, 0.f, 0.f};
            }
    }

    // fixed-order block reduction, one tap at a time: over the columns of a wavefront, then over the wavefronts
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) red[wv][h * 4 + q][lane] = wave_sum_strided(accm[kw][h][kh][q], CT);
            __syncthreads();
            if (wv == 0 && lane < CT && c < g.C) {
#pragma unroll
                for (int h = 0; h < NH; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int e = h * 4 + q, ci = ((sub & ~3) + q) ^ (h ? 7 : 0);     // q = the partner's lane in the quad; mirrored: lane^7's quad
                        wsp[((kh * 3 + kw) * g.Cg + ci) * g.O + c] =
                            (red[0][e][lane] + red[1][e][lane]) + (red[2][e][lane] + red[3][e][lane]);
                    }
            }
            __syncthreads();
        }
}

// ---- host side ---------------------------------------------------------------------------------------------

static inline int cdivx(int a, int b) { return (a + b - 1) / b; }
static int xtune(const char *name, int dflt)
{
    const char *e = tune_env(name);
    return e && *e ? atoi(e) : dflt;
}

bool gconv_nhwc_xchg_supported(const GGeom &g)
{
    if (tune_env("DWCONV_TUNE_GNOXCHG")) return false;
    return g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && (g.Cg == 4 || g.Cg == 8);
}

template <typename T, int CG, int V, int PF>
static hipError_t launch_x(const GGeom &g, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    const int lanes = g.W * (g.C / V);
    const int bs = 256;
    const int nchunks = cdivx(lanes, bs);
    // whole columns per block unless that leaves too few blocks; several images per block when there are plenty,
    // so that the filter entries are loaded once per NI*TH rows
    int TH = g.H;
    while (TH > 7 && (long long)g.N * nchunks * cdivx(g.H, TH) < 1024) TH = (TH + 1) / 2;
    TH = xtune("DWCONV_TUNE_GXTH", TH);
    const int nstrips = cdivx(g.H, TH);
    int NI = 1;
    while (NI < g.N && NI * TH < 28 && (long long)cdivx(g.N, NI * 2) * nchunks * nstrips >= 768) NI *= 2;
    NI = xtune("DWCONV_TUNE_GXNI", NI);
    if (NI < 1 || TH < 1) return hipErrorInvalidValue;
    const long long nb = (long long)cdivx(g.N, NI) * nchunks * nstrips;
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int nt = stream_stores(flip ? "GROUP_NHWC_BWD" : "GROUP_NHWC_FWD", (long long)g.N * g.H * g.W * g.C * sizeof(T), 0);
    if (flip)
        hipLaunchKernelGGL((k_gconv_nhwc_xchg<T, CG, V, PF, true>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)in,
                           (const T *)w, (T *)out, TH, nstrips, nchunks, NI, nblocks, nt);
    else
        hipLaunchKernelGGL((k_gconv_nhwc_xchg<T, CG, V, PF, false>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)in,
                           (const T *)w, (T *)out, TH, nstrips, nchunks, NI, nblocks, nt);
    return hipGetLastError();
}

hipError_t gconv_nhwc_xchg_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    if (!gconv_nhwc_xchg_supported(g)) return hipErrorInvalidValue;
    // one channel per lane (9*CG filter registers): measured faster than two for fp32 groups of 4, and two channels
    // of a group of 8 would need 144 filter registers; bf16 groups of 4 take two (4-byte loads instead of 2-byte ones)
    const int V = g.Cg == 8 ? 1 : xtune("DWCONV_TUNE_GXV", dtype == DT_BF16 ? 2 : 1);
    const int PF = xtune("DWCONV_TUNE_GXPF", 5);     // rows in flight: 4-byte loads need many
#define TRY(T, CGG, VV, PPF) if (g.Cg == CGG && V == VV && PF == PPF) return launch_x<T, CGG, VV, PPF>(g, in, w, out, flip, st)
    if (dtype == DT_F32) {
        TRY(float, 8, 1, 2); TRY(float, 4, 2, 2); TRY(float, 4, 1, 2);
        TRY(float, 8, 1, 3); TRY(float, 4, 2, 3); TRY(float, 4, 1, 3);
        TRY(float, 8, 1, 5); TRY(float, 4, 2, 5); TRY(float, 4, 1, 5);
    } else {
        TRY(bf16_t, 8, 1, 2); TRY(bf16_t, 4, 2, 2); TRY(bf16_t, 4, 1, 2);
        TRY(bf16_t, 8, 1, 5); TRY(bf16_t, 4, 2, 5); TRY(bf16_t, 4, 1, 5);
    }
#undef TRY
    return hipErrorInvalidValue;
}

hipError_t gconv_nhwc_xchg_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int CT, int nctiles,
                                      int nowtiles, int TH, int nstrips, int NI, unsigned nblocks, int J, hipStream_t st)
{
    if (!gconv_nhwc_xchg_supported(g) || CT < g.Cg || CT % g.Cg != 0 || 256 % CT != 0) return hipErrorInvalidValue;
    const bool mm = xtune("DWCONV_TUNE_GXMM", 1) != 0;
#define GOF(T, CGG, MMM) hipLaunchKernelGGL((k_gconv_nhwc_xchg_bwd_filter<T, CGG, 3, MMM>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, (const T *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks, J)
#define TRY(T, CGG) if (g.Cg == CGG) { if (mm) GOF(T, CGG, true); else GOF(T, CGG, false); return hipGetLastError(); }
    if (dtype == DT_F32) {
        TRY(float, 4); TRY(float, 8);
    } else {
        TRY(bf16_t, 4); TRY(bf16_t, 8);
    }
#undef TRY
#undef GOF
    return hipErrorInvalidValue;
}

// ---- 3x3 stride 2: filter-gradient tiling (shared by the workspace query and the launch) and launch -----------------
bool gconv_nhwc_bwd_filter_s2_supported(const GGeom &g)
{
    if (tune_env("DWCONV_TUNE_GNOXCHG")) return false;
    return g.K == 3 && g.s == 2 && g.p == 1 && g.Cg == g.Og && (g.Cg == 4 || g.Cg == 8);
}

static void bwd_filter_s2_tiling(const GGeom &g, int *CT, int *nct, int *nowt, int *TH, int *nst, int *NI, int *ngr)
{
    int ct = g.Cg;
    while (ct < 64 && ct < g.C) ct *= 2;
    const int nc = cdivx(g.C, ct), now = cdivx(g.Wo, 256 / ct);
    // whole columns of dy unless the launch would have too few blocks; several images per block when there are plenty
    int th = g.Ho;
    const long long per_strip = (long long)nc * now * g.N;
    while (th > 4 && per_strip * cdivx(g.Ho, th) < 384) th = (th + 1) / 2;
    int ni = 1;
    while (ni < g.N && per_strip * cdivx(g.Ho, th) / (ni * 2) >= 384) ni *= 2;
    th = xtune("DWCONV_TUNE_GHWTH", th); ni = xtune("DWCONV_TUNE_GHWNI", ni);
    if (th < 1) th = 1;
    if (th > g.Ho) th = g.Ho;
    if (ni < 1) ni = 1;
    if (ni > g.N) ni = g.N;
    const long long J = (long long)g.O * g.Cg * 9;
    while ((long long)now * cdivx(g.Ho, th) * cdivx(g.N, ni) * J * 4 > (64ll << 20)) {
        if (ni < g.N) ni = ni * 2 < g.N ? ni * 2 : g.N; else if (th < g.Ho) th = th * 2 < g.Ho ? th * 2 : g.Ho; else break;
    }
    *CT = ct; *nct = nc; *nowt = now; *TH = th; *nst = cdivx(g.Ho, th); *NI = ni; *ngr = cdivx(g.N, ni);
}

int gconv_nhwc_bwd_filter_s2_parts(const GGeom &g)
{
    int CT, nct, nowt, TH, nst, NI, ngr;
    bwd_filter_s2_tiling(g, &CT, &nct, &nowt, &TH, &nst, &NI, &ngr);
    return nowt * nst * ngr;
}

hipError_t gconv_nhwc_bwd_filter_s2(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts, hipStream_t st)
{
    if (!gconv_nhwc_bwd_filter_s2_supported(g)) return hipErrorInvalidValue;
    int CT, nct, nowt, TH, nst, NI, ngr;
    bwd_filter_s2_tiling(g, &CT, &nct, &nowt, &TH, &nst, &NI, &ngr);
    if (parts != nowt * nst * ngr || CT % g.Cg != 0 || 256 % CT != 0) return hipErrorInvalidValue;
    const long long nb = (long long)nct * nowt * nst * ngr;
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int J = g.O * g.Cg * 9;
#define GOS(T, CGG) hipLaunchKernelGGL((k_gconv_nhwc_xchg_bwd_filter_s2<T, CGG>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                       (const T *)dy, ws, CT, nct, nowt, TH, nst, NI, nblocks, J)
    if (dtype == DT_F32) { if (g.Cg == 4) GOS(float, 4); else GOS(float, 8); }
    else { if (g.Cg == 4) GOS(bf16_t, 4); else GOS(bf16_t, 8); }
#undef GOS
    return hipGetLastError();
}

}  // namespace dwc
