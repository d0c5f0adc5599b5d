// NHWC kernels.  Channels are contiguous, so a lane owns V consecutive channels of one pixel
// column and walks down the rows of its strip: each input row is loaded once per lane (plus the
// left/right neighbour columns, which the L1 serves) and feeds the K output rows it overlaps
// through K-1 rotating accumulators.  A whole image row is one contiguous run of W*C elements,
// so consecutive lanes cover consecutive 16-byte pieces of it, whatever C is.
#include "kernels.hpp"

namespace dwc {

// logical block -> (n, chunk, strip) with strip fastest, after the XCD remap
struct Tile { int n, chunk, strip; };
__device__ __forceinline__ Tile tile_of(unsigned nblocks, int nchunks, int nstrips)
{
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    Tile t;
    t.strip = lb % nstrips; lb /= nstrips;
    t.chunk = lb % nchunks; t.n = lb / nchunks;
    return t;
}

// Register budget of the stride-1 kernel as wavefronts per SIMD (512 VGPRs / budget): filter taps,
// the row ring, the rotating accumulators and one row of outputs, plus addressing.
template <int V, int K, int TW, int PF> constexpr int S1_WAVES()
{
    const int regs = K * K * V + (PF + 1) * (TW + K - 1) * V + (K - 1) * TW * V + TW * V + 24;
    return regs <= 64 ? 8 : regs <= 72 ? 7 : regs <= 84 ? 6 : regs <= 100 ? 5 : regs <= 128 ? 4 : regs <= 168 ? 3 : 2;
}

// ---------------------------------------------------------------------------------------------
// Forward, stride 1, "same" padding (K odd, pad = (K-1)/2, so Wo = W and Ho = H), multiplier 1.
// A lane owns V channels of TW adjacent output columns and walks down the rows of its strip.
// Per input row it loads the TW + K - 1 columns it needs (each element of the row is loaded
// (TW+K-1)/TW times over all lanes; the L1 serves the repeats), PF rows ahead of the row being
// consumed, so that PF * (TW+K-1) loads are in flight per lane.
// FLIP = true reads the filter rotated by 180 degrees, which makes this the backward-data pass
// of the same layer (input = dy, output = dx).
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K, int TW, int PF, bool FLIP>
__global__ __launch_bounds__(256, (S1_WAVES<V, K, TW, PF>())) void k_nhwc_s1(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                 T *__restrict__ y, int TH, int nstrips, int nchunks, unsigned nblocks, int nt)
{
    constexpr int P = (K - 1) / 2;
    constexpr int NC = TW + K - 1;        // input columns per lane
    constexpr int R = PF + 1;             // ring of rows: PF in flight + the one being consumed
    const Tile tl = tile_of(nblocks, nchunks, nstrips);
    const int Q = g.C / V;
    const int nowg = (g.W + TW - 1) / TW;
    const int f = tl.chunk * blockDim.x + threadIdx.x;
    if (f >= nowg * Q) return;
    const int cq = f % Q, ow0 = (f / Q) * TW;

    float wr[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const int sh = FLIP ? K - 1 - kh : kh, sw = FLIP ? K - 1 - kw : kw;
            Vec<T, V>::load(w + (sh * K + sw) * g.C + cq * V, wr[kh][kw]);
        }
    // Out-of-image taps read a valid address (clamped row, the lane's own column) and are zeroed
    // with a select, so the loads are unconditional and can all be issued ahead.
    bool colok[NC];
    int coloff[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int iw = ow0 - P + c;
        colok[c] = iw >= 0 && iw < g.W;
        coloff[c] = (colok[c] ? c : P) * g.C;
    }

    const int oh0 = tl.strip * TH, oh1 = min(g.H, oh0 + TH);
    const int rowstride = g.W * g.C;
    const size_t img = (size_t)tl.n * g.H * rowstride;
    const T *xin = x + img + (ptrdiff_t)(ow0 - P) * g.C + cq * V;
    T *yout = y + img + (size_t)ow0 * g.C + cq * V;

    float acc[K - 1 > 0 ? K - 1 : 1][TW][V];
#pragma unroll
    for (int j = 0; j < K - 1; ++j)
#pragma unroll
        for (int t = 0; t < TW; ++t)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[j][t][v] = 0.f;

    float ring[R][NC][V];
    auto load_row = [&](int r, float (&dst)[NC][V]) {
        const int rr = min(max(r, 0), g.H - 1);
        const bool rowok = rr == r;
        const T *rp = xin + (size_t)rr * rowstride;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            Vec<T, V>::load(rp + coloff[c], dst[c]);
            const bool ok = rowok && colok[c];
#pragma unroll
            for (int v = 0; v < V; ++v) dst[c][v] = ok ? dst[c][v] : 0.f;
        }
    };
    auto consume = [&](int r, const float (&cur)[NC][V]) {
        // input row r is tap row kh of output row r + P - kh
        float out[TW][V];
#pragma unroll
        for (int t = 0; t < TW; ++t)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s = (K > 1) ? acc[0][t][v] : 0.f;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 1][kw][v], cur[t + kw][v], s);
                out[t][v] = s;
            }
#pragma unroll
        for (int j = 0; j < K - 1; ++j)
#pragma unroll
            for (int t = 0; t < TW; ++t)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float s = (j + 1 < K - 1) ? acc[j + 1][t][v] : 0.f;
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 2 - j][kw][v], cur[t + kw][v], s);
                    acc[j][t][v] = s;
                }
        const int oh = r - P;
        if (oh >= oh0) {
#pragma unroll
            for (int t = 0; t < TW; ++t)
                if (TW == 1 || ow0 + t < g.W) store_vec<T, V>(yout + (size_t)oh * rowstride + t * g.C, out[t], nt != 0);
        }
    };

    const int r0 = oh0 - P, r1 = oh1 + P;   // input rows [r0, r1)
#pragma unroll
    for (int j = 0; j < PF; ++j)
        if (r0 + j < r1) load_row(r0 + j, ring[j]);
#pragma unroll 1
    for (int base = r0; base < r1; base += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int r = base + j;
            if (r < r1) {
                if (r + PF < r1) load_row(r + PF, ring[(j + PF) % R]);
                consume(r, ring[j]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Forward, 3x3, stride 2, pad 1, multiplier 1.  A lane owns output column ow and walks down the
// output rows; input row 2*oh+1 is shared by output rows oh (tap row 2) and oh+1 (tap row 0).
// ---------------------------------------------------------------------------------------------
template <typename T, int V>
__global__ __launch_bounds__(256) void k_nhwc_fwd_k3s2(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                       T *__restrict__ y, int TH, int nstrips, int nchunks,
                                                       unsigned nblocks, int nt)
{
    const Tile tl = tile_of(nblocks, nchunks, nstrips);
    const int Q = g.C / V, WoQ = g.Wo * Q;
    const int f = tl.chunk * blockDim.x + threadIdx.x;
    if (f >= WoQ) return;
    const int cq = f % Q, ow = f / Q;

    float wr[3][3][V];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) Vec<T, V>::load(w + (kh * 3 + kw) * g.C + cq * V, wr[kh][kw]);
    bool colok[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = 2 * ow - 1 + kw;
        colok[kw] = iw >= 0 && iw < g.W;
    }
    const int rowstride = g.W * g.C;
    const T *xin = x + (size_t)tl.n * g.H * rowstride + (ptrdiff_t)(2 * ow - 1) * g.C + cq * V;
    T *yout = y + ((size_t)tl.n * g.Ho * g.Wo + ow) * g.C + cq * V;

    auto load_row = [&](int r, float (&dst)[3][V]) {
        const bool rowok = r >= 0 && r < g.H;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            if (rowok && colok[kw]) Vec<T, V>::load(xin + (ptrdiff_t)r * rowstride + kw * g.C, dst[kw]);
            else {
#pragma unroll
                for (int v = 0; v < V; ++v) dst[kw][v] = 0.f;
            }
        }
    };

    const int oh0 = tl.strip * TH, oh1 = min(g.Ho, oh0 + TH);
    float carry[V], re[3][V], ro[3][V];
    load_row(2 * oh0 - 1, ro);
#pragma unroll
    for (int v = 0; v < V; ++v) {
        float s = 0.f;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) s = fmaf(wr[0][kw][v], ro[kw][v], s);
        carry[v] = s;
    }
    for (int oh = oh0; oh < oh1; ++oh) {
        load_row(2 * oh, re);
        load_row(2 * oh + 1, ro);
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float s = carry[v], c = 0.f;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) s = fmaf(wr[1][kw][v], re[kw][v], s);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                s = fmaf(wr[2][kw][v], ro[kw][v], s);
                c = fmaf(wr[0][kw][v], ro[kw][v], c);
            }
            out[v] = s; carry[v] = c;
        }
        store_vec<T, V>(yout + (size_t)oh * g.Wo * g.C, out, nt != 0);
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-data, 3x3, stride 2, pad 1, multiplier 1.  A lane owns dy column b and walks down the
// dy rows a; from dy[a..a+1][b..b+1] it produces the 2x2 block dx[2a..2a+1][2b..2b+1]:
//   dx[2a  ][2b  ] = w11 dy[a][b]
//   dx[2a  ][2b+1] = w10 dy[a][b+1] + w12 dy[a][b]
//   dx[2a+1][2b  ] = w01 dy[a+1][b] + w21 dy[a][b]
//   dx[2a+1][2b+1] = w00 dy[a+1][b+1] + w02 dy[a+1][b] + w20 dy[a][b+1] + w22 dy[a][b]
// Rows 2a+1 >= H and columns 2b+1 >= W do not exist (odd H, W) and are skipped.
// ---------------------------------------------------------------------------------------------
template <typename T, int V>
__global__ __launch_bounds__(256) void k_nhwc_bwd_data_k3s2(Geom g, const T *__restrict__ dy, const T *__restrict__ w,
                                                            T *__restrict__ dx, int TH, int nstrips, int nchunks,
                                                            unsigned nblocks, int nt)
{
    const Tile tl = tile_of(nblocks, nchunks, nstrips);
    const int Q = g.C / V, WoQ = g.Wo * Q;
    const int f = tl.chunk * blockDim.x + threadIdx.x;
    if (f >= WoQ) return;
    const int cq = f % Q, b = f / Q;

    float wr[3][3][V];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) Vec<T, V>::load(w + (kh * 3 + kw) * g.C + cq * V, wr[kh][kw]);

    const bool has_b1 = b + 1 < g.Wo;       // dy column b+1 exists
    const bool col1 = 2 * b + 1 < g.W;      // dx column 2b+1 exists
    const int dyrow = g.Wo * g.C, dxrow = g.W * g.C;
    const T *dyin = dy + ((size_t)tl.n * g.Ho * g.Wo + b) * g.C + cq * V;
    T *dxout = dx + ((size_t)tl.n * g.H * g.W + 2 * b) * g.C + cq * V;

    auto load_row = [&](int a, float (&d0)[V], float (&d1)[V]) {
        if (a < g.Ho) {
            Vec<T, V>::load(dyin + (size_t)a * dyrow, d0);
            if (has_b1) Vec<T, V>::load(dyin + (size_t)a * dyrow + g.C, d1);
            else {
#pragma unroll
                for (int v = 0; v < V; ++v) d1[v] = 0.f;
            }
        } else {
#pragma unroll
            for (int v = 0; v < V; ++v) { d0[v] = 0.f; d1[v] = 0.f; }
        }
    };

    const int a0 = tl.strip * TH, a1 = min(g.Ho, a0 + TH);
    float A0[V], A1[V], B0[V], B1[V];
    load_row(a0, A0, A1);
    for (int a = a0; a < a1; ++a) {
        load_row(a + 1, B0, B1);
        float o00[V], o01[V], o10[V], o11[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            o00[v] = wr[1][1][v] * A0[v];
            o01[v] = fmaf(wr[1][0][v], A1[v], wr[1][2][v] * A0[v]);
            o10[v] = fmaf(wr[0][1][v], B0[v], wr[2][1][v] * A0[v]);
            o11[v] = fmaf(wr[0][0][v], B1[v], fmaf(wr[0][2][v], B0[v], fmaf(wr[2][0][v], A1[v], wr[2][2][v] * A0[v])));
        }
        T *r0p = dxout + (size_t)(2 * a) * dxrow;
        store_vec<T, V>(r0p, o00, nt != 0);
        if (col1) store_vec<T, V>(r0p + g.C, o01, nt != 0);
        if (2 * a + 1 < g.H) {
            store_vec<T, V>(r0p + dxrow, o10, nt != 0);
            if (col1) store_vec<T, V>(r0p + dxrow + g.C, o11, nt != 0);
        }
#pragma unroll
        for (int v = 0; v < V; ++v) { A0[v] = B0[v]; A1[v] = B1[v]; }
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1, multiplier 1.  Block = CT channel-vectors x (256/CT) output columns;
// it owns one strip of output rows of NI consecutive images.  Each lane keeps K*K*V fp32 partial
// sums in registers.  At the end lanes that own the same channels are summed: butterfly shuffles
// inside the wavefront (when CT < 64 a wavefront holds several columns of the same channels),
// then LDS across the 4 wavefronts, all in a fixed order; one partial per block goes to the
// workspace at [part][kh][kw][o].
// S = 1: "same" padding, K odd.  S = 2: K = 3, pad = 1.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K, int S, int PF>
__global__ __launch_bounds__(256) void k_nhwc_bwd_filter(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                         float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                         int TH, int nstrips, int NI, unsigned nblocks)
{
    constexpr int P = (K - 1) / 2;   // also the pad for S == 2, K == 3
    __shared__ float red[4][V][64];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int strip = lb % nstrips; lb /= nstrips;
    const int owtile = lb % nowtiles; lb /= nowtiles;
    const int ctile = lb % nctiles; const int ngroup = lb / nctiles;

    const int OWT = 256 / CT;
    const int tx = threadIdx.x % CT, ty = threadIdx.x / CT;
    const int Q = g.C / V;
    const int cq = ctile * CT + tx, ow = owtile * OWT + ty;
    const bool active = cq < Q && ow < g.Wo;

    float acc[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[kh][kw][v] = 0.f;

    if (active) {
        // Out-of-image taps read a valid address (clamped row, the lane's own column) and are
        // zeroed with a select, so every load is unconditional and can be issued rows ahead.
        bool colok[K];
        int coloff[K];
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const int iw = ow * S - P + kw;
            colok[kw] = iw >= 0 && iw < g.W;
            coloff[kw] = (colok[kw] ? iw : ow * S) * g.C;
        }
        const int xrow = g.W * g.C, dyrow = g.Wo * g.C;
        const int oh0 = strip * TH, oh1 = min(g.Ho, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        for (int n = n0; n < n1; ++n) {
            const T *xin = x + (size_t)n * g.H * xrow + cq * V;
            const T *dyin = dy + ((size_t)n * g.Ho * g.Wo + ow) * g.C + cq * V;
            auto load_x = [&](int r, float (&dst)[K][V]) {
                const int rr = min(max(r, 0), g.H - 1);
                const bool rowok = rr == r;
                const T *rp = xin + (size_t)rr * xrow;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
                    Vec<T, V>::load(rp + coloff[kw], dst[kw]);
                    const bool ok = rowok && colok[kw];
#pragma unroll
                    for (int v = 0; v < V; ++v) dst[kw][v] = ok ? dst[kw][v] : 0.f;
                }
            };
            auto load_dy = [&](int oh, float (&dst)[V]) {
                const int rr = min(max(oh, oh0), oh1 - 1);
                Vec<T, V>::load(dyin + (size_t)rr * dyrow, dst);
                const bool ok = rr == oh;
#pragma unroll
                for (int v = 0; v < V; ++v) dst[v] = ok ? dst[v] : 0.f;
            };
            if constexpr (S == 1) {
                // input row r meets dy row r + P - kh at tap row kh; dyw holds the K live dy rows
                constexpr int R = PF + 1;
                float dyw[K][V];
#pragma unroll
                for (int kh = 0; kh < K; ++kh)
#pragma unroll
                    for (int v = 0; v < V; ++v) dyw[kh][v] = 0.f;
                float xr[R][K][V], dr[R][V];
                const int r0 = oh0 - P, r1 = oh1 + P;
#pragma unroll
                for (int j = 0; j < PF; ++j)
                    if (r0 + j < r1) { load_x(r0 + j, xr[j]); load_dy(r0 + j + P, dr[j]); }
#pragma unroll 1
                for (int base = r0; base < r1; base += R) {
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        const int r = base + j;
                        if (r < r1) {
                            if (r + PF < r1) { load_x(r + PF, xr[(j + PF) % R]); load_dy(r + PF + P, dr[(j + PF) % R]); }
#pragma unroll
                            for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                                for (int v = 0; v < V; ++v) dyw[kh][v] = dyw[kh - 1][v];
#pragma unroll
                            for (int v = 0; v < V; ++v) dyw[0][v] = dr[j][v];
#pragma unroll
                            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                                for (int kw = 0; kw < K; ++kw)
#pragma unroll
                                    for (int v = 0; v < V; ++v)
                                        acc[kh][kw][v] = fmaf(dyw[kh][v], xr[j][kw][v], acc[kh][kw][v]);
                        }
                    }
                }
            } else {
                // output row oh meets input rows 2oh-1, 2oh, 2oh+1; row 2oh+1 is reused by oh+1.
                // The two new rows and the dy row of the next output row are loaded one step ahead.
                float xa[K][V], xb[2][K][V], xc[2][K][V], d[2][V];
                load_x(2 * oh0 - 1, xa);
                load_x(2 * oh0, xb[0]); load_x(2 * oh0 + 1, xc[0]); load_dy(oh0, d[0]);
#pragma unroll 1
                for (int base = oh0; base < oh1; base += 2) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int oh = base + j;
                        if (oh < oh1) {
                            if (oh + 1 < oh1) {
                                load_x(2 * oh + 2, xb[j ^ 1]); load_x(2 * oh + 3, xc[j ^ 1]); load_dy(oh + 1, d[j ^ 1]);
                            }
#pragma unroll
                            for (int kw = 0; kw < K; ++kw)
#pragma unroll
                                for (int v = 0; v < V; ++v) {
                                    acc[0][kw][v] = fmaf(d[j][v], xa[kw][v], acc[0][kw][v]);
                                    acc[1][kw][v] = fmaf(d[j][v], xb[j][kw][v], acc[1][kw][v]);
                                    acc[2][kw][v] = fmaf(d[j][v], xc[j][kw][v], acc[2][kw][v]);
                                    xa[kw][v] = xc[j][kw][v];
                                }
                        }
                    }
                }
            }
        }
    }

    // ---- fixed-order block reduction, one tap at a time ----
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * (K * K * g.C);
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s = wave_sum_strided(acc[kh][kw][v], CT);
                red[wv][v][lane] = s;
            }
            __syncthreads();
            if (wv == 0 && lane < CT && cq < Q) {
                float o[V];
#pragma unroll
                for (int v = 0; v < V; ++v)
                    o[v] = (red[0][v][lane] + red[1][v][lane]) + (red[2][v][lane] + red[3][v][lane]);
#pragma unroll
                for (int v = 0; v < V; ++v) wsp[(kh * K + kw) * g.C + cq * V + v] = o[v];
            }
            __syncthreads();
        }
}

// ---- host side --------------------------------------------------------------------------------

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Block width for the flat (column x channel-vector) mapping: 256 lanes, or 128 when that
// leaves fewer idle lanes in the last chunk of a row.
static inline int flat_block(int WQ)
{
    const int waste256 = ceil_div(WQ, 256) * 256 - WQ, waste128 = ceil_div(WQ, 128) * 128 - WQ;
    return waste128 < waste256 ? 128 : 256;
}

template <typename T, int V, int K, int TW, int PF>
static hipError_t launch_s1(const Geom &g, const void *x, const void *w, void *y, bool flip, int TH, hipStream_t st)
{
    const int lanes = ceil_div(g.W, TW) * (g.C / V);
    const int bs = flat_block(lanes);
    const int nchunks = ceil_div(lanes, bs), nstrips = ceil_div(g.H, TH);
    const unsigned nblocks = (unsigned)g.N * nchunks * nstrips;
    const int nt = stream_stores((long long)g.N * g.H * g.W * g.C * sizeof(T));
    if (flip)
        hipLaunchKernelGGL((k_nhwc_s1<T, V, K, TW, PF, true>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    else
        hipLaunchKernelGGL((k_nhwc_s1<T, V, K, TW, PF, false>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    return hipGetLastError();
}

hipError_t nhwc_s1(const Geom &g, int dtype, int V, const void *x, const void *w, void *y, bool flip, int TH, int TW,
                   int PF, hipStream_t st)
{
#define TRY(T, VV, KK, TTW, PPF) if (g.K == KK && V == VV && TW == TTW && PF == PPF) return launch_s1<T, VV, KK, TTW, PPF>(g, x, w, y, flip, TH, st)
    if (dtype == DT_F32) {
        TRY(float, 4, 3, 1, 1); TRY(float, 4, 3, 1, 2); TRY(float, 4, 3, 1, 3);
        TRY(float, 4, 3, 2, 1); TRY(float, 4, 3, 2, 2); TRY(float, 4, 3, 2, 3);
        TRY(float, 4, 3, 4, 1); TRY(float, 4, 3, 4, 2);
        TRY(float, 4, 3, 7, 1); TRY(float, 4, 3, 7, 2);
        TRY(float, 4, 5, 1, 1); TRY(float, 4, 5, 2, 1);
    } else {
        TRY(bf16_t, 8, 3, 1, 1); TRY(bf16_t, 8, 3, 2, 1); TRY(bf16_t, 8, 3, 2, 2);
        TRY(bf16_t, 4, 3, 1, 1); TRY(bf16_t, 4, 3, 2, 1);
        TRY(bf16_t, 4, 5, 1, 1); TRY(bf16_t, 4, 5, 2, 1);
    }
#undef TRY
    return hipErrorInvalidValue;
}

hipError_t nhwc_k3s2(const Geom &g, int dtype, int V, const void *in, const void *w, void *out, bool bwd, int TH,
                     hipStream_t st)
{
    const int WoQ = g.Wo * (g.C / V);
    const int bs = flat_block(WoQ);
    const int nchunks = ceil_div(WoQ, bs), nstrips = ceil_div(g.Ho, TH);
    const unsigned nblocks = (unsigned)g.N * nchunks * nstrips;
    // forward: a wave's store is one contiguous run, and the pass is read-dominated: stream the output.
    // backward-data writes alternate pixel columns per instruction (partial lines): keep those cached.
    const int nt = bwd ? 0 : stream_stores((long long)g.N * g.Ho * g.Wo * g.C * (dtype == DT_F32 ? 4 : 2));
#define GO(KERNEL, T, VV) hipLaunchKernelGGL((KERNEL<T, VV>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)in, \
                                             (const T *)w, (T *)out, TH, nstrips, nchunks, nblocks, nt)
    if (!bwd) {
        if (dtype == DT_F32) GO(k_nhwc_fwd_k3s2, float, 4);
        else if (V == 8) GO(k_nhwc_fwd_k3s2, bf16_t, 8);
        else GO(k_nhwc_fwd_k3s2, bf16_t, 4);
    } else {
        if (dtype == DT_F32) GO(k_nhwc_bwd_data_k3s2, float, 4);
        else if (V == 8) GO(k_nhwc_bwd_data_k3s2, bf16_t, 8);
        else GO(k_nhwc_bwd_data_k3s2, bf16_t, 4);
    }
#undef GO
    return hipGetLastError();
}

// Tiling of the filter-gradient pass; shared by the workspace query and the launch.
void nhwc_bwd_filter_tiling(const Geom &g, int V, int TH, int NI, int *CT, int *nctiles, int *nowtiles, int *nstrips,
                            int *ngroups)
{
    const int Q = g.C / V;
    int ct = 1;
    while (ct < Q && ct < 64) ct <<= 1;
    *CT = ct;
    *nctiles = ceil_div(Q, ct);
    *nowtiles = ceil_div(g.Wo, 256 / ct);
    *nstrips = ceil_div(g.Ho, TH);
    *ngroups = ceil_div(g.N, NI);
}

hipError_t nhwc_bwd_filter(const Geom &g, int dtype, int V, const void *x, const void *dy, float *ws, int TH, int NI,
                           hipStream_t st)
{
    int CT, nctiles, nowtiles, nstrips, ngroups;
    nhwc_bwd_filter_tiling(g, V, TH, NI, &CT, &nctiles, &nowtiles, &nstrips, &ngroups);
    const unsigned nblocks = (unsigned)nctiles * nowtiles * nstrips * ngroups;
#define GO(T, VV, KK, SS) hipLaunchKernelGGL((k_nhwc_bwd_filter<T, VV, KK, SS, 2>), dim3(nblocks), dim3(256), 0, st, g, \
                                             (const T *)x, (const T *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks)
    if (dtype == DT_F32) {
        if (g.K == 3 && g.s == 1) GO(float, 4, 3, 1);
        else if (g.K == 3 && g.s == 2) GO(float, 4, 3, 2);
        else if (g.K == 5 && g.s == 1) GO(float, 4, 5, 1);
        else return hipErrorInvalidValue;
    } else {
        if (g.K == 3 && g.s == 1 && V == 8) GO(bf16_t, 8, 3, 1);
        else if (g.K == 3 && g.s == 1) GO(bf16_t, 4, 3, 1);
        else if (g.K == 3 && g.s == 2 && V == 8) GO(bf16_t, 8, 3, 2);
        else if (g.K == 3 && g.s == 2) GO(bf16_t, 4, 3, 2);
        else if (g.K == 5 && g.s == 1) GO(bf16_t, 4, 5, 1);
        else return hipErrorInvalidValue;
    }
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
