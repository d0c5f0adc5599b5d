// NHWC kernels.  Channels are contiguous, so a lane owns V consecutive channels of one pixel
// column and walks down the rows of its strip: each input row is loaded once per lane (plus the
// left/right neighbour columns, which the L1 serves) and feeds the K output rows it overlaps
// through K-1 rotating accumulators.  A whole image row is one contiguous run of W*C elements,
// so consecutive lanes cover consecutive 16-byte pieces of it, whatever C is.
#include "kernels.hpp"
#include <stdlib.h>

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
template <int V, int K, int PF> constexpr int S1_WAVES()
{
    // (counted as if every row of the ring were widened to fp32: a tighter budget for bf16, whose ring
    // stays packed, made the compiler spill and cost 40 %)
    const int regs = K * K * V + (PF + 1) * K * V + (K - 1) * V + V + 24;
    return regs <= 64 ? 8 : regs <= 72 ? 7 : regs <= 84 ? 6 : regs <= 100 ? 5 : regs <= 128 ? 4 : regs <= 168 ? 3 : 2;
}

// ---------------------------------------------------------------------------------------------
// Forward, stride 1, "same" padding (K odd, pad = (K-1)/2, so Wo = W and Ho = H), multiplier 1.
// A lane owns V channels of one output column and walks down the rows of its strip.  Per input
// row it loads the K columns it needs, PF rows ahead of the row being consumed; the loads are
// unconditional (clamped addresses) and nothing touches a loaded value until its row is consumed,
// so PF*K loads stay in flight per lane.  Padding costs nothing per row: taps on columns outside
// the image have their weights zeroed once per lane, rows outside the image are skipped by a
// branch that is uniform over the block.
// FLIP = true reads the filter rotated by 180 degrees, which makes this the backward-data pass
// of the same layer (input = dy, output = dx).
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K, int PF, bool FLIP, int M>
__global__ __launch_bounds__(256, (S1_WAVES<V, K, PF>())) void k_nhwc_s1(
    Geom g, const T *__restrict__ x, const T *__restrict__ w, T *__restrict__ y, int TH, int nstrips, int nchunks,
    unsigned nblocks, int nt)
{
    constexpr int P = (K - 1) / 2;
    constexpr int R = PF + 1;             // ring of rows: PF in flight + the one being consumed
    const Tile tl = tile_of(nblocks, nchunks, nstrips);
    // A lane owns V consecutive OUTPUT channels of the layer (o = cq*V ...), which read V/M input
    // channels.  Forward: load V/M channels of x, store V channels of y.  Backward-data: load V
    // channels of dy, add the M outputs that share an input channel, store V/M channels of dx.
    constexpr int VI = FLIP ? V : V / M;      // channels per lane in the tensor that is read
    constexpr int VO = FLIP ? V / M : V;      // channels per lane in the tensor that is written
    const int Q = g.O / V;
    const int f = tl.chunk * blockDim.x + threadIdx.x;
    if (f >= g.W * Q) return;
    const int cq = f % Q, ow = f / Q;
    const int CI = FLIP ? g.O : g.C, CO = FLIP ? g.C : g.O;   // channels per pixel, read / written

    int coloff[K];
    float wr[K][K][V];
#pragma unroll
    for (int kw = 0; kw < K; ++kw) {
        const int iw = ow - P + kw;
        const bool ok = iw >= 0 && iw < g.W;
        coloff[kw] = (ok ? iw - ow : 0) * CI;
#pragma unroll
        for (int kh = 0; kh < K; ++kh) {
            const int sh = FLIP ? K - 1 - kh : kh, sw = FLIP ? K - 1 - kw : kw;
            Vec<T, V>::load(w + (sh * K + sw) * g.O + cq * V, wr[kh][kw]);
#pragma unroll
            for (int v = 0; v < V; ++v) wr[kh][kw][v] = ok ? wr[kh][kw][v] : 0.f;
        }
    }

    const int oh0 = tl.strip * TH, oh1 = min(g.H, oh0 + TH);
    const int rowstride = g.W * CI, orowstride = g.W * CO;
    const T *xin = x + (size_t)tl.n * g.H * rowstride + (size_t)ow * CI + cq * VI;
    T *yout = y + (size_t)tl.n * g.H * orowstride + (size_t)ow * CO + cq * VO;

    float acc[K - 1 > 0 ? K - 1 : 1][V];
#pragma unroll
    for (int j = 0; j < K - 1; ++j)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[j][v] = 0.f;

    // Valid input rows of the strip are [ra, rb).  Rows above the image only rotate zero
    // accumulators, so the walk simply starts at ra; rows below the image are an epilogue
    // without loads.  The main loop is branch-free: R rows per trip, loads clamped to row rb-1
    // (a few redundant re-loads of the last row at the end of a strip).
    const int r0 = oh0 - P, r1 = oh1 + P;
    const int ra = max(r0, 0), rb = min(r1, g.H);
    // the ring keeps rows as loaded (bf16 packed) and widens them when the row is consumed
    RawVec<T, VI> ring[R][K];
    auto load_row = [&](int r, RawVec<T, VI> (&dst)[K]) {
        const T *rp = xin + (size_t)min(r, rb - 1) * rowstride;
#pragma unroll
        for (int kw = 0; kw < K; ++kw) dst[kw].load(rp + coloff[kw]);
    };
    auto emit = [&](int oh, const float (&out)[V]) {
        if constexpr (VO == V) {
            store_vec<T, V>(yout + (size_t)oh * orowstride, out, nt != 0);
        } else {
            float red[VO];
#pragma unroll
            for (int c = 0; c < VO; ++c) {
                float t = out[c * M];
#pragma unroll
                for (int q = 1; q < M; ++q) t += out[c * M + q];
                red[c] = t;
            }
            store_vec<T, VO>(yout + (size_t)oh * orowstride, red, nt != 0);
        }
    };
    auto consume = [&](int r, const RawVec<T, VI> (&raw)[K]) {
        // input row r is tap row kh of output row r + P - kh
        float cur[K][VI];
#pragma unroll
        for (int kw = 0; kw < K; ++kw) raw[kw].get(cur[kw]);
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float s = (K > 1) ? acc[0][v] : 0.f;
#pragma unroll
            for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 1][kw][v], cur[kw][FLIP ? v : v / M], s);
            out[v] = s;
        }
#pragma unroll
        for (int j = 0; j < K - 1; ++j)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s = (j + 1 < K - 1) ? acc[j + 1][v] : 0.f;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 2 - j][kw][v], cur[kw][FLIP ? v : v / M], s);
                acc[j][v] = s;
            }
        const int oh = r - P;
        if (oh >= oh0) emit(oh, out);
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
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            out[v] = (K > 1) ? acc[0][v] : 0.f;
#pragma unroll
            for (int j = 0; j < K - 1; ++j) acc[j][v] = (j + 1 < K - 1) ? acc[j + 1][v] : 0.f;
        }
        const int oh = r - P;
        if (oh >= oh0) emit(oh, out);
    }
}

// ---------------------------------------------------------------------------------------------
// Stride 1, "same" padding, multiplier 1, TWO output columns per lane.  The 5x5 walk on two channels per lane
// is bound by the number of memory instructions (five 4-byte loads and a store per 50 multiply-adds); with two
// adjacent columns a lane loads K+1 input columns for two outputs and the same filter registers serve both.
// Rows are read through a buffer view of the image: the row offset is a scalar, the column offsets are loop
// invariants, and a column outside the image is read at an offset outside the view, which returns the zero of the
// padding (the filter cannot carry the zeros here, since a tap meets different columns for the two outputs).
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K, int PF, bool FLIP, int NCOL>
__global__ __launch_bounds__(256) void k_nhwc_s1_2col(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                      T *__restrict__ y, int TH, int nstrips, int nchunks,
                                                      unsigned nblocks, int nt)
{
    constexpr int P = (K - 1) / 2;
    constexpr int R = PF + 1;
    constexpr int NC = K + NCOL - 1;      // input columns per lane
    const Tile tl = tile_of(nblocks, nchunks, nstrips);
    const int Q = g.C / V, W2 = (g.W + NCOL - 1) / NCOL;
    const int f = tl.chunk * blockDim.x + threadIdx.x;
    if (f >= W2 * Q) return;
    const int cq = f % Q, ow = (f / Q) * NCOL;     // the last lane of a row may own fewer than NCOL columns

    // byte offset of each input column inside an image row; a column outside the image gets an offset beyond the
    // view, which reads as zero (the padding)
    uint32_t coloff[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const int iw = ow - P + j;
        coloff[j] = (iw >= 0 && iw < g.W) ? (uint32_t)(iw * g.C + cq * V) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
    }
    float wr[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const int sh = FLIP ? K - 1 - kh : kh, sw = FLIP ? K - 1 - kw : kw;
            Vec<T, V>::load(w + (sh * K + sw) * g.C + cq * V, wr[kh][kw]);
        }

    const int oh0 = tl.strip * TH, oh1 = min(g.H, oh0 + TH);
    const int rowstride = g.W * g.C;
    const uint32_t rowbytes = (uint32_t)rowstride * (uint32_t)sizeof(T);
    const BufView xin(x + (size_t)tl.n * g.H * rowstride, (uint32_t)g.H * rowbytes);      // the image: below 4 GiB
    const BufView yout(y + (size_t)tl.n * g.H * rowstride, (uint32_t)g.H * rowbytes);
    const uint32_t outoff = (uint32_t)(ow * g.C + cq * V) * (uint32_t)sizeof(T), colbytes = (uint32_t)g.C * (uint32_t)sizeof(T);

    float acc[K - 1][NCOL][V];
#pragma unroll
    for (int j = 0; j < K - 1; ++j)
#pragma unroll
        for (int c = 0; c < NCOL; ++c)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[j][c][v] = 0.f;

    const int r0 = oh0 - P, r1 = oh1 + P;
    const int ra = max(r0, 0), rb = min(r1, g.H);
    RawVec<T, V> ring[R][NC];
    auto load_row = [&](int r, RawVec<T, V> (&dst)[NC]) {
        const uint32_t rowoff = (uint32_t)min(r, rb - 1) * rowbytes;
#pragma unroll
        for (int j = 0; j < NC; ++j) dst[j].load_buf(xin, coloff[j], rowoff);
    };
    auto emit = [&](int oh, const float (&out)[NCOL][V]) {
#pragma unroll
        for (int c = 0; c < NCOL; ++c)
            if (ow + c < g.W) store_buf<T, V>(yout, outoff + c * colbytes, (uint32_t)oh * rowbytes, out[c], nt != 0);
    };
    auto consume = [&](int r, const RawVec<T, V> (&raw)[NC]) {
        float cur[NC][V];
#pragma unroll
        for (int j = 0; j < NC; ++j) raw[j].get(cur[j]);
        float out[NCOL][V];
#pragma unroll
        for (int c = 0; c < NCOL; ++c)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s = acc[0][c][v];
#pragma unroll
                for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 1][kw][v], cur[c + kw][v], s);
                out[c][v] = s;
            }
#pragma unroll
        for (int j = 0; j < K - 1; ++j)
#pragma unroll
            for (int c = 0; c < NCOL; ++c)
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float s = (j + 1 < K - 1) ? acc[j + 1][c][v] : 0.f;
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 2 - j][kw][v], cur[c + kw][v], s);
                    acc[j][c][v] = s;
                }
        const int oh = r - P;
        if (oh >= oh0) emit(oh, out);
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
    for (int r = rb; r < r1; ++r) {
        float out[NCOL][V];
#pragma unroll
        for (int c = 0; c < NCOL; ++c)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                out[c][v] = acc[0][c][v];
#pragma unroll
                for (int j = 0; j < K - 1; ++j) acc[j][c][v] = (j + 1 < K - 1) ? acc[j + 1][c][v] : 0.f;
            }
        const int oh = r - P;
        if (oh >= oh0) emit(oh, out);
    }
}

// ---------------------------------------------------------------------------------------------
// Forward, 3x3, stride 2, pad 1, multiplier 1.  A lane owns output column ow and walks down the
// output rows; input row 2*oh+1 is shared by output rows oh (tap row 2) and oh+1 (tap row 0).
// The two input rows of the next output row are loaded while the current one is computed.
// Padding as in the stride-1 kernel: zeroed weights for columns, uniform branches for rows.
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
    int coloff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int iw = 2 * ow - 1 + kw;
        const bool ok = iw >= 0 && iw < g.W;
        coloff[kw] = (ok ? iw : 2 * ow) * g.C;
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            Vec<T, V>::load(w + (kh * 3 + kw) * g.C + cq * V, wr[kh][kw]);
#pragma unroll
            for (int v = 0; v < V; ++v) wr[kh][kw][v] = ok ? wr[kh][kw][v] : 0.f;
        }
    }
    const int rowstride = g.W * g.C;
    const T *xin = x + (size_t)tl.n * g.H * rowstride + cq * V;
    T *yout = y + ((size_t)tl.n * g.Ho * g.Wo + ow) * g.C + cq * V;

    auto load_row = [&](int r, float (&dst)[3][V]) {
        const T *rp = xin + (size_t)min(max(r, 0), g.H - 1) * rowstride;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) Vec<T, V>::load(rp + coloff[kw], dst[kw]);
    };
    auto dot = [&](const float (&wk)[3][V], const float (&row)[3][V], float (&sum)[V]) {
#pragma unroll
        for (int v = 0; v < V; ++v)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) sum[v] = fmaf(wk[kw][v], row[kw][v], sum[v]);
    };

    // Output rows [oh0, ohb) have both input rows 2oh and 2oh+1 inside the image (all of them when
    // H is even); an odd H leaves one last row without its bottom tap row.  The main loop is
    // branch-free: two output rows per trip, the next pair of input rows loaded (clamped) ahead.
    const int oh0 = tl.strip * TH, oh1 = min(g.Ho, oh0 + TH);
    const int ohb = min(oh1, g.H / 2);
    float carry[V], re[2][3][V], ro[2][3][V];
#pragma unroll
    for (int v = 0; v < V; ++v) carry[v] = 0.f;
    if (2 * oh0 - 1 >= 0) {
        float top[3][V];
        load_row(2 * oh0 - 1, top);
        dot(wr[0], top, carry);
    }
    load_row(2 * oh0, re[0]);
    load_row(2 * oh0 + 1, ro[0]);
    auto step = [&](int oh, int j) {
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) { out[v] = carry[v]; carry[v] = 0.f; }
        dot(wr[1], re[j], out);
        dot(wr[2], ro[j], out);
        dot(wr[0], ro[j], carry);
        store_vec<T, V>(yout + (size_t)oh * g.Wo * g.C, out, nt != 0);
    };
    int oh = oh0;
#pragma unroll 1
    for (; oh + 2 <= ohb; oh += 2) {
        load_row(2 * oh + 2, re[1]); load_row(2 * oh + 3, ro[1]);
        step(oh, 0);
        load_row(2 * oh + 4, re[0]); load_row(2 * oh + 5, ro[0]);
        step(oh + 1, 1);
    }
    if (oh < ohb) {
        load_row(2 * oh + 2, re[1]);
        step(oh, 0);
        ++oh;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
#pragma unroll
            for (int v = 0; v < V; ++v) re[0][kw][v] = re[1][kw][v];
    }
    if (oh < oh1) {
        // odd H: the last output row has no input row 2oh+1
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) out[v] = carry[v];
        dot(wr[1], re[0], out);
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
// Rows 2a+1 >= H and columns 2b+1 >= W do not exist (odd H, W) and are skipped.  A missing
// column b+1 zeroes the weights that multiply it; a missing row a+1 is a block-uniform branch.
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

    const bool has_b1 = b + 1 < g.Wo;       // dy column b+1 exists
    const bool col1 = 2 * b + 1 < g.W;      // dx column 2b+1 exists
    float wr[3][3][V];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            Vec<T, V>::load(w + (kh * 3 + kw) * g.C + cq * V, wr[kh][kw]);
            if (kw == 0) {
#pragma unroll
                for (int v = 0; v < V; ++v) wr[kh][kw][v] = has_b1 ? wr[kh][kw][v] : 0.f;   // w?0 multiplies dy[.][b+1]
            }
        }
    const int dyrow = g.Wo * g.C, dxrow = g.W * g.C;
    const int off1 = has_b1 ? g.C : 0;
    const T *dyin = dy + ((size_t)tl.n * g.Ho * g.Wo + b) * g.C + cq * V;
    T *dxout = dx + ((size_t)tl.n * g.H * g.W + 2 * b) * g.C + cq * V;

    auto load_row = [&](int a, float (&d0)[V], float (&d1)[V]) {
        const T *rp = dyin + (size_t)min(a, g.Ho - 1) * dyrow;
        Vec<T, V>::load(rp, d0);
        Vec<T, V>::load(rp + off1, d1);
    };

    // dy rows [a0, ab) have a row a+1 below them; the last dy row of the image (a = Ho-1) does not
    // and is handled after the loop.  Main loop: three dy rows per trip, branch-free, row a+2
    // loaded (clamped) while rows a and a+1 are used.
    const int a0 = tl.strip * TH, a1 = min(g.Ho, a0 + TH);
    const int ab = min(a1, g.Ho - 1);
    float ring0[3][V], ring1[3][V];    // ring of three dy rows: column b and column b+1
    auto emit = [&](int a, const float (&A0)[V], const float (&A1)[V], const float (&B0)[V], const float (&B1)[V],
                    bool has_below) {
        float o00[V], o01[V], o10[V], o11[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            o00[v] = wr[1][1][v] * A0[v];
            o01[v] = fmaf(wr[1][0][v], A1[v], wr[1][2][v] * A0[v]);
            o10[v] = wr[2][1][v] * A0[v];
            o11[v] = fmaf(wr[2][0][v], A1[v], wr[2][2][v] * A0[v]);
        }
        if (has_below) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                o10[v] = fmaf(wr[0][1][v], B0[v], o10[v]);
                o11[v] = fmaf(wr[0][0][v], B1[v], fmaf(wr[0][2][v], B0[v], o11[v]));
            }
        }
        T *r0p = dxout + (size_t)(2 * a) * dxrow;
        store_vec<T, V>(r0p, o00, nt != 0);
        if (col1) store_vec<T, V>(r0p + g.C, o01, nt != 0);
        if (2 * a + 1 < g.H) {
            store_vec<T, V>(r0p + dxrow, o10, nt != 0);
            if (col1) store_vec<T, V>(r0p + dxrow + g.C, o11, nt != 0);
        }
    };
    load_row(a0, ring0[0], ring1[0]);
    load_row(a0 + 1, ring0[1], ring1[1]);
    int a = a0;
#pragma unroll 1
    for (; a + 3 <= ab; a += 3) {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            load_row(a + j + 2, ring0[(j + 2) % 3], ring1[(j + 2) % 3]);
            emit(a + j, ring0[j], ring1[j], ring0[(j + 1) % 3], ring1[(j + 1) % 3], true);
        }
    }
    // up to two more rows with a row below, then possibly the image's last dy row
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        if (a + j < a1) {
            if (j < 2) load_row(a + j + 2, ring0[(j + 2) % 3], ring1[(j + 2) % 3]);
            emit(a + j, ring0[j], ring1[j], ring0[(j + 1) % 3], ring1[(j + 1) % 3], a + j + 1 < g.Ho);
        }
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
template <typename T, int V, int K, int S, int PF, int M, bool FLAT = false>
__global__ __launch_bounds__(256, (PF <= 2 && K == 3 && S == 1 && sizeof(T) == 4) ? 4 : 1) void k_nhwc_bwd_filter(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                         float *__restrict__ ws, int CT, int nctiles, int nowtiles,
                                                         int TH, int nstrips, int NI, unsigned nblocks)
{
    constexpr int P = (K - 1) / 2;   // also the pad for S == 2, K == 3
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
    const bool active = cq < Q && ow < g.Wo;

    float acc[K][K][V];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw)
#pragma unroll
            for (int v = 0; v < V; ++v) acc[kh][kw][v] = 0.f;

    if (active) {
        // Loads are unconditional (clamped rows) and untouched until consumed, so they stay in flight across
        // iterations.  Rows outside the image or the strip are handled by peeling the first and last few rows off
        // the main loop (the conditions are uniform over the block).  Columns outside the image:
        //  * 5x5 (BUF): loads go through a buffer view of the image; the row offset is a scalar, the column offsets
        //    are loop invariants, and a column outside the image is read at an offset outside the view, which
        //    returns zero, so its taps accumulate nothing.  That takes the 64-bit address arithmetic (six adds per
        //    50 multiply-adds) out of a walk that is bound by its vector-ALU work: 4 % faster.
        //  * 3x3: flat loads at clamped columns (the views measured 3-14 % slower there); the lane accumulates
        //    whatever the clamped address holds and zeroes those taps' sums once, after the walk.
        constexpr bool BUF = K == 5;
        bool colok[K];
        uint32_t coloff[K];      // BUF: bytes inside an image row
        int coloff_e[K];         // flat loads: elements from the start of the row
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const int iw = ow * S - P + kw;
            colok[kw] = iw >= 0 && iw < g.W;
            coloff[kw] = colok[kw] ? (uint32_t)(iw * g.C + cq * VX) * (uint32_t)sizeof(T) : BufView::OUTSIDE;
            coloff_e[kw] = (colok[kw] ? iw : ow * S) * g.C;
        }
        const uint32_t dyoff = (uint32_t)(ow * g.O + cq * V) * (uint32_t)sizeof(T);
        const int xrow = g.W * g.C, dyrow = g.Wo * g.O;
        const uint32_t xrowbytes = (uint32_t)xrow * (uint32_t)sizeof(T), dyrowbytes = (uint32_t)dyrow * (uint32_t)sizeof(T);
        const uint32_t ximg = (uint32_t)g.H * xrowbytes, dyimg = (uint32_t)g.Ho * dyrowbytes;      // an image: at most 2 GiB
        // one row of x (K columns) and one of dy for image nn, rows already clamped
        auto load_rows_x = [&](int nn, int r, RawVec<T, VX> (&dst)[K]) {
            if constexpr (BUF) {
                const BufView xin(x + (size_t)nn * g.H * xrow, ximg);
#pragma unroll
                for (int kw = 0; kw < K; ++kw) dst[kw].load_buf(xin, coloff[kw], (uint32_t)r * xrowbytes);
            } else {
                const T *xin = x + (size_t)nn * g.H * xrow + cq * VX;
                const T *rp = xin + (size_t)r * xrow;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) dst[kw].load(rp + coloff_e[kw]);
            }
        };
        auto load_row_dy = [&](int nn, int oh, RawVec<T, V> &dst) {
            if constexpr (BUF) dst.load_buf(BufView(dy + (size_t)nn * g.Ho * dyrow, dyimg), dyoff, (uint32_t)oh * dyrowbytes);
            else {
                const T *dyin = dy + ((size_t)nn * g.Ho * g.Wo + ow) * g.O + cq * V;
                dst.load(dyin + (size_t)oh * dyrow);
            }
        };
        const int oh0 = strip * TH, oh1 = min(g.Ho, oh0 + TH);
        const int n0 = ngroup * NI, n1 = min(g.N, n0 + NI);
        if constexpr (S == 1 && FLAT) {
            // FLAT (3x3 bf16 on small planes, where it measured 10 % faster; on large planes and for 5x5 it measured
            // 4-17 % slower than the per-image walk below): one flat sequence of steps over (image, row): step (n, r), r = oh0-P .. oh1+P-1, takes dy row r+P into
            // the window of K live dy rows (a zero row once r+P is below the strip) and, when x row r is inside the
            // image, accumulates it against the window: input row r meets dy row r+P-kh at tap row kh.  The loads of
            // step s+PF are issued at step s and stay as loaded (packed for bf16) until they are used, ACROSS image
            // boundaries: a walk that starts over with every image waits one full memory latency per image, which on
            // 14- or 19-row planes is as long as the image's arithmetic.  Every condition is uniform over the block.
            constexpr int R = PF + 1;
            const int r0 = oh0 - P, rend = oh1 + P;
            const int total = (n1 - n0) * (rend - r0);
            float dyw[K][V];
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int v = 0; v < V; ++v) dyw[kh][v] = 0.f;
            int pn = n0, pr = r0;          // the step whose loads are issued next
            auto issue = [&](RawVec<T, VX> (&xd)[K], RawVec<T, V> &dd) {
                const int nn = min(pn, n1 - 1);
                load_rows_x(nn, min(max(pr, 0), g.H - 1), xd);
                load_row_dy(nn, min(max(pr + P, oh0), oh1 - 1), dd);
                if (++pr == rend) { pr = r0; ++pn; }
            };
            int cr = r0;                   // row of the step being consumed
            auto consume = [&](const RawVec<T, VX> (&xd)[K], const RawVec<T, V> &dd) {
                float dv[V];
                dd.get(dv);
                if (cr + P >= oh1) {       // the new dy row is below the strip: it belongs to the next block's sums
#pragma unroll
                    for (int v = 0; v < V; ++v) dv[v] = 0.f;
                }
                if (cr == r0) {            // a new image: nothing of the previous one may stay in the window
#pragma unroll
                    for (int kh = 0; kh < K; ++kh)
#pragma unroll
                        for (int v = 0; v < V; ++v) dyw[kh][v] = 0.f;
                }
#pragma unroll
                for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                    for (int v = 0; v < V; ++v) dyw[kh][v] = dyw[kh - 1][v];
#pragma unroll
                for (int v = 0; v < V; ++v) dyw[0][v] = dv[v];
                if (cr >= 0 && cr < g.H) {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        float xv[VX];
                        xd[kw].get(xv);
#pragma unroll
                        for (int kh = 0; kh < K; ++kh)
#pragma unroll
                            for (int v = 0; v < V; ++v) acc[kh][kw][v] = fmaf(dyw[kh][v], xv[v / M], acc[kh][kw][v]);
                    }
                }
                if (++cr == rend) cr = r0;
            };
            RawVec<T, VX> xr[R][K];
            RawVec<T, V> dr[R];
#pragma unroll
            for (int j = 0; j < PF; ++j) issue(xr[j], dr[j]);
            int st = 0;
#pragma unroll 1
            for (; st + R <= total; st += R) {
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    issue(xr[(j + PF) % R], dr[(j + PF) % R]);
                    consume(xr[j], dr[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < R - 1; ++j)
                if (st + j < total) consume(xr[j], dr[j]);
        } else {
        for (int n = n0; n < n1; ++n) {
            // rows are loaded ahead and stay as loaded (packed for bf16) until they are accumulated
            auto load_xr = [&](int r, RawVec<T, VX> (&dst)[K]) { load_rows_x(n, min(max(r, 0), g.H - 1), dst); };
            auto load_dr = [&](int oh, RawVec<T, V> &dst) { load_row_dy(n, min(max(oh, oh0), oh1 - 1), dst); };
            if constexpr (S == 1) {
                // input row r meets dy row r + P - kh at tap row kh; dyw holds the K live dy rows
                // The main loop takes R rows per trip.  R = K lets the window of live dy rows come back to the same
                // registers after every trip (a trip of PF + 1 = 3 rows on a 5-row window costs a register copy per
                // window entry and row); only PF + 1 of the R ring slots are live at any time.
                constexpr int R = (K > PF + 1) ? K : PF + 1;
                float dyw[K][V];
#pragma unroll
                for (int kh = 0; kh < K; ++kh)
#pragma unroll
                    for (int v = 0; v < V; ++v) dyw[kh][v] = 0.f;
                auto push_dy = [&](const float (&d)[V]) {
#pragma unroll
                    for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                        for (int v = 0; v < V; ++v) dyw[kh][v] = dyw[kh - 1][v];
#pragma unroll
                    for (int v = 0; v < V; ++v) dyw[0][v] = d[v];
                };
                auto push_raw = [&](const RawVec<T, V> &d) {
                    float dv[V];
                    d.get(dv);
                    push_dy(dv);
                };
                auto accumulate = [&](const RawVec<T, VX> (&xr)[K]) {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        float xv[VX];
                        xr[kw].get(xv);
#pragma unroll
                        for (int kh = 0; kh < K; ++kh)
#pragma unroll
                            for (int v = 0; v < V; ++v) acc[kh][kw][v] = fmaf(dyw[kh][v], xv[v / M], acc[kh][kw][v]);
                    }
                };
                const int r0 = oh0 - P, r1 = oh1 + P;
                const int ra = max(r0, 0), rb = min(r1, g.H);       // x rows inside the image
                const int rm = min(rb, oh1 - P);                     // rows whose new dy row r+P is inside the strip
                float zero[V];
#pragma unroll
                for (int v = 0; v < V; ++v) zero[v] = 0.f;
                // 5x5 bf16: the image's first loads all go out together, i.e. the first PF rows of the walk and the
                // dy rows of the (up to P) rows above the image, which enter the window without anything being
                // accumulated: one memory latency per image instead of one per row above it plus one for the walk.
                // The other variants have no registers to spare for it (the fp32 3x3 kernel would spill).
                constexpr bool TOGETHER = K == 5 && sizeof(T) == 2;
                RawVec<T, VX> xr[R][K];
                RawVec<T, V> dr[R];
                if constexpr (TOGETHER) {
                    RawVec<T, V> above[P];
#pragma unroll
                    for (int j = 0; j < PF; ++j) { load_xr(ra + j, xr[j]); load_dr(ra + j + P, dr[j]); }
#pragma unroll
                    for (int i = 0; i < P; ++i)
                        if (r0 + i < ra) load_dr(r0 + i + P, above[i]);
#pragma unroll
                    for (int i = 0; i < P; ++i)
                        if (r0 + i < ra) {
                            if (r0 + i + P >= oh1) push_dy(zero);
                            else push_raw(above[i]);
                        }
                } else {
                    // rows above the image: their dy rows enter the window, nothing is accumulated
                    for (int r = r0; r < ra; ++r) {
                        RawVec<T, V> d;
                        load_dr(r + P, d);
                        if (r + P >= oh1) push_dy(zero);
                        else push_raw(d);
                    }
#pragma unroll
                    for (int j = 0; j < PF; ++j) { load_xr(ra + j, xr[j]); load_dr(ra + j + P, dr[j]); }
                }
                int base = ra;
#pragma unroll 1
                for (; base + R <= rm; base += R) {
#pragma unroll
                    for (int j = 0; j < R; ++j) {
                        load_xr(base + j + PF, xr[(j + PF) % R]);
                        load_dr(base + j + PF + P, dr[(j + PF) % R]);
                        push_raw(dr[j]);
                        accumulate(xr[j]);
                    }
                }
                // remaining rows: those still inside [ra, rm) use their prefetched dy row (and keep the ring
                // filled: a load past the last row is clamped and never used), the last ones (new dy row below the
                // strip) push zeros
#pragma unroll
                for (int j = 0; j < R - 1; ++j) {
                    if (base + j < rm) {
                        if (j + PF < R - 1) { load_xr(base + j + PF, xr[(j + PF) % R]); load_dr(base + j + PF + P, dr[(j + PF) % R]); }
                        push_raw(dr[j]);
                        accumulate(xr[j]);
                    }
                }
                for (int r = max(rm, ra); r < rb; ++r) {
                    RawVec<T, VX> xt[K];
                    load_xr(r, xt);
                    push_dy(zero);
                    accumulate(xt);
                }
            } else {
                // output row oh meets input rows 2oh-1, 2oh, 2oh+1; row 2oh+1 is reused by oh+1.
                // Rows [oh0, ohb) have all of 2oh, 2oh+1 inside the image; an odd H leaves one last
                // row without its bottom tap row.  The next output row's loads are issued ahead and stay
                // as loaded (packed for bf16) until the row is accumulated.
                const int ohb = min(oh1, g.H / 2);
                RawVec<T, VX> xa[K], xb[2][K], xc[2][K];
                RawVec<T, V> d[2];
                if (2 * oh0 - 1 >= 0) load_xr(2 * oh0 - 1, xa);
                else {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) xa[kw].zero();
                }
                load_xr(2 * oh0, xb[0]); load_xr(2 * oh0 + 1, xc[0]); load_dr(oh0, d[0]);
                auto tap_row = [&](int kh, const RawVec<T, VX> (&xr)[K], const float (&dv)[V]) {
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        float xv[VX];
                        xr[kw].get(xv);
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[kh][kw][v] = fmaf(dv[v], xv[v / M], acc[kh][kw][v]);
                    }
                };
                auto step = [&](int j) {
                    float dv[V];
                    d[j].get(dv);
                    tap_row(0, xa, dv); tap_row(1, xb[j], dv); tap_row(2, xc[j], dv);
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) xa[kw] = xc[j][kw];
                };
                int oh = oh0;
#pragma unroll 1
                for (; oh + 2 <= ohb; oh += 2) {
                    load_xr(2 * oh + 2, xb[1]); load_xr(2 * oh + 3, xc[1]); load_dr(oh + 1, d[1]);
                    step(0);
                    load_xr(2 * oh + 4, xb[0]); load_xr(2 * oh + 5, xc[0]); load_dr(oh + 2, d[0]);
                    step(1);
                }
                if (oh < ohb) {
                    load_xr(2 * oh + 2, xb[1]); load_dr(oh + 1, d[1]);
                    step(0);
                    ++oh;
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) xb[0][kw] = xb[1][kw];
                    d[0] = d[1];
                }
                if (oh < oh1) {
                    // odd H: the last output row has no input row 2oh+1
                    float dv[V];
                    d[0].get(dv);
                    tap_row(0, xa, dv); tap_row(1, xb[0], dv);
                }
            }
        }
        }
        if constexpr (!BUF) {
            // taps on columns outside the image accumulated clamped data: drop them
#pragma unroll
            for (int kw = 0; kw < K; ++kw)
                if (!colok[kw]) {
#pragma unroll
                    for (int kh = 0; kh < K; ++kh)
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[kh][kw][v] = 0.f;
                }
        }
    }

    // ---- fixed-order block reduction ----
    const int part = (ngroup * nstrips + strip) * nowtiles + owtile;
    float *wsp = ws + (size_t)part * (K * K * g.O);
    block_reduce_taps<K, V>(acc, CT, red, [&](int kh, int kw, int v, float total) {
        if (cq < Q) wsp[(kh * K + kw) * g.O + cq * V + v] = total;
    });
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

template <typename T, int V, int K, int PF, int M>
static hipError_t launch_s1(const Geom &g, const void *x, const void *w, void *y, bool flip, int TH, hipStream_t st)
{
    const int lanes = g.W * (g.O / V);
    const int bs = flat_block(lanes);
    const int nchunks = ceil_div(lanes, bs), nstrips = ceil_div(g.H, TH);
    const unsigned nblocks = (unsigned)g.N * nchunks * nstrips;
    const int nt = stream_stores(flip ? "NHWC_S1_BWD" : "NHWC_S1_FWD", (long long)g.N * g.H * g.W * (flip ? g.C : g.O) * sizeof(T), 0);
    if (flip)
        hipLaunchKernelGGL((k_nhwc_s1<T, V, K, PF, true, M>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    else
        hipLaunchKernelGGL((k_nhwc_s1<T, V, K, PF, false, M>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    return hipGetLastError();
}

template <typename T, int V, int K, int PF, int NCOL>
static hipError_t launch_s1_2col(const Geom &g, const void *x, const void *w, void *y, bool flip, int TH, hipStream_t st)
{
    const int lanes = ((g.W + NCOL - 1) / NCOL) * (g.C / V);
    const int bs = flat_block(lanes);
    const int nchunks = ceil_div(lanes, bs), nstrips = ceil_div(g.H, TH);
    const unsigned nblocks = (unsigned)g.N * nchunks * nstrips;
    const int nt = stream_stores(flip ? "NHWC_S1_BWD" : "NHWC_S1_FWD", (long long)g.N * g.H * g.W * g.C * sizeof(T), 0);
    if (flip)
        hipLaunchKernelGGL((k_nhwc_s1_2col<T, V, K, PF, true, NCOL>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    else
        hipLaunchKernelGGL((k_nhwc_s1_2col<T, V, K, PF, false, NCOL>), dim3(nblocks), dim3(bs), 0, st, g, (const T *)x,
                           (const T *)w, (T *)y, TH, nstrips, nchunks, nblocks, nt);
    return hipGetLastError();
}

hipError_t nhwc_s1(const Geom &g, int dtype, int V, const void *x, const void *w, void *y, bool flip, int TH, int PF,
                   hipStream_t st)
{
    // bf16 5x5 on two channels per lane: two output columns per lane (fewer memory instructions)
    if (dtype == DT_BF16 && g.m == 1 && g.K == 5 && V == 2 && !tune_env("DWCONV_TUNE_NO2COL")) {
        const char *e = tune_env("DWCONV_TUNE_NCOL");
        const int ncol = e ? atoi(e) : 2;
        if (ncol == 4) return launch_s1_2col<bf16_t, 2, 5, 2, 4>(g, x, w, y, flip, TH, st);
        if (ncol == 3) return launch_s1_2col<bf16_t, 2, 5, 2, 3>(g, x, w, y, flip, TH, st);
        if (PF == 1) return launch_s1_2col<bf16_t, 2, 5, 1, 2>(g, x, w, y, flip, TH, st);
        return launch_s1_2col<bf16_t, 2, 5, 2, 2>(g, x, w, y, flip, TH, st);
    }
#define TRY(T, VV, KK, PPF) if (g.m == 1 && g.K == KK && V == VV && PF == PPF) return launch_s1<T, VV, KK, PPF, 1>(g, x, w, y, flip, TH, st)
    // channel multiplier 2: 3x3, two rows ahead
    if (g.m == 2 && g.K == 3) {
        if (dtype == DT_F32 && V == 4) return launch_s1<float, 4, 3, 2, 2>(g, x, w, y, flip, TH, st);
        if (dtype == DT_BF16 && V == 8) return launch_s1<bf16_t, 8, 3, 2, 2>(g, x, w, y, flip, TH, st);
        if (dtype == DT_BF16 && V == 4) return launch_s1<bf16_t, 4, 3, 2, 2>(g, x, w, y, flip, TH, st);
        return hipErrorInvalidValue;
    }
    if (dtype == DT_F32) {
        TRY(float, 4, 3, 1); TRY(float, 4, 3, 2); TRY(float, 4, 3, 3); TRY(float, 4, 3, 4);
        TRY(float, 4, 5, 1); TRY(float, 4, 5, 2);
    } else {
        TRY(bf16_t, 8, 3, 1); TRY(bf16_t, 8, 3, 2); TRY(bf16_t, 8, 3, 3);
        TRY(bf16_t, 4, 3, 1); TRY(bf16_t, 4, 3, 2); TRY(bf16_t, 4, 3, 3);
        TRY(bf16_t, 2, 5, 1); TRY(bf16_t, 2, 5, 2);
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
    const int nt = bwd ? stream_stores("NHWC_S2_BWD", (long long)g.N * g.H * g.W * g.C * (dtype == DT_F32 ? 4 : 2), 0)
                       : stream_stores("NHWC_S2_FWD", (long long)g.N * g.Ho * g.Wo * g.C * (dtype == DT_F32 ? 4 : 2), 0);
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
    const int Q = g.O / V;
    // Lanes of a block: CT channel-vectors x 256/CT columns, up to 64 vectors (1 KB of a pixel) wide;
    // narrower channel tiles with more columns measured slower.
    const int cap = 64;
    int ct = 1;
    while (ct < Q && ct < cap) ct <<= 1;
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
#define GO(T, VV, KK, SS) hipLaunchKernelGGL((k_nhwc_bwd_filter<T, VV, KK, SS, 2, 1>), dim3(nblocks), dim3(256), 0, st, g, \
                                             (const T *)x, (const T *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks)
#define GOM2(T, VV) hipLaunchKernelGGL((k_nhwc_bwd_filter<T, VV, 3, 1, 2, 2>), dim3(nblocks), dim3(256), 0, st, g, \
                                       (const T *)x, (const T *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks)
    if (g.m == 2) {
        if (!(g.K == 3 && g.s == 1)) return hipErrorInvalidValue;
        if (dtype == DT_F32 && V == 4) GOM2(float, 4);
        else if (dtype == DT_BF16 && V == 8) GOM2(bf16_t, 8);
        else if (dtype == DT_BF16 && V == 4) GOM2(bf16_t, 4);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
#undef GOM2
    if (dtype == DT_F32) {
        if (g.K == 3 && g.s == 1) GO(float, 4, 3, 1);
        else if (g.K == 3 && g.s == 2) GO(float, 4, 3, 2);
        else if (g.K == 5 && g.s == 1) GO(float, 4, 5, 1);
        else return hipErrorInvalidValue;
    } else {
        // packed dot products over row pairs: 5x5 (459 against 480 us per step over the nine bf16 layers at batch 256) and
        // 3x3 with four channels per lane (142 against 151 us over six layers); with eight channels per lane the
        // multiply-add form is faster (204 against 209 us over three layers) unless DWCONV_TUNE_DOT2K3=1
        if (nhwc_bwd_filter_dot2_supported(g, V) && (g.K == 5 || V == 4 || tune_env("DWCONV_TUNE_DOT2K3")))
            return nhwc_bwd_filter_dot2(g, V, x, dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks, st);
        if (g.K == 3 && g.s == 1 && V == 8) GO(bf16_t, 8, 3, 1);
        else if (g.K == 3 && g.s == 1 && g.H <= 28)
            hipLaunchKernelGGL((k_nhwc_bwd_filter<bf16_t, 4, 3, 1, 2, 1, true>), dim3(nblocks), dim3(256), 0, st, g, (const bf16_t *)x,
                               (const bf16_t *)dy, ws, CT, nctiles, nowtiles, TH, nstrips, NI, nblocks);
        else if (g.K == 3 && g.s == 1) GO(bf16_t, 4, 3, 1);
        else if (g.K == 3 && g.s == 2 && V == 8) GO(bf16_t, 8, 3, 2);
        else if (g.K == 3 && g.s == 2) GO(bf16_t, 4, 3, 2);
        else if (g.K == 5 && g.s == 1 && V == 2) GO(bf16_t, 2, 5, 1);
        else return hipErrorInvalidValue;
    }
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
