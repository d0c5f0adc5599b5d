// NCHW "row-walk" kernels for planes whose rows are a whole number of 16-byte vectors.
// A lane owns V adjacent columns of one plane and walks down the rows of its strip.  Per input
// row it loads one aligned V-wide vector plus the few neighbour elements left and right of it
// (the L1 serves those), rows ahead of the row being consumed.  The vector ALU budget is what
// shapes these kernels: at full HBM rate a CU retires about one output element per clock and can
// issue 64 lane-operations per clock, so everything besides the K*K multiply-adds per element
// (addressing, edge handling) is amortised over the V outputs of a lane.
#include "kernels.hpp"
#include <stdlib.h>

namespace dwc {

static inline int ceil_div_h(int a, int b) { return (a + b - 1) / b; }

// Rows per group of the whole-line write-out for output rows of W elements of esz bytes: the
// smallest group that is a whole number of 128-byte lines, capped at 4 rows (rows of 112 bytes
// then make groups of whole 64-byte half lines, which measured as good).  0: not applicable
// (rows that are whole lines by themselves, or too short).
static int row_group(int W, int esz)
{
    int rs = 1;
    while (rs <= 4 && (rs * W * esz) % 128 != 0) rs <<= 1;
    if (rs == 8) rs = 4;
    return (rs == 2 || rs == 4) ? rs : 0;
}

// flat lane index -> (plane, strip, vector column)
struct Lane { int plane, strip, c4; bool valid; };
__device__ __forceinline__ Lane lane_of(unsigned nblocks, int ncols, int nstrips, int nplanes)
{
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const unsigned f = lb * 256u + threadIdx.x;
    Lane l;
    const unsigned ps = f / (unsigned)ncols;
    l.c4 = f - ps * ncols;
    l.plane = ps / (unsigned)nstrips;
    l.strip = ps - l.plane * nstrips;
    l.valid = l.plane < nplanes;
    return l;
}

// ---------------------------------------------------------------------------------------------
// Whole-line write-out through LDS.  An output row of a plane is not a whole number of 128-byte
// lines, but RS consecutive rows are (RS = 2 for rows of 448 bytes, 4 for 224), and they are
// contiguous in memory.  Each lane parks the 16-byte vectors it produces for RS successive rows of
// its work item in LDS; then the block's 256 * RS vectors are written in memory order with
// streaming stores: entry e = tid + 256 k belongs to the work item of lane e / RS, and inside an
// item the entries run over (row, vector column) like the addresses do.  Two LDS buffers alternate,
// so one barrier per RS rows is enough.  Every lane of the block must take part (no early exit), the
// rows per strip must be a multiple of RS, and all lanes must produce rows in lockstep.
// ---------------------------------------------------------------------------------------------
template <typename T, int RS>
struct LineWriter {
    int idx[RS], rows[RS];
    T *ptr[RS];
    int slot, buf, done;      // uniform over the block

    // lanes are laid flat over (plane, strip, vector column); W4 vectors per row, VE elements per
    // vector, TH output rows per strip, H x W output planes
    __device__ __forceinline__ void init(unsigned lb, int W4, int VE, int nstrips, int nplanes, int TH, int H, int W, T *out)
    {
#pragma unroll
        for (int k = 0; k < RS; ++k) {
            const int e = threadIdx.x + 256 * k;
            const int l = e / RS;
            const unsigned psl = (lb * 256u + l) / (unsigned)W4;
            const long long first = (long long)psl * W4 - (long long)lb * 256;
            const int a = first > 0 ? (int)first : 0;
            const int b = first + W4 < 256 ? (int)(first + W4) : 256;
            const int cnt = b - a, rel = e - RS * a;
            const int srow = rel / cnt, ll = a + rel - srow * cnt;
            const int c4l = (int)((long long)ll - first);
            const int pl = psl / (unsigned)nstrips, stl = psl - pl * nstrips;
            const int o0 = stl * TH, o1 = min(H, o0 + TH);
            idx[k] = srow * 256 + ll;
            rows[k] = pl < nplanes ? o1 - (o0 + srow) : 0;     // rows from this entry's first one to the strip's end
            ptr[k] = out + ((size_t)min(pl, nplanes - 1) * H + (o0 + srow)) * W + c4l * VE;
        }
        slot = 0; buf = 0; done = 0;
    }

    // the lane's vector of the next row of its item; writes out after every RS-th row
    __device__ __forceinline__ void put(u4v_t (&stage)[2][RS * 256], const u4v_t &pk, int W)
    {
        stage[buf][slot * 256 + threadIdx.x] = pk;
        if (++slot == RS) {
            __syncthreads();
#pragma unroll
            for (int k = 0; k < RS; ++k)
                if (done < rows[k]) {
                    const u4v_t v = stage[buf][idx[k]];
                    __builtin_nontemporal_store(v, reinterpret_cast<u4v_t *>(ptr[k] + (size_t)done * W));
                }
            slot = 0; buf ^= 1; done += RS;
        }
    }
};

template <typename T>
__device__ __forceinline__ u4v_t pack16(const float (&r)[16 / sizeof(T)])
{
    u4v_t pk;
    if constexpr (sizeof(T) == 4) {
        pk.x = __float_as_uint(r[0]); pk.y = __float_as_uint(r[1]); pk.z = __float_as_uint(r[2]); pk.w = __float_as_uint(r[3]);
    } else {
        pk.x = pack2_bf16(r[0], r[1]);
        pk.y = pack2_bf16(r[2], r[3]);
        pk.z = pack2_bf16(r[4], r[5]);
        pk.w = pack2_bf16(r[6], r[7]);
    }
    return pk;
}

// ---------------------------------------------------------------------------------------------
// Forward, stride 1, "same" padding (K odd, pad (K-1)/2), any multiplier; FLIP = filter rotated
// by 180 degrees = backward-data of the same layer (multiplier 1).
// A lane owns V adjacent columns and walks TH + 2P input rows with K-1 rotating accumulators; the
// ring holds raw loads (clamped addresses), padding is applied when a row is consumed, and every
// lane walks the same number of rows (lanes of a shorter last strip, and lanes past the last plane,
// run on with their stores masked).
// RS > 0: whole-line write-out of RS-row groups (needs 16-byte vectors, TH % RS == 0, H % RS == 0);
// RS == 0: each lane stores its vector directly (streamed if nt).
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K, int PF, bool FLIP, int RS>
__global__ __launch_bounds__(256) void k_nchwd_s1(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                  T *__restrict__ y, int TH, int nstrips, unsigned nblocks, int nt)
{
    static_assert(RS == 0 || sizeof(T) * V == 16, "whole-line write-out: one 16-byte vector per lane and row");
    constexpr int P = (K - 1) / 2;
    constexpr int NW = V + 2 * P;
    constexpr int R = PF + 1;
    __shared__ u4v_t stage[2][RS > 0 ? RS * 256 : 1];
    const int W4 = g.W / V;
    const int nplanes = g.N * g.O;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const unsigned f = lb * 256u + threadIdx.x;
    const unsigned ps = f / (unsigned)W4;
    const int c4 = f - ps * W4;
    int plane = ps / (unsigned)nstrips;
    const int strip = ps - plane * nstrips;
    const bool valid = plane < nplanes;
    if (!valid) plane = nplanes - 1;      // lanes past the end compute on the last plane; nothing of theirs is stored
    const int n = plane / g.O, o = plane - n * g.O;
    const int plane_in = n * g.C + o / g.m;

    float wr[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) wr[kh][kw] = ldf(w + (o * K + (FLIP ? K - 1 - kh : kh)) * K + (FLIP ? K - 1 - kw : kw));

    const bool has_left = c4 > 0, has_right = c4 < W4 - 1;
    const T *xin = x + (size_t)plane_in * g.H * g.W + c4 * V;
    T *yout = y + (size_t)plane * g.H * g.W + c4 * V;
    const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);

    LineWriter<T, (RS > 0 ? RS : 1)> lw;
    if constexpr (RS > 0) lw.init(lb, W4, V, nstrips, nplanes, TH, g.H, g.W, y);

    int loff[P > 0 ? P : 1], roff[P > 0 ? P : 1];
#pragma unroll
    for (int i = 0; i < P; ++i) { loff[i] = has_left ? -(P - i) : 0; roff[i] = has_right ? V + i : V - 1; }

    float ring[R][NW];
    auto load_row = [&](int r, float (&dst)[NW]) {
        const T *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
        float mid[V];
        Vec<T, V>::load(rp, mid);
#pragma unroll
        for (int i = 0; i < P; ++i) { dst[i] = ldf(rp + loff[i]); dst[P + V + i] = ldf(rp + roff[i]); }
#pragma unroll
        for (int v = 0; v < V; ++v) dst[P + v] = mid[v];
    };

    float acc[K - 1 > 0 ? K - 1 : 1][V];
#pragma unroll
    for (int j = 0; j < K - 1; ++j)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[j][v] = 0.f;

    auto consume = [&](int idx, int r, const float (&raw)[NW]) {
        const bool rowok = r >= 0 && r < g.H;
        float cur[NW];
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const bool ok = rowok && (i < P ? has_left : (i >= P + V ? has_right : true));
            cur[i] = ok ? raw[i] : 0.f;
        }
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float s = (K > 1) ? acc[0][v] : 0.f;
#pragma unroll
            for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 1][kw], cur[v + kw], s);
            out[v] = s;
        }
#pragma unroll
        for (int jj = 0; jj < K - 1; ++jj)
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s = (jj + 1 < K - 1) ? acc[jj + 1][v] : 0.f;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) s = fmaf(wr[K - 2 - jj][kw], cur[v + kw], s);
                acc[jj][v] = s;
            }
        if (idx >= 2 * P) {        // the row just finished is output row oh0 + idx - 2P
            if constexpr (RS > 0) lw.put(stage, pack16<T>(out), g.W);
            else if (valid && r - P < oh1) store_vec<T, V>(yout + (size_t)(r - P) * g.W, out, nt != 0);
        }
    };

    const int r0 = oh0 - P, nrows = TH + 2 * P;
#pragma unroll
    for (int j = 0; j < PF; ++j) load_row(r0 + j, ring[j]);
    int i = 0;
#pragma unroll 1
    for (; i + R <= nrows; i += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            load_row(r0 + i + j + PF, ring[(j + PF) % R]);
            consume(i + j, r0 + i + j, ring[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < R - 1; ++j)
        if (i + j < nrows) consume(i + j, r0 + i + j, ring[j]);
}

// ---------------------------------------------------------------------------------------------
// bf16 stride-1 walk on packed pairs.  In NCHW two adjacent columns share a 32-bit word, and
// gfx950 multiplies two bf16 pairs and adds both products to an fp32 accumulator in one
// instruction (v_dot2c_f32_bf16), so the row stays packed: no widening, and a K-tap row of an
// output costs ceil((K+1)/2) instructions instead of K.  A lane owns 8 columns = 4 words, plus the
// aligned word left and right of them (columns -2,-1 and 8,9): P[i] = columns (2i-2, 2i-1).
// Output column j reads columns j-P..j+P, which start in word (j-P+2)/2 at half (j+P)&1; the
// filter row is packed twice, once for each starting half, with a zero in the unused half.
// Accumulation is fp32 as in the other kernels; products of bf16 values are exact in fp32.
// RS > 0: whole-line write-out of RS-row groups (LineWriter); RS == 0: direct 16-byte stores.
// ---------------------------------------------------------------------------------------------
template <int V, int K, int PF, bool FLIP, int RS>
__global__ __launch_bounds__(256) void k_nchwd_s1_bf16x8(Geom g, const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                         bf16_t *__restrict__ y, int TH, int nstrips, unsigned nblocks)
{
    static_assert((V == 8 || V == 4) && (RS == 0 || V == 8), "8 columns per lane, or 4 without the whole-line write-out");
    constexpr int P = (K - 1) / 2, R = PF + 1;
    constexpr int NP = V / 2 + 2;                   // words per row and lane
    constexpr int NT = (K + 2) / 2;                 // packed words per filter row (either starting half)
    static_assert(K == 3 || K == 5, "left and right neighbours must fit one word each");
    __shared__ u4v_t stage[2][(RS > 0 ? RS : 1) * 256];
    const int W4 = g.W / V;
    const int nplanes = g.N * g.O;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const unsigned f = lb * 256u + threadIdx.x;
    const unsigned ps = f / (unsigned)W4;
    const int c4 = f - ps * W4;
    int plane = ps / (unsigned)nstrips;
    const int strip = ps - plane * nstrips;
    const bool valid = plane < nplanes;
    if (!valid) plane = nplanes - 1;      // lanes past the end compute on the last plane; nothing of theirs is stored
    const int n = plane / g.O, o = plane - n * g.O;
    const int plane_in = n * g.C + o / g.m;

    // filter rows packed for both starting halves: wp[kh][q][t], q = (j + P) & 1
    uint32_t wp[K][2][NT];
#pragma unroll
    for (int kh = 0; kh < K; ++kh) {
        uint32_t wv[K];
#pragma unroll
        for (int kw = 0; kw < K; ++kw) wv[kw] = w[(o * K + (FLIP ? K - 1 - kh : kh)) * K + (FLIP ? K - 1 - kw : kw)];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int k0 = 2 * t - q, k1 = 2 * t + 1 - q;       // taps in the low and the high half
                const uint32_t lo = (k0 >= 0 && k0 < K) ? wv[k0 < 0 ? 0 : (k0 < K ? k0 : 0)] : 0u;
                const uint32_t hi = (k1 >= 0 && k1 < K) ? wv[k1 < 0 ? 0 : (k1 < K ? k1 : 0)] : 0u;
                wp[kh][q][t] = lo | (hi << 16);
            }
    }

    const bool has_left = c4 > 0, has_right = c4 < W4 - 1;
    const bf16_t *xin = x + (size_t)plane_in * g.H * g.W + c4 * V;
    bf16_t *yout = y + (size_t)plane * g.H * g.W + c4 * V;
    const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
    const int loff = has_left ? -2 : 0, roff = has_right ? V : V - 2;     // clamped into the lane's own words

    LineWriter<bf16_t, (RS > 0 ? RS : 1)> lw;
    if constexpr (RS > 0) lw.init(lb, W4, V, nstrips, nplanes, TH, g.H, g.W, y);

    uint32_t ring[R][NP];
    auto load_row = [&](int r, uint32_t (&dst)[NP]) {
        const bf16_t *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
        if constexpr (V == 8) {
            const uint4 mid = *reinterpret_cast<const uint4 *>(rp);
            dst[1] = mid.x; dst[2] = mid.y; dst[3] = mid.z; dst[4] = mid.w;
        } else {
            const uint2 mid = *reinterpret_cast<const uint2 *>(rp);
            dst[1] = mid.x; dst[2] = mid.y;
        }
        dst[0] = *reinterpret_cast<const uint32_t *>(rp + loff);
        dst[NP - 1] = *reinterpret_cast<const uint32_t *>(rp + roff);
    };

    float acc[K - 1][V];
#pragma unroll
    for (int j = 0; j < K - 1; ++j)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[j][v] = 0.f;

    // contribution of input row `cur` through filter row kh to the lane's 8 outputs, added to `s`
    auto tap_row = [&](int kh, const uint32_t (&cur)[NP], float (&s)[V]) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int q = (j + P) & 1, i0 = (j - P + 2) >> 1;
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (2 * t - q < K && 2 * t + 1 - q >= 0) s[j] = dot2_bf16(cur[i0 + t], wp[kh][q][t], s[j]);
        }
    };

    auto consume = [&](int idx, int r, const uint32_t (&raw)[NP]) {
        const bool rowok = r >= 0 && r < g.H;
        uint32_t cur[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const bool ok = rowok && (i == 0 ? has_left : (i == NP - 1 ? has_right : true));
            cur[i] = ok ? raw[i] : 0u;
        }
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) out[v] = acc[0][v];
        tap_row(K - 1, cur, out);
#pragma unroll
        for (int jj = 0; jj < K - 1; ++jj) {
            float s[V];
#pragma unroll
            for (int v = 0; v < V; ++v) s[v] = (jj + 1 < K - 1) ? acc[jj + 1][v] : 0.f;
            tap_row(K - 2 - jj, cur, s);
#pragma unroll
            for (int v = 0; v < V; ++v) acc[jj][v] = s[v];
        }
        if (idx >= 2 * P) {        // the row just finished is output row oh0 + idx - 2P
            if constexpr (RS > 0 && V == 8) lw.put(stage, pack16<bf16_t>(out), g.W);
            else {
                const int oh = r - P;
                if (valid && oh < oh1) Vec<bf16_t, V>::store(yout + (size_t)oh * g.W, out);
            }
        }
    };

    const int r0 = oh0 - P, nrows = TH + 2 * P;
#pragma unroll
    for (int j = 0; j < PF; ++j) load_row(r0 + j, ring[j]);
    int i = 0;
#pragma unroll 1
    for (; i + R <= nrows; i += R) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            load_row(r0 + i + j + PF, ring[(j + PF) % R]);
            consume(i + j, r0 + i + j, ring[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < R - 1; ++j)
        if (i + j < nrows) consume(i + j, r0 + i + j, ring[j]);
}

// ---------------------------------------------------------------------------------------------
// Forward, 3x3, stride 2, pad 1, W even.  A lane owns V adjacent output columns and walks down
// the output rows: it needs input columns 2*V*c4 - 1 .. 2*V*c4 + 2V - 1 of rows 2oh-1, 2oh, 2oh+1
// (row 2oh+1 is reused as the top row of output row oh+1).
// RS > 0: whole-line write-out of the output rows in groups of RS; RS == 0: direct stores (streamed if nt).
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int RS>
__global__ __launch_bounds__(256) void k_nchwd_fwd_k3s2(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                        T *__restrict__ y, int TH, int nstrips, unsigned nblocks, int nt)
{
    static_assert(RS == 0 || sizeof(T) * V == 16, "whole-line write-out: one 16-byte output vector per lane and row");
    __shared__ u4v_t stage[2][RS > 0 ? RS * 256 : 1];
    constexpr int NW = 2 * V + 1;
    const int Wo4 = g.Wo / V;
    Lane ln = lane_of(nblocks, Wo4, nstrips, g.N * g.O);
    const bool valid = ln.valid;
    if (!valid) ln.plane = g.N * g.O - 1;     // lanes past the end compute on the last plane; nothing of theirs is stored
    LineWriter<T, (RS > 0 ? RS : 1)> lw;
    if constexpr (RS > 0) lw.init(xcd_remap(blockIdx.x, nblocks), Wo4, V, nstrips, g.N * g.O, TH, g.Ho, g.Wo, y);
    const int n = ln.plane / g.O, o = ln.plane - n * g.O;
    const int plane_in = n * g.C + o / g.m;
    float wr[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wr[kh][kw] = ldf(w + (o * 3 + kh) * 3 + kw);
    const bool has_left = ln.c4 > 0;
    const T *xin = x + (size_t)plane_in * g.H * g.W + ln.c4 * 2 * V;
    T *yout = y + (size_t)ln.plane * g.Ho * g.Wo + ln.c4 * V;
    const int oh0 = ln.strip * TH, oh1 = min(g.Ho, oh0 + TH);
    const int loff = has_left ? -1 : 0;

    // Raw loads (clamped row), masks applied at use: with H = 2*Ho every row 2oh, 2oh+1 of a valid
    // output row is inside the image, so only the left neighbour (first vector of a row) and the
    // row above the image need a select.  Every lane walks TH output rows; lanes past the end of
    // a shorter last strip keep going with their stores masked.
    auto load_row = [&](int r, float (&dst)[NW]) {
        const T *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
        if constexpr (2 * V * sizeof(T) <= 16) {
            // the lane's 2V input columns are one 16-byte vector: consecutive lanes read consecutive vectors
            float ab[2 * V];
            Vec<T, 2 * V>::load(rp, ab);
            dst[0] = ldf(rp + loff);
#pragma unroll
            for (int v = 0; v < 2 * V; ++v) dst[1 + v] = ab[v];
        } else {
            float a[V], b[V];
            Vec<T, V>::load(rp, a);
            Vec<T, V>::load(rp + V, b);
            dst[0] = ldf(rp + loff);
#pragma unroll
            for (int v = 0; v < V; ++v) { dst[1 + v] = a[v]; dst[1 + V + v] = b[v]; }
        }
    };

    float carry[V], re[2][NW], ro[2][NW];
    {
        float top[NW];
        load_row(2 * oh0 - 1, top);
        const bool topok = oh0 > 0;
        const float l = has_left ? top[0] : 0.f;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float t = fmaf(wr[0][0], v == 0 ? l : top[2 * v], fmaf(wr[0][1], top[2 * v + 1], wr[0][2] * top[2 * v + 2]));
            carry[v] = topok ? t : 0.f;
        }
    }
    load_row(2 * oh0, re[0]);
    load_row(2 * oh0 + 1, ro[0]);
    auto step = [&](int oh, int j) {
        const float le = has_left ? re[j][0] : 0.f, lo = has_left ? ro[j][0] : 0.f;
        float out[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
            float s = carry[v];
            s = fmaf(wr[1][0], v == 0 ? le : re[j][2 * v], s); s = fmaf(wr[1][1], re[j][2 * v + 1], s); s = fmaf(wr[1][2], re[j][2 * v + 2], s);
            s = fmaf(wr[2][0], v == 0 ? lo : ro[j][2 * v], s); s = fmaf(wr[2][1], ro[j][2 * v + 1], s); s = fmaf(wr[2][2], ro[j][2 * v + 2], s);
            out[v] = s;
            carry[v] = fmaf(wr[0][0], v == 0 ? lo : ro[j][2 * v], fmaf(wr[0][1], ro[j][2 * v + 1], wr[0][2] * ro[j][2 * v + 2]));
        }
        if constexpr (RS > 0) lw.put(stage, pack16<T>(out), g.Wo);
        else if (valid && oh < oh1) store_vec<T, V>(yout + (size_t)oh * g.Wo, out, nt != 0);
    };
    int i = 0;
#pragma unroll 1
    for (; i + 2 <= TH; i += 2) {
        load_row(2 * (oh0 + i) + 2, re[1]); load_row(2 * (oh0 + i) + 3, ro[1]);
        step(oh0 + i, 0);
        load_row(2 * (oh0 + i) + 4, re[0]); load_row(2 * (oh0 + i) + 5, ro[0]);
        step(oh0 + i + 1, 1);
    }
    if (i < TH) step(oh0 + i, 0);
}

// ---------------------------------------------------------------------------------------------
// Backward-data, 3x3, stride 2, pad 1, multiplier 1, W = 2*Wo, H = 2*Ho.  A lane owns V adjacent
// dy columns b and walks down dy rows a; it writes dx columns 2*V*c4 .. 2*V*c4 + 2V - 1 of rows
// 2a and 2a+1 as one 16-byte vector per row (the pass is write-dominated, so the stores are the
// ones kept contiguous across lanes):
//   dx[2a  ][2b  ] = w11 dy[a][b]
//   dx[2a  ][2b+1] = w10 dy[a][b+1] + w12 dy[a][b]
//   dx[2a+1][2b  ] = w01 dy[a+1][b] + w21 dy[a][b]
//   dx[2a+1][2b+1] = w00 dy[a+1][b+1] + w02 dy[a+1][b] + w20 dy[a][b+1] + w22 dy[a][b]
// RS > 0: whole-line write-out (dx rows 2a and 2a+1 are two rows of a group); RS == 0: direct stores.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int RS>
__global__ __launch_bounds__(256) void k_nchwd_bwd_data_k3s2(Geom g, const T *__restrict__ dy, const T *__restrict__ w,
                                                             T *__restrict__ dx, int TH, int nstrips, unsigned nblocks, int nt)
{
    static_assert(sizeof(T) * 2 * V == 16, "one 16-byte dx vector per lane and row");
    __shared__ u4v_t stage[2][RS > 0 ? RS * 256 : 1];
    const int Wo4 = g.Wo / V;
    Lane ln = lane_of(nblocks, Wo4, nstrips, g.N * g.C);
    const bool valid = ln.valid;
    if (!valid) ln.plane = g.N * g.C - 1;     // lanes past the end compute on the last plane; nothing of theirs is stored
    LineWriter<T, (RS > 0 ? RS : 1)> lw;
    if constexpr (RS > 0) lw.init(xcd_remap(blockIdx.x, nblocks), Wo4, 2 * V, nstrips, g.N * g.C, 2 * TH, g.H, g.W, dx);
    T *dxout = dx + (size_t)ln.plane * g.H * g.W + ln.c4 * 2 * V;
    const int o = ln.plane % g.C;
    float wr[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wr[kh][kw] = ldf(w + (o * 3 + kh) * 3 + kw);
    const bool has_right = ln.c4 < Wo4 - 1;
    const T *dyin = dy + (size_t)ln.plane * g.Ho * g.Wo + ln.c4 * V;
    const int a0 = ln.strip * TH, a1 = min(g.Ho, a0 + TH);
    const int roff = has_right ? V : V - 1;

    // Raw loads (clamped row); the row below the image's last dy row and the column right of a
    // row's last vector are masked at use.  Every lane walks TH dy rows, stores masked past the
    // end of a shorter last strip.
    auto load_row = [&](int a, float (&dst)[V + 1]) {
        const T *rp = dyin + (size_t)min(a, g.Ho - 1) * g.Wo;
        float m[V];
        Vec<T, V>::load(rp, m);
        dst[V] = ldf(rp + roff);
#pragma unroll
        for (int v = 0; v < V; ++v) dst[v] = m[v];
    };

    float rows[3][V + 1];
    load_row(a0, rows[0]);
    load_row(a0 + 1, rows[1]);
    auto emit = [&](int a, const float (&Ar)[V + 1], const float (&Br)[V + 1]) {
        const bool below = a + 1 < g.Ho;
        float A[V + 1], B[V + 1];
#pragma unroll
        for (int v = 0; v < V; ++v) { A[v] = Ar[v]; B[v] = below ? Br[v] : 0.f; }
        A[V] = has_right ? Ar[V] : 0.f;
        B[V] = (has_right && below) ? Br[V] : 0.f;
        float ev[2 * V], od[2 * V];   // dx rows 2a and 2a+1, the lane's 2V columns
#pragma unroll
        for (int v = 0; v < V; ++v) {
            ev[2 * v] = wr[1][1] * A[v];
            ev[2 * v + 1] = fmaf(wr[1][0], A[v + 1], wr[1][2] * A[v]);
            od[2 * v] = fmaf(wr[0][1], B[v], wr[2][1] * A[v]);
            od[2 * v + 1] = fmaf(wr[0][0], B[v + 1], fmaf(wr[0][2], B[v], fmaf(wr[2][0], A[v + 1], wr[2][2] * A[v])));
        }
        if constexpr (RS > 0) {
            lw.put(stage, pack16<T>(ev), g.W);
            lw.put(stage, pack16<T>(od), g.W);
        } else if (valid && a < a1) {
            T *rp = dxout + (size_t)(2 * a) * g.W;
            store_vec<T, 2 * V>(rp, ev, nt != 0);
            store_vec<T, 2 * V>(rp + g.W, od, nt != 0);
        }
    };
    int i = 0;
#pragma unroll 1
    for (; i + 3 <= TH; i += 3) {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            load_row(a0 + i + j + 2, rows[(j + 2) % 3]);
            emit(a0 + i + j, rows[j], rows[(j + 1) % 3]);
        }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if (i + j < TH) {
            load_row(a0 + i + j + 2, rows[(j + 2) % 3]);
            emit(a0 + i + j, rows[j], rows[(j + 1) % 3]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1, 3x3, stride S in {1 ("same" pad), 2 (pad 1, W even)}.
// grid = (parts, O).  A block works on ONE output channel: its 256 lanes are laid flat over
// (item, vector column) with nsg = 256 / (vectors per row) (image, strip) work items per round,
// and the block walks `rounds` rounds, so partial sums stay in registers.  At the
// end all 256 lanes hold sums for the same channel: wavefront butterfly, LDS across the four
// wavefronts, one partial per block at ws[part][o][kh][kw].  Fixed order throughout.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int S>
__global__ __launch_bounds__(256) void k_nchwd_bwd_filter_k3(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                             float *__restrict__ ws, int TH, int nstrips, int nsg,
                                                             int rounds)
{
    __shared__ float red[4][9];
    constexpr int NW = (S == 1) ? V + 2 : 2 * V;       // x columns per lane and row; stride 2: the 2V columns under the lane's dy columns
    constexpr int ND = (S == 1) ? V : V + 1;            // dy columns per lane and row; stride 2: and the one to their right
    const int o = blockIdx.y, part = blockIdx.x;
    const int ncols = g.Wo / V;                         // vectors per dy row
    // lanes are laid flat over (item, vector column): nsg = 256 / ncols items per round, no padding
    const int sg = threadIdx.x / ncols, c4 = threadIdx.x - sg * ncols;
    const int nitems = g.N * nstrips;
    const int c_in = o / g.m;
    const bool has_left = c4 > 0, has_right = c4 < ncols - 1;

    float acc[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) acc[kh][kw] = 0.f;

    if (sg < nsg) {
        for (int rd = 0; rd < rounds; ++rd) {
            const int item = (part * rounds + rd) * nsg + sg;
            if (item >= nitems) break;
            const int n = item / nstrips, strip = item - n * nstrips;
            const int oh0 = strip * TH, oh1 = min(g.Ho, oh0 + TH);
            const T *xin = x + ((size_t)n * g.C + c_in) * g.H * g.W + c4 * V * S;
            const T *dyin = dy + ((size_t)n * g.O + o) * g.Ho * g.Wo + c4 * V;
            const int loff = has_left ? -1 : 0, roff = has_right ? V : V - 1;
            // Raw loads with clamped rows; padding (rows outside the image, neighbours outside the
            // row, dy rows past the strip) is applied when the values are used, so the loads of the
            // next row stay in flight while this one is accumulated.  Every lane walks TH rows.
            auto load_x = [&](int r, float (&dst)[NW]) {
                const T *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
                if constexpr (S == 1) {
                    float m[V];
                    Vec<T, V>::load(rp, m);
                    dst[0] = ldf(rp + loff);
                    dst[V + 1] = ldf(rp + roff);
#pragma unroll
                    for (int v = 0; v < V; ++v) dst[1 + v] = m[v];
                } else {
                    float a[V], b[V];
                    Vec<T, V>::load(rp, a);
                    Vec<T, V>::load(rp + V, b);
#pragma unroll
                    for (int v = 0; v < V; ++v) { dst[v] = a[v]; dst[V + v] = b[v]; }
                }
            };
            auto mask_x = [&](int r, float (&row)[NW]) {
                const bool rowok = r >= 0 && r < g.H;
#pragma unroll
                for (int i = 0; i < NW; ++i) {
                    const bool ok = rowok && (S == 2 ? true : (i == 0 ? has_left : (i == V + 1 ? has_right : true)));
                    row[i] = ok ? row[i] : 0.f;
                }
            };
            auto load_dy = [&](int oh, float (&dst)[ND]) {
                const T *rp = dyin + (size_t)min(oh, g.Ho - 1) * g.Wo;
                float m[V];
                Vec<T, V>::load(rp, m);
#pragma unroll
                for (int v = 0; v < V; ++v) dst[v] = m[v];
                if constexpr (S == 2) dst[V] = ldf(rp + roff);
            };
            // x rows oh*S-1, oh*S, oh*S+1 meet dy row oh at tap rows 0, 1, 2.
            float xa[NW], xb[NW], xc[3][NW], d[3][ND], xs[2][NW];
            load_x(oh0 * S - 1, xa);
            mask_x(oh0 * S - 1, xa);
            if constexpr (S == 1) {
                load_x(oh0, xb);
                mask_x(oh0, xb);
                // two rows ahead: while row oh is accumulated, rows oh+2 and oh+3 are in flight
                load_x(oh0 + 1, xc[0]); load_dy(oh0, d[0]);
                load_x(oh0 + 2, xc[1]); load_dy(oh0 + 1, d[1]);
                auto step = [&](int oh, int j) {
                    mask_x(oh + 1, xc[j]);
                    const bool dok = oh < oh1;
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        const float dv = dok ? d[j][v] : 0.f;
#pragma unroll
                        for (int kw = 0; kw < 3; ++kw) {
                            acc[0][kw] = fmaf(dv, xa[v + kw], acc[0][kw]);
                            acc[1][kw] = fmaf(dv, xb[v + kw], acc[1][kw]);
                            acc[2][kw] = fmaf(dv, xc[j][v + kw], acc[2][kw]);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < NW; ++i) { xa[i] = xb[i]; xb[i] = xc[j][i]; }
                };
                int i = 0;
#pragma unroll 1
                for (; i + 3 <= TH; i += 3) {
#pragma unroll
                    for (int j = 0; j < 3; ++j) {
                        load_x(oh0 + i + j + 3, xc[(j + 2) % 3]); load_dy(oh0 + i + j + 2, d[(j + 2) % 3]);
                        step(oh0 + i + j, j);
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (i + j < TH) step(oh0 + i + j, j);
            } else {
                load_x(2 * oh0, xs[0]); load_x(2 * oh0 + 1, xc[0]); load_dy(oh0, d[0]);
                // summed per x column (the sum over all lanes is the same as per dy column): x column 2b meets dy[oh][b]
                // at tap column 1, x column 2b+1 meets dy[oh][b] at tap column 2 and dy[oh][b+1] at tap column 0, so a lane
                // needs no x neighbour and every x element is loaded by exactly one lane
                auto step = [&](int oh, int j) {
                    // rows 2oh and 2oh+1 are inside the image for every valid oh (H = 2*Ho)
                    const bool dok = oh < oh1;
                    float D[V + 1];
#pragma unroll
                    for (int v = 0; v < V; ++v) D[v] = dok ? d[j][v] : 0.f;
                    D[V] = (dok && has_right) ? d[j][V] : 0.f;
#pragma unroll
                    for (int v = 0; v < V; ++v) {
                        acc[0][1] = fmaf(D[v], xa[2 * v], acc[0][1]);
                        acc[1][1] = fmaf(D[v], xs[j][2 * v], acc[1][1]);
                        acc[2][1] = fmaf(D[v], xc[j][2 * v], acc[2][1]);
                        acc[0][2] = fmaf(D[v], xa[2 * v + 1], acc[0][2]);
                        acc[1][2] = fmaf(D[v], xs[j][2 * v + 1], acc[1][2]);
                        acc[2][2] = fmaf(D[v], xc[j][2 * v + 1], acc[2][2]);
                        acc[0][0] = fmaf(D[v + 1], xa[2 * v + 1], acc[0][0]);
                        acc[1][0] = fmaf(D[v + 1], xs[j][2 * v + 1], acc[1][0]);
                        acc[2][0] = fmaf(D[v + 1], xc[j][2 * v + 1], acc[2][0]);
                    }
#pragma unroll
                    for (int i = 0; i < NW; ++i) xa[i] = xc[j][i];
                };
                int i = 0;
#pragma unroll 1
                for (; i + 2 <= TH; i += 2) {
                    load_x(2 * (oh0 + i) + 2, xs[1]); load_x(2 * (oh0 + i) + 3, xc[1]); load_dy(oh0 + i + 1, d[1]);
                    step(oh0 + i, 0);
                    load_x(2 * (oh0 + i) + 4, xs[0]); load_x(2 * (oh0 + i) + 5, xc[0]); load_dy(oh0 + i + 2, d[0]);
                    step(oh0 + i + 1, 1);
                }
                if (i < TH) step(oh0 + i, 0);
            }
        }
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const float s = wave_sum(acc[kh][kw]);
            if (lane == 0) red[wv][kh * 3 + kw] = s;
        }
    __syncthreads();
    if (threadIdx.x < 9) {
        const int t = threadIdx.x;
        ws[((size_t)part * g.O + o) * 9 + t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1, K x K (K odd), stride 1, "same" padding: same block organisation as the
// 3x3 kernel above (one channel per block, sub-groups take (image, strip) items, one partial per
// block), written input-row-major: x row r meets dy row r + P - kh at tap row kh, so a lane keeps
// the K live dy rows in a shifting window and K*K partial sums.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int K>
__global__ __launch_bounds__(256) void k_nchwd_bwd_filter_s1(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                             float *__restrict__ ws, int TH, int nstrips, int nsg,
                                                             int rounds)
{
    __shared__ float red[4][K * K];
    constexpr int P = (K - 1) / 2;
    constexpr int NW = V + 2 * P;
    const int o = blockIdx.y, part = blockIdx.x;
    const int ncols = g.W / V;
    const int sg = threadIdx.x / ncols, c4 = threadIdx.x - sg * ncols;
    const int nitems = g.N * nstrips;
    const int c_in = o / g.m;
    const bool has_left = c4 > 0, has_right = c4 < ncols - 1;

    float acc[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) acc[kh][kw] = 0.f;

    if (sg < nsg) {
        int loff[P], roff[P];
#pragma unroll
        for (int i = 0; i < P; ++i) { loff[i] = has_left ? -(P - i) : 0; roff[i] = has_right ? V + i : V - 1; }
        for (int rd = 0; rd < rounds; ++rd) {
            const int item = (part * rounds + rd) * nsg + sg;
            if (item >= nitems) break;
            const int n = item / nstrips, strip = item - n * nstrips;
            const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
            const T *xin = x + ((size_t)n * g.C + c_in) * g.H * g.W + c4 * V;
            const T *dyin = dy + ((size_t)n * g.O + o) * g.H * g.W + c4 * V;
            auto load_row = [&](int r, float (&xd)[NW], float (&dd)[V]) {
                const T *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
                float m[V];
                Vec<T, V>::load(rp, m);
#pragma unroll
                for (int i = 0; i < P; ++i) { xd[i] = ldf(rp + loff[i]); xd[P + V + i] = ldf(rp + roff[i]); }
#pragma unroll
                for (int v = 0; v < V; ++v) xd[P + v] = m[v];
                Vec<T, V>::load(dyin + (size_t)min(max(r + P, 0), g.H - 1) * g.W, dd);
            };
            float dyw[K][V];
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int v = 0; v < V; ++v) dyw[kh][v] = 0.f;
            float xr[2][NW], dr[2][V];
            auto step = [&](int r, int j) {
                const bool rowok = r >= 0 && r < g.H;
                const bool dok = r + P >= oh0 && r + P < oh1;
                float xv[NW];
#pragma unroll
                for (int i = 0; i < NW; ++i) {
                    const bool ok = rowok && (i < P ? has_left : (i >= P + V ? has_right : true));
                    xv[i] = ok ? xr[j][i] : 0.f;
                }
#pragma unroll
                for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                    for (int v = 0; v < V; ++v) dyw[kh][v] = dyw[kh - 1][v];
#pragma unroll
                for (int v = 0; v < V; ++v) dyw[0][v] = dok ? dr[j][v] : 0.f;
#pragma unroll
                for (int kh = 0; kh < K; ++kh)
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        float sacc = acc[kh][kw];
#pragma unroll
                        for (int v = 0; v < V; ++v) sacc = fmaf(dyw[kh][v], xv[v + kw], sacc);
                        acc[kh][kw] = sacc;
                    }
            };
            const int r0 = oh0 - P, nrows = TH + 2 * P;
            load_row(r0, xr[0], dr[0]);
            int i = 0;
#pragma unroll 1
            for (; i + 2 <= nrows; i += 2) {
                load_row(r0 + i + 1, xr[1], dr[1]);
                step(r0 + i, 0);
                load_row(r0 + i + 2, xr[0], dr[0]);
                step(r0 + i + 1, 1);
            }
            if (i < nrows) step(r0 + i, 0);
        }
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const float s = wave_sum(acc[kh][kw]);
            if (lane == 0) red[wv][kh * K + kw] = s;
        }
    __syncthreads();
    if (threadIdx.x < K * K) {
        const int t = threadIdx.x;
        ws[((size_t)part * g.O + o) * (K * K) + t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1 for bf16, stride 1, on packed pairs (see k_nchwd_s1_bf16x8): the dy row
// and the x row both stay packed, and one v_dot2c_f32_bf16 adds dy[2m] x[2m+e] + dy[2m+1] x[2m+1+e]
// to the tap's fp32 sum.  For an even column offset e = kw - P the x pair is a word as loaded; for
// an odd one it straddles two words and is built once per x row with a funnel shift (V/2 + 1 of
// them serve every odd offset).  Same block structure and reduction as k_nchwd_bwd_filter_s1.
// ---------------------------------------------------------------------------------------------
template <int V, int K>
__global__ __launch_bounds__(256) void k_nchwd_bwd_filter_s1_bf16(Geom g, const bf16_t *__restrict__ x,
                                                                  const bf16_t *__restrict__ dy, float *__restrict__ ws,
                                                                  int TH, int nstrips, int nsg, int rounds)
{
    static_assert((V == 8 || V == 4) && (K == 3 || K == 5), "packed pairs with one neighbour word on each side");
    __shared__ float red[4][K * K];
    constexpr int P = (K - 1) / 2;
    constexpr int NP = V / 2 + 2;       // x words per row and lane: columns -2 .. V+1
    constexpr int ND = V / 2;           // dy words per row and lane
    const int o = blockIdx.y, part = blockIdx.x;
    const int ncols = g.W / V;
    const int sg = threadIdx.x / ncols, c4 = threadIdx.x - sg * ncols;
    const int nitems = g.N * nstrips;
    const int c_in = o / g.m;
    const bool has_left = c4 > 0, has_right = c4 < ncols - 1;

    float acc[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) acc[kh][kw] = 0.f;

    if (sg < nsg) {
        const int loff = has_left ? -2 : 0, roff = has_right ? V : V - 2;
        for (int rd = 0; rd < rounds; ++rd) {
            const int item = (part * rounds + rd) * nsg + sg;
            if (item >= nitems) break;
            const int n = item / nstrips, strip = item - n * nstrips;
            const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
            const bf16_t *xin = x + ((size_t)n * g.C + c_in) * g.H * g.W + c4 * V;
            const bf16_t *dyin = dy + ((size_t)n * g.O + o) * g.H * g.W + c4 * V;
            auto load_words = [&](const bf16_t *p, uint32_t *dst) {
                if constexpr (V == 8) { const uint4 q = *reinterpret_cast<const uint4 *>(p); dst[0] = q.x; dst[1] = q.y; dst[2] = q.z; dst[3] = q.w; }
                else { const uint2 q = *reinterpret_cast<const uint2 *>(p); dst[0] = q.x; dst[1] = q.y; }
            };
            auto load_row = [&](int r, uint32_t (&xd)[NP], uint32_t (&dd)[ND]) {
                const bf16_t *rp = xin + (size_t)min(max(r, 0), g.H - 1) * g.W;
                load_words(rp, &xd[1]);
                xd[0] = *reinterpret_cast<const uint32_t *>(rp + loff);
                xd[NP - 1] = *reinterpret_cast<const uint32_t *>(rp + roff);
                load_words(dyin + (size_t)min(max(r + P, 0), g.H - 1) * g.W, &dd[0]);
            };
            uint32_t dyw[K][ND];
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int m = 0; m < ND; ++m) dyw[kh][m] = 0u;
            uint32_t xr[2][NP], dr[2][ND];
            auto step = [&](int r, int j) {
                const bool rowok = r >= 0 && r < g.H;
                const bool dok = r + P >= oh0 && r + P < oh1;
                uint32_t xe[NP], xo[NP - 1];       // aligned words; words shifted by one column: xo[i] = columns (2i-1, 2i)
#pragma unroll
                for (int i = 0; i < NP; ++i) {
                    const bool ok = rowok && (i == 0 ? has_left : (i == NP - 1 ? has_right : true));
                    xe[i] = ok ? xr[j][i] : 0u;
                }
#pragma unroll
                for (int i = 0; i < NP - 1; ++i) xo[i] = __builtin_amdgcn_alignbit(xe[i + 1], xe[i], 16);
#pragma unroll
                for (int kh = K - 1; kh > 0; --kh)
#pragma unroll
                    for (int m = 0; m < ND; ++m) dyw[kh][m] = dyw[kh - 1][m];
#pragma unroll
                for (int m = 0; m < ND; ++m) dyw[0][m] = dok ? dr[j][m] : 0u;
#pragma unroll
                for (int kh = 0; kh < K; ++kh)
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        const int e = kw - P;            // x column = dy column + e
                        float sacc = acc[kh][kw];
#pragma unroll
                        for (int m = 0; m < ND; ++m) {
                            // dy columns (2m, 2m+1) meet x columns (2m+e, 2m+1+e)
                            const uint32_t xw = (e & 1) ? xo[m + (e + 1) / 2] : xe[m + 1 + e / 2];
                            sacc = dot2_bf16(dyw[kh][m], xw, sacc);
                        }
                        acc[kh][kw] = sacc;
                    }
            };
            const int r0 = oh0 - P, nrows = TH + 2 * P;
            load_row(r0, xr[0], dr[0]);
            int i = 0;
#pragma unroll 1
            for (; i + 2 <= nrows; i += 2) {
                load_row(r0 + i + 1, xr[1], dr[1]);
                step(r0 + i, 0);
                load_row(r0 + i + 2, xr[0], dr[0]);
                step(r0 + i + 1, 1);
            }
            if (i < nrows) step(r0 + i, 0);
        }
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const float s = wave_sum(acc[kh][kw]);
            if (lane == 0) red[wv][kh * K + kw] = s;
        }
    __syncthreads();
    if (threadIdx.x < K * K) {
        const int t = threadIdx.x;
        ws[((size_t)part * g.O + o) * (K * K) + t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    }
}

// ---------------------------------------------------------------------------------------------
// Fused backward pass, NCHW, 3x3, stride 1, pad 1, multiplier 1: the input gradient dx and the
// stage-1 partial sums of the filter gradient from one walk over dy and x (dy is read once).
// Block structure of the filter-gradient kernel above: grid = (parts, C), a block works on one
// channel, lanes flat over (item, vector column) with nsg (image, strip) items per round.  Step t
// of the walk takes dy row t with its left and right neighbour column, and x row t+1 (own columns):
//   input gradient:  dx[r][c] = sum_{kh,kw} w[kh][kw] dy[r+1-kh][c+1-kw]; dy row t is tap row 0, 1, 2
//     of dx rows t-1, t, t+1 (two rotating accumulators; the filter is uniform over the block);
//   filter gradient, summed per x column instead of per dy column: x column c meets dy[t][c+1-kw] at
//     tap column kw and x rows t-1, t, t+1 (a three-row window of the lane's own columns) at tap rows
//     0, 1, 2.  The dy neighbours are there for the input gradient anyway, so x needs none: four load
//     instructions per step instead of six.  Only dy rows inside the item's own strip count (the products
//     are masked), while the input gradient needs the true halo rows.
// dx leaves through the whole-line write-out (RS rows per group; needs TH % RS == 0, H % RS == 0),
// so every lane of the block walks every round in lockstep: lanes without an item (the last few
// lanes of the block, a partly filled last round) run on clamped addresses with everything masked.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int RS>
__global__ __launch_bounds__(256) void k_nchwd_bwd_fused_k3s1(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                              const T *__restrict__ w, T *__restrict__ dx,
                                                              float *__restrict__ ws, int TH, int nstrips, int nsg,
                                                              int rounds)
{
    static_assert(sizeof(T) * V == 16, "whole-line write-out: one 16-byte vector per lane and row");
    __shared__ float red[4][9];
    __shared__ u4v_t stage[2][RS * 256];
    constexpr int NW = V + 2;
    const int o = blockIdx.y, part = blockIdx.x;
    const int ncols = g.W / V;
    const int sg = threadIdx.x / ncols, c4 = threadIdx.x - sg * ncols;
    const int nitems = g.N * nstrips;
    const bool has_left = c4 > 0, has_right = c4 < ncols - 1;
    const int loff = has_left ? -1 : 0, roff = has_right ? V : V - 1;
    const size_t plane = (size_t)g.H * g.W;

    float wr[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wr[kh][kw] = ldf(w + (o * 3 + kh) * 3 + kw);

    float acc[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) acc[kh][kw] = 0.f;

    LineWriter<T, RS> lw;
    lw.slot = 0; lw.buf = 0; lw.done = 0;

    for (int rd = 0; rd < rounds; ++rd) {
        const int item0 = (part * rounds + rd) * nsg;
        const int item = item0 + sg;
        const bool live = sg < nsg && item < nitems;
        const int itc = min(item, nitems - 1);                 // clamped: loads stay in bounds
        const int n = itc / nstrips, strip = itc - n * nstrips;
        const int oh0 = strip * TH, oh1 = min(g.H, oh0 + TH);
        const T *xin = x + ((size_t)n * g.C + o) * plane + c4 * V;
        const T *dyin = dy + ((size_t)n * g.C + o) * plane + c4 * V;
        // write-out entries of this round: entry e = tid + 256 k belongs to the item slot of lane e / RS;
        // inside an item entries run over (row, vector column)
#pragma unroll
        for (int k = 0; k < RS; ++k) {
            const int e = threadIdx.x + 256 * k;
            const int l = e / RS;
            const int sgl = l / ncols, a = sgl * ncols;
            const int rel = e - RS * a;
            const int srow = rel / ncols, c4l = rel - srow * ncols;
            const int iteml = item0 + sgl;
            const bool ok = sgl < nsg && iteml < nitems;
            const int itl = min(iteml, nitems - 1);
            const int nl = itl / nstrips, stl = itl - nl * nstrips;
            const int o0 = stl * TH, o1 = min(g.H, o0 + TH);
            lw.idx[k] = min(srow, RS - 1) * 256 + min(a + c4l, 255);
            lw.rows[k] = ok ? o1 - (o0 + srow) : 0;
            lw.ptr[k] = dx + (((size_t)nl * g.C + o) * g.H + min(o0 + srow, g.H - 1)) * g.W + c4l * V;
        }
        lw.done = 0;

        auto load_row = [&](int t, float (&dd)[NW], float (&xd)[V]) {
            const T *dp = dyin + (size_t)min(max(t, 0), g.H - 1) * g.W;
            const T *xp = xin + (size_t)min(max(t + 1, 0), g.H - 1) * g.W;
            float m[V];
            Vec<T, V>::load(dp, m);
            dd[0] = ldf(dp + loff); dd[V + 1] = ldf(dp + roff);
#pragma unroll
            for (int v = 0; v < V; ++v) dd[1 + v] = m[v];
            Vec<T, V>::load(xp, xd);
        };

        // xw[kh] = x row t-1+kh at the lane's columns (zero outside the image); x row t0 enters ahead of the first step
        float A0[V], A1[V], xw[3][V];
        const int t0 = oh0 - 1;
        {
            float f[V];
            Vec<T, V>::load(xin + (size_t)max(t0, 0) * g.W, f);
#pragma unroll
            for (int v = 0; v < V; ++v) { A0[v] = 0.f; A1[v] = 0.f; xw[0][v] = 0.f; xw[1][v] = 0.f; xw[2][v] = t0 >= 0 ? f[v] : 0.f; }
        }

        float dr[2][NW], xr[2][V];
        auto consume = [&](int step, int t, const float (&dd)[NW], const float (&xd)[V]) {
            const bool dyok = t >= 0 && t < g.H;
            const bool mine = live && t >= oh0 && t < oh1;
            const bool xok = t + 1 < g.H;
            float d[NW];
#pragma unroll
            for (int i = 0; i < NW; ++i) {
                const bool colok = i == 0 ? has_left : (i == V + 1 ? has_right : true);
                d[i] = (dyok && colok) ? dd[i] : 0.f;
            }
            // input gradient: dx column c (window index c + 1) reads dy columns c+1-kw = window index c + 2 - kw
            float out[V];
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float s0 = A0[v], s1 = A1[v], s2 = 0.f;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    s0 = fmaf(wr[0][kw], d[v + 2 - kw], s0);
                    s1 = fmaf(wr[1][kw], d[v + 2 - kw], s1);
                    s2 = fmaf(wr[2][kw], d[v + 2 - kw], s2);
                }
                out[v] = s0; A0[v] = s1; A1[v] = s2;
            }
            // dx row t-1 = oh0 + step - 2 leaves at steps 2 .. TH+1, the same for every lane (rows past the
            // strip's end are masked in the write-out)
            if (step >= 2 && step < TH + 2) lw.put(stage, pack16<T>(out), g.W);
            // filter gradient: x column c (index v) against dy column c+1-kw (window index v + 2 - kw)
#pragma unroll
            for (int v = 0; v < V; ++v) { xw[0][v] = xw[1][v]; xw[1][v] = xw[2][v]; xw[2][v] = xok ? xd[v] : 0.f; }
            float dm[NW];
#pragma unroll
            for (int i = 0; i < NW; ++i) dm[i] = mine ? d[i] : 0.f;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    float sacc = acc[kh][kw];
#pragma unroll
                    for (int v = 0; v < V; ++v) sacc = fmaf(dm[v + 2 - kw], xw[kh][v], sacc);
                    acc[kh][kw] = sacc;
                }
        };

        // steps t = oh0-1 .. oh0+TH for every lane (the same count, whatever the strip's real height)
        const int nsteps = TH + 2;
        load_row(t0, dr[0], xr[0]);
        int i = 0;
#pragma unroll 1
        for (; i + 2 <= nsteps; i += 2) {
            load_row(t0 + i + 1, dr[1], xr[1]);
            consume(i, t0 + i, dr[0], xr[0]);
            load_row(t0 + i + 2, dr[0], xr[0]);
            consume(i + 1, t0 + i + 1, dr[1], xr[1]);
        }
        if (i < nsteps) consume(i, t0 + i, dr[0], xr[0]);
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const float s = wave_sum(acc[kh][kw]);
            if (lane == 0) red[wv][kh * 3 + kw] = s;
        }
    __syncthreads();
    if (threadIdx.x < 9) {
        const int t = threadIdx.x;
        ws[((size_t)part * g.C + o) * 9 + t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    }
}

// ---------------------------------------------------------------------------------------------
// Fused backward pass, NCHW, 3x3, stride 2, pad 1, multiplier 1, W = 2*Wo, H = 2*Ho.  Block structure of
// the stride-1 fused kernel above (grid = (parts, C), lanes flat over (item, vector column), rounds of nsg
// (image, strip) items).  A lane owns V adjacent dy columns b and the 2V x / dx columns 2b, 2b+1 under them,
// and walks the TH dy rows a of its strip; step a holds dy rows a and a+1 (the lane's columns and the one to
// their right) and x rows 2a-1, 2a, 2a+1 (the lane's own 2V columns, one 16-byte vector per row):
//   input gradient: dx rows 2a and 2a+1 as in k_nchwd_bwd_data_k3s2, through the whole-line write-out;
//   filter gradient, summed per x column: x column 2b meets dy[a][b] at tap column 1, x column 2b+1 meets
//     dy[a][b] at tap column 2 and dy[a][b+1] at tap column 0; x rows 2a-1, 2a, 2a+1 are tap rows 0, 1, 2,
//     and row 2a+1 stays as the top row of step a+1.  Every x element is loaded by exactly one lane.
// dy is read once: the pass moves 2|x| + |y| elements.  Every lane walks TH steps in lockstep (whole-line
// write-out); lanes without an item and steps past a shorter last strip run on clamped rows, masked.
// Needs (2 TH) % RS == 0 and H % RS == 0.
// ---------------------------------------------------------------------------------------------
template <typename T, int V, int RS>
__global__ __launch_bounds__(256) void k_nchwd_bwd_fused_k3s2(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                              const T *__restrict__ w, T *__restrict__ dx,
                                                              float *__restrict__ ws, int TH, int nstrips, int nsg,
                                                              int rounds)
{
    static_assert(sizeof(T) * 2 * V == 16, "one 16-byte x / dx vector per lane and row");
    __shared__ float red[4][9];
    __shared__ u4v_t stage[2][RS * 256];
    constexpr int XV = 2 * V;
    const int o = blockIdx.y, part = blockIdx.x;
    const int ncols = g.Wo / V;
    const int sg = threadIdx.x / ncols, c4 = threadIdx.x - sg * ncols;
    const int nitems = g.N * nstrips;
    const bool has_right = c4 < ncols - 1;
    const int roff = has_right ? V : V - 1;
    const size_t xplane = (size_t)g.H * g.W, dyplane = (size_t)g.Ho * g.Wo;

    float wr[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wr[kh][kw] = ldf(w + (o * 3 + kh) * 3 + kw);

    float acc[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) acc[kh][kw] = 0.f;

    LineWriter<T, RS> lw;
    lw.slot = 0; lw.buf = 0; lw.done = 0;

    for (int rd = 0; rd < rounds; ++rd) {
        const int item0 = (part * rounds + rd) * nsg;
        const int item = item0 + sg;
        const bool live = sg < nsg && item < nitems;
        const int itc = min(item, nitems - 1);                 // clamped: loads stay in bounds
        const int n = itc / nstrips, strip = itc - n * nstrips;
        const int a0 = strip * TH, a1 = min(g.Ho, a0 + TH);
        const T *xin = x + ((size_t)n * g.C + o) * xplane + c4 * XV;
        const T *dyin = dy + ((size_t)n * g.C + o) * dyplane + c4 * V;
        // write-out entries of this round (dx rows of 2 TH per item, W / XV vectors per row = ncols)
#pragma unroll
        for (int k = 0; k < RS; ++k) {
            const int e = threadIdx.x + 256 * k;
            const int l = e / RS;
            const int sgl = l / ncols, a = sgl * ncols;
            const int rel = e - RS * a;
            const int srow = rel / ncols, c4l = rel - srow * ncols;
            const int iteml = item0 + sgl;
            const bool ok = sgl < nsg && iteml < nitems;
            const int itl = min(iteml, nitems - 1);
            const int nl = itl / nstrips, stl = itl - nl * nstrips;
            const int o0 = stl * 2 * TH, o1 = min(g.H, o0 + 2 * TH);
            lw.idx[k] = min(srow, RS - 1) * 256 + min(a + c4l, 255);
            lw.rows[k] = ok ? o1 - (o0 + srow) : 0;
            lw.ptr[k] = dx + (((size_t)nl * g.C + o) * g.H + min(o0 + srow, g.H - 1)) * g.W + c4l * XV;
        }
        lw.done = 0;

        auto load_dy = [&](int a, float (&dst)[V + 1]) {
            const T *rp = dyin + (size_t)min(a, g.Ho - 1) * g.Wo;
            float m[V];
            Vec<T, V>::load(rp, m);
            dst[V] = ldf(rp + roff);
#pragma unroll
            for (int v = 0; v < V; ++v) dst[v] = m[v];
        };
        auto load_x = [&](int r, float (&dst)[XV]) { Vec<T, XV>::load(xin + (size_t)min(max(r, 0), g.H - 1) * g.W, dst); };

        // xa = x row 2a-1 (zero above the image), kept from the previous step's row 2a+1; dA, dB = dy rows a, a+1
        float xa[XV], xe[2][XV], xo[2][XV], dA[V + 1], dB[V + 1], dC[V + 1];
        load_x(2 * a0 - 1, xa);
#pragma unroll
        for (int i = 0; i < XV; ++i) xa[i] = a0 > 0 ? xa[i] : 0.f;
        load_dy(a0, dA); load_dy(a0 + 1, dB);
        load_x(2 * a0, xe[0]); load_x(2 * a0 + 1, xo[0]);

        auto step = [&](int a, const float (&Ar)[V + 1], const float (&Br)[V + 1], const float (&X1)[XV], const float (&X2)[XV]) {
            const bool below = a + 1 < g.Ho;
            const bool mine = live && a < a1;
            float A[V + 1], B[V + 1];
#pragma unroll
            for (int v = 0; v < V; ++v) { A[v] = Ar[v]; B[v] = below ? Br[v] : 0.f; }
            A[V] = has_right ? Ar[V] : 0.f;
            B[V] = (has_right && below) ? Br[V] : 0.f;
            float ev[XV], od[XV];   // dx rows 2a and 2a+1, the lane's 2V columns
#pragma unroll
            for (int v = 0; v < V; ++v) {
                ev[2 * v] = wr[1][1] * A[v];
                ev[2 * v + 1] = fmaf(wr[1][0], A[v + 1], wr[1][2] * A[v]);
                od[2 * v] = fmaf(wr[0][1], B[v], wr[2][1] * A[v]);
                od[2 * v + 1] = fmaf(wr[0][0], B[v + 1], fmaf(wr[0][2], B[v], fmaf(wr[2][0], A[v + 1], wr[2][2] * A[v])));
            }
            lw.put(stage, pack16<T>(ev), g.W);
            lw.put(stage, pack16<T>(od), g.W);
            // filter gradient (only dy rows of the lane's own strip and item)
            float D[V + 1];
#pragma unroll
            for (int v = 0; v <= V; ++v) D[v] = mine ? A[v] : 0.f;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                acc[0][1] = fmaf(D[v], xa[2 * v], acc[0][1]);
                acc[1][1] = fmaf(D[v], X1[2 * v], acc[1][1]);
                acc[2][1] = fmaf(D[v], X2[2 * v], acc[2][1]);
                acc[0][2] = fmaf(D[v], xa[2 * v + 1], acc[0][2]);
                acc[1][2] = fmaf(D[v], X1[2 * v + 1], acc[1][2]);
                acc[2][2] = fmaf(D[v], X2[2 * v + 1], acc[2][2]);
                acc[0][0] = fmaf(D[v + 1], xa[2 * v + 1], acc[0][0]);
                acc[1][0] = fmaf(D[v + 1], X1[2 * v + 1], acc[1][0]);
                acc[2][0] = fmaf(D[v + 1], X2[2 * v + 1], acc[2][0]);
            }
#pragma unroll
            for (int i = 0; i < XV; ++i) xa[i] = X2[i];
        };

        // every lane walks TH steps; the rows of the next step are loaded while this one is computed
        auto advance = [&](int a, int j) {
            load_dy(a + 2, dC);
            load_x(2 * a + 2, xe[j ^ 1]); load_x(2 * a + 3, xo[j ^ 1]);
            step(a, dA, dB, xe[j], xo[j]);
#pragma unroll
            for (int v = 0; v <= V; ++v) { dA[v] = dB[v]; dB[v] = dC[v]; }
        };
        int i = 0;
#pragma unroll 1
        for (; i + 2 <= TH; i += 2) {
            advance(a0 + i, 0);
            advance(a0 + i + 1, 1);
        }
        if (i < TH) advance(a0 + i, 0);
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const float s = wave_sum(acc[kh][kw]);
            if (lane == 0) red[wv][kh * 3 + kw] = s;
        }
    __syncthreads();
    if (threadIdx.x < 9) {
        const int t = threadIdx.x;
        ws[((size_t)part * g.C + o) * 9 + t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
    }
}

// ---- host side --------------------------------------------------------------------------------

// vector width for the direct kernels (0 = not applicable): rows must be whole 16-byte vectors;
// bf16 rows that are only a multiple of 4 use 8-byte vectors.
int nchwd_vec(const Geom &g, int dtype, int pass)
{
    const bool s1 = g.s == 1 && (g.K == 3 || g.K == 5) && g.p == (g.K - 1) / 2;
    const bool s2 = g.s == 2 && g.K == 3 && g.p == 1 && g.W % 2 == 0 && g.H % 2 == 0;
    if (!s1 && !s2) return 0;
    if (pass == 1 && g.m != 1) return 0;
    if (pass == 2 && g.K != 3 && !(g.K == 5 && s1)) return 0;
    if (pass == 2 && g.O > 65535) return 0;      // the filter-gradient launches put the channel on gridDim.y
    if (g.H < 16) return 0;                      // small planes go to the LDS-tile kernels
    const int wv = s1 ? g.W : g.Wo;              // the dimension that lanes split into vectors
    if (s2 && pass == 1) {                       // dy columns per lane; dx is stored 2V wide
        if (dtype == DT_F32) return wv % 2 == 0 ? 2 : 0;
        return wv % 4 == 0 ? 4 : 0;
    }
    if (s2 && pass == 0) {
        // forward: 16-byte output vectors when the whole-line write-out applies; otherwise the lane's
        // 2V input columns are one 16-byte vector
        const int esz = dtype == DT_F32 ? 4 : 2, rs = row_group(g.Wo, esz);
        if (rs && g.Ho % rs == 0 && wv % (16 / esz) == 0) return 16 / esz;
        if (dtype == DT_F32) return wv % 2 == 0 ? 2 : 0;
        return wv % 4 == 0 ? 4 : 0;
    }
    if (dtype == DT_F32) return wv % 4 == 0 ? 4 : (s2 && wv % 2 == 0 ? 2 : 0);
    return wv % 8 == 0 ? 8 : (wv % 4 == 0 ? 4 : 0);
}

template <typename T, int V, int K>
static hipError_t go_s1(const Geom &g, const void *x, const void *w, void *y, bool flip, int TH, hipStream_t st)
{
    const long long out_bytes = (long long)g.N * g.O * g.H * g.W * sizeof(T);
    if constexpr (sizeof(T) * V == 16) {
        // whole-line write-out, streamed: rows grouped so that a group is a whole number of lines
        const int rs = row_group(g.W, (int)sizeof(T));
        if (rs >= 2 && g.H % rs == 0 && stream_stores(flip ? "NCHW_S1_BWD" : "NCHW_S1_FWD", out_bytes, 0)) {
            TH = (TH + rs - 1) / rs * rs;
            const int nstrips = ceil_div_h(g.H, TH);
            const long long lanes = (long long)g.N * g.O * nstrips * (g.W / V);
            const unsigned nblocks = (unsigned)((lanes + 255) / 256);
#define GOL(FL, RSV) hipLaunchKernelGGL((k_nchwd_s1<T, V, K, 2, FL, RSV>), dim3(nblocks), dim3(256), 0, st, g, \
                                        (const T *)x, (const T *)w, (T *)y, TH, nstrips, nblocks, 1)
#define GOB(FL, RSV) hipLaunchKernelGGL((k_nchwd_s1_bf16x8<V, K, 2, FL, RSV>), dim3(nblocks), dim3(256), 0, st, g, \
                                        (const bf16_t *)x, (const bf16_t *)w, (bf16_t *)y, TH, nstrips, nblocks)
            if constexpr (sizeof(T) == 2 && V == 8) {      // bf16: packed-pair arithmetic
                if (!tune_env("DWCONV_TUNE_NODOT")) {
                    if (rs == 2) { if (flip) GOB(true, 2); else GOB(false, 2); }
                    else { if (flip) GOB(true, 4); else GOB(false, 4); }
                    return hipGetLastError();
                }
            }
            if (rs == 2) { if (flip) GOL(true, 2); else GOL(false, 2); }
            else { if (flip) GOL(true, 4); else GOL(false, 4); }
#undef GOL
            return hipGetLastError();
        }
    }
    const int nstrips = ceil_div_h(g.H, TH);
    const long long lanes = (long long)g.N * g.O * nstrips * (g.W / V);
    const unsigned nblocks = (unsigned)((lanes + 255) / 256);
    // rows that are whole lines by themselves can be streamed as they are; otherwise a wave's store
    // covers pieces of several rows (partial lines) and stays cached
    if constexpr (sizeof(T) == 2) {
        if (!tune_env("DWCONV_TUNE_NODOT")) {
            if (flip) GOB(true, 0); else GOB(false, 0);
            return hipGetLastError();
        }
    }
#undef GOB
    const int whole = (g.W * (int)sizeof(T)) % 128 == 0;
    const int nt = whole ? stream_stores(flip ? "NCHW_S1_BWD" : "NCHW_S1_FWD", out_bytes, 0) : 0;
    if (flip)
        hipLaunchKernelGGL((k_nchwd_s1<T, V, K, 2, true, 0>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, (const T *)w,
                           (T *)y, TH, nstrips, nblocks, nt);
    else
        hipLaunchKernelGGL((k_nchwd_s1<T, V, K, 2, false, 0>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, (const T *)w,
                           (T *)y, TH, nstrips, nblocks, nt);
    return hipGetLastError();
}

hipError_t nchwd_s1(const Geom &g, int dtype, int V, const void *x, const void *w, void *y, bool flip, int TH,
                    hipStream_t st)
{
    if (dtype == DT_F32 && V == 4) return g.K == 3 ? go_s1<float, 4, 3>(g, x, w, y, flip, TH, st) : go_s1<float, 4, 5>(g, x, w, y, flip, TH, st);
    if (dtype == DT_BF16 && V == 8) return g.K == 3 ? go_s1<bf16_t, 8, 3>(g, x, w, y, flip, TH, st) : go_s1<bf16_t, 8, 5>(g, x, w, y, flip, TH, st);
    if (dtype == DT_BF16 && V == 4) return g.K == 3 ? go_s1<bf16_t, 4, 3>(g, x, w, y, flip, TH, st) : go_s1<bf16_t, 4, 5>(g, x, w, y, flip, TH, st);
    return hipErrorInvalidValue;
}

hipError_t nchwd_k3s2(const Geom &g, int dtype, int V, const void *in, const void *w, void *out, bool bwd, int TH,
                      hipStream_t st)
{
    const int nstrips = ceil_div_h(g.Ho, TH);
    const long long lanes = (long long)g.N * g.O * nstrips * (g.Wo / V);
    const unsigned nblocks = (unsigned)((lanes + 255) / 256);
    const int nt = bwd ? stream_stores("NCHW_S2_BWD", (long long)g.N * g.C * g.H * g.W * (dtype == DT_F32 ? 4 : 2), -1)
                       : stream_stores("NCHW_S2_FWD", (long long)g.N * g.O * g.Ho * g.Wo * (dtype == DT_F32 ? 4 : 2));
#define GO(KERNEL, T, VV) hipLaunchKernelGGL((KERNEL<T, VV, 0>), dim3(nblocks), dim3(256), 0, st, g, (const T *)in, \
                                             (const T *)w, (T *)out, TH, nstrips, nblocks, nt)
    if (!bwd) {
        const int esz = dtype == DT_F32 ? 4 : 2;
        const int rs = row_group(g.Wo, esz);
        if (rs && g.Ho % rs == 0 && V * esz == 16 &&
            stream_stores("NCHW_S2_FWD", (long long)g.N * g.O * g.Ho * g.Wo * esz, 0)) {
            const int TH2 = (TH + rs - 1) / rs * rs;
            const int nst = ceil_div_h(g.Ho, TH2);
            const unsigned nb = (unsigned)(((long long)g.N * g.O * nst * (g.Wo / V) + 255) / 256);
#define GOL(T, VV, RSV) hipLaunchKernelGGL((k_nchwd_fwd_k3s2<T, VV, RSV>), dim3(nb), dim3(256), 0, st, g, \
                                           (const T *)in, (const T *)w, (T *)out, TH2, nst, nb, 1)
            if (dtype == DT_F32) { if (rs == 2) GOL(float, 4, 2); else GOL(float, 4, 4); }
            else { if (rs == 2) GOL(bf16_t, 8, 2); else GOL(bf16_t, 8, 4); }
#undef GOL
            return hipGetLastError();
        }
        if (dtype == DT_F32 && V == 4) GO(k_nchwd_fwd_k3s2, float, 4);
        else if (dtype == DT_F32 && V == 2) GO(k_nchwd_fwd_k3s2, float, 2);
        else if (dtype == DT_BF16 && V == 8) GO(k_nchwd_fwd_k3s2, bf16_t, 8);
        else if (dtype == DT_BF16 && V == 4) GO(k_nchwd_fwd_k3s2, bf16_t, 4);
        else return hipErrorInvalidValue;
    } else {
        // V = dy columns per lane; the lane stores 2V dx columns as one 16-byte vector per row
        const int esz = dtype == DT_F32 ? 4 : 2;
        const int rs = row_group(g.W, esz);
        if (rs && g.H % rs == 0 &&
            stream_stores("NCHW_S2_BWD", (long long)g.N * g.C * g.H * g.W * esz, 0)) {
            // whole-line write-out, streamed; 2*TH dx rows per strip must be whole row groups
            const int TH2 = rs == 4 ? (TH + 1) / 2 * 2 : TH;
            const int nst = ceil_div_h(g.Ho, TH2);
            const unsigned nb = (unsigned)(((long long)g.N * g.O * nst * (g.Wo / V) + 255) / 256);
#define GOL(T, VV, RSV) hipLaunchKernelGGL((k_nchwd_bwd_data_k3s2<T, VV, RSV>), dim3(nb), dim3(256), 0, st, g, \
                                           (const T *)in, (const T *)w, (T *)out, TH2, nst, nb, 1)
            if (dtype == DT_F32 && V == 2) { if (rs == 2) GOL(float, 2, 2); else GOL(float, 2, 4); }
            else if (dtype == DT_BF16 && V == 4) { if (rs == 2) GOL(bf16_t, 4, 2); else GOL(bf16_t, 4, 4); }
            else return hipErrorInvalidValue;
#undef GOL
            return hipGetLastError();
        }
        if (dtype == DT_F32 && V == 2) GO(k_nchwd_bwd_data_k3s2, float, 2);
        else if (dtype == DT_BF16 && V == 4) GO(k_nchwd_bwd_data_k3s2, bf16_t, 4);
        else return hipErrorInvalidValue;
    }
#undef GO
    return hipGetLastError();
}

// Filter gradient tiling: sub-group width, rounds per block and number of partials.
void nchwd_bwd_filter_tiling(const Geom &g, int V, int TH, int *nsg_out, int *nstrips, int *rounds, int *parts)
{
    const int ncols = g.Wo / V;
    const int nsg = ncols <= 256 ? 256 / ncols : 0;      // (image, strip) items a block works on per round
    *nsg_out = nsg;
    *nstrips = ceil_div_h(g.Ho, TH);
    if (nsg == 0) { *rounds = 1; *parts = 0; return; }
    const int nitems = g.N * *nstrips;
    // enough blocks for ~8 per CU over the O channels
    const int want_blocks = 2048;
    int want_parts = (want_blocks + g.O - 1) / g.O;
    if (want_parts < 1) want_parts = 1;
    int r = nitems / (nsg * want_parts);
    if (r < 1) r = 1;
    *rounds = r;
    *parts = ceil_div_h(nitems, nsg * r);
}

hipError_t nchwd_bwd_filter(const Geom &g, int dtype, int V, const void *x, const void *dy, float *ws, int TH,
                            hipStream_t st)
{
    int lg, nstrips, rounds, parts;     // lg = items per round
    nchwd_bwd_filter_tiling(g, V, TH, &lg, &nstrips, &rounds, &parts);
    if (lg < 1 || parts < 1) return hipErrorInvalidValue;
    dim3 grid(parts, g.O);
#define GO(T, VV, SS) hipLaunchKernelGGL((k_nchwd_bwd_filter_k3<T, VV, SS>), grid, dim3(256), 0, st, g, (const T *)x, \
                                         (const T *)dy, ws, TH, nstrips, lg, rounds)
    if (g.s == 1 && dtype == DT_BF16 && (g.K == 3 || g.K == 5) && (V == 8 || V == 4) && !(V == 4 && g.K == 3) &&
        !tune_env("DWCONV_TUNE_NODOT")) {
        // bf16: packed-pair arithmetic (3x3 on 4-column lanes measured faster with the two-rows-ahead kernel below)
#define GOD(VV, KK) hipLaunchKernelGGL((k_nchwd_bwd_filter_s1_bf16<VV, KK>), grid, dim3(256), 0, st, g, (const bf16_t *)x, \
                                       (const bf16_t *)dy, ws, TH, nstrips, lg, rounds)
        if (V == 8) { if (g.K == 3) GOD(8, 3); else GOD(8, 5); }
        else GOD(4, 5);
#undef GOD
        return hipGetLastError();
    }
    if (g.s == 1 && g.K == 5) {
#define GO5(T, VV) hipLaunchKernelGGL((k_nchwd_bwd_filter_s1<T, VV, 5>), grid, dim3(256), 0, st, g, (const T *)x, \
                                      (const T *)dy, ws, TH, nstrips, lg, rounds)
        if (dtype == DT_F32 && V == 4) GO5(float, 4);
        else if (dtype == DT_BF16 && V == 8) GO5(bf16_t, 8);
        else if (dtype == DT_BF16 && V == 4) GO5(bf16_t, 4);
        else return hipErrorInvalidValue;
#undef GO5
    } else if (g.s == 1) {
        if (dtype == DT_F32 && V == 4) GO(float, 4, 1);
        else if (dtype == DT_BF16 && V == 8) GO(bf16_t, 8, 1);
        else if (dtype == DT_BF16 && V == 4) GO(bf16_t, 4, 1);
        else return hipErrorInvalidValue;
    } else {
        if (dtype == DT_F32 && V == 4) GO(float, 4, 2);
        else if (dtype == DT_F32 && V == 2) GO(float, 2, 2);
        else if (dtype == DT_BF16 && V == 8) GO(bf16_t, 8, 2);
        else if (dtype == DT_BF16 && V == 4) GO(bf16_t, 4, 2);
        else return hipErrorInvalidValue;
    }
#undef GO
    return hipGetLastError();
}

// Fused backward: same tiling as the filter gradient, strip height a multiple of the row group.
int nchwd_bwd_fused_rs(const Geom &g, int dtype, int V)
{
    if (!(g.K == 3 && g.p == 1 && g.m == 1)) return 0;
    if (g.s == 2) {
        // stride 2: two dy columns per lane in fp32, four in bf16 (the dx columns under them are one 16-byte vector).
        // bf16 on rows of 112 and more only (the 112x112 layer at batch 256: 183 us against 219 for the two passes and
        // their stage 2; the 56x56 layer 108 against 101)
        const bool f = dtype == DT_F32 && V == 2;
        const bool b = dtype == DT_BF16 && V == 4 && g.W >= 112 && !tune_env("DWCONV_TUNE_NOFUSE_NCHW_BF16");
        if (!((f || b) && g.H % 2 == 0 && g.W % 2 == 0 && g.Wo % V == 0)) return 0;
        const int rs = row_group(g.W, f ? 4 : 2);
        return (rs && g.H % rs == 0 && g.Wo / V <= 256) ? rs : 0;
    }
    if (g.s != 1) return 0;
    // bf16 rows of whole 16-byte vectors: 0.3 % of the bf16 step against the two packed-pair passes, one launch fewer
    const bool bf = dtype == DT_BF16 && V == 8 && !tune_env("DWCONV_TUNE_NOFUSE_NCHW_BF16");
    if (!((dtype == DT_F32 && V == 4) || bf)) return 0;
    const int rs = row_group(g.W, dtype == DT_F32 ? 4 : 2);
    return (rs && g.H % rs == 0 && g.W / V <= 256) ? rs : 0;
}

hipError_t nchwd_bwd_fused(const Geom &g, int dtype, int V, const void *x, const void *dy, const void *w, void *dx,
                           float *ws, int TH, hipStream_t st)
{
    const int rs = nchwd_bwd_fused_rs(g, dtype, V);
    if (!rs || (g.s * TH) % rs != 0) return hipErrorInvalidValue;
    int lg, nstrips, rounds, parts;
    nchwd_bwd_filter_tiling(g, V, TH, &lg, &nstrips, &rounds, &parts);
    if (lg < 1 || parts < 1) return hipErrorInvalidValue;
    dim3 grid(parts, g.C);
#define GO(T, VV, RSV) hipLaunchKernelGGL((k_nchwd_bwd_fused_k3s1<T, VV, RSV>), grid, dim3(256), 0, st, g, (const T *)x, \
                                          (const T *)dy, (const T *)w, (T *)dx, ws, TH, nstrips, lg, rounds)
#define GO2(T, VV, RSV) hipLaunchKernelGGL((k_nchwd_bwd_fused_k3s2<T, VV, RSV>), grid, dim3(256), 0, st, g, (const T *)x, \
                                           (const T *)dy, (const T *)w, (T *)dx, ws, TH, nstrips, lg, rounds)
    if (g.s == 2 && dtype == DT_F32) { if (rs == 2) GO2(float, 2, 2); else GO2(float, 2, 4); }
    else if (g.s == 2) { if (rs == 2) GO2(bf16_t, 4, 2); else GO2(bf16_t, 4, 4); }
    else if (dtype == DT_F32) { if (rs == 2) GO(float, 4, 2); else GO(float, 4, 4); }
    else { if (rs == 2) GO(bf16_t, 8, 2); else GO(bf16_t, 8, 4); }
#undef GO
#undef GO2
    return hipGetLastError();
}

}  // namespace dwc
