// Group convolution, NCHW, 3x3 stride 1 pad 1, rows that are whole 4- or 2-column vectors; any number of
// channels per group on either side.
//
// Forward / backward-data (k_gconv_nchw_s1): a block works on one group and OB of its output channels; a
// lane owns V consecutive columns of one (image, strip) and walks the strip's rows.  The group's filters sit
// in LDS as [input channel][tap row][tap column][output channel]: every lane of the block reads the same
// entries (a broadcast).  One step of the walk takes one row of ONE input channel: three loads (the V-column
// vector and its two neighbours), 9*OB weights, 9*OB*V multiply-adds into three rows of accumulators.  The
// loop over input channels is a real loop, so the kernel serves any group size; the row of the next step is
// loaded while the current one is used.  Input rows above and below a strip feed only one or two output
// rows: the rest of their arithmetic is skipped (the step index is uniform over the block).  Backward-data
// is the same walk over dy with the roles of the channels swapped and the taps reversed.
//
// Filter gradient (k_gconv_nchw_bwd_filter): a block works on one input channel b of a group and OB of the
// group's output channels; a lane owns V columns of (image, strip) items and keeps 9*OB sums.  Per output row
// it takes that row of the OB dy planes and one new row of x (a window of three x rows rotates), 9*OB*V
// multiply-adds; rows are loaded two output rows ahead.  At the end the sums are added over the wavefront
// (butterfly), over the four wavefronts through LDS, and the block writes one partial per weight entry; the
// shared second stage adds the partials.
#include "gconv.hpp"

namespace dwc {

template <int OB> struct LdsW;
template <> struct LdsW<4> {
    static __device__ __forceinline__ void get(const float *p, float (&r)[4])
    {
        const float4 q = *reinterpret_cast<const float4 *>(p);
        r[0] = q.x; r[1] = q.y; r[2] = q.z; r[3] = q.w;
    }
};
template <> struct LdsW<8> {
    static __device__ __forceinline__ void get(const float *p, float (&r)[8])
    {
        const float4 q = *reinterpret_cast<const float4 *>(p), t = *reinterpret_cast<const float4 *>(p + 4);
        r[0] = q.x; r[1] = q.y; r[2] = q.z; r[3] = q.w; r[4] = t.x; r[5] = t.y; r[6] = t.z; r[7] = t.w;
    }
};
template <> struct LdsW<2> {
    static __device__ __forceinline__ void get(const float *p, float (&r)[2])
    {
        const float2 q = *reinterpret_cast<const float2 *>(p);
        r[0] = q.x; r[1] = q.y;
    }
};
template <> struct LdsW<1> {
    static __device__ __forceinline__ void get(const float *p, float (&r)[1]) { r[0] = *p; }
};

// One row of one plane as a lane sees it: its V columns and the two neighbours.  Consecutive lanes own consecutive
// column vectors, so the neighbour columns come from the neighbour lanes by a wavefront shuffle when the row is
// used; only the first and the last lane of a wavefront load theirs (a load with one active lane).  This halves
// the vector-memory instructions of the walk (SHFL; without it every lane loads its two neighbours).  Lanes at the two ends of a row get the zero padding instead, so a
// neighbour lane that belongs to another work item is never consulted.
template <typename T, int V, bool SHFL> struct RowIn {
    RawVec<T, V> v;
    T l, r;
    __device__ __forceinline__ void load(const T *row, int col0, int W)
    {
        const int lane = threadIdx.x & 63;
        v.load(row + col0);
        T lv = 0, rv = 0;
        if (!SHFL || lane == 0) lv = row[max(col0 - 1, 0)];
        if (!SHFL || lane == 63) rv = row[min(col0 + V, W - 1)];
        l = lv; r = rv;
    }
    // x[0..V+1] = columns col0-1 .. col0+V, zero outside the row or when the row itself is outside the image
    __device__ __forceinline__ void get(float (&x)[V + 2], bool rowok, int col0, int W) const
    {
        const int lane = threadIdx.x & 63;
        float c[V];
        v.get(c);
        float left = ldf(&l), right = ldf(&r);
        if (SHFL) {
            const float sl = __shfl_up(c[V - 1], 1, 64), sr = __shfl_down(c[0], 1, 64);
            if (lane != 0) left = sl;
            if (lane != 63) right = sr;
        }
        x[0] = (rowok && col0 > 0) ? left : 0.f;
        x[V + 1] = (rowok && col0 + V < W) ? right : 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) x[1 + j] = rowok ? c[j] : 0.f;
    }
};

// Forward / backward-data walk: a loop over the input rows, inside it a loop over the input channels, one row of
// one channel loaded a step ahead, the weights of a step read from LDS as the step runs.  The accumulator rows
// change roles by register moves once per input row.  Few registers (five or more wavefronts per SIMD).  Variants
// with deeper prefetch rings, weights read a sub-step ahead, weights in scalar registers, and a row loop
// unrolled by three to avoid the moves all measured within a few per cent of this one.
template <typename T, int V, int OB, int R, bool FLIP, bool SHFL>
__global__ __launch_bounds__(256) void k_gconv_nchw_s1(GGeom g, const T *__restrict__ in, const T *__restrict__ w,
                                                        T *__restrict__ out, int CI, int CO, int CIN_T, int COUT_T, int TH,
                                                        int nstrips, int ncv, int nlanes, int nlb, unsigned nblocks, int nt)
{
    extern __shared__ __align__(16) float wl[];     // [CI][3][3][OB]
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int nchunks = CO / OB;
    const int chunk = lb % nchunks; lb /= nchunks;
    const int lblk = lb % nlb; const int grp = lb / nlb;

    for (int i = threadIdx.x; i < CI * 9 * OB; i += 256) {
        const int a = i % OB, tap = (i / OB) % 9, b = i / (9 * OB);
        int widx;
        if (!FLIP) widx = ((grp * g.Og + chunk * OB + a) * g.Cg + b) * 9 + tap;
        else       widx = ((grp * g.Og + b) * g.Cg + chunk * OB + a) * 9 + (8 - tap);
        wl[i] = ldf(w + widx);
    }
    __syncthreads();

    const int H = g.H, W = g.W, HW = H * W;
    const int idx = lblk * 256 + threadIdx.x;
    const bool active = idx < nlanes;
    const int id = min(idx, nlanes - 1);
    const int cv = id % ncv, t1 = id / ncv, strip = t1 % nstrips, n = t1 / nstrips;
    const int col0 = cv * V, oh0 = strip * TH, oh1 = min(H, oh0 + TH);
    const T *ibase = in + ((size_t)n * CIN_T + (size_t)grp * CI) * HW;
    T *obase = out + ((size_t)n * COUT_T + (size_t)grp * CO + chunk * OB) * HW + col0;

    float A0[OB][V], A1[OB][V], A2[OB][V];
#pragma unroll
    for (int a = 0; a < OB; ++a)
#pragma unroll
        for (int j = 0; j < V; ++j) { A0[a][j] = 0.f; A1[a][j] = 0.f; A2[a][j] = 0.f; }

    auto fma_row = [&](float (&P)[OB][V], const float *wk, const float (&x)[V + 2]) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            float wv[OB];
            LdsW<OB>::get(wk + kw * OB, wv);
#pragma unroll
            for (int a = 0; a < OB; ++a)
#pragma unroll
                for (int q = 0; q < V; ++q) P[a][q] = fmaf(wv[a], x[q + kw], P[a][q]);
        }
    };

    // R rows (steps of the flat (input row, channel) sequence) are kept in flight: all R are taken out of the
    // ring, the next R loads are issued into it, then the R steps are computed.  What bounds this kernel is the
    // number of bytes in flight (wavefronts x rows ahead x 24 bytes per lane) against the memory latency.
    RowIn<T, V, SHFL> ring[R];
    int lt = 0, lbb = 0;                // (row step, channel) of the next load; uniform over the block
    auto issue = [&](RowIn<T, V, SHFL> &slot) {
        const int rn = min(max(oh0 - 1 + lt, 0), H - 1);      // clamped: loads past the walk's end are unused
        slot.load(ibase + (size_t)lbb * HW + (size_t)rn * W, col0, W);
        if (++lbb == CI) { lbb = 0; ++lt; }
    };
#pragma unroll
    for (int j = 0; j < R; ++j) issue(ring[j]);
#pragma unroll 1
    for (int t = 0; t < TH + 2; ++t) {
        const int r = oh0 - 1 + t;
        const bool rowok = r >= 0 && r < H;
        const bool f0 = t <= TH - 1, f1 = t >= 1 && t <= TH, f2 = t >= 2;   // uniform over the block
#pragma unroll 1
        for (int b0 = 0; b0 < CI; b0 += R) {
            float xs[R][V + 2];
#pragma unroll
            for (int j = 0; j < R; ++j) ring[j].get(xs[j], rowok, col0, W);
#pragma unroll
            for (int j = 0; j < R; ++j) issue(ring[j]);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const float *wb = wl + (b0 + j) * 9 * OB;
                if (f0) fma_row(A2, wb, xs[j]);
                if (f1) fma_row(A1, wb + 3 * OB, xs[j]);
                if (f2) fma_row(A0, wb + 6 * OB, xs[j]);
            }
        }
        const int orow = r - 1;
        if (f2 && active && orow < oh1) {
#pragma unroll
            for (int a = 0; a < OB; ++a) store_vec<T, V>(obase + (size_t)a * HW + (size_t)orow * W, A0[a], nt != 0);
        }
#pragma unroll
        for (int a = 0; a < OB; ++a)
#pragma unroll
            for (int q = 0; q < V; ++q) { A0[a][q] = A1[a][q]; A1[a][q] = A2[a][q]; A2[a][q] = 0.f; }
    }
}

// Filter gradient, stage 1.  Block: (group, input channel b, chunk of OB output channels, part).
// WSPLIT: the four wavefronts of a block take four different input channels b and the SAME 64 work items, so the
// dy rows they all need are fetched once per block (the other three reads hit the L1) instead of once per input
// channel from L2; each wavefront then owns its sums and writes its own partial.
template <typename T, int V, int OB, bool SHFL, bool WSPLIT>
__global__ __launch_bounds__(256) void k_gconv_nchw_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                               float *__restrict__ ws, int TH, int nstrips, int ncv,
                                                               int nitems, int parts, unsigned nblocks, int J)
{
    __shared__ float red[4][9 * OB];
    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int nchunks = g.Og / OB;
    const int nbq = WSPLIT ? g.Cg / 4 : g.Cg;
    const int bq = lb % nbq; lb /= nbq;
    const int b = WSPLIT ? bq * 4 + (int)(threadIdx.x >> 6) : bq;
    const int chunk = lb % nchunks; lb /= nchunks;
    const int part = lb % parts; const int grp = lb / parts;
    constexpr int LPB = WSPLIT ? 64 : 256;          // work items per block and iteration
    const int lidx = WSPLIT ? (int)(threadIdx.x & 63) : (int)threadIdx.x;

    const int H = g.H, W = g.W, HW = H * W;
    float acc[OB][3][3];
#pragma unroll
    for (int a = 0; a < OB; ++a)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) acc[a][kh][kw] = 0.f;

    for (int item = part * LPB + lidx; item < nitems; item += parts * LPB) {
        const int cv = item % ncv, t1 = item / ncv, strip = t1 % nstrips, n = t1 / nstrips;
        const int col0 = cv * V, oh0 = strip * TH, oh1 = min(H, oh0 + TH);
        const T *xp = x + ((size_t)n * g.C + (size_t)grp * g.Cg + b) * HW;
        const T *dp = dy + ((size_t)n * g.O + (size_t)grp * g.Og + chunk * OB) * HW + col0;

        // window of three x rows: X0 = row oh-1, X1 = row oh, X2 = row oh+1
        float X0[V + 2], X1[V + 2], X2[V + 2];
        {
            RowIn<T, V, SHFL> q;
            q.load(xp + (size_t)max(oh0 - 1, 0) * W, col0, W);
            q.get(X1, oh0 - 1 >= 0, col0, W);
            q.load(xp + (size_t)oh0 * W, col0, W);
            q.get(X2, true, col0, W);
        }
        // two output rows ahead: slot j holds x row oh+1 and the dy rows oh of output row oh = oh0 + j (mod 2)
        RowIn<T, V, SHFL> xn[2];
        RawVec<T, V> dn[2][OB];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            xn[j].load(xp + (size_t)min(oh0 + j + 1, H - 1) * W, col0, W);
#pragma unroll
            for (int a = 0; a < OB; ++a) dn[j][a].load(dp + (size_t)a * HW + (size_t)min(oh0 + j, H - 1) * W);
        }
        for (int oh = oh0; oh < oh1; oh += 2) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int cur = oh + j;
                const bool valid = cur < oh1;           // an odd strip height leaves one empty step at the end
#pragma unroll
                for (int q = 0; q < V + 2; ++q) { X0[q] = X1[q]; X1[q] = X2[q]; }
                xn[j].get(X2, cur + 1 < H, col0, W);
                float d[OB][V];
#pragma unroll
                for (int a = 0; a < OB; ++a) {
                    dn[j][a].get(d[a]);
#pragma unroll
                    for (int q = 0; q < V; ++q) d[a][q] = valid ? d[a][q] : 0.f;
                }
                xn[j].load(xp + (size_t)min(cur + 3, H - 1) * W, col0, W);
#pragma unroll
                for (int a = 0; a < OB; ++a) dn[j][a].load(dp + (size_t)a * HW + (size_t)min(cur + 2, H - 1) * W);
#pragma unroll
                for (int a = 0; a < OB; ++a)
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                        for (int q = 0; q < V; ++q) {
                            acc[a][0][kw] = fmaf(d[a][q], X0[q + kw], acc[a][0][kw]);
                            acc[a][1][kw] = fmaf(d[a][q], X1[q + kw], acc[a][1][kw]);
                            acc[a][2][kw] = fmaf(d[a][q], X2[q + kw], acc[a][2][kw]);
                        }
            }
        }
    }

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int a = 0; a < OB; ++a)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const float s = wave_sum(acc[a][kh][kw]);
                if (lane == 0) red[wv][(a * 3 + kh) * 3 + kw] = s;
            }
    __syncthreads();
    if (WSPLIT) {
        // every wavefront holds the finished sums of its own input channel
        if (lane < 9 * OB) {
            const int e = lane, a = e / 9, tap = e % 9;
            const int o = grp * g.Og + chunk * OB + a;
            ws[(size_t)part * J + ((size_t)o * g.Cg + b) * 9 + tap] = red[wv][e];
        }
    } else if (threadIdx.x < 9 * OB) {
        const int e = threadIdx.x, a = e / 9, tap = e % 9;
        const int o = grp * g.Og + chunk * OB + a;
        ws[(size_t)part * J + ((size_t)o * g.Cg + b) * 9 + tap] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    }
}

// ---- host side ---------------------------------------------------------------------------------------------

static int gtune(const char *name, int dflt)
{
    const char *e = tune_env(name);
    return e && *e ? atoi(e) : dflt;
}
static int pick_ob(int CO)
{
    const int cap = gtune("DWCONV_TUNE_GOB", 4);
    return (CO % 4 == 0 && cap >= 4) ? 4 : ((CO % 2 == 0 && cap >= 2) ? 2 : 1);
}
// columns per lane; the forward / backward-data walk measured faster with two columns per lane on rows of up
// to 56 elements (fewer registers, more wavefronts in flight), the filter gradient with four throughout
static int pick_v(int W, bool walk = false)
{
    const int cap = gtune("DWCONV_TUNE_GV", walk && W <= 56 ? 2 : 4);
    return (W % 4 == 0 && cap >= 4) ? 4 : (W % 2 == 0 ? 2 : 0);
}

bool gconv_nchw_supported(const GGeom &g)
{
    if (!(g.K == 3 && g.s == 1 && g.p == 1)) return false;
    if (pick_v(g.W) == 0) return false;
    // the group's filters for one block have to fit in LDS with room to spare
    const int ob_f = pick_ob(g.Og), ob_b = pick_ob(g.Cg);
    if ((long long)g.Cg * 9 * ob_f * 4 > 32768 || (long long)g.Og * 9 * ob_b * 4 > 32768) return false;
    return true;
}

// strip height: the tallest of whole plane / 28 / 14 / 7 rows that still gives the launch about two
// blocks per compute unit
static int gconv_pick_th(const GGeom &g, long long blocks_per_lane_block_row, bool walk, int v = 0)
{
    const int forced = gtune("DWCONV_TUNE_GTH", 0);
    if (forced > 0) return forced < g.H ? forced : g.H;
    const int cands[4] = {g.H, 28, 14, 7};
    const int ncv = g.W / (v > 0 ? v : pick_v(g.W, walk));
    const long long want = gtune("DWCONV_TUNE_GBLOCKS", 512);
    for (int i = 0; i < 4; ++i) {
        const int th = cands[i] < g.H ? cands[i] : g.H;
        const long long nlanes = (long long)g.N * ((g.H + th - 1) / th) * ncv;
        if (((nlanes + 255) / 256) * blocks_per_lane_block_row >= want) return th;
    }
    return g.H < 7 ? g.H : 7;
}

hipError_t gconv_nchw_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    if (!gconv_nchw_supported(g)) return hipErrorInvalidValue;
    const int CI = flip ? g.Og : g.Cg, CO = flip ? g.Cg : g.Og;
    const int CIN_T = flip ? g.O : g.C, COUT_T = flip ? g.C : g.O;
    int V = pick_v(g.W, true);
    // bf16 on wide rows: eight columns per lane, so that a lane's accesses are 16 bytes as in fp32
    if (dtype == DT_BF16 && V == 4 && g.W % 8 == 0 && gtune("DWCONV_TUNE_GV8", 1) != 0) V = 8;
    // all eight output channels of a group of 8 in one block on two-column lanes (the input is then read once)
    const int OB = (V == 2 && CO == 8 && gtune("DWCONV_TUNE_GOB8", 1) != 0) ? 8 : pick_ob(CO);
    const int nchunks = CO / OB;
    const int TH = gconv_pick_th(g, (long long)g.G * nchunks, true, V);
    const int nstrips = (g.H + TH - 1) / TH, ncv = g.W / V;
    const long long nl = (long long)g.N * nstrips * ncv;
    const long long nlb = (nl + 255) / 256;
    const long long nb = nlb * g.G * nchunks;
    if (nl >= (1ll << 31) || nb >= (1ll << 31)) return hipErrorInvalidValue;
    const int nlanes = (int)nl;
    const unsigned nblocks = (unsigned)nb;
    const size_t lds = (size_t)CI * 9 * OB * sizeof(float);
    const int esz = dtype == DT_F32 ? 4 : 2;
    const int nt = stream_stores(flip ? "GROUP_NCHW_BWD" : "GROUP_NCHW_FWD", (long long)g.N * COUT_T * g.H * g.W * esz);
    // rows in flight per lane: R must divide the channels read per group
    int R = CI % 4 == 0 ? 4 : (CI % 2 == 0 ? 2 : 1);
    const int rcap = gtune("DWCONV_TUNE_GR", 4);
    while (R > rcap) R /= 2;
#define GO5(T, VV, OBB, RR)                                                                                                 \
    do {                                                                                                                    \
        if (flip) hipLaunchKernelGGL((k_gconv_nchw_s1<T, VV, OBB, RR, true, (VV == 2)>), dim3(nblocks), dim3(256), lds, st, g, \
                                     (const T *)in, (const T *)w, (T *)out, CI, CO, CIN_T, COUT_T, TH, nstrips, ncv, nlanes, \
                                     (int)nlb, nblocks, nt);                                                                \
        else hipLaunchKernelGGL((k_gconv_nchw_s1<T, VV, OBB, RR, false, (VV == 2)>), dim3(nblocks), dim3(256), lds, st, g,  \
                                (const T *)in, (const T *)w, (T *)out, CI, CO, CIN_T, COUT_T, TH, nstrips, ncv, nlanes,     \
                                (int)nlb, nblocks, nt);                                                                     \
    } while (0)
#define GO3(T, VV, OBB) do { if (R == 4) GO5(T, VV, OBB, 4); else if (R == 2) GO5(T, VV, OBB, 2); else GO5(T, VV, OBB, 1); } while (0)
#define GO2(T, VV) do { if (OB == 4) GO3(T, VV, 4); else if (OB == 2) GO3(T, VV, 2); else GO3(T, VV, 1); } while (0)
    if (OB == 8) { if (dtype == DT_F32) GO3(float, 2, 8); else GO3(bf16_t, 2, 8); }
    else if (dtype == DT_F32) { if (V == 4) GO2(float, 4); else GO2(float, 2); }
    else                 { if (V == 8) GO2(bf16_t, 8); else if (V == 4) GO2(bf16_t, 4); else GO2(bf16_t, 2); }
#undef GO2
#undef GO3
#undef GO5
    return hipGetLastError();
}

// Filter-gradient tiling: strip height, and partials per weight entry (each part = 256 lanes that stride
// over the (image, strip, column-vector) items).
static bool gconv_nchw_wsplit(const GGeom &g) { return g.Cg % 4 == 0 && gtune("DWCONV_TUNE_GWSPLIT", 1) != 0; }

static void gconv_nchw_bwd_filter_tiling(const GGeom &g, int *TH, int *nstrips, int *nitems, int *parts)
{
    const int OB = pick_ob(g.Og);
    const bool ws = gconv_nchw_wsplit(g);
    const long long per_part_row = (long long)g.G * (ws ? g.Cg / 4 : g.Cg) * (g.Og / OB);
    const int th = gconv_pick_th(g, per_part_row, false);
    const int ns = (g.H + th - 1) / th;
    const long long ni = (long long)g.N * ns * (g.W / pick_v(g.W));
    // about 2048 blocks in the launch (1024 measured better for the wavefront-split kernel on groups of 4), each
    // lane with at least one item, a bounded number of partials
    long long p = (gtune("DWCONV_TUNE_GWBLOCKS", ws && g.Cg == 4 ? 1024 : 2048) + per_part_row - 1) / per_part_row;
    const long long maxp = ws ? (ni + 63) / 64 : (ni + 255) / 256;
    if (p > maxp) p = maxp;
    if (p > (ws ? 128 : 64)) p = ws ? 128 : 64;
    if (p < 1) p = 1;
    *TH = th; *nstrips = ns; *nitems = (int)(ni < (1ll << 31) ? ni : 0); *parts = (int)p;
}

int gconv_nchw_bwd_filter_parts(const GGeom &g)
{
    int TH, ns, ni, parts;
    gconv_nchw_bwd_filter_tiling(g, &TH, &ns, &ni, &parts);
    return parts;
}

hipError_t gconv_nchw_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts,
                                 hipStream_t st)
{
    if (!gconv_nchw_supported(g)) return hipErrorInvalidValue;
    int TH, nstrips, nitems, p2;
    gconv_nchw_bwd_filter_tiling(g, &TH, &nstrips, &nitems, &p2);
    if (p2 != parts || nitems < 1) return hipErrorInvalidValue;
    const int OB = pick_ob(g.Og), V = pick_v(g.W);
    const bool wsplit = gconv_nchw_wsplit(g);
    const long long nb = (long long)g.G * parts * (g.Og / OB) * (wsplit ? g.Cg / 4 : g.Cg);
    if (nb >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)nb;
    const int J = g.O * g.Cg * 9;
    // neighbour columns by wavefront shuffle: measured faster for groups of 8 and on 14-wide rows, slower on 28
    const bool shfl = gtune("DWCONV_TUNE_GWSHFL", (g.Cg >= 8 || g.W <= 14) ? 1 : 0) != 0;
#define GOK(T, VV, OBB, SH, WS) hipLaunchKernelGGL((k_gconv_nchw_bwd_filter<T, VV, OBB, SH, WS>), dim3(nblocks), dim3(256), 0, st, \
                                                   g, (const T *)x, (const T *)dy, ws, TH, nstrips, g.W / VV, nitems, parts, nblocks, J)
#define GO3(T, VV, OBB)                                                                                                     \
    do {                                                                                                                    \
        if (shfl && wsplit) GOK(T, VV, OBB, true, true);                                                                    \
        else if (shfl) GOK(T, VV, OBB, true, false);                                                                        \
        else if (wsplit) GOK(T, VV, OBB, false, true);                                                                      \
        else GOK(T, VV, OBB, false, false);                                                                                 \
    } while (0)
#define GO2(T, VV) do { if (OB == 4) GO3(T, VV, 4); else if (OB == 2) GO3(T, VV, 2); else GO3(T, VV, 1); } while (0)
    if (dtype == DT_F32) { if (V == 4) GO2(float, 4); else GO2(float, 2); }
    else                 { if (V == 4) GO2(bf16_t, 4); else GO2(bf16_t, 2); }
#undef GO2
#undef GO3
#undef GOK
    return hipGetLastError();
}

}  // namespace dwc
