// NCHW kernels.  A (n, channel) plane is H*W contiguous elements, and any run of whole rows of it
// is one contiguous range.  A block takes a few "units" (a strip of output rows of one plane; the
// whole plane when it is small), copies the input rows each unit needs into LDS with aligned
// 16-byte loads issued back to back (every lane has all its loads in flight before its first
// wait), computes from LDS with one lane per column, stages the outputs in LDS, and writes them
// back as aligned 16-byte stores.  Halo rows shared by neighbouring strips come from L2.
#include "kernels.hpp"

namespace dwc {

enum { MODE_FWD = 0, MODE_BWD_S2 = 1 };

struct TileGeom {
    int TR;        // rows per unit: output rows (forward, filter gradient) or dy rows (backward-data stride 2)
    int nstrips;   // units per plane
    int wp_log2;   // lanes per unit = 1 << wp_log2 >= Wo (a lane owns one output / dy column)
    int U;         // units per block = 256 >> wp_log2 (at most 32)
    int LIN;       // floats reserved per unit in the input LDS area (multiple of 8)
    int LOUT;      // floats reserved per unit in the second LDS area (outputs, or dy for the filter gradient)
    int nunits;    // units per launch (forward/backward-data) or per image (filter gradient)
    int NI;        // filter gradient: images per block
    float inv_lvin, inv_lvout;   // 1 / (16-byte vectors per unit area), to split a flat vector index
};

template <typename T> struct Elems { static constexpr int VE = 16 / sizeof(T); };

struct Unit {
    int o;               // output channel of the plane
    int oh0, oh1;        // unit rows [oh0, oh1) (output rows, or dy rows in MODE_BWD_S2)
    int r_lo;            // first input row held in LDS
    int gi0, gilen;      // input range in elements
    int go0, golen;      // second range: output (or dy for the filter gradient)
};

// A unit's global range [g0, g0+len) sits in LDS with element e at area[e - a0], a0 = g0 rounded down to
// 16 bytes, so that aligned 16-byte global vectors map to aligned LDS vectors.

// LDS -> global: elements of the vector outside [g0, g1) belong to another unit and are skipped.
template <typename T>
__device__ __forceinline__ void store_vec_from_lds(T *__restrict__ dst, int g0, int g1, int a, const float *lds)
{
    constexpr int VE = Elems<T>::VE;
    float v[VE];
#pragma unroll
    for (int j = 0; j < VE; j += 4) {
        float4 q = *reinterpret_cast<const float4 *>(lds + j);
        v[j] = q.x; v[j + 1] = q.y; v[j + 2] = q.z; v[j + 3] = q.w;
    }
    if (a >= g0 && a + VE <= g1) {
        Vec<T, VE>::store(dst + a, v);
    } else {
#pragma unroll
        for (int j = 0; j < VE; ++j)
            if (a + j >= g0 && a + j < g1) stf(dst + a + j, v[j]);
    }
}

// Unit `ug` of image-independent index space: plane = ug / nstrips (over N*O planes), strip = rest.
template <int K, int S, int MODE>
__device__ __forceinline__ Unit unit_of(const Geom &g, const TileGeom &tg, int ug)
{
    Unit u;
    const int plane_out = ug / tg.nstrips, strip = ug - plane_out * tg.nstrips;
    const int n = plane_out / g.O;
    u.o = plane_out - n * g.O;
    const int plane_in = n * g.C + u.o / g.m;
    u.oh0 = strip * tg.TR;
    u.oh1 = min(g.Ho, u.oh0 + tg.TR);
    if (MODE == MODE_FWD) {
        u.r_lo = min(g.H - 1, max(0, u.oh0 * S - g.p));
        const int r_hi = min(g.H - 1, (u.oh1 - 1) * S - g.p + K - 1);
        const int rows_in = max(0, r_hi - u.r_lo + 1);
        u.gi0 = (plane_in * g.H + u.r_lo) * g.W;
        u.gilen = rows_in * g.W;
        u.go0 = (plane_out * g.Ho + u.oh0) * g.Wo;
        u.golen = (u.oh1 - u.oh0) * g.Wo;
    } else {
        // input = dy rows [oh0, min(Ho, oh1+1)), output = dx rows [2*oh0, min(H, 2*oh1))
        u.r_lo = u.oh0;
        const int rows_in = min(g.Ho, u.oh1 + 1) - u.oh0;
        u.gi0 = (plane_out * g.Ho + u.oh0) * g.Wo;
        u.gilen = rows_in * g.Wo;
        const int x0 = 2 * u.oh0, x1 = min(g.H, 2 * u.oh1);
        u.go0 = (plane_in * g.H + x0) * g.W;
        u.golen = max(0, x1 - x0) * g.W;
    }
    return u;
}

// Cooperative copy of every unit's input range into its LDS area.  Each lane first issues all of
// its (up to BATCH) 16-byte loads, then writes them to LDS, so the loads overlap each other.
template <typename T>
__device__ __forceinline__ void tile_load(const T *__restrict__ src, int total, const Unit *units, int nu, int LA,
                                          float inv_lv, bool second, float *area)
{
    constexpr int VE = Elems<T>::VE;
    constexpr int BATCH = 16 / VE * 2;      // 8 vectors of fp32, 4 of bf16: 32 registers either way
    const int lv = LA / VE;
    const int nvec = nu * lv;
    for (int base = 0; base < nvec; base += BATCH * 256) {
        float v[BATCH][VE];
        int dst[BATCH];
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            const int idx = base + it * 256 + (int)threadIdx.x;
            dst[it] = -1;
            if (idx < nvec) {
                const int u = __float2int_rd((idx + 0.5f) * inv_lv), i = idx - u * lv;
                const int g0 = second ? units[u].go0 : units[u].gi0, len = second ? units[u].golen : units[u].gilen;
                const int a = (g0 & ~(VE - 1)) + i * VE;
                if (a < g0 + len) {
                    dst[it] = u * LA + i * VE;
                    if (a + VE <= total) Vec<T, VE>::load(src + a, v[it]);
                    else {
#pragma unroll
                        for (int j = 0; j < VE; ++j) v[it][j] = (a + j < total) ? ldf(src + a + j) : 0.f;
                    }
                }
            }
        }
#pragma unroll
        for (int it = 0; it < BATCH; ++it)
            if (dst[it] >= 0) {
#pragma unroll
                for (int j = 0; j < VE; j += 4)
                    *reinterpret_cast<float4 *>(area + dst[it] + j) = make_float4(v[it][j], v[it][j + 1], v[it][j + 2], v[it][j + 3]);
            }
    }
}

template <typename T>
__device__ __forceinline__ void tile_store(T *__restrict__ dst, const Unit *units, int nu, int LA, float inv_lv,
                                           const float *area)
{
    constexpr int VE = Elems<T>::VE;
    const int lv = LA / VE;
    for (int idx = threadIdx.x; idx < nu * lv; idx += 256) {
        const int u = __float2int_rd((idx + 0.5f) * inv_lv), i = idx - u * lv;
        const int g0 = units[u].go0, g1 = g0 + units[u].golen;
        const int a = (g0 & ~(VE - 1)) + i * VE;
        if (a < g1) store_vec_from_lds<T>(dst, g0, g1, a, area + u * LA + i * VE);
    }
}

// ---------------------------------------------------------------------------------------------
// Forward for K x K (template), stride S, any pad, any multiplier.  FLIP rotates the filter by
// 180 degrees: with "same" padding, stride 1 and multiplier 1 that is the backward-data pass.
// ---------------------------------------------------------------------------------------------
template <typename T, int K, int S, bool FLIP>
__global__ __launch_bounds__(256) void k_nchw_fwd(Geom g, TileGeom tg, const T *__restrict__ x, const T *__restrict__ w,
                                                  T *__restrict__ y, unsigned nblocks)
{
    extern __shared__ float4 smem4[];
    __shared__ Unit units[32];
    float *lin = reinterpret_cast<float *>(smem4);
    float *lout = lin + tg.U * tg.LIN;
    constexpr int VE = Elems<T>::VE;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int ug0 = lb * tg.U;
    const int nu = min(tg.U, tg.nunits - ug0);
    if ((int)threadIdx.x < nu) units[threadIdx.x] = unit_of<K, S, MODE_FWD>(g, tg, ug0 + threadIdx.x);
    __syncthreads();

    tile_load<T>(x, g.N * g.C * g.H * g.W, units, nu, tg.LIN, tg.inv_lvin, false, lin);
    __syncthreads();

    {
        const int u = threadIdx.x >> tg.wp_log2, c = threadIdx.x & ((1 << tg.wp_log2) - 1);
        if (u < nu && c < g.Wo) {
            const Unit un = units[u];
            float wr[K][K];
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int kw = 0; kw < K; ++kw)
                    wr[kh][kw] = ldf(w + (un.o * K + (FLIP ? K - 1 - kh : kh)) * K + (FLIP ? K - 1 - kw : kw));
            const float *base = lin + u * tg.LIN + (un.gi0 & (VE - 1));     // element (r_lo, 0)
            float *obase = lout + u * tg.LOUT + (un.go0 & (VE - 1));         // element (oh0, 0)
            const int iw0 = c * S - g.p;
            // out-of-image taps read a clamped (valid) LDS address and are zeroed with a select
            bool colok[K];
            int coff[K];
#pragma unroll
            for (int kw = 0; kw < K; ++kw) {
                colok[kw] = iw0 + kw >= 0 && iw0 + kw < g.W;
                coff[kw] = colok[kw] ? iw0 + kw : 0;
            }
            const int r_hi = un.r_lo + un.gilen / g.W - 1;   // last input row held in LDS
            auto read_row = [&](int r, float (&row)[K]) {
                const int rr = min(max(r, un.r_lo), r_hi);
                const bool rowok = rr == r && r_hi >= un.r_lo;
                const float *rp = base + (rowok ? rr - un.r_lo : 0) * g.W;
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
                    const float t = rp[coff[kw]];
                    row[kw] = (rowok && colok[kw]) ? t : 0.f;
                }
            };
            if constexpr (S == 1) {
                // input row r is tap row kh of output row r + p - kh: K-1 rotating partial sums
                float acc[K - 1 > 0 ? K - 1 : 1];
#pragma unroll
                for (int j = 0; j < K - 1; ++j) acc[j] = 0.f;
                const int r0 = un.oh0 - g.p, r1 = un.oh1 - g.p + K - 1;     // rows [r0, r1)
#pragma unroll 4
                for (int r = r0; r < r1; ++r) {
                    float row[K];
                    read_row(r, row);
                    float out = (K > 1) ? acc[0] : 0.f;
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) out = fmaf(wr[K - 1][kw], row[kw], out);
#pragma unroll
                    for (int j = 0; j < K - 1; ++j) {
                        float t = (j + 1 < K - 1) ? acc[j + 1] : 0.f;
#pragma unroll
                        for (int kw = 0; kw < K; ++kw) t = fmaf(wr[K - 2 - j][kw], row[kw], t);
                        acc[j] = t;
                    }
                    const int oh = r + g.p - (K - 1);
                    if (oh >= un.oh0) obase[(oh - un.oh0) * g.Wo + c] = out;
                }
            } else {
#pragma unroll 2
                for (int oh = un.oh0; oh < un.oh1; ++oh) {
                    float rows[K][K];
#pragma unroll
                    for (int kh = 0; kh < K; ++kh) read_row(oh * S - g.p + kh, rows[kh]);
                    float acc = 0.f;
#pragma unroll
                    for (int kh = 0; kh < K; ++kh)
#pragma unroll
                        for (int kw = 0; kw < K; ++kw) acc = fmaf(wr[kh][kw], rows[kh][kw], acc);
                    obase[(oh - un.oh0) * g.Wo + c] = acc;
                }
            }
        }
    }
    __syncthreads();

    tile_store<T>(y, units, nu, tg.LOUT, tg.inv_lvout, lout);
}

// ---------------------------------------------------------------------------------------------
// Backward-data, 3x3, stride 2, pad 1, multiplier 1.  A lane owns dy column b and walks down the
// unit's dy rows a; from dy[a..a+1][b..b+1] it produces the 2x2 block dx[2a..2a+1][2b..2b+1]
// (same tap table as the NHWC kernel).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_nchw_bwd_data_k3s2(Geom g, TileGeom tg, const T *__restrict__ dy,
                                                            const T *__restrict__ w, T *__restrict__ dx, unsigned nblocks)
{
    extern __shared__ float4 smem4[];
    __shared__ Unit units[32];
    float *lin = reinterpret_cast<float *>(smem4);
    float *lout = lin + tg.U * tg.LIN;
    constexpr int VE = Elems<T>::VE;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int ug0 = lb * tg.U;
    const int nu = min(tg.U, tg.nunits - ug0);
    if ((int)threadIdx.x < nu) units[threadIdx.x] = unit_of<3, 2, MODE_BWD_S2>(g, tg, ug0 + threadIdx.x);
    __syncthreads();

    tile_load<T>(dy, g.N * g.O * g.Ho * g.Wo, units, nu, tg.LIN, tg.inv_lvin, false, lin);
    __syncthreads();

    {
        const int u = threadIdx.x >> tg.wp_log2, b = threadIdx.x & ((1 << tg.wp_log2) - 1);
        if (u < nu && b < g.Wo) {
            const Unit un = units[u];
            float wr[3][3];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) wr[kh][kw] = ldf(w + (un.o * 3 + kh) * 3 + kw);
            const float *base = lin + u * tg.LIN + (un.gi0 & (VE - 1));     // dy element (oh0, 0)
            float *obase = lout + u * tg.LOUT + (un.go0 & (VE - 1));         // dx element (2*oh0, 0)
            const bool has_b1 = b + 1 < g.Wo, col1 = 2 * b + 1 < g.W;
            float A0 = base[b], A1 = has_b1 ? base[b + 1] : 0.f;
            for (int a = un.oh0; a < un.oh1; ++a) {
                float B0 = 0.f, B1 = 0.f;
                if (a + 1 < g.Ho) {
                    const float *rp = base + (a + 1 - un.oh0) * g.Wo;
                    B0 = rp[b];
                    B1 = has_b1 ? rp[b + 1] : 0.f;
                }
                float *op = obase + (2 * (a - un.oh0)) * g.W + 2 * b;
                op[0] = wr[1][1] * A0;
                if (col1) op[1] = fmaf(wr[1][0], A1, wr[1][2] * A0);
                if (2 * a + 1 < g.H) {
                    op[g.W] = fmaf(wr[0][1], B0, wr[2][1] * A0);
                    if (col1) op[g.W + 1] = fmaf(wr[0][0], B1, fmaf(wr[0][2], B0, fmaf(wr[2][0], A1, wr[2][2] * A0)));
                }
                A0 = B0; A1 = B1;
            }
        }
    }
    __syncthreads();

    tile_store<T>(dx, units, nu, tg.LOUT, tg.inv_lvout, lout);
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1.  Units are (output channel, strip) pairs of ONE image; the block loops
// over NI consecutive images, keeping K*K fp32 partial sums per lane in registers.  At the end
// the lanes of a unit are summed with butterfly shuffles (and through LDS when a unit spans more
// than one wavefront), in a fixed order, and lane 0 of the unit writes the unit's partial to the
// workspace at [part][o][kh][kw], part = image group * nstrips + strip.
// ---------------------------------------------------------------------------------------------
template <typename T, int K, int S>
__global__ __launch_bounds__(256) void k_nchw_bwd_filter(Geom g, TileGeom tg, const T *__restrict__ x,
                                                         const T *__restrict__ dy, float *__restrict__ ws,
                                                         int nublocks, unsigned nblocks)
{
    extern __shared__ float4 smem4[];
    __shared__ Unit units[32];
    __shared__ float red[4][K * K];
    float *lin = reinterpret_cast<float *>(smem4);
    float *ldy = lin + tg.U * tg.LIN;
    constexpr int VE = Elems<T>::VE;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int ublock = lb % nublocks, ngroup = lb / nublocks;
    const int ug0 = ublock * tg.U;                       // unit index within an image
    const int nu = min(tg.U, tg.nunits - ug0);
    const int n0 = ngroup * tg.NI, n1 = min(g.N, n0 + tg.NI);
    const int WP = 1 << tg.wp_log2;
    const int u = threadIdx.x >> tg.wp_log2, c = threadIdx.x & (WP - 1);
    const bool active = u < nu && c < g.Wo;

    float acc[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) acc[kh][kw] = 0.f;
    const int iw0 = c * S - g.p;
    bool colok[K];
#pragma unroll
    for (int kw = 0; kw < K; ++kw) colok[kw] = iw0 + kw >= 0 && iw0 + kw < g.W;

    for (int n = n0; n < n1; ++n) {
        __syncthreads();   // the previous image's LDS contents are no longer needed
        if ((int)threadIdx.x < nu) units[threadIdx.x] = unit_of<K, S, MODE_FWD>(g, tg, n * tg.nunits + ug0 + threadIdx.x);
        __syncthreads();
        tile_load<T>(x, g.N * g.C * g.H * g.W, units, nu, tg.LIN, tg.inv_lvin, false, lin);
        tile_load<T>(dy, g.N * g.O * g.Ho * g.Wo, units, nu, tg.LOUT, tg.inv_lvout, true, ldy);
        __syncthreads();
        if (active) {
            const Unit un = units[u];
            const float *base = lin + u * tg.LIN + (un.gi0 & (VE - 1));
            const float *dbase = ldy + u * tg.LOUT + (un.go0 & (VE - 1));
            for (int oh = un.oh0; oh < un.oh1; ++oh) {
                const float d = dbase[(oh - un.oh0) * g.Wo + c];
#pragma unroll
                for (int kh = 0; kh < K; ++kh) {
                    const int ih = oh * S - g.p + kh;
                    if (ih >= 0 && ih < g.H) {
                        const float *rp = base + (ih - un.r_lo) * g.W + iw0;
#pragma unroll
                        for (int kw = 0; kw < K; ++kw)
                            if (colok[kw]) acc[kh][kw] = fmaf(d, rp[kw], acc[kh][kw]);
                    }
                }
            }
        }
    }

    // ---- fixed-order reduction over the lanes of each unit ----
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int strip = (ug0 + u) % tg.nstrips, o = (ug0 + u) / tg.nstrips;
    const int part = ngroup * tg.nstrips + strip;
    const int J = g.O * K * K;
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            float s = acc[kh][kw];
            for (int off = min(WP, 64) >> 1; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
            acc[kh][kw] = s;
        }
    if (WP <= 64) {
        if (u < nu && c == 0) {
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int kw = 0; kw < K; ++kw) ws[(size_t)part * J + (o * K + kh) * K + kw] = acc[kh][kw];
        }
    } else {
        // a unit spans WP/64 wavefronts (2 or 4): combine their sums through LDS
        __syncthreads();
        if (lane == 0) {
#pragma unroll
            for (int kh = 0; kh < K; ++kh)
#pragma unroll
                for (int kw = 0; kw < K; ++kw) red[wv][kh * K + kw] = acc[kh][kw];
        }
        __syncthreads();
        const int wpu = WP >> 6;   // wavefronts per unit
        if (u < nu && c == 0) {
#pragma unroll
            for (int t = 0; t < K * K; ++t) {
                float s = red[wv][t];
                for (int j = 1; j < wpu; ++j) s += red[wv + j][t];
                ws[(size_t)part * J + o * K * K + t] = s;
            }
        }
    }
}

// ---- host side --------------------------------------------------------------------------------

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

// Tiling of the forward / filter-gradient passes (mode 0) or of backward-data stride 2 (mode 1).
// Returns false when the tile does not fit (then the caller uses another kernel).
bool nchw_tiling(const Geom &g, int mode, int TR, TileGeom *tg, size_t *lds_bytes)
{
    int wp = 3;
    while ((1 << wp) < g.Wo) ++wp;
    if (wp > 8) return false;            // more than 256 columns per row
    tg->wp_log2 = wp;
    tg->U = 256 >> wp;
    if (TR > g.Ho) TR = g.Ho;
    if (TR < 1) TR = 1;
    tg->TR = TR;
    tg->nstrips = ceil_div(g.Ho, TR);
    if (mode == MODE_FWD) {
        const int rows_in = min(g.H, (TR - 1) * g.s + g.K);
        tg->LIN = round_up(rows_in * g.W + 16, 8);
        tg->LOUT = round_up(TR * g.Wo + 16, 8);
    } else {
        tg->LIN = round_up((TR + 1) * g.Wo + 16, 8);
        tg->LOUT = round_up(2 * TR * g.W + 16, 8);
    }
    tg->nunits = g.N * g.O * tg->nstrips;
    tg->NI = 1;
    tg->inv_lvin = tg->inv_lvout = 1.0f;   // set per dtype at launch
    *lds_bytes = (size_t)tg->U * (tg->LIN + tg->LOUT) * sizeof(float);
    return *lds_bytes <= 60 * 1024;
}

template <typename T>
static void set_inv(TileGeom &tg)
{
    constexpr int VE = Elems<T>::VE;
    tg.inv_lvin = 1.0f / (float)(tg.LIN / VE);
    tg.inv_lvout = 1.0f / (float)(tg.LOUT / VE);
}

template <typename T, int K, int S>
static hipError_t launch_fwd_t(const Geom &g, TileGeom tg, size_t lds, const void *x, const void *w, void *y, bool flip,
                               hipStream_t st)
{
    set_inv<T>(tg);
    const unsigned nblocks = (unsigned)ceil_div(tg.nunits, tg.U);
    if (flip)
        hipLaunchKernelGGL((k_nchw_fwd<T, K, S, true>), dim3(nblocks), dim3(256), lds, st, g, tg, (const T *)x,
                           (const T *)w, (T *)y, nblocks);
    else
        hipLaunchKernelGGL((k_nchw_fwd<T, K, S, false>), dim3(nblocks), dim3(256), lds, st, g, tg, (const T *)x,
                           (const T *)w, (T *)y, nblocks);
    return hipGetLastError();
}

bool nchw_fwd_supported(const Geom &g, int TR)
{
    TileGeom tg; size_t lds;
    if (!((g.K == 3 || g.K == 5) && (g.s == 1 || g.s == 2))) return false;
    return nchw_tiling(g, MODE_FWD, TR, &tg, &lds);
}

hipError_t nchw_fwd(const Geom &g, int dtype, const void *x, const void *w, void *y, bool flip, int TR, hipStream_t st)
{
    TileGeom tg;
    size_t lds;
    if (!nchw_tiling(g, MODE_FWD, TR, &tg, &lds)) return hipErrorInvalidValue;
#define TRY(KK, SS) if (g.K == KK && g.s == SS) return dtype == DT_F32 ? launch_fwd_t<float, KK, SS>(g, tg, lds, x, w, y, flip, st) \
                                                                        : launch_fwd_t<bf16_t, KK, SS>(g, tg, lds, x, w, y, flip, st)
    TRY(3, 1); TRY(3, 2); TRY(5, 1); TRY(5, 2);
#undef TRY
    return hipErrorInvalidValue;
}

bool nchw_bwd_data_k3s2_supported(const Geom &g, int TR)
{
    TileGeom tg; size_t lds;
    return g.K == 3 && g.s == 2 && g.p == 1 && g.m == 1 && nchw_tiling(g, MODE_BWD_S2, TR, &tg, &lds);
}

hipError_t nchw_bwd_data_k3s2(const Geom &g, int dtype, const void *dy, const void *w, void *dx, int TR, hipStream_t st)
{
    TileGeom tg;
    size_t lds;
    if (!nchw_tiling(g, MODE_BWD_S2, TR, &tg, &lds)) return hipErrorInvalidValue;
    const unsigned nblocks = (unsigned)ceil_div(tg.nunits, tg.U);
    if (dtype == DT_F32) {
        set_inv<float>(tg);
        hipLaunchKernelGGL(k_nchw_bwd_data_k3s2<float>, dim3(nblocks), dim3(256), lds, st, g, tg, (const float *)dy,
                           (const float *)w, (float *)dx, nblocks);
    } else {
        set_inv<bf16_t>(tg);
        hipLaunchKernelGGL(k_nchw_bwd_data_k3s2<bf16_t>, dim3(nblocks), dim3(256), lds, st, g, tg, (const bf16_t *)dy,
                           (const bf16_t *)w, (bf16_t *)dx, nblocks);
    }
    return hipGetLastError();
}

// Filter gradient: returns the number of partials per dw element (0 if unsupported).
int nchw_bwd_filter_parts(const Geom &g, int TR, int NI)
{
    TileGeom tg; size_t lds;
    if (!((g.K == 3 || g.K == 5) && (g.s == 1 || g.s == 2))) return 0;
    if (!nchw_tiling(g, MODE_FWD, TR, &tg, &lds)) return 0;
    return ceil_div(g.N, NI) * tg.nstrips;
}

template <typename T, int K, int S>
static hipError_t launch_bwd_filter_t(const Geom &g, TileGeom tg, size_t lds, const void *x, const void *dy, float *ws,
                                      hipStream_t st)
{
    set_inv<T>(tg);
    const int nublocks = ceil_div(tg.nunits, tg.U);
    const unsigned nblocks = (unsigned)nublocks * ceil_div(g.N, tg.NI);
    hipLaunchKernelGGL((k_nchw_bwd_filter<T, K, S>), dim3(nblocks), dim3(256), lds, st, g, tg, (const T *)x,
                       (const T *)dy, ws, nublocks, nblocks);
    return hipGetLastError();
}

hipError_t nchw_bwd_filter(const Geom &g, int dtype, const void *x, const void *dy, float *ws, int TR, int NI,
                           hipStream_t st)
{
    TileGeom tg;
    size_t lds;
    if (!nchw_tiling(g, MODE_FWD, TR, &tg, &lds)) return hipErrorInvalidValue;
    tg.nunits = g.O * tg.nstrips;     // per image
    tg.NI = NI;
#define TRY(KK, SS) if (g.K == KK && g.s == SS) return dtype == DT_F32 ? launch_bwd_filter_t<float, KK, SS>(g, tg, lds, x, dy, ws, st) \
                                                                        : launch_bwd_filter_t<bf16_t, KK, SS>(g, tg, lds, x, dy, ws, st)
    TRY(3, 1); TRY(3, 2); TRY(5, 1); TRY(5, 2);
#undef TRY
    return hipErrorInvalidValue;
}

}  // namespace dwc
