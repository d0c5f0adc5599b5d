// NCHW kernels for small planes (rows of 7, 14 or 28 elements, and 4 or 8 for 3x3; 3x3 filters, 5x5 at stride 1;
// multiplier 1).
// Rows this short are not whole 16-byte vectors, but consecutive planes are contiguous, so a block
// takes a run of whole planes as ONE flat range: aligned 16-byte loads into LDS (all of a lane's
// loads issued before its first wait), then one lane per (plane, output row) computes the whole
// row from LDS with the row width known at compile time (every tap is a multiply-add with a
// fixed LDS offset, nothing else), stages it in LDS, and the block writes the flat output range
// back with aligned 16-byte stores.
#include "kernels.hpp"

namespace dwc {

template <typename T> struct ElemsS { static constexpr int VE = 16 / sizeof(T); };

// Flat range [g0, g1) of `src` -> lds[e - a0], a0 = g0 rounded down to a 16-byte boundary.
// Everything that can be decided for the whole block is: batches past the range are skipped by a uniform
// branch, lanes past the range in the last batch re-load its last vector (and do not commit it), and the
// element-wise path exists only for a range whose last vector sticks out of the tensor.  Per-lane branches
// around every vector cost these kernels a tenth of their time.
template <typename T, int VE>
__device__ __forceinline__ void flat_load_vec(const T *__restrict__ src, int total, int a0, int nvec, int idx, bool whole,
                                              float (&v)[VE])
{
    const int a = a0 + min(idx, nvec - 1) * VE;
    if (whole) { Vec<T, VE>::load(src + a, v); return; }        // uniform branch: the usual case has no lane mask at all
    if (a + VE <= total) Vec<T, VE>::load(src + a, v);
    else {
#pragma unroll
        for (int j = 0; j < VE; ++j) { const float t = ldf(src + min(a + j, total - 1)); v[j] = (a + j < total) ? t : 0.f; }
    }
}
template <int VE>
__device__ __forceinline__ void flat_commit_vec(float *lds, int nvec, int first, const float (&v)[VE])
{
    const int idx = first + (int)threadIdx.x;
    if (first + 256 <= nvec) {                          // uniform: whole batches commit without a lane mask
#pragma unroll
        for (int j = 0; j < VE; j += 4)
            *reinterpret_cast<float4 *>(lds + idx * VE + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
    } else if (idx < nvec) {
#pragma unroll
        for (int j = 0; j < VE; j += 4)
            *reinterpret_cast<float4 *>(lds + idx * VE + j) = make_float4(v[j], v[j + 1], v[j + 2], v[j + 3]);
    }
}

template <typename T>
__device__ __forceinline__ void flat_load(const T *__restrict__ src, int total, int g0, int g1, float *lds)
{
    constexpr int VE = ElemsS<T>::VE;
    constexpr int BATCH = 16 / VE * 2;
    const int a0 = g0 & ~(VE - 1);
    const int nvec = (g1 - a0 + VE - 1) / VE;
    const bool whole = a0 + nvec * VE <= total;         // uniform
    for (int base = 0; base < nvec; base += BATCH * 256) {
        float v[BATCH][VE];
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            if (base + it * 256 >= nvec) break;          // uniform over the block
            flat_load_vec<T, VE>(src, total, a0, nvec, base + it * 256 + (int)threadIdx.x, whole, v[it]);
        }
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            if (base + it * 256 >= nvec) break;
            flat_commit_vec<VE>(lds, nvec, base + it * 256, v[it]);
        }
    }
}

// The same in two halves, so that the loads of the next range can be in flight while the block computes on the
// current one: issue into registers (up to BATCH 16-byte vectors per lane, kept as loaded: bf16 stays packed, which
// halves the registers a stage in flight costs), commit to LDS (widening bf16 there).
template <typename T> struct FlatRegs { static constexpr int BATCH = 16 / ElemsS<T>::VE * 2; uint4 raw[BATCH]; };
template <typename T>
__device__ __forceinline__ void flat_issue(const T *__restrict__ src, int total, int g0, int g1, FlatRegs<T> &r)
{
    constexpr int VE = ElemsS<T>::VE;
    const int a0 = g0 & ~(VE - 1);
    const int nvec = (g1 - a0 + VE - 1) / VE;
    const bool whole = a0 + nvec * VE <= total;
#pragma unroll
    for (int it = 0; it < FlatRegs<T>::BATCH; ++it) {
        if (it * 256 >= nvec) break;                     // uniform over the block
        const int a = a0 + min(it * 256 + (int)threadIdx.x, nvec - 1) * VE;
        if (whole || a + VE <= total) r.raw[it] = *reinterpret_cast<const uint4 *>(src + a);
        else {                                           // the last vector of a tensor whose size is not a multiple of VE
            uint32_t wds[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < VE; ++j) {
                const T t = src[min(a + j, total - 1)];
                uint32_t bits;
                if constexpr (sizeof(T) == 4) bits = __float_as_uint(t); else bits = (uint32_t)t;
                if (a + j >= total) bits = 0u;
                if constexpr (sizeof(T) == 4) wds[j] = bits; else wds[j / 2] |= bits << (16 * (j & 1));
            }
            r.raw[it] = make_uint4(wds[0], wds[1], wds[2], wds[3]);
        }
    }
}
template <typename T>
__device__ __forceinline__ void flat_commit(int g0, int g1, const FlatRegs<T> &r, float *lds)
{
    constexpr int VE = ElemsS<T>::VE;
    const int a0 = g0 & ~(VE - 1);
    const int nvec = (g1 - a0 + VE - 1) / VE;
#pragma unroll
    for (int it = 0; it < FlatRegs<T>::BATCH; ++it) {
        if (it * 256 >= nvec) break;                     // uniform over the block
        const uint4 q = r.raw[it];
        float v[VE];
        if constexpr (sizeof(T) == 4) {
            v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
        } else {
            v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
            v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
            v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
            v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
        }
        flat_commit_vec<VE>(lds, nvec, it * 256, v);
    }
}

// lds[e - a0] -> flat range [g0, g1) of dst; the first and last vector may be partial.
template <typename T>
__device__ __forceinline__ void flat_store(T *__restrict__ dst, int g0, int g1, const float *lds, bool stream)
{
    constexpr int VE = ElemsS<T>::VE;
    const int a0 = g0 & ~(VE - 1);
    const int nvec = (g1 - a0 + VE - 1) / VE;
    const bool aligned = ((g0 | g1) & (VE - 1)) == 0;   // uniform: no partial vector at either end
    auto one = [&](int idx, bool plain) {
        const int a = a0 + idx * VE;
        float v[VE];
#pragma unroll
        for (int j = 0; j < VE; j += 4) {
            const float4 q = *reinterpret_cast<const float4 *>(lds + idx * VE + j);
            v[j] = q.x; v[j + 1] = q.y; v[j + 2] = q.z; v[j + 3] = q.w;
        }
        if (plain || (a >= g0 && a + VE <= g1)) store_vec<T, VE>(dst + a, v, stream);
        else {
#pragma unroll
            for (int j = 0; j < VE; ++j)
                if (a + j >= g0 && a + j < g1) stf(dst + a + j, v[j]);
        }
    };
    for (int first = 0; first < nvec; first += 256) {    // uniform trip count
        const int idx = first + (int)threadIdx.x;
        if (aligned && first + 256 <= nvec) one(idx, true);          // uniform: a whole batch of whole vectors
        else if (idx < nvec) one(idx, false);
    }
}

// ---------------------------------------------------------------------------------------------
// Forward K x K (K odd), pad (K-1)/2, stride S, row width W (template).  FLIP: filter rotated by 180 degrees
// (backward-data of the stride-1 layer).  U planes per block, one lane per (plane, output row).
// ---------------------------------------------------------------------------------------------
// TPB tiles of U planes per block, one after the other (tile lb*TPB + i): the next tile's planes are loaded into
// registers while the current tile is computed from LDS and written out, so a block's memory latency is paid once.
// INPLACE: the outputs (a lane's whole row, held in registers) go back into the LDS area of the inputs once every
// lane has read its rows, which halves the block's LDS and doubles the blocks per CU on 28-wide planes.
// CG > 1 (3x3 stride 1): a group convolution with CG channels per group on both sides (Section V-B).  The planes of a group
// are neighbours in memory and a tile holds whole groups (U a multiple of CG), so the lane of output plane o adds up the CG
// input planes of its group from the same staged tile; filter [O][CG][3][3].
template <typename T, int K, int S, int W, bool FLIP, bool INPLACE, int CG = 1>
__global__ __launch_bounds__(256) void k_nchws_fwd(Geom g, const T *__restrict__ x, const T *__restrict__ w,
                                                   T *__restrict__ y, int U, int nplanes, unsigned nblocks, int nt, int TPB)
{
    static_assert(CG == 1 || (K == 3 && (S == 1 || (S == 2 && !FLIP))), "group form: 3x3, stride 1 or the stride-2 forward");
    extern __shared__ float4 smem4[];
    constexpr int VE = ElemsS<T>::VE;
    constexpr int P = (K - 1) / 2;
    constexpr int WO = (W + 2 * P - K) / S + 1;
    const int HW = g.H * W, HoWo = g.Ho * WO;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    float *lin = reinterpret_cast<float *>(smem4);
    float *lout = INPLACE ? lin : lin + ((U * HW + 2 * VE + 3) & ~3);
    const int total = g.N * g.C * HW;
    const int p = threadIdx.x / g.Ho, oh = threadIdx.x - p * g.Ho;

    // TPB == 0: a single tile whose planes do not fit the register staging (more than 8192 elements): loaded straight into LDS
    const int ntl = TPB > 0 ? TPB : 1;
    FlatRegs<T> regs;
    if (TPB > 0) {
        const int q0 = (int)(lb * ntl) * U, nq = min(U, nplanes - q0);
        flat_issue<T>(x, total, q0 * HW, (q0 + nq) * HW, regs);
    }
    for (int ti = 0; ti < ntl; ++ti) {
    const int p0 = (int)(lb * ntl + ti) * U;
    if (p0 >= nplanes) break;                       // uniform over the block
    const int np = min(U, nplanes - p0);
    const int gi0 = p0 * HW, go0 = p0 * HoWo;
    if (ti > 0) __syncthreads();                    // the previous tile's write-out has read lout, its compute lin
    if (TPB > 0) flat_commit<T>(gi0, gi0 + np * HW, regs, lin);
    else flat_load<T>(x, total, gi0, gi0 + np * HW, lin);
    __syncthreads();
    if (ti + 1 < ntl && p0 + U < nplanes) {
        const int q0 = p0 + U, nq = min(U, nplanes - q0);
        flat_issue<T>(x, total, q0 * HW, (q0 + nq) * HW, regs);
    }

    float out[WO];
    if (p < np) {
        const int c = (p0 + p) % g.C;
#pragma unroll
        for (int j = 0; j < WO; ++j) out[j] = 0.f;
#pragma unroll
        for (int ci = 0; ci < CG; ++ci) {
        float wr[K][K];
        // taps on rows outside the image are dropped by zeroing their weights (the row address is clamped)
#pragma unroll
        for (int kh = 0; kh < K; ++kh) {
            const int ih = oh * S - P + kh;
            const bool ok = ih >= 0 && ih < g.H;
#pragma unroll
            for (int kw = 0; kw < K; ++kw) {
                const int tap = (FLIP ? K - 1 - kh : kh) * K + (FLIP ? K - 1 - kw : kw);
                int widx;
                if constexpr (CG == 1) widx = c * K * K + tap;
                else if constexpr (!FLIP) widx = (c * CG + ci) * K * K + tap;               // w[o = c][ci]
                else widx = ((c - c % CG + ci) * CG + c % CG) * K * K + tap;                 // w[o = the group's ci-th][the lane's channel]
                const float t = ldf(w + widx);
                wr[kh][kw] = ok ? t : 0.f;
            }
        }
        // the plane read: the lane's own (depthwise), or plane ci of the lane's group (p0 is a multiple of CG)
        const float *pl = lin + (gi0 & (VE - 1)) + (CG == 1 ? p : p - p % CG + ci) * HW;
#pragma unroll
        for (int kh = 0; kh < K; ++kh) {
            const int ih = min(max(oh * S - P + kh, 0), g.H - 1);
            const float *rp = pl + ih * W;
            float row[W];
#pragma unroll
            for (int i = 0; i < W; ++i) row[i] = rp[i];
#pragma unroll
            for (int j = 0; j < WO; ++j)
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
                    const int iw = j * S - P + kw;
                    if (iw >= 0 && iw < W) out[j] = fmaf(wr[kh][kw], row[iw], out[j]);
                }
        }
        }
        if constexpr (!INPLACE) {
            float *op = lout + (go0 & (VE - 1)) + p * HoWo + oh * WO;
#pragma unroll
            for (int j = 0; j < WO; ++j) op[j] = out[j];
        }
    }
    if constexpr (INPLACE) {
        __syncthreads();                            // every lane has read its input rows
        if (p < np) {
            float *op = lout + (go0 & (VE - 1)) + p * HoWo + oh * WO;
#pragma unroll
            for (int j = 0; j < WO; ++j) op[j] = out[j];
        }
    }
    __syncthreads();

    flat_store<T>(y, go0, go0 + np * HoWo, lout, nt != 0);
    }
}

// ---------------------------------------------------------------------------------------------
// Backward-data 3x3, stride 2, pad 1, dx row width W (template, even), dy row width W/2.
// One lane per (plane, dy row a): writes dx rows 2a and 2a+1.
// ---------------------------------------------------------------------------------------------
// CG > 1: group convolution with CG channels per group on both sides; the lane of input plane c adds up the CG dy planes of
// its group (a tile holds whole groups), filter [O][CG][3][3].
template <typename T, int W, int CG = 1>
__global__ __launch_bounds__(256) void k_nchws_bwd_data_s2(Geom g, const T *__restrict__ dy, const T *__restrict__ w,
                                                           T *__restrict__ dx, int U, int nplanes, unsigned nblocks, int nt)
{
    extern __shared__ float4 smem4[];
    constexpr int VE = ElemsS<T>::VE;
    constexpr int WO = W / 2;
    const int HW = g.H * W, HoWo = g.Ho * WO;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int p0 = lb * U, np = min(U, nplanes - p0);
    float *lin = reinterpret_cast<float *>(smem4);
    float *lout = lin + ((U * HoWo + 2 * VE + 3) & ~3);
    const int gi0 = p0 * HoWo, go0 = p0 * HW;

    flat_load<T>(dy, g.N * g.O * HoWo, gi0, gi0 + np * HoWo, lin);
    __syncthreads();

    const int p = threadIdx.x / g.Ho, a = threadIdx.x - p * g.Ho;
    if (p < np) {
        const int c = (p0 + p) % g.C;
        const bool has_b = a + 1 < g.Ho;
        float ev[W], od[W];                       // dx rows 2a and 2a+1
#pragma unroll
        for (int i = 0; i < W; ++i) { ev[i] = 0.f; od[i] = 0.f; }
#pragma unroll
        for (int o = 0; o < CG; ++o) {
            float wr[3][3];
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    // depthwise: the lane's own filter; groups: output channel o of the lane's group against the lane's input channel
                    const int widx = CG == 1 ? (c * 3 + kh) * 3 + kw : (((c - c % CG + o) * CG + c % CG) * 3 + kh) * 3 + kw;
                    wr[kh][kw] = ldf(w + widx);
                }
            const float *pl = lin + (gi0 & (VE - 1)) + (CG == 1 ? p : p - p % CG + o) * HoWo;
            const float *ra = pl + a * WO, *rb = pl + (has_b ? a + 1 : a) * WO;
            float A[WO + 1], B[WO + 1];
#pragma unroll
            for (int i = 0; i < WO; ++i) { A[i] = ra[i]; const float t = rb[i]; B[i] = has_b ? t : 0.f; }
            A[WO] = 0.f; B[WO] = 0.f;
#pragma unroll
            for (int b = 0; b < WO; ++b) {
                ev[2 * b] = fmaf(wr[1][1], A[b], ev[2 * b]);
                ev[2 * b + 1] = fmaf(wr[1][0], A[b + 1], fmaf(wr[1][2], A[b], ev[2 * b + 1]));
                od[2 * b] = fmaf(wr[0][1], B[b], fmaf(wr[2][1], A[b], od[2 * b]));
                od[2 * b + 1] = fmaf(wr[0][0], B[b + 1], fmaf(wr[0][2], B[b], fmaf(wr[2][0], A[b + 1], fmaf(wr[2][2], A[b], od[2 * b + 1]))));
            }
        }
        float *op = lout + (go0 & (VE - 1)) + p * HW + (2 * a) * W;
#pragma unroll
        for (int i = 0; i < W; ++i) { op[i] = ev[i]; op[W + i] = od[i]; }
    }
    __syncthreads();

    flat_store<T>(dx, go0, go0 + np * HW, lout, nt != 0);
}

// ---------------------------------------------------------------------------------------------
// Backward-filter stage 1, K x K (K odd), pad (K-1)/2, stride S, x row width W (template).  A block owns U
// consecutive channels and walks NI images; a lane owns (channel, output row) and keeps its K*K
// partial sums in registers across the images.  At the end the rows of a channel are added in
// row order through LDS and one partial per block is written at ws[part][c][kh][kw].
// ---------------------------------------------------------------------------------------------
// CG > 1 (3x3 stride 1): group convolution with CG channels per group on both sides; the lane of output plane o keeps
// 9 sums for each of the CG input planes of its group (all in the block's tile: U is a multiple of CG); partial sums
// at ws[part][o][ci][kh][kw].
template <typename T, int K, int S, int W, int CG = 1>
__global__ __launch_bounds__(256) void k_nchws_bwd_filter(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                          float *__restrict__ ws, int U, int NI, int ncblocks,
                                                          unsigned nblocks)
{
    static_assert(CG == 1 || K == 3, "group form: 3x3");
    extern __shared__ float4 smem4[];
    constexpr int VE = ElemsS<T>::VE;
    constexpr int P = (K - 1) / 2;
    constexpr int WO = (W + 2 * P - K) / S + 1;
    const int HW = g.H * W, HoWo = g.Ho * WO;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int cblk = lb % ncblocks, part = lb / ncblocks;
    const int c0 = cblk * U, nc = min(U, g.C - c0);
    const int n0 = part * NI, n1 = min(g.N, n0 + NI);
    float *lx = reinterpret_cast<float *>(smem4);
    float *ld = lx + ((U * HW + 2 * VE + 3) & ~3);

    const int p = threadIdx.x / g.Ho, oh = threadIdx.x - p * g.Ho;
    float acc[CG][K][K];
#pragma unroll
    for (int ci = 0; ci < CG; ++ci)
#pragma unroll
        for (int kh = 0; kh < K; ++kh)
#pragma unroll
            for (int kw = 0; kw < K; ++kw) acc[ci][kh][kw] = 0.f;
    bool rowok[K];
    int rowi[K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh) {
        const int ih = oh * S - P + kh;
        rowok[kh] = ih >= 0 && ih < g.H;
        rowi[kh] = min(max(ih, 0), g.H - 1);
    }

    // the next image's planes are loaded into registers while this one is accumulated from LDS
    FlatRegs<T> rx, rd;
    {
        const int gx0 = (n0 * g.C + c0) * HW, gd0 = (n0 * g.O + c0) * HoWo;
        flat_issue<T>(x, g.N * g.C * HW, gx0, gx0 + nc * HW, rx);
        flat_issue<T>(dy, g.N * g.O * HoWo, gd0, gd0 + nc * HoWo, rd);
    }
    for (int n = n0; n < n1; ++n) {
        const int gx0 = (n * g.C + c0) * HW, gd0 = (n * g.O + c0) * HoWo;
        __syncthreads();
        flat_commit<T>(gx0, gx0 + nc * HW, rx, lx);
        flat_commit<T>(gd0, gd0 + nc * HoWo, rd, ld);
        __syncthreads();
        if (n + 1 < n1) {
            const int hx0 = ((n + 1) * g.C + c0) * HW, hd0 = ((n + 1) * g.O + c0) * HoWo;
            flat_issue<T>(x, g.N * g.C * HW, hx0, hx0 + nc * HW, rx);
            flat_issue<T>(dy, g.N * g.O * HoWo, hd0, hd0 + nc * HoWo, rd);
        }
        if (p < nc) {
            const float *dp = ld + (gd0 & (VE - 1)) + p * HoWo + oh * WO;
            float d[WO];
#pragma unroll
            for (int j = 0; j < WO; ++j) d[j] = dp[j];
#pragma unroll
            for (int ci = 0; ci < CG; ++ci) {
                // the x plane: the lane's own (depthwise), or plane ci of the lane's group (c0 is a multiple of CG)
                const float *xp = lx + (gx0 & (VE - 1)) + (CG == 1 ? p : p - p % CG + ci) * HW;
#pragma unroll
                for (int kh = 0; kh < K; ++kh) {
                    const float *rp = xp + rowi[kh] * W;
                    float row[W];
#pragma unroll
                    for (int i = 0; i < W; ++i) { const float t = rp[i]; row[i] = rowok[kh] ? t : 0.f; }
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        float s = acc[ci][kh][kw];
#pragma unroll
                        for (int j = 0; j < WO; ++j) {
                            const int iw = j * S - P + kw;
                            if (iw >= 0 && iw < W) s = fmaf(d[j], row[iw], s);
                        }
                        acc[ci][kh][kw] = s;
                    }
                }
            }
        }
    }

    // rows of a channel are added in row order (fixed), through LDS; one input channel of the group at a time
    float *red = lx;     // 256 * K*K floats, reusing the staging areas (the host sizes the LDS for it)
#pragma unroll
    for (int ci = 0; ci < CG; ++ci) {
        __syncthreads();
#pragma unroll
        for (int kh = 0; kh < K; ++kh)
#pragma unroll
            for (int kw = 0; kw < K; ++kw) red[threadIdx.x * (K * K) + kh * K + kw] = (p < nc) ? acc[ci][kh][kw] : 0.f;
        __syncthreads();
        for (int idx = threadIdx.x; idx < nc * K * K; idx += 256) {
            const int pc = idx / (K * K), t = idx - pc * (K * K);
            float s = 0.f;
            for (int r = 0; r < g.Ho; ++r) s += red[(pc * g.Ho + r) * (K * K) + t];
            ws[(((size_t)part * g.O + c0 + pc) * CG + ci) * (K * K) + t] = s;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Fused backward pass, 3x3, stride 1, pad 1, row width W (template): the planes of x and dy of one
// image are staged in LDS once and serve both gradients.  Block and lane mapping of the
// filter-gradient kernel above (U consecutive channels, NI images; a lane owns (channel, row)):
// the lane accumulates its 9 partial sums from the x rows around its dy row, and it computes row
// `oh` of dx from the dy rows around it with the rotated filter; the dx planes go to a third
// LDS area and leave as one flat range with aligned 16-byte streaming stores.
// INPLACE (28-wide rows, where three areas would leave a block four channels): the dx rows wait in
// registers until every lane has read its x rows and then take x's place in LDS.
// ---------------------------------------------------------------------------------------------
template <typename T, int W, bool INPLACE>
__global__ __launch_bounds__(256) void k_nchws_bwd_fused(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                         const T *__restrict__ w, T *__restrict__ dx,
                                                         float *__restrict__ ws, int U, int NI, int ncblocks,
                                                         unsigned nblocks, int nt)
{
    extern __shared__ float4 smem4[];
    constexpr int VE = ElemsS<T>::VE;
    constexpr int K = 3;
    const int HW = g.H * W;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int cblk = lb % ncblocks, part = lb / ncblocks;
    const int c0 = cblk * U, nc = min(U, g.C - c0);
    const int n0 = part * NI, n1 = min(g.N, n0 + NI);
    const int area = (U * HW + 2 * VE + 3) & ~3;
    float *lx = reinterpret_cast<float *>(smem4);
    float *ld = lx + area;
    float *lo = INPLACE ? lx : ld + area;

    const int p = threadIdx.x / g.H, oh = threadIdx.x - p * g.H;
    const bool own = p < nc;
    float acc[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) acc[kh][kw] = 0.f;
    bool rowok[K];
    int rowi[K];
    float wr[K][K];          // rotated filter of the lane's channel, rows outside the image zeroed
#pragma unroll
    for (int kh = 0; kh < K; ++kh) {
        const int ih = oh - 1 + kh;
        rowok[kh] = ih >= 0 && ih < g.H;
        rowi[kh] = min(max(ih, 0), g.H - 1);
#pragma unroll
        for (int kw = 0; kw < K; ++kw) {
            const float t = ldf(w + ((c0 + min(p, nc - 1)) * K + (K - 1 - kh)) * K + (K - 1 - kw));
            wr[kh][kw] = rowok[kh] ? t : 0.f;
        }
    }

    FlatRegs<T> rx, rd;
    {
        const int g0 = (n0 * g.C + c0) * HW;
        flat_issue<T>(x, g.N * g.C * HW, g0, g0 + nc * HW, rx);
        flat_issue<T>(dy, g.N * g.C * HW, g0, g0 + nc * HW, rd);
    }
    for (int n = n0; n < n1; ++n) {
        const int g0 = (n * g.C + c0) * HW;       // x, dy and dx planes of this image and channel block: the same flat range
        __syncthreads();                          // the previous image's dx has left the staging area
        flat_commit<T>(g0, g0 + nc * HW, rx, lx);
        flat_commit<T>(g0, g0 + nc * HW, rd, ld);
        __syncthreads();
        if (n + 1 < n1) {
            const int h0 = ((n + 1) * g.C + c0) * HW;
            flat_issue<T>(x, g.N * g.C * HW, h0, h0 + nc * HW, rx);
            flat_issue<T>(dy, g.N * g.C * HW, h0, h0 + nc * HW, rd);
        }
        float out[W];
        if (own) {
            const int off = (g0 & (VE - 1)) + p * HW;
            const float *xp = lx + off, *dpl = ld + off;
            // filter gradient: dy row oh against x rows oh-1, oh, oh+1
            float d[W];
#pragma unroll
            for (int j = 0; j < W; ++j) d[j] = dpl[oh * W + j];
#pragma unroll
            for (int kh = 0; kh < K; ++kh) {
                const float *rp = xp + rowi[kh] * W;
                float row[W];
#pragma unroll
                for (int i = 0; i < W; ++i) { const float t = rp[i]; row[i] = rowok[kh] ? t : 0.f; }
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
                    float s = acc[kh][kw];
#pragma unroll
                    for (int j = 0; j < W; ++j) {
                        const int iw = j - 1 + kw;
                        if (iw >= 0 && iw < W) s = fmaf(d[j], row[iw], s);
                    }
                    acc[kh][kw] = s;
                }
            }
            // input gradient: row oh of dx = rotated filter over dy rows oh-1, oh, oh+1
#pragma unroll
            for (int j = 0; j < W; ++j) out[j] = 0.f;
#pragma unroll
            for (int kh = 0; kh < K; ++kh) {
                const float *rp = dpl + rowi[kh] * W;
                float row[W];
#pragma unroll
                for (int i = 0; i < W; ++i) row[i] = (kh == 1) ? d[i] : rp[i];
#pragma unroll
                for (int j = 0; j < W; ++j)
#pragma unroll
                    for (int kw = 0; kw < K; ++kw) {
                        const int iw = j - 1 + kw;
                        if (iw >= 0 && iw < W) out[j] = fmaf(wr[kh][kw], row[iw], out[j]);
                    }
            }
            if constexpr (!INPLACE) {
                float *op = lo + off + oh * W;
#pragma unroll
                for (int j = 0; j < W; ++j) op[j] = out[j];
            }
        }
        if constexpr (INPLACE) {
            __syncthreads();                      // every lane has read its x rows
            if (own) {
                float *op = lo + (g0 & (VE - 1)) + p * HW + oh * W;
#pragma unroll
                for (int j = 0; j < W; ++j) op[j] = out[j];
            }
        }
        __syncthreads();
        flat_store<T>(dx, g0, g0 + nc * HW, lo, nt != 0);
    }

    // rows of a channel are added in row order (fixed), through LDS
    __syncthreads();
    float *red = lx;     // 256 * 9 floats across the staging areas (the host sizes the LDS for it)
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) red[threadIdx.x * (K * K) + kh * K + kw] = own ? acc[kh][kw] : 0.f;
    __syncthreads();
    for (int idx = threadIdx.x; idx < nc * K * K; idx += 256) {
        const int pc = idx / (K * K), t = idx - pc * (K * K);
        float s = 0.f;
        for (int r = 0; r < g.H; ++r) s += red[(pc * g.H + r) * (K * K) + t];
        ws[((size_t)part * g.C + c0 + pc) * (K * K) + t] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// Fused backward pass, 3x3, stride 2, pad 1, x row width W (template, even; H even): block mapping of
// the kernel above, one lane per (channel, dy row a).  The lane adds dy row a against x rows 2a-1,
// 2a, 2a+1 into its 9 partial sums and computes dx rows 2a and 2a+1 from dy rows a and a+1.  The dx
// rows stay in registers until every lane has read its x rows, then take the place of x in LDS and
// leave as one flat range: two staging areas instead of three, which is what lets a block of
// 28-wide planes keep ten channels.
// ---------------------------------------------------------------------------------------------
template <typename T, int W>
__global__ __launch_bounds__(256) void k_nchws_bwd_fused_s2(Geom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                            const T *__restrict__ w, T *__restrict__ dx,
                                                            float *__restrict__ ws, int U, int NI, int ncblocks,
                                                            unsigned nblocks, int nt)
{
    extern __shared__ float4 smem4[];
    constexpr int VE = ElemsS<T>::VE;
    constexpr int K = 3, WO = W / 2;
    const int HW = g.H * W, HoWo = g.Ho * WO;
    const unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int cblk = lb % ncblocks, part = lb / ncblocks;
    const int c0 = cblk * U, nc = min(U, g.C - c0);
    const int n0 = part * NI, n1 = min(g.N, n0 + NI);
    float *lx = reinterpret_cast<float *>(smem4);                 // x planes, then the dx planes
    float *ld = lx + ((U * HW + 2 * VE + 3) & ~3);

    const int p = threadIdx.x / g.Ho, a = threadIdx.x - p * g.Ho;
    const bool own = p < nc;
    const bool has_up = a > 0, has_b = a + 1 < g.Ho;
    float acc[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) acc[kh][kw] = 0.f;
    float wr[K][K];
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) wr[kh][kw] = ldf(w + ((c0 + min(p, nc - 1)) * K + kh) * K + kw);

    FlatRegs<T> rx, rd;
    {
        const int gx0 = (n0 * g.C + c0) * HW, gd0 = (n0 * g.C + c0) * HoWo;
        flat_issue<T>(x, g.N * g.C * HW, gx0, gx0 + nc * HW, rx);
        flat_issue<T>(dy, g.N * g.C * HoWo, gd0, gd0 + nc * HoWo, rd);
    }
    for (int n = n0; n < n1; ++n) {
        const int gx0 = (n * g.C + c0) * HW, gd0 = (n * g.C + c0) * HoWo;
        __syncthreads();                          // the previous image's dx has left the staging area
        flat_commit<T>(gx0, gx0 + nc * HW, rx, lx);
        flat_commit<T>(gd0, gd0 + nc * HoWo, rd, ld);
        __syncthreads();
        if (n + 1 < n1) {
            const int hx0 = ((n + 1) * g.C + c0) * HW, hd0 = ((n + 1) * g.C + c0) * HoWo;
            flat_issue<T>(x, g.N * g.C * HW, hx0, hx0 + nc * HW, rx);
            flat_issue<T>(dy, g.N * g.C * HoWo, hd0, hd0 + nc * HoWo, rd);
        }
        float o0[W], o1[W];                       // dx rows 2a and 2a+1
        if (own) {
            const float *xp = lx + (gx0 & (VE - 1)) + p * HW;
            const float *dp = ld + (gd0 & (VE - 1)) + p * HoWo;
            float A[WO + 1], B[WO + 1];           // dy rows a and a+1, a zero to their right
            const float *ra = dp + a * WO, *rb = dp + (has_b ? a + 1 : a) * WO;
#pragma unroll
            for (int j = 0; j < WO; ++j) { A[j] = ra[j]; const float t = rb[j]; B[j] = has_b ? t : 0.f; }
            A[WO] = 0.f; B[WO] = 0.f;
            // filter gradient: x rows 2a-1, 2a, 2a+1; dy column j meets x column 2j-1+kw
#pragma unroll
            for (int kh = 0; kh < K; ++kh) {
                const int ih = 2 * a - 1 + kh;
                const float *rp = xp + (kh == 0 && !has_up ? 0 : ih) * W;
                float row[W];
#pragma unroll
                for (int i = 0; i < W; ++i) { const float t = rp[i]; row[i] = (kh == 0 && !has_up) ? 0.f : t; }
#pragma unroll
                for (int kw = 0; kw < K; ++kw) {
                    float sacc = acc[kh][kw];
#pragma unroll
                    for (int j = 0; j < WO; ++j) {
                        const int iw = 2 * j - 1 + kw;
                        if (iw >= 0 && iw < W) sacc = fmaf(A[j], row[iw], sacc);
                    }
                    acc[kh][kw] = sacc;
                }
            }
            // input gradient (Eq. 3 at stride 2): rows 2a, 2a+1
#pragma unroll
            for (int b = 0; b < WO; ++b) {
                o0[2 * b] = wr[1][1] * A[b];
                o0[2 * b + 1] = fmaf(wr[1][0], A[b + 1], wr[1][2] * A[b]);
                o1[2 * b] = fmaf(wr[0][1], B[b], wr[2][1] * A[b]);
                o1[2 * b + 1] = fmaf(wr[0][0], B[b + 1], fmaf(wr[0][2], B[b], fmaf(wr[2][0], A[b + 1], wr[2][2] * A[b])));
            }
        }
        __syncthreads();                          // every lane has read its x rows
        if (own) {
            float *op = lx + (gx0 & (VE - 1)) + p * HW + (2 * a) * W;
#pragma unroll
            for (int i = 0; i < W; ++i) { op[i] = o0[i]; op[W + i] = o1[i]; }
        }
        __syncthreads();
        flat_store<T>(dx, gx0, gx0 + nc * HW, lx, nt != 0);
    }

    // rows of a channel are added in row order (fixed), through LDS
    __syncthreads();
    float *red = lx;     // 256 * 9 floats across the staging areas (the host sizes the LDS for it)
#pragma unroll
    for (int kh = 0; kh < K; ++kh)
#pragma unroll
        for (int kw = 0; kw < K; ++kw) red[threadIdx.x * (K * K) + kh * K + kw] = own ? acc[kh][kw] : 0.f;
    __syncthreads();
    for (int idx = threadIdx.x; idx < nc * K * K; idx += 256) {
        const int pc = idx / (K * K), t = idx - pc * (K * K);
        float sum = 0.f;
        for (int r = 0; r < g.Ho; ++r) sum += red[(pc * g.Ho + r) * (K * K) + t];
        ws[((size_t)part * g.C + c0 + pc) * (K * K) + t] = sum;
    }
}

// ---- host side --------------------------------------------------------------------------------

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Row widths with a compiled instance; the pass needs 3x3, pad 1, multiplier 1 and H small enough
// that one lane per output row fills a block with at least 8 planes.
bool nchws_supported(const Geom &g, int pass)
{
    if (g.m != 1) return false;
    const bool k3 = g.K == 3 && g.p == 1 && (g.s == 1 || g.s == 2);
    const bool k5 = g.K == 5 && g.p == 2 && g.s == 1;   // 5x5 stride 1 (backward-data runs the forward kernel with the rotated filter)
    if (!k3 && !k5) return false;
    if (!(g.W == 7 || g.W == 14 || g.W == 28 || (g.K == 3 && (g.W == 8 || (g.W == 4 && g.s == 1))))) return false;
    if (g.s == 2 && (g.W % 2 != 0 || g.H % 2 != 0)) return false;
    if (g.Ho > 32 || g.H > 32) return false;
    return true;
}

static int planes_per_block(const Geom &g) { return 256 / g.Ho; }

static size_t lds_bytes_for(int U, int in_plane, int out_plane, int ve)
{
    return (size_t)(((U * in_plane + 2 * ve + 3) & ~3) + U * out_plane + 2 * ve + 4) * sizeof(float);
}

template <typename T>
static hipError_t go_fwd(const Geom &g, const void *x, const void *w, void *y, bool flip, hipStream_t st, int cg = 1)
{
    constexpr int VE = ElemsS<T>::VE;
    int U = planes_per_block(g);
    if (cg > 1 && !(g.K == 3 && (g.s == 1 || (g.s == 2 && !flip && (g.W == 14 || g.W == 28))) &&
                    (g.W == 7 || g.W == 14 || g.W == 28) && g.C % cg == 0))
        return hipErrorInvalidValue;
    const int HW = g.H * g.W, HoWo = g.Ho * g.Wo;
    while (U > 1 && lds_bytes_for(U, HW, HoWo, VE) > 60 * 1024) --U;
    // a tile's planes must fit the register staging that lets the next tile load while this one is computed (8192
    // elements): the 28-wide stride-2 forward takes 10 planes per tile instead of 15 and is 13 % faster for it
    while (U > 1 && U * HW + VE > 8192) --U;
    if (const char *e = tune_env("DWCONV_TUNE_SU")) { if (atoi(e) >= 1 && atoi(e) < U) U = atoi(e); }
    if (cg > 1) { U -= U % cg; if (U < cg) return hipErrorInvalidValue; }       // whole groups per tile
    // outputs back into the input area when two areas would leave room for at most three blocks per CU
    bool inplace = g.W == 28 && lds_bytes_for(U, HW, HoWo, VE) > 40 * 1024;
    if (const char *e = tune_env("DWCONV_TUNE_SINPLACE")) inplace = g.W == 28 && atoi(e) != 0;
    const size_t lds = inplace ? lds_bytes_for(U, HW, 0, VE) : lds_bytes_for(U, HW, HoWo, VE);
    const int nplanes = g.N * g.C;
    const int ntiles = cdiv(nplanes, U);
    // tiles per block: two on large launches (measured against 1, 3 and 4 on the 14x14 and 7x7 layers at batch 128:
    // 3 to 10 % on the input gradient and the 7x7 forward; three tiles leave a short last round of blocks and lose)
    int tpb = ntiles >= 2048 ? 2 : 1;
    if (const char *e = tune_env("DWCONV_TUNE_STPB")) tpb = atoi(e);
    if (tpb < 1) tpb = 1;
    if (tpb > 8) tpb = 8;
    if (U * HW + VE > 8192) tpb = 0;            // too large for the register staging: one tile per block, loaded straight into LDS
    const unsigned nblocks = (unsigned)cdiv(ntiles, tpb > 0 ? tpb : 1);
    // the block writes one contiguous range with whole 16-byte vectors: streamed
    const int nt = stream_stores(flip ? "NCHW_SMALL_BWD" : "NCHW_SMALL_FWD", (long long)nplanes * HoWo * sizeof(T), 0);
#define GO(KK, SS, WW, FL, IP) hipLaunchKernelGGL((k_nchws_fwd<T, KK, SS, WW, FL, IP>), dim3(nblocks), dim3(256), lds, st, g, \
                                                  (const T *)x, (const T *)w, (T *)y, U, nplanes, nblocks, nt, tpb)
#define PICK(KK, SS, WW) if (g.K == KK && g.s == SS && g.W == WW && !inplace) { if (flip) GO(KK, SS, WW, true, false); else GO(KK, SS, WW, false, false); return hipGetLastError(); }
#define PICKIP(KK, SS, WW) if (g.K == KK && g.s == SS && g.W == WW && inplace) { if (flip) GO(KK, SS, WW, true, true); else GO(KK, SS, WW, false, true); return hipGetLastError(); }
#define GOG(WW, FL, IP, CGG) hipLaunchKernelGGL((k_nchws_fwd<T, 3, 1, WW, FL, IP, CGG>), dim3(nblocks), dim3(256), lds, st, g, \
                                                (const T *)x, (const T *)w, (T *)y, U, nplanes, nblocks, nt, tpb)
#define PICKG(WW, IP, CGG) if (cg == CGG && g.W == WW && inplace == IP) { if (flip) GOG(WW, true, IP, CGG); else GOG(WW, false, IP, CGG); return hipGetLastError(); }
#define PICKGW(CGG) PICKG(7, false, CGG) PICKG(14, false, CGG) PICKG(28, false, CGG) PICKG(28, true, CGG)
#define GOG2(WW, IP, CGG) hipLaunchKernelGGL((k_nchws_fwd<T, 3, 2, WW, false, IP, CGG>), dim3(nblocks), dim3(256), lds, st, g, \
                                             (const T *)x, (const T *)w, (T *)y, U, nplanes, nblocks, nt, tpb)
#define PICKG2(WW, IP, CGG) if (cg == CGG && g.W == WW && inplace == IP) { GOG2(WW, IP, CGG); return hipGetLastError(); }
#define PICKGW2(CGG) PICKG2(14, false, CGG) PICKG2(28, false, CGG) PICKG2(28, true, CGG)
    if (cg > 1 && g.s == 2) {
        PICKGW2(2) PICKGW2(4) PICKGW2(8)
        return hipErrorInvalidValue;
    }
    if (cg > 1) {
        PICKGW(2) PICKGW(4) PICKGW(8)
        return hipErrorInvalidValue;
    }
#undef PICKGW2
#undef PICKG2
#undef GOG2
#undef PICKGW
#undef PICKG
#undef GOG
    PICK(3, 1, 7) PICK(3, 1, 14) PICK(3, 1, 28) PICK(3, 2, 14) PICK(3, 2, 28) PICK(5, 1, 7) PICK(5, 1, 14) PICK(5, 1, 28)
    PICK(3, 1, 4) PICK(3, 1, 8) PICK(3, 2, 8)
    PICKIP(3, 1, 28) PICKIP(3, 2, 28) PICKIP(5, 1, 28)
#undef PICKIP
#undef PICK
#undef GO
    return hipErrorInvalidValue;
}

hipError_t nchws_fwd(const Geom &g, int dtype, const void *x, const void *w, void *y, bool flip, hipStream_t st)
{
    return dtype == DT_F32 ? go_fwd<float>(g, x, w, y, flip, st) : go_fwd<bf16_t>(g, x, w, y, flip, st);
}

// Group convolution on small planes: 3x3 stride 1 pad 1, cg = 2, 4 or 8 channels per group on both sides, rows of 7, 14 or 28.
bool nchws_group_supported(const Geom &g, int cg)
{
    if (!(g.K == 3 && g.p == 1 && g.m == 1 && (cg == 2 || cg == 4 || cg == 8) && g.C % cg == 0 && g.H <= 32)) return false;
    if (g.s == 1) return (g.W == 7 || g.W == 14 || g.W == 28) && 256 / g.H >= cg;
    // stride 2: even maps with rows of 14 or 28; a block has one lane per (plane, dy row)
    return g.s == 2 && (g.W == 14 || g.W == 28) && g.H % 2 == 0 && 256 / g.Ho >= cg;
}

hipError_t nchws_group_fwd(const Geom &g, int cg, int dtype, const void *x, const void *w, void *y, bool flip, hipStream_t st)
{
    if (!nchws_group_supported(g, cg)) return hipErrorInvalidValue;
    return dtype == DT_F32 ? go_fwd<float>(g, x, w, y, flip, st, cg) : go_fwd<bf16_t>(g, x, w, y, flip, st, cg);
}

template <typename T>
static hipError_t go_bwd_data_s2(const Geom &g, const void *dy, const void *w, void *dx, hipStream_t st, int cg = 1)
{
    constexpr int VE = ElemsS<T>::VE;
    int U = planes_per_block(g);
    const int HW = g.H * g.W, HoWo = g.Ho * g.Wo;
    while (U > 1 && lds_bytes_for(U, HoWo, HW, VE) > 60 * 1024) --U;
    if (cg > 1) { U -= U % cg; if (U < cg) return hipErrorInvalidValue; }       // whole groups per tile
    const size_t lds = lds_bytes_for(U, HoWo, HW, VE);
    const int nplanes = g.N * g.C;
    const unsigned nblocks = (unsigned)cdiv(nplanes, U);
    const int nt = stream_stores("NCHW_SMALL_BWD", (long long)nplanes * HW * sizeof(T), 0);
#define GO(WW) hipLaunchKernelGGL((k_nchws_bwd_data_s2<T, WW>), dim3(nblocks), dim3(256), lds, st, g, (const T *)dy, \
                                  (const T *)w, (T *)dx, U, nplanes, nblocks, nt)
#define GOG(WW, CGG) hipLaunchKernelGGL((k_nchws_bwd_data_s2<T, WW, CGG>), dim3(nblocks), dim3(256), lds, st, g, (const T *)dy, \
                                        (const T *)w, (T *)dx, U, nplanes, nblocks, nt)
#define PICKG(CGG) if (cg == CGG) { if (g.W == 14) GOG(14, CGG); else if (g.W == 28) GOG(28, CGG); else return hipErrorInvalidValue; \
                                    return hipGetLastError(); }
    if (cg > 1) {
        PICKG(2) PICKG(4) PICKG(8)
        return hipErrorInvalidValue;
    }
#undef PICKG
#undef GOG
    if (g.W == 14) GO(14);
    else if (g.W == 28) GO(28);
    else if (g.W == 8) GO(8);
    else return hipErrorInvalidValue;
#undef GO
    return hipGetLastError();
}

hipError_t nchws_bwd_data_s2(const Geom &g, int dtype, const void *dy, const void *w, void *dx, hipStream_t st)
{
    return dtype == DT_F32 ? go_bwd_data_s2<float>(g, dy, w, dx, st) : go_bwd_data_s2<bf16_t>(g, dy, w, dx, st);
}

hipError_t nchws_group_bwd_data_s2(const Geom &g, int cg, int dtype, const void *dy, const void *w, void *dx, hipStream_t st)
{
    if (!nchws_group_supported(g, cg) || g.s != 2) return hipErrorInvalidValue;
    return dtype == DT_F32 ? go_bwd_data_s2<float>(g, dy, w, dx, st, cg) : go_bwd_data_s2<bf16_t>(g, dy, w, dx, st, cg);
}

// planes (channels) per block and images per block for the filter gradient
void nchws_bwd_filter_tiling(const Geom &g, int dtype, int *U, int *NI, int *parts, int cg)
{
    const int ve = dtype == DT_F32 ? 4 : 8;
    int u = planes_per_block(g);
    if (u > g.C) u = g.C;
    const int HW = g.H * g.W, HoWo = g.Ho * g.Wo;
    while (u > 1 && lds_bytes_for(u, HW, HoWo, ve) > 60 * 1024) --u;
    // a block's planes of one image must fit the register staging of the loader (8192 elements per tensor)
    while (u > 1 && (u * HW + ve > 8192 || u * HoWo + ve > 8192)) --u;
    if (cg > 1 && u >= cg) u -= u % cg;            // group convolution: whole groups per block
    *U = u;
    // Images per block.  Planes of 14x14 and smaller: about 1000 blocks in the launch but at most four images per
    // block (a block that walks four images instead of one writes a quarter of the partial sums and pays the block
    // reduction once: 9 % on the 14x14 layers, a third on the 7x7 layer; eight measured slower again); larger planes:
    // about 2048 blocks
    const int ncb = cdiv(g.C, u);
    int ni = HW <= 196 ? (int)(((long long)g.N * ncb + 512) / 1024) : (int)(((long long)g.N * ncb) / 2048);
    if (HW <= 196 && ni > 4) ni = 4;
    if (ni < 1) ni = 1;
    if (ni > g.N) ni = g.N;
    *NI = ni;
    *parts = cdiv(g.N, ni);
}

template <typename T>
static hipError_t go_bwd_filter(const Geom &g, const void *x, const void *dy, float *ws, int U, int NI, hipStream_t st,
                                int cg = 1)
{
    constexpr int VE = ElemsS<T>::VE;
    const int HW = g.H * g.W, HoWo = g.Ho * g.Wo;
    size_t lds = lds_bytes_for(U, HW, HoWo, VE);
    if (lds < 256 * (size_t)(g.K * g.K) * sizeof(float)) lds = 256 * (size_t)(g.K * g.K) * sizeof(float);
    const int ncb = cdiv(g.C, U);
    const unsigned nblocks = (unsigned)ncb * cdiv(g.N, NI);
#define GO(KK, SS, WW) hipLaunchKernelGGL((k_nchws_bwd_filter<T, KK, SS, WW>), dim3(nblocks), dim3(256), lds, st, g, \
                                          (const T *)x, (const T *)dy, ws, U, NI, ncb, nblocks)
#define GOG(WW, CGG) hipLaunchKernelGGL((k_nchws_bwd_filter<T, 3, 1, WW, CGG>), dim3(nblocks), dim3(256), lds, st, g, \
                                        (const T *)x, (const T *)dy, ws, U, NI, ncb, nblocks)
#define GOG2(WW, CGG) hipLaunchKernelGGL((k_nchws_bwd_filter<T, 3, 2, WW, CGG>), dim3(nblocks), dim3(256), lds, st, g, \
                                         (const T *)x, (const T *)dy, ws, U, NI, ncb, nblocks)
#define PICKG(CGG) if (cg == CGG) { if (g.s == 2) { if (g.W == 14) GOG2(14, CGG); else if (g.W == 28) GOG2(28, CGG); else return hipErrorInvalidValue; } \
                                    else if (g.W == 7) GOG(7, CGG); else if (g.W == 14) GOG(14, CGG); else if (g.W == 28) GOG(28, CGG); \
                                    else return hipErrorInvalidValue; return hipGetLastError(); }
    if (cg > 1) {
        if (!(g.K == 3 && (g.s == 1 || g.s == 2)) || U % cg != 0) return hipErrorInvalidValue;
        PICKG(2) PICKG(4) PICKG(8) // groups of 8 only where the row-walk filter gradient cannot run (7-wide rows): it measured faster
        return hipErrorInvalidValue;
    }
#undef PICKG
#undef GOG2
#undef GOG
    if (g.K == 3 && g.s == 1 && g.W == 7) GO(3, 1, 7);
    else if (g.K == 3 && g.s == 1 && g.W == 14) GO(3, 1, 14);
    else if (g.K == 3 && g.s == 1 && g.W == 28) GO(3, 1, 28);
    else if (g.K == 3 && g.s == 2 && g.W == 14) GO(3, 2, 14);
    else if (g.K == 3 && g.s == 2 && g.W == 28) GO(3, 2, 28);
    else if (g.K == 5 && g.s == 1 && g.W == 7) GO(5, 1, 7);
    else if (g.K == 5 && g.s == 1 && g.W == 14) GO(5, 1, 14);
    else if (g.K == 5 && g.s == 1 && g.W == 28) GO(5, 1, 28);
    else if (g.K == 3 && g.s == 1 && g.W == 4) GO(3, 1, 4);
    else if (g.K == 3 && g.s == 1 && g.W == 8) GO(3, 1, 8);
    else if (g.K == 3 && g.s == 2 && g.W == 8) GO(3, 2, 8);
    else return hipErrorInvalidValue;
#undef GO
    return hipGetLastError();
}

hipError_t nchws_bwd_filter(const Geom &g, int dtype, const void *x, const void *dy, float *ws, int U, int NI,
                            hipStream_t st)
{
    return dtype == DT_F32 ? go_bwd_filter<float>(g, x, dy, ws, U, NI, st) : go_bwd_filter<bf16_t>(g, x, dy, ws, U, NI, st);
}

hipError_t nchws_group_bwd_filter(const Geom &g, int cg, int dtype, const void *x, const void *dy, float *ws, int U, int NI,
                                  hipStream_t st)
{
    if (!nchws_group_supported(g, cg)) return hipErrorInvalidValue;
    return dtype == DT_F32 ? go_bwd_filter<float>(g, x, dy, ws, U, NI, st, cg) : go_bwd_filter<bf16_t>(g, x, dy, ws, U, NI, st, cg);
}

// Fused backward on small planes: tiling of the filter gradient, with U bounded by the three LDS areas.
bool nchws_bwd_fused_supported(const Geom &g)
{
    if (!(nchws_supported(g, 2) && g.K == 3 && g.p == 1 && g.m == 1)) return false;
    if (g.s == 1) return true;                      // 28-wide rows with the dx planes in x's LDS area
    return g.W == 28 || g.W == 14 || g.W == 8;      // stride 2 (even H and W by nchws_supported)
}

static size_t lds_bytes_fused(int U, int plane, int ve, int areas = 3)
{
    const size_t area = (size_t)((U * plane + 2 * ve + 3) & ~3);
    size_t b = ((size_t)areas * area + 4) * sizeof(float);
    return b < 256 * 9 * sizeof(float) ? 256 * 9 * sizeof(float) : b;
}
// stride 2: the x area (which the dx planes reuse) and the dy area
static size_t lds_bytes_fused_s2(int U, int in_plane, int out_plane, int ve)
{
    const size_t b = lds_bytes_for(U, in_plane, out_plane, ve);
    return b < 256 * 9 * sizeof(float) ? 256 * 9 * sizeof(float) : b;
}

void nchws_bwd_fused_tiling(const Geom &g, int dtype, int *U, int *NI, int *parts)
{
    nchws_bwd_filter_tiling(g, dtype, U, NI, parts);       // U within the LDS and register staging of x and dy
    const int ve = dtype == DT_F32 ? 4 : 8;
    if (g.s == 1)
        while (*U > 1 && lds_bytes_fused(*U, g.H * g.W, ve, g.W == 28 ? 2 : 3) > 60 * 1024) --*U;
    const int ncb = cdiv(g.C, *U);
    int ni = (int)(((long long)g.N * ncb) / 2048);
    if (ni < 1) ni = 1;
    if (ni > g.N) ni = g.N;
    *NI = ni;
    *parts = cdiv(g.N, ni);
}

template <typename T>
static hipError_t go_bwd_fused(const Geom &g, const void *x, const void *dy, const void *w, void *dx, float *ws, int U,
                               int NI, hipStream_t st)
{
    constexpr int VE = ElemsS<T>::VE;
    const size_t lds = g.s == 1 ? lds_bytes_fused(U, g.H * g.W, VE, g.W == 28 ? 2 : 3)
                                : lds_bytes_fused_s2(U, g.H * g.W, g.Ho * g.Wo, VE);
    const int ncb = cdiv(g.C, U);
    const unsigned nblocks = (unsigned)ncb * cdiv(g.N, NI);
    const int nt = stream_stores("NCHW_SMALL_BWD", (long long)g.N * g.C * g.H * g.W * sizeof(T), 0);
    if (g.s == 2) {
        if (U * g.Ho > 256 || U * g.H * g.W + VE > 8192 || lds > 64 * 1024) return hipErrorInvalidValue;
#define GO2(WW) hipLaunchKernelGGL((k_nchws_bwd_fused_s2<T, WW>), dim3(nblocks), dim3(256), lds, st, g, (const T *)x, \
                                   (const T *)dy, (const T *)w, (T *)dx, ws, U, NI, ncb, nblocks, nt)
        if (g.W == 28) GO2(28);
        else if (g.W == 14) GO2(14);
        else if (g.W == 8) GO2(8);
        else return hipErrorInvalidValue;
#undef GO2
        return hipGetLastError();
    }
#define GO(WW, IP) hipLaunchKernelGGL((k_nchws_bwd_fused<T, WW, IP>), dim3(nblocks), dim3(256), lds, st, g, (const T *)x, \
                                      (const T *)dy, (const T *)w, (T *)dx, ws, U, NI, ncb, nblocks, nt)
    if (g.W == 14) GO(14, false);
    else if (g.W == 7) GO(7, false);
    else if (g.W == 8) GO(8, false);
    else if (g.W == 4) GO(4, false);
    else if (g.W == 28) { if (U * g.H > 256 || lds > 64 * 1024) return hipErrorInvalidValue; GO(28, true); }
    else return hipErrorInvalidValue;
#undef GO
    return hipGetLastError();
}

hipError_t nchws_bwd_fused(const Geom &g, int dtype, const void *x, const void *dy, const void *w, void *dx, float *ws,
                           int U, int NI, hipStream_t st)
{
    if (!nchws_bwd_fused_supported(g)) return hipErrorInvalidValue;
    return dtype == DT_F32 ? go_bwd_fused<float>(g, x, dy, w, dx, ws, U, NI, st)
                           : go_bwd_fused<bf16_t>(g, x, dy, w, dx, ws, U, NI, st);
}

}  // namespace dwc
