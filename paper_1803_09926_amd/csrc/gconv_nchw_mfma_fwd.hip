// Group convolution, NCHW, 3x3 stride 1 pad 1: forward (Eq. 2 with the sum over a group's input channels) and
// backward-data (Eq. 3) on the matrix cores, for 4 or 8 channels per group on both sides and 14x14, 28x28 or 56x56 planes, and
// for 2 channels per group on 112x112 planes.
//
// y[o][p] = sum over (b, tap) of w[o][b][tap] * x[b][p + tap] is a matrix product with the output channels as rows and
// the pixels as columns.  In a 4x4 matrix instruction a block of four lanes is four consecutive pixels of a row: the
// lane's A operand is the filter entry of ITS output channel of the quad (a register that never changes), its B
// operand the input value at ITS pixel, and D[i][j] (register i of lane j) collects y[output channel i][pixel j].
// fp32: one (input channel, tap) per instruction (4x4x1).  bf16: the inner dimension of 4x4x4 is four input channels,
// the lane packs its pixel's four values (read one by one from the channel planes) into two registers.
//
// The block stages eight consecutive input channels (one group of 8, two groups of 4, four groups of 2) of one "fill"
// in LDS exactly as the filter gradient does (gconv_nchw_mfma.hip: flat 16-byte loads one or two fills ahead in
// registers, a gap of zeros after each row, zero rows at the plane's edge), and the eight output planes of the fill in
// a second LDS area, written back as flat 16-byte stores.  A fill is an image (28x28), four images as a 2 x 2 mosaic of
// that geometry (14x14), or a strip of rows with the rows above and below it (56x56: 14 rows; 112x112: 14 rows in
// bf16, 7 in fp32).  A wavefront owns one output quad and half of the fill's pixels; its lanes are the pixels of a
// row and its gap (28-wide: two rows side by side; 112-wide: half a row, the neighbour pixels then come from LDS), and
// it walks the input rows downwards: an input row adds to three output rows (three accumulators that change roles),
// the pixel to the left and right comes from the neighbour lanes by a lane permute, and an output row leaves for LDS
// when its last input row is done.  With two channels per group a quad is two groups and the lane's filter entries
// for the other group's planes are zero (a block-diagonal 4x4 tile).  Backward-data is the same walk over dy with the
// filter transposed within the group and the taps reversed.
#include "gconv_mfma.hpp"

namespace dwc {

template <typename T, int CG, int W, int H, bool FLIP>
__global__ __launch_bounds__(256) void k_gconv_nchws_mfma_fwd(GGeom g, const T *__restrict__ in, const T *__restrict__ w,
                                                              T *__restrict__ out, int parts, int nfills, unsigned nblocks)
{
    using L = PlaneFill<W, H, (int)sizeof(T)>;
    static_assert(CG == 2 || CG == 4 || CG == 8, "groups of 2, 4 or 8");
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int CPV = F32 ? 1 : 2;                // four-pixel vectors of a 16-byte chunk
    constexpr int XCH = 8 * L::XROWS * L::VPR / CPV, YCH = 8 * L::RS * L::VPR / CPV;     // chunks of a fill
    constexpr int XPASS = (XCH + 255) / 256, YPASS = (YCH + 255) / 256;
    constexpr int AREA_Y = L::MOSAIC ? 4 * 8 * H * W : 8 * L::RS * W;       // output planes of the fill, rows packed (mosaic: image after image)
    constexpr int EPC = 4 * CPV, CPI = XCH / 4;    // elements of a chunk; mosaic: chunks of one image's eight planes
    constexpr int LEAD = 16 / (int)sizeof(T);       // zeros before the first plane: the pixel left of its first one
    __shared__ __align__(16) T lds_all[LEAD + L::AREA_X + AREA_Y];
    T *lds = lds_all + LEAD;
    // fills ahead in registers; fp32 strips: one (two would leave registers for one wavefront per SIMD only)
    constexpr int DEPTH = (F32 && L::STRIP) ? 1 : 2;

    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int part = lb % parts, cb = lb / parts;   // cb: the block's channel octet
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    T *ylds = lds + L::AREA_X;

    for (int i = tid; i < (LEAD + L::AREA_X) * (int)sizeof(T) / 16; i += 256) reinterpret_cast<u4raw_t *>(lds_all)[i] = u4raw_t{0u, 0u, 0u, 0u};

    struct Where { int plane, row, cv; };
    auto where = [](int v, int rows) { Where q; q.plane = v / (rows * L::VPR); const int rem = v % (rows * L::VPR); q.row = rem / L::VPR; q.cv = rem % L::VPR; return q; };

    // DEPTH fills ahead in registers; every load is issued unconditionally (see the filter gradient)
    struct Stage { u4raw_t x[XPASS]; uint32_t xok; };
    auto gload = [&](Stage &s, int f) {
        const int ff = f < nfills ? f : part;
        const int n = ff / L::NSTRIP, r0 = (ff % L::NSTRIP) * L::RS;
        const T *xs = in + ((size_t)n * g.C + (size_t)cb * 8) * (H * W);
        s.xok = 0xffffffffu;
#pragma unroll
        for (int p = 0; p < XPASS; ++p) {
            const int q = min(p * 256 + tid, XCH - 1);
            if constexpr (L::MOSAIC) {
                // four images per fill, each image's eight planes one flat range (a batch that is not a multiple of four
                // repeats its last image; those outputs are not stored)
                const int ni = min(ff * 4 + q / CPI, g.N - 1);
                s.x[p] = *reinterpret_cast<const u4raw_t *>(in + ((size_t)ni * g.C + (size_t)cb * 8) * (H * W) + (size_t)(q % CPI) * EPC);
            } else if constexpr (L::STRIP) {
                const Where wq = where(q * CPV, L::XROWS);
                const int rg = r0 - 1 + wq.row;
                if (rg < 0 || rg >= H) s.xok &= ~(1u << p);
                s.x[p] = *reinterpret_cast<const u4raw_t *>(xs + (size_t)wq.plane * (H * W) + min(max(rg, 0), H - 1) * W + wq.cv * 4);
            } else {
                s.x[p] = *reinterpret_cast<const u4raw_t *>(xs + (size_t)q * (4 * CPV));
            }
        }
    };
    auto lstore = [&](const Stage &s) {
#pragma unroll
        for (int p = 0; p < XPASS; ++p) {
            const int q = p * 256 + tid;
            if ((p + 1) * 256 <= XCH || q < XCH) {
                const bool ok = (s.xok >> p) & 1u;
                const u4raw_t v = {ok ? s.x[p].x : 0u, ok ? s.x[p].y : 0u, ok ? s.x[p].z : 0u, ok ? s.x[p].w : 0u};
                constexpr int RSH = L::STRIP ? 0 : 1;
                if constexpr (L::MOSAIC) {
                    // rows of 14 are not whole chunks: element by element (plane, row, column of its image; the image's
                    // place in the mosaic)
                    const int a4 = q / CPI, e0 = (q % CPI) * EPC;
                    const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int k = 0; k < EPC; ++k) {
                        const int e = e0 + k, plane = e / (H * W), rem = e % (H * W);
                        T *dst = lds + plane * L::PPX + ((a4 >> 1) * 16 + 1 + rem / W) * L::WP + (a4 & 1) * 16 + rem % W;
                        if constexpr (F32) *dst = __uint_as_float(wd[k]);
                        else *dst = (T)(wd[k >> 1] >> ((k & 1) * 16));
                    }
                } else if constexpr (F32) {
                    const Where wq = where(q, L::XROWS);
                    *reinterpret_cast<u4raw_t *>(lds + wq.plane * L::PPX + (wq.row + RSH) * L::WP + wq.cv * 4) = v;
                } else {
                    const Where w0 = where(2 * q, L::XROWS), w1 = where(2 * q + 1, L::XROWS);
                    *reinterpret_cast<u2raw_t *>(lds + w0.plane * L::PPX + (w0.row + RSH) * L::WP + w0.cv * 4) = u2raw_t{v.x, v.y};
                    *reinterpret_cast<u2raw_t *>(lds + w1.plane * L::PPX + (w1.row + RSH) * L::WP + w1.cv * 4) = u2raw_t{v.z, v.w};
                }
            }
        }
    };
    // the fill's output planes: LDS (rows packed, plane after plane) -> global, 16 bytes per lane
    auto ystore = [&](int f) {
        const int n = f / L::NSTRIP, r0 = (f % L::NSTRIP) * L::RS;
        T *ys = out + ((size_t)n * g.C + (size_t)cb * 8) * (H * W);
#pragma unroll
        for (int p = 0; p < YPASS; ++p) {
            const int q = p * 256 + tid;
            if ((p + 1) * 256 <= YCH || q < YCH) {
                const u4raw_t v = *reinterpret_cast<const u4raw_t *>(ylds + (size_t)q * (4 * CPV));
                if constexpr (L::MOSAIC) {
                    const int ni = f * 4 + q / CPI;
                    if (ni < g.N) *reinterpret_cast<u4raw_t *>(out + ((size_t)ni * g.C + (size_t)cb * 8) * (H * W) + (size_t)(q % CPI) * EPC) = v;
                } else if constexpr (L::STRIP) {
                    const Where wq = where(q * CPV, L::RS);
                    *reinterpret_cast<u4raw_t *>(ys + (size_t)wq.plane * (H * W) + (r0 + wq.row) * W + wq.cv * 4) = v;
                } else {
                    *reinterpret_cast<u4raw_t *>(ys + (size_t)q * (4 * CPV)) = v;
                }
            }
        }
    };

    // The wavefront's task: one output quad of the octet and half of the fill's pixels.  Rows of up to 64 lanes (pixels and
    // the gap after them): SPW streams side by side, the upper or the lower half of the fill's rows.  Rows of 128 lanes: the
    // left or the right half of every row.
    constexpr int LPS = L::WP;                        // lanes of a row
    constexpr bool WIDE = LPS > 64;
    constexpr int RPS = WIDE ? L::RS : L::RS / 2 / (WIDE ? 1 : L::SPW);          // output rows of a stream
    static_assert(WIDE || L::RS % (2 * L::SPW) == 0, "whole streams");
    const int oq = wv & 1, half = wv >> 1;            // oq: the output quad of the octet
    const int col = WIDE ? half * 64 + lane : lane % LPS;
    const int row0 = WIDE ? 0 : half * (L::RS / 2) + (lane / LPS) * RPS;         // the stream's first output row within the fill
    const bool colok = L::MOSAIC ? (col & 15) < W : col < W;
    // Neighbour pixels.  Narrow rows: from the lanes one below and one above by a lane permute; lane 0 has none to its left
    // and starts a row (zero), every other stream start has the previous stream's gap there (zero), and a row's last pixel
    // has its own gap.  Wide rows: read from LDS like the pixel itself (the element before a row is the previous row's gap).
    const int up = ((lane - 1) & 63) * 4, dn = ((lane + 1) & 63) * 4;
    const uint32_t lmask = lane == 0 ? 0u : 0xffffffffu;
    // The quad's input planes.  Groups of 8: the whole octet.  Groups of 4: the quad's own four planes.  Groups of 2: the
    // quad is two groups, its four planes are their inputs, and a lane's filter entries for the other group's planes are
    // zero (a block-diagonal 4x4 filter tile).
    constexpr int CI = CG == 8 ? 8 : 4;
    const int cin0 = CG == 8 ? 0 : oq * 4;            // first input plane within the octet
    const T *xpl = lds + cin0 * L::PPX + L::xrow(row0) * L::WP + col;
    // output planes in LDS: plane pitch YPP, row pitch W (mosaic: the lane's image first)
    constexpr int YPP = L::MOSAIC ? H * W : L::RS * W;
    T *ypl = L::MOSAIC ? ylds + ((row0 / 14) * 2 + (col >> 4)) * (8 * H * W) + (oq * 4) * YPP + (row0 % 14) * W + (col & 15)
                       : ylds + (oq * 4) * YPP + row0 * W + col;

    // The lane's filter entries: output channel i = lane & 3 of the quad, every input plane of the quad, every tap.
    // Forward: w[o][b][tap].  Backward-data: the output of this pass is x's channel, the input dy's: w[b][o][8 - tap].
    const int li = lane & 3;
    const int grp = CG == 8 ? cb : CG == 4 ? cb * 2 + oq : cb * 4 + oq * 2 + li / 2;
    const int oi = CG == 8 ? oq * 4 + li : CG == 4 ? li : li % 2;     // the lane's output channel within its group
    float wf[F32 ? CI * 9 : 1];
    uint32_t wb[F32 ? 1 : (CI / 4) * 9 * 2];
#pragma unroll
    for (int b = 0; b < CI; ++b)
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int bg = CG == 2 ? b % 2 : b;                       // the plane's channel within the lane's group
            const bool mine = CG != 2 || b / 2 == li / 2;             // ... if it is one of that group's
            const size_t idx = !FLIP ? (((size_t)grp * CG + oi) * CG + bg) * 9 + tap : (((size_t)grp * CG + bg) * CG + oi) * 9 + (8 - tap);
            if constexpr (F32) {
                const float v = w[idx];
                wf[b * 9 + tap] = mine ? v : 0.f;
            } else {
                const uint32_t v = w[idx];
                const uint32_t hw = mine ? v : 0u;
                uint32_t &dst = wb[((b / 4) * 9 + tap) * 2 + (b % 4) / 2];
                if (b % 2 == 0) dst = hw; else dst |= hw << 16;
            }
        }

    v4f_t acc[3];

    auto fill = [&](Stage &s, int f) {
        lstore(s);
        __syncthreads();
        gload(s, f + DEPTH * parts);
        // input row t (relative to the stream's first output row) adds tap row kh to output row t + 1 - kh
#pragma unroll
        for (int t = -1; t <= RPS; ++t) {
            v4f_t &a0 = acc[(t + 4) % 3], &a1 = acc[(t + 3) % 3], &a2 = acc[(t + 2) % 3];     // output rows t+1, t, t-1
            const bool k0 = t + 1 < RPS, k1 = t >= 0 && t < RPS, k2 = t - 1 >= 0;
            if (k0) a0 = v4f_t{0.f, 0.f, 0.f, 0.f};                                             // output row t+1 starts here
            if constexpr (F32) {
#pragma unroll
                for (int b = 0; b < CI; ++b) {
                    const float *px = xpl + b * L::PPX + t * L::WP;
                    const uint32_t c = __float_as_uint(px[0]);
                    float X[3];
                    X[1] = __uint_as_float(c);
                    if constexpr (WIDE) {
                        X[0] = px[-1]; X[2] = px[1];
                    } else {
                        X[0] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)c) & lmask);
                        X[2] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)c));
                    }
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        if (k0) a0 = __builtin_amdgcn_mfma_f32_4x4x1f32(wf[b * 9 + kw], X[kw], a0, 0, 0, 0);
                        if (k1) a1 = __builtin_amdgcn_mfma_f32_4x4x1f32(wf[b * 9 + 3 + kw], X[kw], a1, 0, 0, 0);
                        if (k2) a2 = __builtin_amdgcn_mfma_f32_4x4x1f32(wf[b * 9 + 6 + kw], X[kw], a2, 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int bq = 0; bq < CI / 4; ++bq) {
                    const T *px = xpl + (bq * 4) * L::PPX + t * L::WP;
                    auto four = [&](int d) {          // the quad's four channels at the pixel d columns away
                        const uint32_t c0 = px[d], c1 = px[L::PPX + d], c2 = px[2 * L::PPX + d], c3 = px[3 * L::PPX + d];
                        return u2w_t{c0 | (c1 << 16), c2 | (c3 << 16)};
                    };
                    u2w_t X[3];
                    X[1] = four(0);
                    if constexpr (WIDE) {
                        X[0] = four(-1); X[2] = four(1);
                    } else {
                        X[0] = u2w_t{(uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)X[1].x) & lmask, (uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)X[1].y) & lmask};
                        X[2] = u2w_t{(uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)X[1].x), (uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)X[1].y)};
                    }
#pragma unroll
                    for (int kw = 0; kw < 3; ++kw) {
                        const v4s_t bv = __builtin_bit_cast(v4s_t, X[kw]);
                        auto A = [&](int tap) { return __builtin_bit_cast(v4s_t, u2w_t{wb[(bq * 9 + tap) * 2], wb[(bq * 9 + tap) * 2 + 1]}); };
                        if (k0) a0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(A(kw), bv, a0, 0, 0, 0);
                        if (k1) a1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(A(3 + kw), bv, a1, 0, 0, 0);
                        if (k2) a2 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(A(6 + kw), bv, a2, 0, 0, 0);
                    }
                }
            }
            if (k2 && colok) {                              // output row t-1 is complete
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (F32) ypl[i * YPP + (t - 1) * W] = a2[i];
                    else ypl[i * YPP + (t - 1) * W] = f32_to_bf16(a2[i]);
                }
            }
        }
        __syncthreads();                               // the input rows are free, the output planes complete
        ystore(f);
    };

    Stage sa, sb;
    int f = part;
    gload(sa, f);                                      // part < parts <= nfills
    if constexpr (DEPTH == 2) gload(sb, f + parts);
    __syncthreads();                                   // the zeros are in place
    if constexpr (DEPTH == 2) {
        while (f < nfills) {
            fill(sa, f);
            f += parts;
            if (f >= nfills) break;
            fill(sb, f);
            f += parts;
        }
    } else {
        for (; f < nfills; f += parts) fill(sa, f);
    }
}

// ---- host side ---------------------------------------------------------------------------------------------

bool gconv_nchws_mfma_fwd_supported(const GGeom &g)
{
    if (tune_env("DWCONV_TUNE_GNOSMMF")) return false;
    if (!(g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && g.C % 8 == 0)) return false;
    if (g.H == 112 && g.W == 112) return g.Cg == 2 && !tune_env("DWCONV_TUNE_GNOSMMF112");
    return ((g.H == 14 && g.W == 14) || (g.H == 28 && g.W == 28) || (g.H == 56 && g.W == 56)) && (g.Cg == 4 || g.Cg == 8);
}

hipError_t gconv_nchws_mfma_fwd(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st)
{
    if (!gconv_nchws_mfma_fwd_supported(g)) return hipErrorInvalidValue;
    // fills (images, or 14-row strips of 56x56 images) dealt to about 512 blocks, all resident at once
    int target = 512;
    if (const char *e = tune_env("DWCONV_TUNE_GSMFBLOCKS")) if (atoi(e) > 0) target = atoi(e);
    const int octets = g.C / 8, nf = g.W == 14 ? (g.N + 3) / 4 : g.N * (g.W == 56 ? 4 : g.W == 112 ? (dtype == DT_F32 ? 16 : 8) : 1);
    int p = (target + octets - 1) / octets;
    if (p > nf) p = nf;
    if (p < 1) p = 1;
    const int per = (nf + p - 1) / p;
    const int bpo = (nf + per - 1) / per;
    const unsigned nblocks = (unsigned)octets * (unsigned)bpo;
#define GO3(T, CGG, WW, FL) hipLaunchKernelGGL((k_gconv_nchws_mfma_fwd<T, CGG, WW, WW, FL>), dim3(nblocks), dim3(256), 0, st, g, (const T *)in, \
                                               (const T *)w, (T *)out, bpo, nf, nblocks)
#define GO2(T, CGG, WW) do { if (flip) GO3(T, CGG, WW, true); else GO3(T, CGG, WW, false); } while (0)
#define GO1(T, CGG) do { if (g.W == 14) GO2(T, CGG, 14); else if (g.W == 28) GO2(T, CGG, 28); else GO2(T, CGG, 56); } while (0)
    if (g.W == 112) { if (dtype == DT_F32) GO2(float, 2, 112); else GO2(bf16_t, 2, 112); }
    else if (dtype == DT_F32) { if (g.Cg == 8) GO1(float, 8); else GO1(float, 4); }
    else                      { if (g.Cg == 8) GO1(bf16_t, 8); else GO1(bf16_t, 4); }
#undef GO1
#undef GO2
#undef GO3
    return hipGetLastError();
}

}  // namespace dwc
