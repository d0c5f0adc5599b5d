// Group convolution, NCHW, 3x3 stride 1 pad 1: filter gradient (Eq. 4 with the sum over a group's channel pairs) on the
// matrix cores, for 4 or 8 channels per group on both sides and 28x28 or 56x56 planes, and for 2 channels per group
// on 112x112 planes; the same kernel can be fed from NHWC tensors (template switch).
//
// Per pixel a group of 8 needs 8*8*9 multiply-adds for 16 loaded values: on the vector ALU this pass is bound by
// arithmetic (about a third of the memory rate).  The sum over pixels is a matrix product dW[o][b][tap] =
// sum_p dy[o][p] * x[b][p + tap], and the 4x4 matrix instructions compute 16 independent 4x4 products per
// wavefront: a block of four lanes holds four channels at one pixel position (fp32: one pixel, 4x4x1; bf16: four
// consecutive pixels of a row as the four-element inner dimension, 4x4x4, exactly the 8 bytes a lane reads from
// its plane).  A = the dy values of the lane's output channel, B = the x values of the lane's input channel at the
// tap's offset, D[i][j] (register i of lane j) = the sum for (output channel i, input channel j) of the quad pair.
//
// A thread block works on eight consecutive channels (one group of 8, two groups of 4, four groups of 2) of one
// "fill" at a time: an image (28x28) or a strip of rows of an image (56x56: 14 rows; 112x112: 14 rows in bf16, 7 in
// fp32).  The eight x planes and eight dy planes come in as 16-byte loads (28x28: one flat range, the planes being
// contiguous in NCHW), one or two fills ahead in registers, and are laid out in LDS with a gap of zeros after every
// row and the rows above and below in place (zeros at the plane's edge), so every tap's operand is an unconditional
// LDS read at a constant offset from the position (the padding supplies the zeros of Eq. 4's border).
//
// A wavefront's 16 positions (4 pixels each) are streams of rows: 28-wide, two streams of eight (the seven vectors of
// a row and the gap after it, where dy is zero); 56-wide, one stream of 16; 112-wide, half a row (the row's two halves
// go to two wavefronts).  A stream walks down its rows and keeps the three x rows of the taps in registers: a step
// reads one new x row and one dy row from LDS; the one pixel left and right of a position's four is the neighbour
// lane's vector, fetched by a lane permute instead of a second LDS read (single-word reads at a stride of four words
// use a quarter of the banks); on 112-wide rows the wavefront's first and last position read theirs from LDS.
// Groups of 8: the four wavefronts take the four (input quad, output quad) pairs and all rows of the fill, 9
// accumulators each.  Groups of 4: two wavefronts per group, the upper and the lower half of the rows (two partial
// sums per block).  Groups of 2: a quad is two groups, two wavefronts per quad (left and right half of the rows), and
// only the sums of channel pairs of the same group are written.  At the end a wavefront adds its 16 blocks with a
// shuffle butterfly and writes its entries of the block's partial; the shared second stage adds the partials in a
// fixed order.
//
// NHWC feed: the block's eight channels of a pixel are 16 contiguous bytes (fp32: 32); they are loaded as such and
// scattered to their planes in LDS one element each; everything after that is unchanged, and the partial sums are
// written in the NHWC filter's layout.
#include "gconv_mfma.hpp"

namespace dwc {

template <typename T, int CG, int W, int H, bool NHWC>
__global__ __launch_bounds__(256) void k_gconv_nchws_mfma_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                     float *__restrict__ ws, int parts, int nfills, unsigned nblocks,
                                                                     int J)
{
    using L = PlaneFill<W, H, (int)sizeof(T)>;
    static_assert(CG == 2 || CG == 4 || CG == 8, "groups of 2, 4 or 8");
    constexpr bool WIDE = L::WP > 64;               // a row's 32 positions span two wavefronts
    // dy rows: with the gap of zeros after each row, or (wide rows, to fit LDS) packed, the gap positions zeroed when read
    constexpr int DROW = WIDE ? W : L::WP, PPD = WIDE ? L::RS * W : L::PPD, AREA_D = 8 * PPD;
    constexpr int LEAD = 16 / (int)sizeof(T);       // zeros before the first plane: the pixel left of its first one
    // fills ahead in registers; fp32 strips and wide rows: one (two would leave registers for one wavefront per SIMD only)
    constexpr int DEPTH = ((L::STRIP && (sizeof(T) == 4 || WIDE)) || (L::MOSAIC && sizeof(T) == 4)) ? 1 : 2;
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int CPV = F32 ? 1 : 2;                // four-pixel vectors of a 16-byte chunk
    constexpr int HPP = F32 ? 2 : 1;                // NHWC: 16-byte chunks of a pixel's eight channels
    constexpr int EPC = 4 * CPV;                    // elements of a chunk
    constexpr int XCH = 8 * L::XROWS * L::VPR / CPV, DCH = 8 * L::RS * L::VPR / CPV;     // chunks of a fill
    constexpr int XPASS = (XCH + 255) / 256, DPASS = (DCH + 255) / 256;
    __shared__ __align__(16) T lds_all[LEAD + L::AREA_X + AREA_D];    // x planes, then dy planes
    T *lds = lds_all + LEAD;

    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    // cb: the block's channel octet.  NHWC: the octets of one image run side by side (they share its cache lines)
    const int part = NHWC ? lb / (g.C / 8) : lb % parts, cb = NHWC ? lb % (g.C / 8) : lb / parts;
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);

    for (int i = tid; i < (LEAD + L::AREA_X + AREA_D) * (int)sizeof(T) / 16; i += 256) reinterpret_cast<u4raw_t *>(lds_all)[i] = u4raw_t{0u, 0u, 0u, 0u};

    // where four-pixel vector v of a fill's x (dy) rows lives: plane, row within the loaded rows, vector within the row
    struct Where { int plane, row, cv; };
    auto where = [](int v, int rows) { Where q; q.plane = v / (rows * L::VPR); const int rem = v % (rows * L::VPR); q.row = rem / L::VPR; q.cv = rem % L::VPR; return q; };

    // DEPTH fills ahead in registers.  Every load is issued unconditionally (lanes past the end of the last pass and
    // blocks past their last fill repeat a valid address and drop the result; a row outside the plane reads the
    // nearest row inside and is zeroed on its way to LDS): the number of loads in flight is then the same on every
    // path, and the wait before a fill's LDS writes covers that fill's loads only.
    struct Stage { u4raw_t x[XPASS], d[DPASS]; uint32_t xok; };      // xok: per pass, the x chunk is inside the plane (mosaic: the dy chunk's image exists)
    auto gload = [&](Stage &s, int f) {
        const int ff = f < nfills ? f : part;
        const int n = ff / L::NSTRIP, r0 = (ff % L::NSTRIP) * L::RS;
        const T *xs = x + ((size_t)n * g.C + (size_t)cb * 8) * (H * W);
        const T *ds = dy + ((size_t)n * g.O + (size_t)cb * 8) * (H * W);
        s.xok = 0xffffffffu;
        if constexpr (L::MOSAIC) {
            // four images per fill, each image's eight planes one flat range; past the end of the batch the last image is
            // read again and its dy dropped
            static_assert(!NHWC && XCH == DCH, "mosaic fills are NCHW, x and dy of one shape");
            constexpr int CPI = XCH / 4;
#pragma unroll
            for (int p = 0; p < XPASS; ++p) {
                const int q = min(p * 256 + tid, XCH - 1), ni = ff * 4 + q / CPI;
                if (ni >= g.N) s.xok &= ~(1u << p);
                const size_t off = ((size_t)min(ni, g.N - 1) * g.C + (size_t)cb * 8) * (H * W) + (size_t)(q % CPI) * EPC;
                s.x[p] = *reinterpret_cast<const u4raw_t *>(x + off);
                s.d[p] = *reinterpret_cast<const u4raw_t *>(dy + off);
            }
            return;
        }
        if constexpr (NHWC) {
            // a chunk is one pixel's eight channels (fp32: four of them): 16 bytes every C elements
#pragma unroll
            for (int p = 0; p < XPASS; ++p) {
                const int q = min(p * 256 + tid, XCH - 1), pq = q / HPP, hs = q % HPP;
                const int rg = (L::STRIP ? r0 - 1 : 0) + pq / W;
                if (rg < 0 || rg >= H) s.xok &= ~(1u << p);
                s.x[p] = *reinterpret_cast<const u4raw_t *>(x + (((size_t)n * H + min(max(rg, 0), H - 1)) * W + pq % W) * g.C + cb * 8 + hs * 4);
            }
#pragma unroll
            for (int p = 0; p < DPASS; ++p) {
                const int q = min(p * 256 + tid, DCH - 1), pq = q / HPP, hs = q % HPP;
                s.d[p] = *reinterpret_cast<const u4raw_t *>(dy + (((size_t)n * H + r0 + pq / W) * W + pq % W) * g.O + cb * 8 + hs * 4);
            }
            return;
        }
#pragma unroll
        for (int p = 0; p < XPASS; ++p) {
            const int q = min(p * 256 + tid, XCH - 1);
            if constexpr (L::STRIP) {
                const Where wq = where(q * CPV, L::XROWS);
                const int rg = r0 - 1 + wq.row;
                if (rg < 0 || rg >= H) s.xok &= ~(1u << p);
                s.x[p] = *reinterpret_cast<const u4raw_t *>(xs + (size_t)wq.plane * (H * W) + min(max(rg, 0), H - 1) * W + wq.cv * 4);
            } else {
                s.x[p] = *reinterpret_cast<const u4raw_t *>(xs + (size_t)q * (4 * CPV));      // the planes whole: one flat range
            }
        }
#pragma unroll
        for (int p = 0; p < DPASS; ++p) {
            const int q = min(p * 256 + tid, DCH - 1);
            if constexpr (L::STRIP) {
                const Where wq = where(q * CPV, L::RS);
                s.d[p] = *reinterpret_cast<const u4raw_t *>(ds + (size_t)wq.plane * (H * W) + (r0 + wq.row) * W + wq.cv * 4);
            } else {
                s.d[p] = *reinterpret_cast<const u4raw_t *>(ds + (size_t)q * (4 * CPV));
            }
        }
    };
    auto put = [&](T *area, int pitch, int rowpitch, int rowshift, int rows, int q, u4raw_t v) {
        if constexpr (F32) {
            const Where wq = where(q, rows);
            *reinterpret_cast<u4raw_t *>(area + wq.plane * pitch + (wq.row + rowshift) * rowpitch + wq.cv * 4) = v;
        } else {
            const Where w0 = where(2 * q, rows), w1 = where(2 * q + 1, rows);
            *reinterpret_cast<u2raw_t *>(area + w0.plane * pitch + (w0.row + rowshift) * rowpitch + w0.cv * 4) = u2raw_t{v.x, v.y};
            *reinterpret_cast<u2raw_t *>(area + w1.plane * pitch + (w1.row + rowshift) * rowpitch + w1.cv * 4) = u2raw_t{v.z, v.w};
        }
    };
    // NHWC: the chunk's channels go to their planes one element each (consecutive lanes are consecutive pixels of a row)
    auto scatter = [&](T *area, int pitch, int rowpitch, int rowshift, int q, u4raw_t v) {
        const int pq = q / HPP, hs = q % HPP;
        T *dst = area + (hs * 4) * pitch + (pq / W + rowshift) * rowpitch + pq % W;
        if constexpr (F32) {
            dst[0] = __uint_as_float(v.x); dst[pitch] = __uint_as_float(v.y); dst[2 * pitch] = __uint_as_float(v.z); dst[3 * pitch] = __uint_as_float(v.w);
        } else {
            dst[0] = (T)v.x; dst[pitch] = (T)(v.x >> 16); dst[2 * pitch] = (T)v.y; dst[3 * pitch] = (T)(v.y >> 16);
            dst[4 * pitch] = (T)v.z; dst[5 * pitch] = (T)(v.z >> 16); dst[6 * pitch] = (T)v.w; dst[7 * pitch] = (T)(v.w >> 16);
        }
    };
    // mosaic: rows of 14 are not whole chunks, so element by element: plane, row and column within its image, the image's
    // place in the mosaic (x: one zero row above and below each sub-plane; dy: the 28 virtual rows)
    auto mosaic_put = [&](int q, u4raw_t vx, u4raw_t vd) {
        constexpr int CPI = XCH / 4;
        const int a4 = q / CPI, e0 = (q % CPI) * EPC;
        const uint32_t wx[4] = {vx.x, vx.y, vx.z, vx.w}, wd[4] = {vd.x, vd.y, vd.z, vd.w};
#pragma unroll
        for (int k = 0; k < EPC; ++k) {
            const int e = e0 + k, plane = e / (H * W), rem = e % (H * W), r = rem / W, c = (a4 & 1) * 16 + rem % W;
            T *dx_ = lds + plane * L::PPX + ((a4 >> 1) * 16 + 1 + r) * L::WP + c;
            T *dd_ = lds + L::AREA_X + plane * PPD + ((a4 >> 1) * 14 + r) * DROW + c;
            if constexpr (F32) { *dx_ = __uint_as_float(wx[k]); *dd_ = __uint_as_float(wd[k]); }
            else { *dx_ = (T)(wx[k >> 1] >> ((k & 1) * 16)); *dd_ = (T)(wd[k >> 1] >> ((k & 1) * 16)); }
        }
    };
    auto lstore = [&](const Stage &s) {
        if constexpr (L::MOSAIC) {
#pragma unroll
            for (int p = 0; p < XPASS; ++p) {
                const int q = p * 256 + tid;
                if ((p + 1) * 256 <= XCH || q < XCH) {
                    const bool ok = (s.xok >> p) & 1u;
                    const u4raw_t d = s.d[p];
                    mosaic_put(q, s.x[p], u4raw_t{ok ? d.x : 0u, ok ? d.y : 0u, ok ? d.z : 0u, ok ? d.w : 0u});
                }
            }
            return;
        }
        if constexpr (NHWC) {
#pragma unroll
            for (int p = 0; p < XPASS; ++p) {
                const int q = p * 256 + tid;
                if ((p + 1) * 256 <= XCH || q < XCH) {
                    const bool ok = (s.xok >> p) & 1u;
                    const u4raw_t v = s.x[p];
                    scatter(lds, L::PPX, L::WP, L::STRIP ? 0 : 1, q, u4raw_t{ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u});
                }
            }
#pragma unroll
            for (int p = 0; p < DPASS; ++p) {
                const int q = p * 256 + tid;
                if ((p + 1) * 256 <= DCH || q < DCH) scatter(lds + L::AREA_X, PPD, DROW, 0, q, s.d[p]);
            }
            return;
        }
#pragma unroll
        for (int p = 0; p < XPASS; ++p) {
            const int q = p * 256 + tid;
            if ((p + 1) * 256 <= XCH || q < XCH) {
                const bool ok = (s.xok >> p) & 1u;
                const u4raw_t v = s.x[p];
                put(lds, L::PPX, L::WP, L::STRIP ? 0 : 1, L::XROWS, q, u4raw_t{ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u});
            }
        }
#pragma unroll
        for (int p = 0; p < DPASS; ++p) {
            const int q = p * 256 + tid;
            if ((p + 1) * 256 <= DCH || q < DCH) put(lds + L::AREA_X, PPD, DROW, 0, L::RS, q, s.d[p]);
        }
    };

    // The wavefront's task: quads of x and dy planes within the octet, and its rows.  Its 16 positions are SPW streams:
    // the vectors of a row and the gap after it (dy reads zeros there); a stream walks down RPS rows, one row per step,
    // and keeps the three x rows of the taps in registers, so a step reads one new x row and one dy row.  Groups of 8:
    // the wavefront walks all RS rows of the fill.  Groups of 4: the group's two wavefronts take the upper and the
    // lower half of them.
    // Wide rows (two wavefronts per row, groups of 2): the quad is two groups, the wavefront takes the left or the right
    // 16 positions of every row of the fill, and only the sums of channel pairs of the same group are kept at the end.
    constexpr int RPW = (CG == 8 || WIDE) ? L::RS : L::RS / 2, RPS = WIDE ? RPW : RPW / (WIDE ? 1 : L::SPW);
    static_assert(WIDE || RPW % L::SPW == 0, "whole streams");
    static_assert(WIDE == (CG == 2), "groups of 2 on wide rows only");
    const int xq = wv & 1, dq = CG == 8 ? wv >> 1 : wv & 1;
    const int half = wv >> 1;
    const int slot = lane >> 2;
    const int pos = WIDE ? half * 16 + slot : slot % (L::WP / 4);                 // the position within its row
    const int row0 = WIDE ? 0 : (CG == 8 ? 0 : half * RPW) + (slot / (L::WP / 4)) * RPS;
    const T *xpl = lds + (xq * 4 + (lane & 3)) * L::PPX + L::xrow(row0) * L::WP + pos * 4;
    const bool dvalid = !WIDE || pos < L::VPR;         // packed dy rows have no gap: those positions read a real vector and drop it
    const T *dpl = lds + L::AREA_X + (dq * 4 + (lane & 3)) * PPD + row0 * DROW + (dvalid ? pos : 0) * 4;
    // the neighbour positions' vectors come from the lanes four below and four above; position 0 has no left neighbour
    // in the wavefront and starts a row (zero); the last position of a row is a gap, whatever it gets meets a zero of dy
    const int up = ((lane - 4) & 63) * 4, dn = ((lane + 4) & 63) * 4;
    const uint32_t lmask = lane < 4 ? 0u : 0xffffffffu;

    v4f_t acc[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) acc[kh][kw] = v4f_t{0.f, 0.f, 0.f, 0.f};

    // one x row of the lane's position as the B operands of the three tap columns
    struct XRow { float f[6]; u2w_t b[3]; };
    auto xrow = [&](int t, XRow &X) {
        if constexpr (F32) {
            const u4raw_t v = *reinterpret_cast<const u4raw_t *>(xpl + t * L::WP);
            uint32_t lw = (uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)v.w) & lmask;
            uint32_t rw = (uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)v.x);
            if constexpr (WIDE) {       // the wavefront's first and last position: the neighbour is in the other wavefront (or the gap)
                if (slot == 0) lw = __float_as_uint(xpl[t * L::WP - 1]);
                if (slot == 15) rw = __float_as_uint(xpl[t * L::WP + 4]);
            }
            X.f[0] = __uint_as_float(lw);
            X.f[5] = __uint_as_float(rw);
            X.f[1] = __uint_as_float(v.x); X.f[2] = __uint_as_float(v.y); X.f[3] = __uint_as_float(v.z); X.f[4] = __uint_as_float(v.w);
        } else {
            const u2raw_t v = *reinterpret_cast<const u2raw_t *>(xpl + t * L::WP);                  // columns c .. c+3
            uint32_t lw = (uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)v.y) & lmask;             // columns c-2, c-1
            uint32_t rw = (uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)v.x);                     // columns c+4, c+5
            if constexpr (WIDE) {
                if (slot == 0) lw = *reinterpret_cast<const uint32_t *>(xpl + t * L::WP - 2);
                if (slot == 15) rw = *reinterpret_cast<const uint32_t *>(xpl + t * L::WP + 4);
            }
            const uint32_t p0 = __builtin_amdgcn_alignbyte(v.x, lw, 2);             // c-1, c
            const uint32_t p1 = __builtin_amdgcn_alignbyte(v.y, v.x, 2);            // c+1, c+2
            const uint32_t p2 = __builtin_amdgcn_alignbyte(rw, v.y, 2);             // c+3, c+4
            X.b[0] = u2w_t{p0, p1}; X.b[1] = u2w_t{v.x, v.y}; X.b[2] = u2w_t{p1, p2};
        }
    };
    // dy row t against the x rows t-1, t, t+1
    auto step = [&](int t, const XRow &X0, const XRow &X1, const XRow &X2) {
        if constexpr (F32) {
            u4raw_t dr = *reinterpret_cast<const u4raw_t *>(dpl + t * DROW);
            if (!dvalid) dr = u4raw_t{0u, 0u, 0u, 0u};
            const float d[4] = {__uint_as_float(dr.x), __uint_as_float(dr.y), __uint_as_float(dr.z), __uint_as_float(dr.w)};
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    acc[0][kw] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[c], X0.f[c + kw], acc[0][kw], 0, 0, 0);
                    acc[1][kw] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[c], X1.f[c + kw], acc[1][kw], 0, 0, 0);
                    acc[2][kw] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[c], X2.f[c + kw], acc[2][kw], 0, 0, 0);
                }
        } else {
            u2raw_t dr = *reinterpret_cast<const u2raw_t *>(dpl + t * DROW);
            if (!dvalid) dr = u2raw_t{0u, 0u};
            const v4s_t a = __builtin_bit_cast(v4s_t, dr);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                acc[0][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X0.b[kw]), acc[0][kw], 0, 0, 0);
                acc[1][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X1.b[kw]), acc[1][kw], 0, 0, 0);
                acc[2][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X2.b[kw]), acc[2][kw], 0, 0, 0);
            }
        }
    };
    auto fill = [&](Stage &s, int f) {
        lstore(s);
        __syncthreads();
        gload(s, f + DEPTH * parts);
        XRow R[3];
        xrow(-1, R[0]);
        xrow(0, R[1]);
#pragma unroll
        for (int t = 0; t < RPS; ++t) {
            xrow(t + 1, R[(t + 2) % 3]);
            step(t, R[t % 3], R[(t + 1) % 3], R[(t + 2) % 3]);
        }
        __syncthreads();                               // every wavefront is done with this fill's rows
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

    // the 16 blocks of the wavefront hold 16 partial sums of the same entries: butterfly over the block index
    const int pidx = CG == 8 ? part : part * 2 + half;      // groups of 4 and 2: the two wavefronts of a quad write a partial each
    float *wsp = ws + (size_t)pidx * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = acc[kh][kw][i];
                s += __shfl_xor(s, 4, 64); s += __shfl_xor(s, 8, 64); s += __shfl_xor(s, 16, 64); s += __shfl_xor(s, 32, 64);
                if (lane < 4 && (CG != 2 || (lane >> 1) == (i >> 1))) {        // groups of 2: pairs of the same group only
                    const int o = cb * 8 + dq * 4 + i, b = CG == 8 ? xq * 4 + lane : CG == 4 ? lane : lane & 1;
                    if constexpr (NHWC) wsp[((size_t)(kh * 3 + kw) * CG + b) * g.O + o] = s;     // the filter's layout: [tap][input channel][O]
                    else wsp[((size_t)o * CG + b) * 9 + kh * 3 + kw] = s;
                }
            }
}

// ---- host side ---------------------------------------------------------------------------------------------

bool gconv_nchws_mfma_bwd_filter_supported(const GGeom &g, int dtype, bool nhwc)
{
    if (tune_env("DWCONV_TUNE_GNOSMM")) return false;
    if (!(g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && g.C % 8 == 0)) return false;
    // 112x112 with groups of 2: bf16 only (254 -> 182 us at batch 256); in fp32 the 7-row strips that fit LDS tie with the
    // row walk (192 us at batch 128), which stays
    // NHWC: 16 bytes per pixel and octet are fetched, a strided pattern that runs at half the speed of the NCHW form's flat
    // ranges; it pays where the lane-exchange kernel is bound by arithmetic: bf16 groups of 8 (28x28 at batch 256:
    // 159 -> 102 us; groups of 4 and fp32 measured 15 to 40 % slower than the earlier kernels and stay there)
    if (nhwc && (tune_env("DWCONV_TUNE_GNOSMMNHWC") || !((dtype == DT_BF16 && g.Cg == 8) || tune_env("DWCONV_TUNE_GSMMNHWCALL")))) return false;
    if (g.H == 112 && g.W == 112) return !nhwc && g.Cg == 2 && (dtype == DT_BF16 || tune_env("DWCONV_TUNE_GSMM112F32")) && !tune_env("DWCONV_TUNE_GNOSMM112");
    if (g.H == 14 && g.W == 14) return !nhwc && (g.Cg == 4 || g.Cg == 8);
    return ((g.H == 28 && g.W == 28) || (g.H == 56 && g.W == 56)) && (g.Cg == 4 || g.Cg == 8);
}

// fills (28x28: images; 56x56: strips of 14 rows of an image) are dealt to `parts` blocks per channel octet, about 512
// blocks in the launch (two per compute unit, all resident at once; 1024 measured 15 % slower: the first loads and the
// final reduction of a block are not overlapped with anything of its own), every block the same number of fills where
// the batch allows it
static int nchws_mfma_fills(const GGeom &g, int dtype) { return g.W == 14 ? (g.N + 3) / 4 : g.N * (g.W == 56 ? 4 : g.W == 112 ? (dtype == DT_F32 ? 16 : 8) : 1); }
static int nchws_mfma_blocks_per_octet(const GGeom &g, int dtype)
{
    int target = 512;
    if (const char *e = tune_env("DWCONV_TUNE_GSMBLOCKS")) if (atoi(e) > 0) target = atoi(e);
    const int octets = g.C / 8, nf = nchws_mfma_fills(g, dtype);
    int p = (target + octets - 1) / octets;
    if (p > nf) p = nf;
    if (p < 1) p = 1;
    const int per = (nf + p - 1) / p;
    return (nf + per - 1) / per;
}

int gconv_nchws_mfma_bwd_filter_parts(const GGeom &g, int dtype) { return nchws_mfma_blocks_per_octet(g, dtype) * (g.Cg == 8 ? 1 : 2); }

hipError_t gconv_nchws_mfma_bwd_filter(const GGeom &g, int dtype, bool nhwc, const void *x, const void *dy, float *ws, int parts,
                                       hipStream_t st)
{
    if (!gconv_nchws_mfma_bwd_filter_supported(g, dtype, nhwc) || parts != gconv_nchws_mfma_bwd_filter_parts(g, dtype)) return hipErrorInvalidValue;
    const int bpo = nchws_mfma_blocks_per_octet(g, dtype);
    const unsigned nblocks = (unsigned)(g.C / 8) * (unsigned)bpo;
    const int J = g.O * g.Cg * 9;
#define GOL(T, CGG, WW, NH) hipLaunchKernelGGL((k_gconv_nchws_mfma_bwd_filter<T, CGG, WW, WW, NH>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                               (const T *)dy, ws, bpo, nchws_mfma_fills(g, dtype), nblocks, J)
#define GOW(T, CGG, WW) do { if (nhwc) GOL(T, CGG, WW, true); else GOL(T, CGG, WW, false); } while (0)
#define GO(T, CGG) do { if (g.W == 14) GOL(T, CGG, 14, false); else if (g.W == 28) GOW(T, CGG, 28); else GOW(T, CGG, 56); } while (0)
    if (g.W == 112) { if (dtype == DT_F32) GOL(float, 2, 112, false); else GOL(bf16_t, 2, 112, false); }
    else if (dtype == DT_F32) { if (g.Cg == 8) GO(float, 8); else GO(float, 4); }
    else                      { if (g.Cg == 8) GO(bf16_t, 8); else GO(bf16_t, 4); }
#undef GOW
#undef GOL
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
