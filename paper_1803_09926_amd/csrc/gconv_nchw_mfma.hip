// Group convolution, NCHW, 3x3 stride 1 pad 1: filter gradient (Eq. 4 with the sum over a group's channel pairs) on the
// matrix cores, for 4 or 8 channels per group on both sides and 28x28 planes.
//
// Per pixel a group of 8 needs 8*8*9 multiply-adds for 16 loaded values: on the vector ALU this pass is bound by
// arithmetic (about a third of the memory rate).  The sum over pixels is a matrix product dW[o][b][tap] =
// sum_p dy[o][p] * x[b][p + tap], and the 4x4 matrix instructions compute 16 independent 4x4 products per
// wavefront: a block of four lanes holds four channels at one pixel position (fp32: one pixel, 4x4x1; bf16: four
// consecutive pixels of a row as the four-element inner dimension, 4x4x4, exactly the 8 bytes a lane reads from
// its plane).  A = the dy values of the lane's output channel, B = the x values of the lane's input channel at the
// tap's offset, D[i][j] (register i of lane j) = the sum for (output channel i, input channel j) of the quad pair.
//
// A thread block works on eight consecutive channels (one group of 8, or two groups of 4) of one image at a time:
// the eight x planes and eight dy planes (contiguous in NCHW) come in as flat 16-byte loads, two images ahead in
// registers, and are laid out in LDS with a four-element zero gap after every row and a zero row between planes,
// so every tap's operand is an unconditional LDS read at a constant offset from the position (the padding supplies
// the zeros of Eq. 4's border).  A wavefront's 16 positions are two streams of eight: the seven 4-pixel vectors of a
// row and the gap after it (dy is zero there).  A stream walks down its rows and keeps the three x rows of the taps
// in registers: a step reads one new x row and one dy row from LDS; the one pixel left and right of a position's
// four is the neighbour lane's vector, fetched by a lane permute instead of a second LDS read (single-word reads at
// a stride of four words use a quarter of the banks).  Groups of 8: the four wavefronts take the four (input quad,
// output quad) pairs and the whole plane (streams of 14 rows), 9 accumulators each.  Groups of 4: two wavefronts
// per group, the upper and the lower half of the plane (two partial sums per block).  At the end a
// wavefront adds its 16 blocks with a shuffle butterfly and writes its entries of the block's partial; the shared
// second stage adds the partials in a fixed order.
#include "gconv_mfma.hpp"

namespace dwc {

template <int W, int H> struct SmallPlaneLds {
    static constexpr int WP = W + 4;                // row pitch: the row, then four zeros
    static constexpr int PADP = 16;                 // planes staggered over the LDS banks
    static constexpr int PP = (H + 1) * WP + PADP;  // plane pitch: the rows, one zero row, the stagger (zeros)
    static constexpr int LEAD = WP + 4;             // zeros before the first plane (the row above it)
    static constexpr int AREA = LEAD + 8 * PP;      // elements of one tensor's eight planes
    static constexpr int V4 = H * W / 4;            // four-pixel vectors of a plane
    // element offset of four-pixel vector v of the eight planes (v = plane * V4 + index in the plane)
    static __device__ __forceinline__ int offset(int v)
    {
        const int plane = v / V4, rem = v % V4, r = rem / (W / 4), cv = rem % (W / 4);
        return LEAD + plane * PP + r * WP + cv * 4;
    }
};

template <typename T, int CG, int W, int H>
__global__ __launch_bounds__(256) void k_gconv_nchws_mfma_bwd_filter(GGeom g, const T *__restrict__ x, const T *__restrict__ dy,
                                                                     float *__restrict__ ws, int parts, unsigned nblocks, int J)
{
    using L = SmallPlaneLds<W, H>;
    static_assert(L::WP == 32 && H % 2 == 0 && (CG == 4 || CG == 8), "rows of seven vectors and a gap: eight positions; groups of 4 or 8");
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int EPC = 16 / (int)sizeof(T);        // elements of a 16-byte chunk
    constexpr int NCH = 8 * H * W / EPC;            // chunks of one tensor's eight planes
    constexpr int NPASS = (NCH + 255) / 256;
    __shared__ __align__(16) T lds[2 * L::AREA];    // x planes, then dy planes

    unsigned lb = xcd_remap(blockIdx.x, nblocks);
    const int part = lb % parts, cb = lb / parts;   // cb: the block's channel octet
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);

    for (int i = tid; i < 2 * L::AREA * (int)sizeof(T) / 16; i += 256) reinterpret_cast<u4raw_t *>(lds)[i] = u4raw_t{0u, 0u, 0u, 0u};

    // Two images ahead in registers.  Every load is issued unconditionally (lanes past the end of the last pass and
    // blocks past their last image repeat a valid address and drop the result): the number of loads in flight is then
    // the same on every path, and the wait before an image's LDS writes covers that image's loads only.
    struct Stage { u4raw_t x[NPASS], d[NPASS]; };
    auto gload = [&](Stage &s, int n) {
        const int nn = n < g.N ? n : part;
        const T *xs = x + ((size_t)nn * g.C + (size_t)cb * 8) * (H * W);
        const T *ds = dy + ((size_t)nn * g.O + (size_t)cb * 8) * (H * W);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int q = min(p * 256 + tid, NCH - 1);
            s.x[p] = *reinterpret_cast<const u4raw_t *>(xs + (size_t)q * EPC);
            s.d[p] = *reinterpret_cast<const u4raw_t *>(ds + (size_t)q * EPC);
        }
    };
    auto lstore = [&](const Stage &s) {
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int q = p * 256 + tid;
            if ((p + 1) * 256 <= NCH || q < NCH) {
                if constexpr (F32) {
                    const int o = L::offset(q);
                    *reinterpret_cast<u4raw_t *>(lds + o) = s.x[p];
                    *reinterpret_cast<u4raw_t *>(lds + L::AREA + o) = s.d[p];
                } else {
                    const int o0 = L::offset(2 * q), o1 = L::offset(2 * q + 1);
                    *reinterpret_cast<u2raw_t *>(lds + o0) = u2raw_t{s.x[p].x, s.x[p].y};
                    *reinterpret_cast<u2raw_t *>(lds + o1) = u2raw_t{s.x[p].z, s.x[p].w};
                    *reinterpret_cast<u2raw_t *>(lds + L::AREA + o0) = u2raw_t{s.d[p].x, s.d[p].y};
                    *reinterpret_cast<u2raw_t *>(lds + L::AREA + o1) = u2raw_t{s.d[p].z, s.d[p].w};
                }
            }
        }
    };

    // The wavefront's task: quads of x and dy planes within the octet, and its rows.  Its 16 positions are two streams of
    // eight: the seven vectors of a row and the gap after it (dy reads zeros there); a stream walks down RPS rows, one
    // row per step, and keeps the three x rows of the taps in registers, so a step reads one new x row and one dy row.
    // Groups of 8: streams of H/2 rows.  Groups of 4: the group's two wavefronts take the upper and the lower half of
    // the plane, streams of H/4 rows.
    constexpr int RPS = CG == 8 ? H / 2 : H / 4;
    static_assert(H % 4 == 0, "whole streams");
    const int xq = wv & 1, dq = CG == 8 ? wv >> 1 : wv & 1;
    const int half = wv >> 1;
    const int slot = lane >> 2;
    const int row0 = (CG == 8 ? 0 : half * (H / 2)) + (slot >> 3) * RPS;
    const T *xpl = lds + (xq * 4 + (lane & 3)) * L::PP + L::LEAD + row0 * L::WP + (slot & 7) * 4;
    const T *dpl = lds + L::AREA + (dq * 4 + (lane & 3)) * L::PP + L::LEAD + row0 * L::WP + (slot & 7) * 4;
    // the neighbour positions' vectors come from the lanes four below and four above; position 0 has no left neighbour
    // in the wavefront and starts a row (zero); positions 7 and 15 are gaps, whatever they get meets a zero of dy
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
            X.f[0] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)v.w) & lmask);
            X.f[5] = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)v.x));
            X.f[1] = __uint_as_float(v.x); X.f[2] = __uint_as_float(v.y); X.f[3] = __uint_as_float(v.z); X.f[4] = __uint_as_float(v.w);
        } else {
            const u2raw_t v = *reinterpret_cast<const u2raw_t *>(xpl + t * L::WP);                  // columns c .. c+3
            const uint32_t lw = (uint32_t)__builtin_amdgcn_ds_bpermute(up, (int)v.y) & lmask;       // columns c-2, c-1
            const uint32_t rw = (uint32_t)__builtin_amdgcn_ds_bpermute(dn, (int)v.x);               // columns c+4, c+5
            const uint32_t p0 = __builtin_amdgcn_alignbyte(v.x, lw, 2);             // c-1, c
            const uint32_t p1 = __builtin_amdgcn_alignbyte(v.y, v.x, 2);            // c+1, c+2
            const uint32_t p2 = __builtin_amdgcn_alignbyte(rw, v.y, 2);             // c+3, c+4
            X.b[0] = u2w_t{p0, p1}; X.b[1] = u2w_t{v.x, v.y}; X.b[2] = u2w_t{p1, p2};
        }
    };
    // dy row t against the x rows t-1, t, t+1
    auto step = [&](int t, const XRow &X0, const XRow &X1, const XRow &X2) {
        if constexpr (F32) {
            const u4raw_t dr = *reinterpret_cast<const u4raw_t *>(dpl + t * L::WP);
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
            const u2raw_t dr = *reinterpret_cast<const u2raw_t *>(dpl + t * L::WP);
            const v4s_t a = __builtin_bit_cast(v4s_t, dr);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                acc[0][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X0.b[kw]), acc[0][kw], 0, 0, 0);
                acc[1][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X1.b[kw]), acc[1][kw], 0, 0, 0);
                acc[2][kw] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, __builtin_bit_cast(v4s_t, X2.b[kw]), acc[2][kw], 0, 0, 0);
            }
        }
    };
    auto image = [&](Stage &s, int n) {
        lstore(s);
        __syncthreads();
        gload(s, n + 2 * parts);
        XRow R[3];
        xrow(-1, R[0]);
        xrow(0, R[1]);
#pragma unroll
        for (int t = 0; t < RPS; ++t) {
            xrow(t + 1, R[(t + 2) % 3]);
            step(t, R[t % 3], R[(t + 1) % 3], R[(t + 2) % 3]);
        }
        __syncthreads();                               // every wavefront is done with this image's planes
    };

    Stage sa, sb;
    int n = part;
    gload(sa, n);                                      // part < parts <= N
    gload(sb, n + parts);
    __syncthreads();                                   // the zeros are in place
    while (n < g.N) {
        image(sa, n);
        n += parts;
        if (n >= g.N) break;
        image(sb, n);
        n += parts;
    }

    // the 16 blocks of the wavefront hold 16 partial sums of the same entries: butterfly over the block index
    const int pidx = CG == 8 ? part : part * 2 + half;
    float *wsp = ws + (size_t)pidx * J;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = acc[kh][kw][i];
                s += __shfl_xor(s, 4, 64); s += __shfl_xor(s, 8, 64); s += __shfl_xor(s, 16, 64); s += __shfl_xor(s, 32, 64);
                if (lane < 4) {
                    const int o = cb * 8 + dq * 4 + i, b = (CG == 8 ? xq * 4 : 0) + lane;
                    wsp[((size_t)o * CG + b) * 9 + kh * 3 + kw] = s;
                }
            }
}

// ---- host side ---------------------------------------------------------------------------------------------

bool gconv_nchws_mfma_bwd_filter_supported(const GGeom &g)
{
    if (tune_env("DWCONV_TUNE_GNOSMM")) return false;
    if (!(g.K == 3 && g.s == 1 && g.p == 1 && g.Cg == g.Og && (g.Cg == 4 || g.Cg == 8))) return false;
    return g.H == 28 && g.W == 28 && g.C % 8 == 0;
}

// images are dealt to `parts` blocks per channel octet, about 512 blocks in the launch (two per compute unit: all resident at once; 1024 measured 15 % slower, the first loads and the final reduction of a block are not overlapped with anything of its own), every block the same number
// of images where the batch allows it
static int nchws_mfma_blocks_per_octet(const GGeom &g)
{
    int target = 512;
    if (const char *e = tune_env("DWCONV_TUNE_GSMBLOCKS")) if (atoi(e) > 0) target = atoi(e);
    const int octets = g.C / 8;
    int p = (target + octets - 1) / octets;
    if (p > g.N) p = g.N;
    if (p < 1) p = 1;
    const int per = (g.N + p - 1) / p;
    return (g.N + per - 1) / per;
}

int gconv_nchws_mfma_bwd_filter_parts(const GGeom &g) { return nchws_mfma_blocks_per_octet(g) * (g.Cg == 4 ? 2 : 1); }

hipError_t gconv_nchws_mfma_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts, hipStream_t st)
{
    if (!gconv_nchws_mfma_bwd_filter_supported(g) || parts != gconv_nchws_mfma_bwd_filter_parts(g)) return hipErrorInvalidValue;
    const int bpo = nchws_mfma_blocks_per_octet(g);
    const unsigned nblocks = (unsigned)(g.C / 8) * (unsigned)bpo;
    const int J = g.O * g.Cg * 9;
#define GO(T, CGG) hipLaunchKernelGGL((k_gconv_nchws_mfma_bwd_filter<T, CGG, 28, 28>), dim3(nblocks), dim3(256), 0, st, g, (const T *)x, \
                                      (const T *)dy, ws, bpo, nblocks, J)
    if (dtype == DT_F32) { if (g.Cg == 8) GO(float, 8); else GO(float, 4); }
    else                 { if (g.Cg == 8) GO(bf16_t, 8); else GO(bf16_t, 4); }
#undef GO
    return hipGetLastError();
}

}  // namespace dwc
