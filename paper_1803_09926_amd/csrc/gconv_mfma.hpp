// Pieces the matrix-core group-convolution kernels share (gconv_nhwc_mfma.hip, gconv_nhwc_mfma_s2.hip): the lane's input
// vector as loaded, its filter entries as the A operand, and the 4x4 matrix instructions of the two storage types.
// Lane layout of both instructions (16 independent blocks of 4 lanes): A[i][k] comes from lane i of the block, B[k][j]
// from lane j, and D[i][j] is register i of lane j.
#pragma once
#include "gconv.hpp"

namespace dwc {

typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef short v4s_t __attribute__((ext_vector_type(4)));

// The lane's input channels of one pixel, as loaded: LQ quads (fp32: one quad = 16 bytes; bf16: two quads = 16 bytes).
template <typename T> struct LaneIn;
template <> struct LaneIn<float> {
    static constexpr int LQ = 1;
    float c[4];
    __device__ __forceinline__ void load(const BufView &b, uint32_t voff, uint32_t soff)
    {
        const u4raw_t q = b.b128(voff, soff);
        c[0] = __uint_as_float(q.x); c[1] = __uint_as_float(q.y); c[2] = __uint_as_float(q.z); c[3] = __uint_as_float(q.w);
    }
    __device__ __forceinline__ LaneIn sibling() const      // the same registers of the lane four lanes away (the group's other quad)
    {
        LaneIn r;
#pragma unroll
        for (int k = 0; k < 4; ++k) r.c[k] = __shfl_xor(c[k], 4, 64);
        return r;
    }
};
template <> struct LaneIn<bf16_t> {
    static constexpr int LQ = 2;
    uint32_t w[4];
    __device__ __forceinline__ void load(const BufView &b, uint32_t voff, uint32_t soff)
    {
        const u4raw_t q = b.b128(voff, soff);
        w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
    __device__ __forceinline__ LaneIn sibling() const { return *this; }     // never needed: a group of 8 is inside the lane
};

// The lane's filter entries for one (tap, output quad, input quad): A[i][k], i = the lane's output channel, k = 0..3.
template <typename T> struct QuadW;
template <> struct QuadW<float> {
    float a[4];
    __device__ __forceinline__ void set(int k, float v) { a[k] = v; }
    __device__ __forceinline__ void finish() {}
};
template <> struct QuadW<bf16_t> {
    uint32_t w[2];
    __device__ __forceinline__ void set(int k, float v)
    {
        // the filter is stored in bf16, so the upper half of its widened value is the stored value
        const uint32_t h = __float_as_uint(v) >> 16;
        if (k == 0) w[0] = h; else if (k == 1) w[0] |= h << 16; else if (k == 2) w[1] = h; else w[1] |= h << 16;
    }
    __device__ __forceinline__ void finish() {}
};

typedef uint32_t u2w_t __attribute__((ext_vector_type(2)));
// d0 += A2 * B, d1 += A1 * B, d2 += A0 * B for input quad `q` of the lane's vector: one input quad against the filter
// entries of the three tap rows it serves; consecutive instructions go to different accumulators
__device__ __forceinline__ void quad_mma3(v4f_t &d0, v4f_t &d1, v4f_t &d2, const QuadW<float> &a2, const QuadW<float> &a1,
                                          const QuadW<float> &a0, const LaneIn<float> &b, int)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        d0 = __builtin_amdgcn_mfma_f32_4x4x1f32(a2.a[k], b.c[k], d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_4x4x1f32(a1.a[k], b.c[k], d1, 0, 0, 0);
        d2 = __builtin_amdgcn_mfma_f32_4x4x1f32(a0.a[k], b.c[k], d2, 0, 0, 0);
    }
}
__device__ __forceinline__ void quad_mma3(v4f_t &d0, v4f_t &d1, v4f_t &d2, const QuadW<bf16_t> &a2, const QuadW<bf16_t> &a1,
                                          const QuadW<bf16_t> &a0, const LaneIn<bf16_t> &b, int q)
{
    const v4s_t bv = __builtin_bit_cast(v4s_t, u2w_t{b.w[2 * q], b.w[2 * q + 1]});
    d0 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4s_t, u2w_t{a2.w[0], a2.w[1]}), bv, d0, 0, 0, 0);
    d1 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4s_t, u2w_t{a1.w[0], a1.w[1]}), bv, d1, 0, 0, 0);
    d2 = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4s_t, u2w_t{a0.w[0], a0.w[1]}), bv, d2, 0, 0, 0);
}

// d += A * B for input quad `q` of the lane's vector
__device__ __forceinline__ void quad_mma1(v4f_t &d, const QuadW<float> &a, const LaneIn<float> &b, int)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) d = __builtin_amdgcn_mfma_f32_4x4x1f32(a.a[k], b.c[k], d, 0, 0, 0);
}
__device__ __forceinline__ void quad_mma1(v4f_t &d, const QuadW<bf16_t> &a, const LaneIn<bf16_t> &b, int q)
{
    d = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(v4s_t, u2w_t{a.w[0], a.w[1]}),
                                               __builtin_bit_cast(v4s_t, u2w_t{b.w[2 * q], b.w[2 * q + 1]}), d, 0, 0, 0);
}

// The lane's filter entries, wq[oq][tap][iq]: output quad oq of the lane against input quad iq of that quad's group (when
// the group's other quad lives in the neighbouring block, fp32 groups of 8: iq 0 = the lane's own quad, 1 = the
// neighbour's).  MODE 0: forward, A[i][k] = w[tap][ci = k][o = i]; MODE 1: backward-data at stride 1, the filter
// transposed inside the group and rotated, A[i][k] = w[8 - tap][ci = i][o = k]; MODE 2: transposed only.  CG = 2: the
// quad holds two groups.
template <typename T, int CG, int MODE>
__device__ __forceinline__ void load_group_filter(const T *__restrict__ w, int C, int cbase, int j,
                                                  QuadW<T> (&wq)[LaneIn<T>::LQ][9][CG <= 4 ? 1 : CG / 4])
{
    constexpr int LQ = LaneIn<T>::LQ, NQ = CG <= 4 ? 1 : CG / 4;
    constexpr bool SIB = NQ == 2 && LQ == 1;
#pragma unroll
    for (int oq = 0; oq < LQ; ++oq) {
        const int c4 = cbase + 4 * oq, grp0 = c4 / CG * CG, qpos = (c4 - grp0) / 4;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
#pragma unroll
            for (int iq = 0; iq < NQ; ++iq) {
                const int rq = NQ == 1 ? 0 : (SIB ? (qpos ^ iq) : iq);         // that input quad's place in the group
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    size_t idx;
                    if constexpr (CG == 2) {
                        // a quad is two groups of 2: the entries that pair channels of different groups are zero (a
                        // block-diagonal 4x4 tile)
                        if (MODE == 0) idx = (size_t)(tap * 2 + k % 2) * C + c4 + j;
                        else idx = (size_t)((MODE == 1 ? 8 - tap : tap) * 2 + j % 2) * C + c4 + k;
                        const float v = ldf(w + idx);
                        wq[oq][tap][iq].set(k, k / 2 == j / 2 ? v : 0.f);
                        continue;
                    }
                    if (MODE == 0) idx = (size_t)(tap * CG + rq * 4 + k) * C + c4 + j;
                    else idx = (size_t)((MODE == 1 ? 8 - tap : tap) * CG + qpos * 4 + j) * C + grp0 + rq * 4 + k;
                    wq[oq][tap][iq].set(k, ldf(w + idx));
                }
                wq[oq][tap][iq].finish();
            }
    }
}

// ---- NCHW planes staged in LDS (gconv_nchw_mfma.hip, gconv_nchw_mfma_fwd.hip) ------------------------------------
//
// What a block holds in LDS at a time ("fill"): RS rows of eight dy planes and the RS + 2 rows of the eight x planes
// their taps reach.  28x28: the whole plane (the rows above and below it are zeros that are written once).  56x56:
// strips of 14 rows (the rows above and below a strip are loaded, or zeroed at the plane's edge); 112x112 (forward and
// backward-data only): strips of 14 rows in bf16, 7 in fp32.  A row is followed
// by a gap of zeros up to the pitch WP = 16 positions / streams: two rows of 8 positions or one row of 16.
template <int W, int H, int ESZ = 4> struct PlaneFill {
    static_assert((W == 14 && H == 14) || (W == 28 && H == 28) || (W == 56 && H == 56) || (W == 112 && H == 112),
                  "14x14 planes four at a time, 28x28 planes whole, larger planes in strips");
    // 14x14: a fill is four images laid out as a 2 x 2 mosaic of the 28-wide geometry, each row [14 | 2 zeros | 14 | 2
    // zeros] and each column of sub-planes [zero row | 14 rows | zero row] twice: 28 "virtual" rows
    static constexpr bool MOSAIC = W == 14;
    static constexpr bool STRIP = W > 28;
    static constexpr int RS = W <= 28 ? 28 : (W == 56 || ESZ == 2) ? 14 : 7;     // dy rows of a fill
    static constexpr int NSTRIP = MOSAIC ? 1 : H / RS;
    static constexpr int WP = W <= 28 ? 32 : W == 56 ? 64 : 128;     // row pitch in elements
    static constexpr int SPW = 64 / WP;                 // streams (rows walked side by side) of a wavefront; 0: a row spans two
    static constexpr int VPR = MOSAIC ? 7 : W / 4;      // four-pixel vectors of a row (mosaic: of a virtual row's 28 pixels)
    static constexpr int PADP = 16;                     // planes staggered over the LDS banks
    static constexpr int PPX = (RS + (MOSAIC ? 4 : 2)) * WP + PADP;    // x plane pitch: row r0 - 1 first
    // LDS row of virtual row vr of the x planes
    static constexpr __host__ __device__ int xrow(int vr) { return MOSAIC ? (vr / 14) * 16 + 1 + vr % 14 : vr + 1; }
    static constexpr int PPD = RS * WP + PADP;
    static constexpr int XROWS = STRIP ? RS + 2 : RS;   // x rows of a plane that are loaded
    static constexpr int AREA_X = 8 * PPX, AREA_D = 8 * PPD;
};

}  // namespace dwc
