// Shared device-side helpers for the gfx950 depthwise-convolution kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dwc {

// Problem geometry handed to every kernel by value.
struct Geom {
    int N, C, H, W;   // input dims
    int K, s, p, m;   // filter size, stride, pad, channel multiplier
    int O, Ho, Wo;    // O = C*m, output spatial dims
};

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even, through the hardware convert of gfx950 (v_cvt_pk_bf16_f32:
// two values per instruction; the bit-twiddled version costs about eight vector ALU operations per
// value, as much as the nine multiply-adds of a 3x3 output).
typedef float f2v_t __attribute__((ext_vector_type(2)));
typedef __bf16 b2v_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi)
{
    const f2v_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, b2v_t));
}
// c + a.lo * b.lo + a.hi * b.hi on two packed bf16 pairs, accumulated in fp32 (v_dot2c_f32_bf16).
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2v_t, a), __builtin_bit_cast(b2v_t, b), c, false);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack2_bf16(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float ldf(const float *p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void stf(float *p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ---- vector access: V consecutive elements of T as float[V] -----------------------------
template <typename T, int V> struct Vec;

template <> struct Vec<float, 4> {
    static __device__ __forceinline__ void load(const float *p, float (&r)[4])
    {
        float4 v = *reinterpret_cast<const float4 *>(p);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&r)[4])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(r[0], r[1], r[2], r[3]);
    }
};
template <> struct Vec<float, 2> {
    static __device__ __forceinline__ void load(const float *p, float (&r)[2])
    {
        float2 v = *reinterpret_cast<const float2 *>(p);
        r[0] = v.x; r[1] = v.y;
    }
    static __device__ __forceinline__ void store(float *p, const float (&r)[2])
    {
        *reinterpret_cast<float2 *>(p) = make_float2(r[0], r[1]);
    }
};
template <> struct Vec<float, 1> {
    static __device__ __forceinline__ void load(const float *p, float (&r)[1]) { r[0] = *p; }
    static __device__ __forceinline__ void store(float *p, const float (&r)[1]) { *p = r[0]; }
};
template <> struct Vec<bf16_t, 8> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&r)[8])
    {
        uint4 v = *reinterpret_cast<const uint4 *>(p);
        r[0] = __uint_as_float(v.x << 16); r[1] = __uint_as_float(v.x & 0xffff0000u);
        r[2] = __uint_as_float(v.y << 16); r[3] = __uint_as_float(v.y & 0xffff0000u);
        r[4] = __uint_as_float(v.z << 16); r[5] = __uint_as_float(v.z & 0xffff0000u);
        r[6] = __uint_as_float(v.w << 16); r[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&r)[8])
    {
        uint4 v;
        v.x = pack2_bf16(r[0], r[1]);
        v.y = pack2_bf16(r[2], r[3]);
        v.z = pack2_bf16(r[4], r[5]);
        v.w = pack2_bf16(r[6], r[7]);
        *reinterpret_cast<uint4 *>(p) = v;
    }
};
template <> struct Vec<bf16_t, 4> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&r)[4])
    {
        uint2 v = *reinterpret_cast<const uint2 *>(p);
        r[0] = __uint_as_float(v.x << 16); r[1] = __uint_as_float(v.x & 0xffff0000u);
        r[2] = __uint_as_float(v.y << 16); r[3] = __uint_as_float(v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&r)[4])
    {
        uint2 v;
        v.x = pack2_bf16(r[0], r[1]);
        v.y = pack2_bf16(r[2], r[3]);
        *reinterpret_cast<uint2 *>(p) = v;
    }
};
template <> struct Vec<bf16_t, 2> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&r)[2])
    {
        uint32_t v = *reinterpret_cast<const uint32_t *>(p);
        r[0] = __uint_as_float(v << 16); r[1] = __uint_as_float(v & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&r)[2])
    {
        *reinterpret_cast<uint32_t *>(p) = pack2_bf16(r[0], r[1]);
    }
};
template <> struct Vec<bf16_t, 1> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&r)[1]) { r[0] = bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&r)[1]) { *p = f32_to_bf16(r[0]); }
};

// ---- buffer addressing --------------------------------------------------------------------
// A raw buffer descriptor over `bytes` bytes at `base` (one image of a tensor: at most 2 GiB).  A load takes the
// lane's byte offset in a vector register and a wavefront-uniform byte offset in a scalar register, so a walk down
// the rows of an image needs no vector address arithmetic per row; a flat global load takes a 64-bit vector add
// for every address, which the kernels bound by their vector-ALU work (bf16, 5x5) cannot afford.  A read at or
// beyond `bytes` returns zero instead of faulting.  Word 3 of the descriptor is the untyped 32-bit data format of
// this chip family.
typedef uint32_t u4raw_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2raw_t __attribute__((ext_vector_type(2)));
struct BufView {
    // A view covers at most 2 GiB, so this lane offset is outside every view whatever uniform offset is added to
    // it (the sum stays below 4 GiB): the way a lane asks for a zero.
    static constexpr uint32_t OUTSIDE = 0x80000000u;
    __amdgpu_buffer_rsrc_t rsrc;
    // base and bytes must be the same in every lane; they are pinned to scalar registers here, so that a load never
    // falls back to a loop over distinct descriptors when the compiler cannot prove it
    __device__ __forceinline__ BufView(const void *base, uint32_t bytes)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(uniform_ptr(base), 0, (int)uniform(bytes), 0x00020000)) {}
    static __device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
    static __device__ __forceinline__ void *uniform_ptr(const void *p)
    {
        const uint64_t a = (uint64_t)p;
        return (void *)(((uint64_t)uniform((uint32_t)(a >> 32)) << 32) | uniform((uint32_t)a));
    }
    __device__ __forceinline__ uint32_t b32(uint32_t voff, uint32_t soff) const
    {
        return __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)voff, (int)uniform(soff), 0);
    }
    __device__ __forceinline__ u2raw_t b64(uint32_t voff, uint32_t soff) const
    {
        return __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)voff, (int)uniform(soff), 0);
    }
    __device__ __forceinline__ u4raw_t b128(uint32_t voff, uint32_t soff) const
    {
        return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, (int)uniform(soff), 0);
    }
    // stores; NT marks the store non-temporal (cache-policy bit 1 of the instruction)
    template <bool NT> __device__ __forceinline__ void st32(uint32_t d, uint32_t voff, uint32_t soff) const
    {
        __builtin_amdgcn_raw_buffer_store_b32(d, rsrc, (int)voff, (int)uniform(soff), NT ? 2 : 0);
    }
    template <bool NT> __device__ __forceinline__ void st64(u2raw_t d, uint32_t voff, uint32_t soff) const
    {
        __builtin_amdgcn_raw_buffer_store_b64(d, rsrc, (int)voff, (int)uniform(soff), NT ? 2 : 0);
    }
    template <bool NT> __device__ __forceinline__ void st128(u4raw_t d, uint32_t voff, uint32_t soff) const
    {
        __builtin_amdgcn_raw_buffer_store_b128(d, rsrc, (int)voff, (int)uniform(soff), NT ? 2 : 0);
    }
};

// Store V elements; `stream` = true marks the store non-temporal (the output of a large layer is
// not read again by these kernels, so it should not displace the halo rows that are).
// V consecutive elements kept as loaded (bf16 stays packed, two per register) and widened to
// fp32 only where they are used: a prefetch ring of RawVec costs half the registers of a ring of
// floats for bf16.
template <typename T, int V> struct RawVec;
template <int V> struct RawVec<float, V> {
    float v[V];
    __device__ __forceinline__ void load(const float *p) { Vec<float, V>::load(p, v); }
    // V floats at byte offset voff (per lane) + soff (uniform) of the view
    __device__ __forceinline__ void load_buf(const BufView &b, uint32_t voff, uint32_t soff)
    {
        if constexpr (V == 4) { const u4raw_t q = b.b128(voff, soff); v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w); }
        else if constexpr (V == 2) { const u2raw_t q = b.b64(voff, soff); v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y); }
        else { static_assert(V == 1, "float vectors of 1, 2 or 4"); v[0] = __uint_as_float(b.b32(voff, soff)); }
    }
    __device__ __forceinline__ void get(float (&r)[V]) const
    {
#pragma unroll
        for (int i = 0; i < V; ++i) r[i] = v[i];
    }
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = 0.f;
    }
};
template <int V> struct RawVec<bf16_t, V> {
    static_assert(V % 2 == 0, "bf16 vectors are whole 32-bit words");
    uint32_t w[V / 2];
    __device__ __forceinline__ void load(const bf16_t *p)
    {
        if constexpr (V == 8) { const uint4 q = *reinterpret_cast<const uint4 *>(p); w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w; }
        else if constexpr (V == 4) { const uint2 q = *reinterpret_cast<const uint2 *>(p); w[0] = q.x; w[1] = q.y; }
        else { static_assert(V == 2, "bf16 vectors of 2, 4 or 8"); w[0] = *reinterpret_cast<const uint32_t *>(p); }
    }
    __device__ __forceinline__ void load_buf(const BufView &b, uint32_t voff, uint32_t soff)
    {
        if constexpr (V == 8) { const u4raw_t q = b.b128(voff, soff); w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w; }
        else if constexpr (V == 4) { const u2raw_t q = b.b64(voff, soff); w[0] = q.x; w[1] = q.y; }
        else w[0] = b.b32(voff, soff);
    }
    __device__ __forceinline__ void get(float (&r)[V]) const
    {
#pragma unroll
        for (int i = 0; i < V / 2; ++i) { r[2 * i] = __uint_as_float(w[i] << 16); r[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    }
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < V / 2; ++i) w[i] = 0u;
    }
};

template <> struct RawVec<bf16_t, 1> {
    bf16_t w;
    __device__ __forceinline__ void load(const bf16_t *p) { w = *p; }
    __device__ __forceinline__ void get(float (&r)[1]) const { r[0] = bf16_to_f32(w); }
    __device__ __forceinline__ void zero() { w = 0; }
};

typedef float f4v_t __attribute__((ext_vector_type(4)));
typedef uint32_t u4v_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2v_t __attribute__((ext_vector_type(2)));
template <typename T, int V>
__device__ __forceinline__ void store_vec(T *p, const float (&r)[V], bool stream)
{
    if (!stream) { Vec<T, V>::store(p, r); return; }
    if constexpr (sizeof(T) == 4 && V == 4) {
        f4v_t v = {r[0], r[1], r[2], r[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<f4v_t *>(p));
    } else if constexpr (sizeof(T) == 2 && V == 8) {
        u4v_t v;
        v.x = pack2_bf16(r[0], r[1]);
        v.y = pack2_bf16(r[2], r[3]);
        v.z = pack2_bf16(r[4], r[5]);
        v.w = pack2_bf16(r[6], r[7]);
        __builtin_nontemporal_store(v, reinterpret_cast<u4v_t *>(p));
    } else if constexpr (sizeof(T) == 2 && V == 4) {
        u2v_t v;
        v.x = pack2_bf16(r[0], r[1]);
        v.y = pack2_bf16(r[2], r[3]);
        __builtin_nontemporal_store(v, reinterpret_cast<u2v_t *>(p));
    } else {
        Vec<T, V>::store(p, r);
    }
}

// store_vec through a buffer view: V elements at byte offset voff (per lane) + soff (uniform)
template <typename T, int V, bool NT>
__device__ __forceinline__ void store_buf_nt(const BufView &b, uint32_t voff, uint32_t soff, const float (&r)[V])
{
    if constexpr (sizeof(T) == 4) {
        if constexpr (V == 4) { u4raw_t d = {__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2]), __float_as_uint(r[3])}; b.st128<NT>(d, voff, soff); }
        else if constexpr (V == 2) { u2raw_t d = {__float_as_uint(r[0]), __float_as_uint(r[1])}; b.st64<NT>(d, voff, soff); }
        else { static_assert(V == 1, "float vectors of 1, 2 or 4"); b.st32<NT>(__float_as_uint(r[0]), voff, soff); }
    } else {
        if constexpr (V == 8) { u4raw_t d = {pack2_bf16(r[0], r[1]), pack2_bf16(r[2], r[3]), pack2_bf16(r[4], r[5]), pack2_bf16(r[6], r[7])}; b.st128<NT>(d, voff, soff); }
        else if constexpr (V == 4) { u2raw_t d = {pack2_bf16(r[0], r[1]), pack2_bf16(r[2], r[3])}; b.st64<NT>(d, voff, soff); }
        else { static_assert(V == 2, "bf16 vectors of 2, 4 or 8"); b.st32<NT>(pack2_bf16(r[0], r[1]), voff, soff); }
    }
}
template <typename T, int V>
__device__ __forceinline__ void store_buf(const BufView &b, uint32_t voff, uint32_t soff, const float (&r)[V], bool stream)
{
    if (stream) store_buf_nt<T, V, true>(b, voff, soff, r);
    else store_buf_nt<T, V, false>(b, voff, soff, r);
}

// ---- fixed-order reductions -----------------------------------------------------------------
// Butterfly sum over the 64 lanes of a wavefront; every lane ends with the same total and the
// order of additions is fixed by the lane numbers, so the result is reproducible.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Butterfly over lanes whose numbers differ only in the bits at or above `lo_stride`
// (lo_stride a power of two): sums lanes l, l^lo_stride, l^(2*lo_stride), ... up to 32.
__device__ __forceinline__ float wave_sum_strided(float v, int lo_stride)
{
    for (int off = 32; off >= lo_stride; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Block-wide fixed-order sum of K*K*V per-lane partial sums (the end of a filter-gradient walk in the
// NHWC mapping: a block of 4 wavefronts, lane tx + j*CT of every wavefront owns channel vector tx).
// For each value: butterfly over the lanes of a wavefront that own the same channels, then the
// wavefronts 1..3 park their sums in LDS and wavefront 0 adds (w0 + w1) + (w2 + w3) and hands the
// total of tap (kh, kw), channel v to `emit(kh, kw, v, total)` on its lanes below CT.  The values go
// through LDS in chunks of CH, one barrier pair per chunk instead of one per tap: the per-tap form
// cost a block of a 5x5 layer fifty barriers, several microseconds that short walks never won back.
constexpr int reduce_chunk(int nacc)
{
    int ch = nacc < 36 ? nacc : 36;
    while (nacc % ch) --ch;
    return ch;
}
template <int K, int V, typename F>
__device__ __forceinline__ void block_reduce_taps(const float (&acc)[K][K][V], int CT, float *lds, F emit)
{
    constexpr int NACC = K * K * V, CH = reduce_chunk(NACC);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float (*red)[CH][64] = reinterpret_cast<float (*)[CH][64]>(lds);       // [3][CH][64]
#pragma unroll
    for (int c0 = 0; c0 < NACC; c0 += CH) {
        float s[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int e = c0 + i, v = e % V, kw = (e / V) % K, kh = e / (V * K);
            s[i] = wave_sum_strided(acc[kh][kw][v], CT);
        }
        if (wv > 0) {
#pragma unroll
            for (int i = 0; i < CH; ++i) red[wv - 1][i][lane] = s[i];
        }
        __syncthreads();
        if (wv == 0 && lane < CT) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int e = c0 + i, v = e % V, kw = (e / V) % K, kh = e / (V * K);
                emit(kh, kw, v, (s[i] + red[0][i][lane]) + (red[1][i][lane] + red[2][i][lane]));
            }
        }
        if (c0 + CH < NACC) __syncthreads();
    }
}
// floats of LDS that block_reduce_taps needs
template <int K, int V> struct ReduceLds { static constexpr int FLOATS = 3 * reduce_chunk(K * K * V) * 64; };

// The dispatcher launches workgroups round-robin over the 8 XCDs (each with its own L2).
// This maps the hardware block id to a logical one so that each XCD walks a contiguous range
// of logical ids: blocks that share halo rows then share an L2 and run close in time.
__device__ __forceinline__ unsigned xcd_remap(unsigned bid, unsigned nblocks)
{
    const unsigned X = 8;
    unsigned per = nblocks / X, rem = nblocks % X;
    unsigned xcd = bid % X, slot = bid / X;
    // XCDs 0..rem-1 own per+1 logical ids, the rest own per.
    unsigned base = xcd * per + (xcd < rem ? xcd : rem);
    return base + slot;
}

}  // namespace dwc
