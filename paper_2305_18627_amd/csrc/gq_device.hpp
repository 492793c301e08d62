// Device-side building blocks of the Global-QSGD hot path for gfx950 (wave64).
// Internal to the library; the public surface is include/gqsgd.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace gq {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;          // threads per workgroup: four wave64

// f(integral_constant<int, BEGIN>), ..., f(integral_constant<int, END - 1>): a loop whose index is a compile-time
// constant in the body, so that it is unrolled by the language and not at the optimizer's discretion.
template <int BEGIN, int END, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}
constexpr int kMaxWorkers = 64;

// Per-worker device pointers, passed to the kernels by value.
struct GradPtrs { const float *x[kMaxWorkers]; };
struct LevelPtrs { void *lv[kMaxWorkers]; uint32_t *sp[kMaxWorkers]; };
struct LevelCPtrs { const void *lv[kMaxWorkers]; const uint32_t *sp[kMaxWorkers]; };

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  The 32x32->64 products map to v_mad_u64_u32, the two
// three-way xors of a round to v_bitop3_b32; the key schedule depends on the seed only and stays in
// scalar registers.
// ---------------------------------------------------------------------------------------------
struct Words4 { uint32_t w[4]; };

// a ^ b ^ c in one instruction: gfx950's three-input bitwise op with truth table 0x96
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; r++) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    Words4 o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

// The four random words of the coordinates 4*call .. 4*call+3 of one worker (Eq. (2) draws).
__device__ __forceinline__ Words4 random_words(uint64_t seed, uint32_t worker, uint64_t call)
{
    return philox4x32_10((uint32_t)call, (uint32_t)(call >> 32), worker, 0u,
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

// ---------------------------------------------------------------------------------------------
// Per-call constants derived from the norm on the device (Algorithm 1's normalisation, y = |x| / norm).
// ---------------------------------------------------------------------------------------------
struct Scale {
    float scale;   // s / norm (linear) or 2^(s-1) / norm (exponential); 0 if the norm is unusable
    float top;     // s (linear) or 2^(s-1) (exponential) as a float
    float full;    // the norm: |x| >= full is y = 1, the top level with certainty; NaN (never reached) if the norm is unusable
};

template <int SCHEME>
__device__ __forceinline__ Scale make_scale(float norm, int s)
{
    Scale sc;
    sc.top = SCHEME == 0 ? (float)s : __uint_as_float((uint32_t)(127 + s - 1) << 23);
    const float q = sc.top / norm;                          // correctly rounded division
    const bool ok = (norm > 0.0f) && (norm <= 3.402823466e+38f) && (q <= 3.402823466e+38f);
    sc.scale = ok ? q : 0.0f;                               // zero / non-finite norm => every code is 0
    sc.full = ok ? norm : __builtin_nanf("");
    return sc;
}

// ---------------------------------------------------------------------------------------------
// Definition 1 / Eq. (2) for one coordinate.  Both return the signed level as a float whose
// integer conversion is exact; `value` is what is added to the sum, `code` what is stored.
// ---------------------------------------------------------------------------------------------
template <int SCHEME> struct Round;

// min(t, top) for t >= -0, and 0 for a NaN t (a NaN or Inf coordinate times a zero scale, or a NaN
// coordinate): v_med3_f32 returns the smallest of its non-NaN operands when one operand is a NaN, so the
// clamp at the top level and the "a NaN rounds to code 0" rule cost one instruction together.
__device__ __forceinline__ float clamp_nan_to_zero(float t, float top)
{
    return __builtin_amdgcn_fmed3f(t, 0.0f, top);
}

// Linear grid l_u = (s-u)/s: t = y*s lies between h and h+1; the upper one is taken iff U' < t-h.
template <> struct Round<0> {
    static __device__ __forceinline__ float value(float x, const Scale &sc, uint32_t r)
    {
        const float u = (float)r * 0x1.fffffep-33f;                       // U' in [0,1)
        const float ax = __builtin_fabsf(x);
        const float v = __builtin_fmaf(ax, sc.scale, -u);                 // t - U', one rounding
        const float c = clamp_nan_to_zero(__builtin_ceilf(v), sc.top);   // clamp at the top level
        return __builtin_copysignf(ax >= sc.full ? sc.top : c, x);       // y = 1 sits on the top level
    }
    static __device__ __forceinline__ int code_of_value(float value) { return (int)value; }
    static __device__ __forceinline__ int code(float x, const Scale &sc, uint32_t r) { return (int)value(x, sc, r); }
};

// Exponential grid {0} u {2^-j}: z = y*2^(s-1); a binary32 z >= 1 is rounded to a neighbouring power of
// two by adding 23 random bits to its mantissa; z < 1 is first moved to 1+z in [1,2).
template <> struct Round<1> {
    static __device__ __forceinline__ float value(float x, const Scale &sc, uint32_t r)
    {
        const float ax = __builtin_fabsf(x);
        const float z = ax >= sc.full ? sc.top : clamp_nan_to_zero(ax * sc.scale, sc.top);   // y = 1 sits on the top level
        const float one = z < 1.0f ? 1.0f : 0.0f;
        const float w = z + one;
        const uint32_t b = __float_as_uint(w) + (r >> 9);
        const float p2 = __uint_as_float(b & 0x7F800000u) - one;          // 0, 1, 2, 4, ..
        return __builtin_copysignf(p2, x);
    }
    // value = +-2^(k-1) or 0  ->  code = +-k or 0
    static __device__ __forceinline__ int code_of_value(float value)
    {
        const uint32_t b = __float_as_uint(value);
        const int k = max((int)((b >> 23) & 0xFFu) - 126, 0);
        return (b >> 31) ? -k : k;
    }
    // The code without the detour over the value: the rounded w = z (+1 if z < 1) has exponent field E, and
    // k = E - 126 for z >= 1 (value 2^(E-127)), k = E - 127 for z < 1 (value 0 or 1).
    static __device__ __forceinline__ int code(float x, const Scale &sc, uint32_t r)
    {
        const float ax = __builtin_fabsf(x);
        const float z = ax >= sc.full ? sc.top : clamp_nan_to_zero(ax * sc.scale, sc.top);   // y = 1 sits on the top level
        const bool small = z < 1.0f;
        const float w = z + (small ? 1.0f : 0.0f);
        const uint32_t b = __float_as_uint(w) + (r >> 9);
        const int k = (int)(b >> 23) - (small ? 127 : 126);
        return x < 0.0f ? -k : k;
    }
};

// Four consecutive coordinates of a gradient (vector v); nvalid < 4 of them exist at the ragged end, zeros beyond.
__device__ __forceinline__ f32x4 load_coords(const float *x, int64_t v, int nvalid)
{
    if (nvalid == 4) return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(x) + v);
    f32x4 a = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *t = x + (v << 2);
    if (nvalid > 0) a.x = t[0];
    if (nvalid > 1) a.y = t[1];
    if (nvalid > 2) a.z = t[2];
    return a;
}

// Four int8 codes as one word, coordinate i in byte i.
__device__ __forceinline__ uint32_t pack_bytes(const int *q)
{
    return (uint32_t)(q[0] & 255) | ((uint32_t)(q[1] & 255) << 8) | ((uint32_t)(q[2] & 255) << 16) | ((uint32_t)(q[3] & 255) << 24);
}

// Short draws: coordinate j of a vector takes the low (j even) or high (j odd) half of word j / 2 of the vector's pair
// of Philox words, moved to the top of a 32-bit word with zeros below.
__device__ __forceinline__ uint32_t short_draw(const uint32_t *pair, int j)
{
    return (j & 1) ? (pair[j >> 1] & 0xFFFF0000u) : (pair[j >> 1] << 16);
}

// ---------------------------------------------------------------------------------------------
// Wave reductions for the norm: DPP inside a row of 16 lanes (quad permutes, then the two mirror
// patterns), ds_swizzle across the two rows of a half wave, readlane across the halves.
// Every lane of the wave must be active.  The result is uniform.
// ---------------------------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ uint32_t dpp32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL> __device__ __forceinline__ double dpp64(double v)
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = dpp32<CTRL>((uint32_t)b), hi = dpp32<CTRL>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ uint32_t swizzle_xor16(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);   // bit-mask mode: lane ^ 16
}
constexpr int kDppQuadXor1 = 0xB1;     // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;     // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // row_half_mirror: lane i <-> 7-i of each 8
constexpr int kDppMirror = 0x140;      // row_mirror:      lane i <-> 15-i of each 16

// Short draws (16 random bits per coordinate): one Philox call serves the eight coordinates of two
// neighbouring vectors 2c and 2c+1.  To keep every load and store of a wave contiguous, a wave takes 128
// consecutive vectors and lane l owns vectors l ("A") and 64 + l ("B") of them.  Even lane 2i runs the call
// of vectors 2i, 2i+1 of the A half, odd lane 2i+1 the call of vectors 2i, 2i+1 of the B half, and the two
// lanes swap the half of the words the other needs (one DPP exchange of two registers).  Afterwards
// word pair `a` rounds the lane's A vector and `b` its B vector; coordinate j of a vector takes the low
// (j even) or high (j odd) half of word j / 2 of its pair, moved to the top of a 32-bit word with zeros
// below, so that the rounding rules apply unchanged.  Every lane of the wave must be active.
struct ShortDraws { uint32_t a[2], b[2]; };
__device__ __forceinline__ ShortDraws share_short_draws(const Words4 &r, bool odd)
{
    const uint32_t got0 = dpp32<kDppQuadXor1>(odd ? r.w[0] : r.w[2]);
    const uint32_t got1 = dpp32<kDppQuadXor1>(odd ? r.w[1] : r.w[3]);
    ShortDraws o;
    o.a[0] = odd ? got0 : r.w[0]; o.a[1] = odd ? got1 : r.w[1];
    o.b[0] = odd ? r.w[2] : got0; o.b[1] = odd ? r.w[3] : got1;
    return o;
}

__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp64<kDppQuadXor1>(v);
    v += dpp64<kDppQuadXor2>(v);
    v += dpp64<kDppHalfMirror>(v);
    v += dpp64<kDppMirror>(v);
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = swizzle_xor16((uint32_t)b), hi = swizzle_xor16((uint32_t)(b >> 32));
    v += __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    const uint64_t t = (uint64_t)__double_as_longlong(v);
    const uint32_t lo0 = __builtin_amdgcn_readlane((int)(uint32_t)t, 0), hi0 = __builtin_amdgcn_readlane((int)(uint32_t)(t >> 32), 0);
    const uint32_t lo1 = __builtin_amdgcn_readlane((int)(uint32_t)t, 32), hi1 = __builtin_amdgcn_readlane((int)(uint32_t)(t >> 32), 32);
    return __longlong_as_double((long long)(((uint64_t)hi0 << 32) | lo0)) +
           __longlong_as_double((long long)(((uint64_t)hi1 << 32) | lo1));
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
    v = max(v, dpp32<kDppQuadXor1>(v));
    v = max(v, dpp32<kDppQuadXor2>(v));
    v = max(v, dpp32<kDppHalfMirror>(v));
    v = max(v, dpp32<kDppMirror>(v));
    v = max(v, swizzle_xor16(v));
    return max((uint32_t)__builtin_amdgcn_readlane((int)v, 0), (uint32_t)__builtin_amdgcn_readlane((int)v, 32));
}

}  // namespace gq
