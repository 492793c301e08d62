// Algorithm 1's aggregation step and Eq. (1) on MI355X (gfx950): the integer sum of stored codes and its
// dequantisation.  The contract of the entry points is stated in include/gqsgd.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 1's aggregation step on stored codes.  Same ownership as the fused kernel: a lane owns four
// coordinates, i.e. one 32-bit (8-bit codes) or 16-bit (4-bit codes) word of every worker's level
// buffer and a nibble of its sign words; loads and the 128-bit stores of a wave are contiguous.
// =============================================================================================
constexpr int kAggBlock = 128;

template <int SCHEME, int PACK>
__global__ void __launch_bounds__(kAggBlock)
int_aggregate_kernel(LevelCPtrs L, int K, int64_t d, int64_t v_begin, void *__restrict__ agg_out, int agg_fmt)
{
    constexpr bool kNibble = (PACK == GQ_PACK_I4 || PACK == GQ_PACK_U4_SIGNPLANE);
    constexpr bool kPlane = (PACK == GQ_PACK_U8_SIGNPLANE || PACK == GQ_PACK_U4_SIGNPLANE);
    // Packed two's-complement nibbles are decoded through a 256-entry LDS table indexed by a byte: the
    // entry holds the integer values of both nibbles, each biased by 128, in its two 16-bit halves, so
    // that one 32-bit add accumulates two coordinates (K * 192 < 2^16, no carry between the halves).
    constexpr bool kLut = (PACK == GQ_PACK_I4);
    constexpr int kBias = 128;
    __shared__ uint32_t lut[kLut ? 256 : 1];
    if (kLut) {
        for (int b = threadIdx.x; b < 256; b += kAggBlock) {
            uint32_t e = 0;
            for (int h = 0; h < 2; h++) {
                const int q = ((int)((uint32_t)b << (28 - 4 * h))) >> 28;
                const int mag = (int)((1u << abs(q)) >> 1);
                const int val = SCHEME == 0 ? q : (q < 0 ? -mag : mag);
                e |= (uint32_t)(val + kBias) << (16 * h);
            }
            lut[b] = e;
        }
        __syncthreads();
    }
    const int64_t v = v_begin + (int64_t)blockIdx.x * kAggBlock + threadIdx.x;     // v_begin is a multiple of 8
    const int64_t nfull = d >> 2;
    const int nvalid = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
    if (nvalid == 0) return;

    struct Unit { uint32_t codes, signs; };
    auto fetch = [&](int w) {
        Unit t;
        if (!kNibble) {
            if (nvalid == 4) {
                t.codes = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(L.lv[w]) + v);
            } else {
                const uint8_t *b = reinterpret_cast<const uint8_t *>(L.lv[w]) + (v << 2);
                t.codes = 0;
                for (int i = 0; i < nvalid; i++) t.codes |= (uint32_t)b[i] << (8 * i);
            }
        } else {
            if (nvalid == 4) {
                t.codes = __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(L.lv[w]) + v);
            } else {
                const uint8_t *b = reinterpret_cast<const uint8_t *>(L.lv[w]) + (v << 1);
                t.codes = b[0];
                if (nvalid == 3) t.codes |= (uint32_t)b[1] << 8;
            }
        }
        t.signs = kPlane ? (L.sp[w][v >> 3] >> (4 * (int)(v & 7))) & 15u : 0u;
        return t;
    };
    int a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    auto value = [&](const Unit &t, int i) {
        int q;
        if (PACK == GQ_PACK_I8)      q = (int)(int8_t)(t.codes >> (8 * i));
        else if (PACK == GQ_PACK_I4) q = ((int)(t.codes << (28 - 4 * i))) >> 28;
        else if (PACK == GQ_PACK_U8_SIGNPLANE) q = (int)((t.codes >> (8 * i)) & 255u);
        else                         q = (int)((t.codes >> (4 * i)) & 15u);
        if (SCHEME == 0) return (kPlane && ((t.signs >> i) & 1u)) ? -q : q;
        const bool neg = kPlane ? (((t.signs >> i) & 1u) != 0u) : (q < 0);
        const int mag = (int)((1u << abs(q)) >> 1);                  // 2^(k-1), 0 for k = 0
        return neg ? -mag : mag;
    };
    uint32_t s01 = 0, s23 = 0;
    auto add = [&](const Unit &t) {
        if (kLut) {
            s01 += lut[t.codes & 255u];
            s23 += lut[(t.codes >> 8) & 255u];
        } else {
            a0 += value(t, 0); a1 += value(t, 1); a2 += value(t, 2); a3 += value(t, 3);
        }
    };
    // eight workers' loads are issued before the first is consumed
    int w = 0;
    for (; w + 8 <= K; w += 8) {
        Unit t[8];
#pragma unroll
        for (int j = 0; j < 8; j++) t[j] = fetch(w + j);
#pragma unroll
        for (int j = 0; j < 8; j++) add(t[j]);
    }
    for (; w + 2 <= K; w += 2) {
        const Unit t0 = fetch(w), t1 = fetch(w + 1);
        add(t0); add(t1);
    }
    for (; w < K; w++) add(fetch(w));
    if (kLut) {
        a0 = (int)(s01 & 0xFFFFu) - K * kBias; a1 = (int)(s01 >> 16) - K * kBias;
        a2 = (int)(s23 & 0xFFFFu) - K * kBias; a3 = (int)(s23 >> 16) - K * kBias;
    }

    if (agg_fmt == GQ_AGG_I32) {
        if (nvalid == 4) {
            const i32x4 o = {a0, a1, a2, a3};
            __builtin_nontemporal_store(o, reinterpret_cast<i32x4 *>(agg_out) + v);
        } else {
            int *o = reinterpret_cast<int *>(agg_out) + (v << 2);
            o[0] = a0;
            if (nvalid > 1) o[1] = a1;
            if (nvalid > 2) o[2] = a2;
        }
    } else {
        if (nvalid == 4) {
            const i16x4 o = {(short)a0, (short)a1, (short)a2, (short)a3};
            __builtin_nontemporal_store(o, reinterpret_cast<i16x4 *>(agg_out) + v);
        } else {
            short *o = reinterpret_cast<short *>(agg_out) + (v << 2);
            o[0] = (short)a0;
            if (nvalid > 1) o[1] = (short)a1;
            if (nvalid > 2) o[2] = (short)a2;
        }
    }
}

// =============================================================================================
// Algorithm 1's aggregation step on packed 4-bit codes, for workgroups that lie wholly inside the buffer.  The
// one-vector-per-lane kernel above moves two bytes per lane and load, which leaves it bound by
// instruction issue, not by HBM.  Here a lane owns EIGHT coordinates: one 32-bit load of codes (and one
// byte of sign bits) per worker.  Every byte of codes, together with its two sign bits in the sign-plane
// format, indexes an LDS table whose entry holds the integer values of both coordinates, each biased to
// be non-negative, in its two 16-bit halves: one table read and one 32-bit add accumulate two
// coordinates (the biased sums stay below 2^16 for K <= 64: at most (64 + 128) * 64 resp. (15 + 16) * 64).
// 32-bit sums are staged in LDS so that the workgroup writes two contiguous runs of 16 bytes per thread;
// 16-bit sums are 16 bytes per lane already.  Not for the exponential grid in the sign-plane format
// (values up to 2^14 do not fit the halves): that combination keeps the kernel above.
// =============================================================================================
constexpr int kNibBlock = 128;
constexpr int kNibCoords = 8;

template <int SCHEME, bool PLANE>
__global__ void __launch_bounds__(kNibBlock)
int_aggregate_nibble_kernel(LevelCPtrs L, int K, void *__restrict__ agg_out, int agg_fmt)
{
    static_assert(!(SCHEME == 1 && PLANE), "exponential sign-plane values do not fit 16-bit halves");
    constexpr int kEntries = PLANE ? 1024 : 256;
    constexpr int kBias = PLANE ? 16 : 128;
    __shared__ uint32_t lut[kEntries];
    __shared__ int stage[kNibBlock * kNibCoords];
    for (int e = threadIdx.x; e < kEntries; e += kNibBlock) {
        uint32_t entry = 0;
        for (int h = 0; h < 2; h++) {
            const int nibble = (e >> (4 * h)) & 15;
            int val;
            if (PLANE) {
                val = nibble;                                             // linear magnitude
                if ((e >> (8 + h)) & 1) val = -val;
            } else {
                const int q = (nibble ^ 8) - 8;                           // two's complement nibble
                const int mag = (int)((1u << abs(q)) >> 1);               // 2^(k-1), 0 for k = 0
                val = SCHEME == 0 ? q : (q < 0 ? -mag : mag);
            }
            entry |= (uint32_t)(val + kBias) << (16 * h);
        }
        lut[e] = entry;
    }
    __syncthreads();
    const int64_t u = (int64_t)blockIdx.x * kNibBlock + threadIdx.x;      // eight coordinates 8u .. 8u+7

    uint32_t s01 = 0, s23 = 0, s45 = 0, s67 = 0;
    auto add = [&](uint32_t c, uint32_t sb) {
        if (PLANE) {
            s01 += lut[(c & 255u) | ((sb & 3u) << 8)];
            s23 += lut[((c >> 8) & 255u) | ((sb & 12u) << 6)];
            s45 += lut[((c >> 16) & 255u) | ((sb & 48u) << 4)];
            s67 += lut[(c >> 24) | ((sb & 192u) << 2)];
        } else {
            s01 += lut[c & 255u];
            s23 += lut[(c >> 8) & 255u];
            s45 += lut[(c >> 16) & 255u];
            s67 += lut[c >> 24];
        }
    };
    auto codes_of = [&](int w) { return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(L.lv[w]) + u); };
    auto signs_of = [&](int w) { return PLANE ? (uint32_t)reinterpret_cast<const uint8_t *>(L.sp[w])[u] : 0u; };
    int w = 0;
    for (; w + 8 <= K; w += 8) {                     // eight workers' loads are issued before the first is consumed
        uint32_t c[8], sb[8];
#pragma unroll
        for (int j = 0; j < 8; j++) { c[j] = codes_of(w + j); sb[j] = signs_of(w + j); }
#pragma unroll
        for (int j = 0; j < 8; j++) add(c[j], sb[j]);
    }
    if (w + 4 <= K) {
        uint32_t c[4], sb[4];
#pragma unroll
        for (int j = 0; j < 4; j++) { c[j] = codes_of(w + j); sb[j] = signs_of(w + j); }
#pragma unroll
        for (int j = 0; j < 4; j++) add(c[j], sb[j]);
        w += 4;
    }
    if (w + 2 <= K) {
        const uint32_t c0 = codes_of(w), c1 = codes_of(w + 1), b0 = signs_of(w), b1 = signs_of(w + 1);
        add(c0, b0); add(c1, b1);
        w += 2;
    }
    if (w < K) add(codes_of(w), signs_of(w));
    const int off = K * kBias;
    const int a0 = (int)(s01 & 0xFFFFu) - off, a1 = (int)(s01 >> 16) - off, a2 = (int)(s23 & 0xFFFFu) - off, a3 = (int)(s23 >> 16) - off;
    const int a4 = (int)(s45 & 0xFFFFu) - off, a5 = (int)(s45 >> 16) - off, a6 = (int)(s67 & 0xFFFFu) - off, a7 = (int)(s67 >> 16) - off;
    if (agg_fmt == GQ_AGG_I16) {
        const u32x4 o = {((uint32_t)a0 & 0xFFFFu) | ((uint32_t)a1 << 16), ((uint32_t)a2 & 0xFFFFu) | ((uint32_t)a3 << 16),
                         ((uint32_t)a4 & 0xFFFFu) | ((uint32_t)a5 << 16), ((uint32_t)a6 & 0xFFFFu) | ((uint32_t)a7 << 16)};
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(agg_out) + u);
    } else {
        const int t = (int)threadIdx.x;
        *reinterpret_cast<i32x4 *>(&stage[8 * t]) = i32x4{a0, a1, a2, a3};
        *reinterpret_cast<i32x4 *>(&stage[8 * t + 4]) = i32x4{a4, a5, a6, a7};
        __syncthreads();
        i32x4 *out = reinterpret_cast<i32x4 *>(agg_out) + (int64_t)blockIdx.x * (kNibBlock * kNibCoords / 4);
        __builtin_nontemporal_store(*reinterpret_cast<const i32x4 *>(&stage[4 * t]), out + t);
        __builtin_nontemporal_store(*reinterpret_cast<const i32x4 *>(&stage[4 * (kNibBlock + t)]), out + kNibBlock + t);
    }
}

// =============================================================================================
// Eq. (1): out = norm * A / (n * unit).
// =============================================================================================
template <typename T>
__global__ void __launch_bounds__(kBlock)
dequantize_kernel(const T *__restrict__ agg, int64_t d, const float *__restrict__ norm, float deq_div,
                  float *__restrict__ out)
{
    typedef T tx4 __attribute__((ext_vector_type(4)));
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t nfull = d >> 2;
    const int nvalid = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
    if (nvalid == 0) return;
    const float nrm = *norm;
    const float c = (nrm > 0.0f && nrm <= 3.402823466e+38f) ? nrm / deq_div : 0.0f;
    if (nvalid == 4) {
        const tx4 a = __builtin_nontemporal_load(reinterpret_cast<const tx4 *>(agg) + v);
        const f32x4 o = {(float)a.x * c, (float)a.y * c, (float)a.z * c, (float)a.w * c};
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(out) + v);
    } else {
        for (int i = 0; i < nvalid; i++) out[(v << 2) + i] = (float)agg[(v << 2) + i] * c;
    }
}

}  // namespace gq

using namespace gq;

extern "C" {

gq_status gq_int_aggregate(const void *const *levels, const uint32_t *const *signplanes, int K, int64_t d,
                           const gq_params *p, void *agg_out, void *hip_stream)
{
    gq_status st = check_params(p, true, true);
    if (st != GQ_OK) return st;
    if (!levels || K < 1 || K > GQ_MAX_WORKERS || d < 0) return GQ_ERR_INVALID_ARG;
    st = gq_check_width(p, K);
    if (st != GQ_OK) return st;
    const bool plane = p->pack >= GQ_PACK_U8_SIGNPLANE;
    if (plane && !signplanes) return GQ_ERR_INVALID_ARG;
    LevelCPtrs L;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(levels[i], 16)) return GQ_ERR_INVALID_ARG;
        L.lv[i] = levels[i];
        L.sp[i] = nullptr;
        if (plane) {
            if (d > 0 && !aligned(signplanes[i], 4)) return GQ_ERR_INVALID_ARG;
            L.sp[i] = signplanes[i];
        }
    }
    if (d > 0 && !aligned(agg_out, 16)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t nvec = (d + 3) / 4;
    // packed 4-bit codes: the workgroups that lie wholly inside the buffer take the eight-coordinates-per-lane
    // kernel, the ragged rest (fewer than 1024 coordinates) the general one
    int64_t v_begin = 0;
    const bool nibble_lut = p->pack == GQ_PACK_I4 || (p->pack == GQ_PACK_U4_SIGNPLANE && p->scheme == GQ_LINEAR);
    if (nibble_lut) {
        const int64_t wide_blocks = d / (kNibBlock * kNibCoords);
        if (!grid_fits(wide_blocks, kNibBlock)) return GQ_ERR_INVALID_ARG;
        if (wide_blocks > 0) {
            const dim3 wgrid((unsigned)wide_blocks), wblock(kNibBlock);
            if (p->pack == GQ_PACK_U4_SIGNPLANE) hipLaunchKernelGGL((int_aggregate_nibble_kernel<0, true>), wgrid, wblock, 0, s, L, K, agg_out, p->agg);
            else if (p->scheme == GQ_LINEAR) hipLaunchKernelGGL((int_aggregate_nibble_kernel<0, false>), wgrid, wblock, 0, s, L, K, agg_out, p->agg);
            else hipLaunchKernelGGL((int_aggregate_nibble_kernel<1, false>), wgrid, wblock, 0, s, L, K, agg_out, p->agg);
            if (launched() != GQ_OK) return GQ_ERR_DEVICE;
            v_begin = wide_blocks * (kNibBlock * kNibCoords / 4);
            if (v_begin >= nvec) return GQ_OK;
        }
    }
    const int64_t blocks = (nvec - v_begin + kAggBlock - 1) / kAggBlock;
    if (!grid_fits(blocks, kAggBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kAggBlock);
#define GQ_AGG(SC, PK) hipLaunchKernelGGL((int_aggregate_kernel<SC, PK>), grid, block, 0, s, L, K, d, v_begin, agg_out, p->agg)
    if (p->scheme == GQ_LINEAR) {
        switch (p->pack) {
        case GQ_PACK_I8: GQ_AGG(0, GQ_PACK_I8); break;
        case GQ_PACK_I4: GQ_AGG(0, GQ_PACK_I4); break;
        case GQ_PACK_U8_SIGNPLANE: GQ_AGG(0, GQ_PACK_U8_SIGNPLANE); break;
        default: GQ_AGG(0, GQ_PACK_U4_SIGNPLANE); break;
        }
    } else {
        switch (p->pack) {
        case GQ_PACK_I8: GQ_AGG(1, GQ_PACK_I8); break;
        case GQ_PACK_I4: GQ_AGG(1, GQ_PACK_I4); break;
        case GQ_PACK_U8_SIGNPLANE: GQ_AGG(1, GQ_PACK_U8_SIGNPLANE); break;
        default: GQ_AGG(1, GQ_PACK_U4_SIGNPLANE); break;
        }
    }
#undef GQ_AGG
    return launched();
}

gq_status gq_dequantize(const void *agg, int64_t d, const float *norm, const gq_params *p, int K, float *out,
                        void *hip_stream)
{
    const gq_status st = check_params(p, false, true);
    if (st != GQ_OK) return st;
    if (K < 1 || K > GQ_MAX_WORKERS || d < 0 || !aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    if (d > 0 && (!aligned(agg, 16) || !aligned(out, 16))) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    const int64_t nvec = (d + 3) / 4;
    const int64_t blocks = (nvec + kBlock - 1) / kBlock;
    if (!grid_fits(blocks, kBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kBlock);
    const float div = dequant_divisor(p, K);
    hipStream_t s = (hipStream_t)hip_stream;
    if (p->agg == GQ_AGG_I32)
        hipLaunchKernelGGL(dequantize_kernel<int>, grid, block, 0, s, (const int *)agg, d, norm, div, out);
    else
        hipLaunchKernelGGL(dequantize_kernel<short>, grid, block, 0, s, (const short *)agg, d, norm, div, out);
    return launched();
}

}  // extern "C"
