// Kernels and C entry points of the Global-QSGD hot path for MI355X (gfx950).
// The contract of every entry point is stated in include/gqsgd.h.
//
// Data layout.  Every buffer is a flat array in HBM.  A lane always owns four consecutive
// coordinates of a gradient (one 128-bit load per worker), which are also the four words of one
// Philox call, so that a wave reads 1 KiB of contiguous gradient per worker and load.  All traffic is
// streaming with no reuse: nothing is staged through LDS except the few words of the reductions.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"

namespace gq {

struct GradPtrs { const float *x[kMaxWorkers]; };
struct LevelPtrs { void *lv[kMaxWorkers]; uint32_t *sp[kMaxWorkers]; };
struct LevelCPtrs { const void *lv[kMaxWorkers]; const uint32_t *sp[kMaxWorkers]; };

// =============================================================================================
// Algorithm 1 line 1: global norm.  Pass 1 reduces the gradients to 8-byte partials (a uint32 bit
// pattern for the max norm, a binary64 sum of squares otherwise); pass 2 folds the partials in a
// fixed order in one block and writes the norm and the status word.  No atomics: reproducible.
//
// Pass 1 comes in two shapes.  (inf,inf) and (2,2) do not need per-worker results, so a block
// takes a contiguous tile of coordinates and reads it from ALL workers, K 128-bit loads in flight
// per lane -- the access pattern of the fused kernel, which streams fastest.  (2,inf) needs one
// sum per worker: there a block strides over a single worker's gradient.
// =============================================================================================
constexpr int kNormTileBlock = 128;            // threads per block, tile shape
constexpr int kNormTileVec = 4;                // 128-bit vectors per lane and worker in one tile
constexpr int kNormMaxTileBlocks = 1 << 16;    // cap on the number of tile partials
constexpr int kNormVecPerThread = 8;           // per-worker shape: target loads per thread
constexpr int kNormMaxBlocksPerWorker = 1024;
constexpr int kNormFinalBlock = 1024;

static inline int norm_blocks_per_worker(int64_t d)
{
    const int64_t nvec = d / 4;
    int64_t b = (nvec + (int64_t)kBlock * kNormVecPerThread - 1) / ((int64_t)kBlock * kNormVecPerThread);
    if (b < 1) b = 1;
    if (b > kNormMaxBlocksPerWorker) b = kNormMaxBlocksPerWorker;
    return (int)b;
}

// tiles of kNormTileBlock*kNormTileVec vectors; a block takes `tiles_per_block` consecutive tiles
static inline void norm_tile_shape(int64_t d, int64_t *blocks, int64_t *tiles_per_block)
{
    const int64_t nvec = d / 4;
    const int64_t per_tile = (int64_t)kNormTileBlock * kNormTileVec;
    int64_t tiles = (nvec + per_tile - 1) / per_tile;
    if (tiles < 1) tiles = 1;
    const int64_t tpb = (tiles + kNormMaxTileBlocks - 1) / kNormMaxTileBlocks;
    *tiles_per_block = tpb;
    *blocks = (tiles + tpb - 1) / tpb;
}

__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// Per-lane accumulator of either norm, and its reduction over the block into one 8-byte word.
template <bool MAXNORM> struct NormAcc {
    uint32_t m0 = 0, m1 = 0, m2 = 0, m3 = 0;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    __device__ __forceinline__ void take(const f32x4 &a)
    {
        if (MAXNORM) {
            // |x| compared as unsigned bit patterns: ordered like the values, NaN above Inf above finite
            m0 = max(m0, abs_bits(a.x)); m1 = max(m1, abs_bits(a.y));
            m2 = max(m2, abs_bits(a.z)); m3 = max(m3, abs_bits(a.w));
        } else {
            const double x0 = a.x, x1 = a.y, x2 = a.z, x3 = a.w;   // squares are exact in binary64
            a0 = __builtin_fma(x0, x0, a0); a1 = __builtin_fma(x1, x1, a1);
            a2 = __builtin_fma(x2, x2, a2); a3 = __builtin_fma(x3, x3, a3);
        }
    }
    // every thread of the block must call this; the result is valid in thread 0
    template <int BLOCK> __device__ __forceinline__ uint64_t block_reduce(uint64_t *sh) const
    {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        uint64_t mine;
        if (MAXNORM) mine = wave_max(max(max(m0, m1), max(m2, m3)));
        else         mine = (uint64_t)__double_as_longlong(wave_sum((a0 + a1) + (a2 + a3)));
        if (lane == 0) sh[wave] = mine;
        __syncthreads();
        uint64_t r = sh[0];
        for (int i = 1; i < BLOCK / 64; i++) {
            if (MAXNORM) r = max(r, sh[i]);
            else r = (uint64_t)__double_as_longlong(__longlong_as_double((long long)r) + __longlong_as_double((long long)sh[i]));
        }
        return r;
    }
};

template <bool MAXNORM, int KT>
__global__ void __launch_bounds__(kNormTileBlock)
norm_tile_kernel(GradPtrs P, int K, int64_t d, int64_t tiles_per_block, uint64_t *__restrict__ partial)
{
    const int64_t nvec = d >> 2;
    const int Kc = KT > 0 ? KT : K;
    NormAcc<MAXNORM> acc;
    int64_t base = (int64_t)blockIdx.x * tiles_per_block * (kNormTileBlock * kNormTileVec) + threadIdx.x;
    for (int64_t t = 0; t < tiles_per_block; t++, base += kNormTileBlock * kNormTileVec) {
#pragma unroll
        for (int j = 0; j < kNormTileVec; j++) {
            const int64_t v = base + (int64_t)j * kNormTileBlock;
            if (v < nvec) {
                if (KT > 0) {
                    f32x4 g[KT > 0 ? KT : 1];                   // all K loads in flight (measured best, also at K = 32)
#pragma unroll
                    for (int w = 0; w < KT; w++) g[w] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w]) + v);
#pragma unroll
                    for (int w = 0; w < KT; w++) acc.take(g[w]);
                } else {
                    int w = 0;
                    for (; w + 4 <= Kc; w += 4) {
                        const f32x4 g0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w]) + v);
                        const f32x4 g1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w + 1]) + v);
                        const f32x4 g2 = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w + 2]) + v);
                        const f32x4 g3 = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w + 3]) + v);
                        acc.take(g0); acc.take(g1); acc.take(g2); acc.take(g3);
                    }
                    for (; w < Kc; w++) acc.take(__builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w]) + v));
                }
            }
        }
    }
    if (blockIdx.x == 0 && (int64_t)threadIdx.x < (d & 3)) {     // ragged tail: up to three coordinates per worker
        for (int w = 0; w < Kc; w++) {
            const f32x4 a = {P.x[w][(nvec << 2) + threadIdx.x], 0.0f, 0.0f, 0.0f};
            acc.take(a);
        }
    }
    __shared__ uint64_t sh[kNormTileBlock / 64];
    const uint64_t r = acc.template block_reduce<kNormTileBlock>(sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = r;
}

template <bool MAXNORM>
__global__ void __launch_bounds__(kBlock) norm_partial_kernel(GradPtrs P, int64_t d, int bpw, uint64_t *partial)
{
    const int worker = blockIdx.x / bpw;
    const int blk = blockIdx.x - worker * bpw;
    const float *x = P.x[worker];
    const f32x4 *xv = reinterpret_cast<const f32x4 *>(x);
    const int64_t nvec = d >> 2;
    const int64_t step = (int64_t)bpw * kBlock;
    int64_t v = (int64_t)blk * kBlock + threadIdx.x;
    NormAcc<MAXNORM> acc;
    for (; v + 3 * step < nvec; v += 4 * step) {
        const f32x4 b0 = __builtin_nontemporal_load(xv + v);
        const f32x4 b1 = __builtin_nontemporal_load(xv + v + step);
        const f32x4 b2 = __builtin_nontemporal_load(xv + v + 2 * step);
        const f32x4 b3 = __builtin_nontemporal_load(xv + v + 3 * step);
        acc.take(b0); acc.take(b1); acc.take(b2); acc.take(b3);
    }
    for (; v < nvec; v += step) acc.take(__builtin_nontemporal_load(xv + v));
    if (blk == 0 && (int64_t)threadIdx.x < (d & 3)) {            // ragged tail: up to three coordinates
        const f32x4 a = {x[(nvec << 2) + threadIdx.x], 0.0f, 0.0f, 0.0f};
        acc.take(a);
    }
    __shared__ uint64_t sh[kBlock / 64];
    const uint64_t r = acc.template block_reduce<kBlock>(sh);
    if (threadIdx.x == 0) partial[blockIdx.x] = r;
}

// Folds `groups` runs of `per_group` partials each.  kind: 0 = (inf,inf), 1 = (2,2), 2 = (2,inf).
__global__ void __launch_bounds__(kNormFinalBlock)
norm_final_kernel(const uint64_t *__restrict__ partial, int groups, int64_t per_group, int kind,
                  float *norm_out, uint32_t *status_flags)
{
    __shared__ uint64_t sh[kNormFinalBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t maxbits = 0;        // kind 0
    double total = 0.0;          // kind 1: sum over groups; kind 2: max over groups
    for (int w = 0; w < groups; w++) {
        const uint64_t *p = partial + (int64_t)w * per_group;
        uint32_t m = 0;
        double a = 0.0, b = 0.0, c = 0.0, e = 0.0;
        int64_t i = threadIdx.x;
        for (; i + 3 * kNormFinalBlock < per_group; i += 4 * kNormFinalBlock) {       // four loads in flight
            const uint64_t p0 = p[i], p1 = p[i + kNormFinalBlock], p2 = p[i + 2 * kNormFinalBlock], p3 = p[i + 3 * kNormFinalBlock];
            if (kind == 0) m = max(max(m, (uint32_t)p0), max(max((uint32_t)p1, (uint32_t)p2), (uint32_t)p3));
            else { a += __longlong_as_double((long long)p0); b += __longlong_as_double((long long)p1);
                   c += __longlong_as_double((long long)p2); e += __longlong_as_double((long long)p3); }
        }
        for (; i < per_group; i += kNormFinalBlock) {
            if (kind == 0) m = max(m, (uint32_t)p[i]);
            else a += __longlong_as_double((long long)p[i]);
        }
        const uint64_t mine = kind == 0 ? (uint64_t)wave_max(m) : (uint64_t)__double_as_longlong(wave_sum((a + b) + (c + e)));
        __syncthreads();
        if (lane == 0) sh[wave] = mine;
        __syncthreads();
        if (kind == 0) {
            for (int j = 0; j < kNormFinalBlock / 64; j++) maxbits = max(maxbits, (uint32_t)sh[j]);
        } else {
            double sw = 0.0;
            for (int j = 0; j < kNormFinalBlock / 64; j++) sw += __longlong_as_double((long long)sh[j]);
            if (kind == 1) total += sw;
            else total = (sw != sw || total != total) ? (sw + total) : (sw > total ? sw : total);  // NaN is sticky
        }
    }
    if (threadIdx.x == 0) {
        const float n = kind == 0 ? __uint_as_float(maxbits) : (float)__builtin_sqrt(total);
        *norm_out = n;
        if (status_flags) {
            uint32_t f = 0;
            if (!(__builtin_fabsf(n) <= 3.402823466e+38f)) f |= 1u;
            if (n == 0.0f) f |= 2u;
            *status_flags = f;
        }
    }
}

// =============================================================================================
// Algorithm 1 lines 2-5 and 9 fused: quantize the K workers' coordinates in registers, add the
// integer values, write the sum (and/or its dequantised mean, Eq. (1), and/or the packed codes).
//   SCHEME      0 linear, 1 exponential
//   KT          compile-time worker count (fully unrolled, K loads in flight), 0 = run-time K
//   LEVELS      also store every worker's packed codes
//   UNIFORM_HI  the high word of the Philox call index is the same for the whole launch
// =============================================================================================
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

// OR over the 8 lanes that share one 32-bit sign word.  Every lane of the wave must be active.
__device__ __forceinline__ uint32_t or_over_8_lanes(uint32_t v)
{
    v |= dpp32<kDppQuadXor1>(v);
    v |= dpp32<kDppQuadXor2>(v);
    v |= dpp32<kDppHalfMirror>(v);
    return v;
}

__device__ __forceinline__ void store_codes(void *lv, uint32_t *sp, int pack, int64_t v, int nvalid, int64_t d,
                                            int q0, int q1, int q2, int q3)
{
    const bool plane = pack >= 2;
    if (plane) {
        const uint32_t nib = (uint32_t)(q0 < 0) | ((uint32_t)(q1 < 0) << 1) | ((uint32_t)(q2 < 0) << 2) |
                             ((uint32_t)(q3 < 0) << 3);
        const uint32_t word = or_over_8_lanes(nib << (4 * (threadIdx.x & 7)));
        if ((threadIdx.x & 7) == 0 && ((v & ~(int64_t)7) << 2) < d) sp[v >> 3] = word;
        q0 = abs(q0); q1 = abs(q1); q2 = abs(q2); q3 = abs(q3);
    }
    if (nvalid == 0) return;
    if (pack == GQ_PACK_I8 || pack == GQ_PACK_U8_SIGNPLANE) {
        const uint32_t w = (uint32_t)(q0 & 255) | ((uint32_t)(q1 & 255) << 8) | ((uint32_t)(q2 & 255) << 16) |
                           ((uint32_t)(q3 & 255) << 24);
        if (nvalid == 4) {
            __builtin_nontemporal_store(w, reinterpret_cast<uint32_t *>(lv) + v);
        } else {
            uint8_t *b = reinterpret_cast<uint8_t *>(lv) + (v << 2);
            for (int i = 0; i < nvalid; i++) b[i] = (uint8_t)(w >> (8 * i));
        }
    } else {
        const uint32_t w = (uint32_t)(q0 & 15) | ((uint32_t)(q1 & 15) << 4) | ((uint32_t)(q2 & 15) << 8) |
                           ((uint32_t)(q3 & 15) << 12);
        if (nvalid == 4) {
            __builtin_nontemporal_store((uint16_t)w, reinterpret_cast<uint16_t *>(lv) + v);
        } else {
            uint8_t *b = reinterpret_cast<uint8_t *>(lv) + (v << 1);
            b[0] = (uint8_t)w;
            if (nvalid == 3) b[1] = (uint8_t)(w >> 8);
        }
    }
}

// Threads per workgroup of the fused kernel.  Small groups retire and refill wave slots at a finer
// grain, which measurably helps the HBM read/write mix of this kernel (64 > 128 > 256 on MI355X).
constexpr int kFusedBlock = 128;

// The integer sum of one lane's four coordinates.  Linear codes are summed as floats (exact: the
// sum stays below 2^24) and converted once; exponential values reach 2^30 and are summed as ints.
template <int SCHEME> struct Acc;
template <> struct Acc<0> {
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    __device__ __forceinline__ void add(float f0, float f1, float f2, float f3) { a0 += f0; a1 += f1; a2 += f2; a3 += f3; }
    __device__ __forceinline__ i32x4 get() const { return i32x4{(int)a0, (int)a1, (int)a2, (int)a3}; }
};
template <> struct Acc<1> {
    int a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    __device__ __forceinline__ void add(float f0, float f1, float f2, float f3) { a0 += (int)f0; a1 += (int)f1; a2 += (int)f2; a3 += (int)f3; }
    __device__ __forceinline__ i32x4 get() const { return i32x4{a0, a1, a2, a3}; }
};

// The launch covers the 4-coordinate vectors v0 <= v < vend of the buffers.  With UNIFORM_HI the
// host guarantees that the Philox call index (call_base + v) does not cross a multiple of 2^32 inside
// the launch, so the high counter word is a scalar: the first round and half of the second are then
// shared by all lanes or all workers and leave the vector ALU.
template <int SCHEME, int KT, bool LEVELS, bool UNIFORM_HI>
__global__ void __launch_bounds__(kFusedBlock)
quantize_aggregate_kernel(GradPtrs P, LevelPtrs L, int K, int64_t d, int64_t v0, int64_t vend, const float *__restrict__ norm, int s,
                          uint64_t seed, uint32_t worker0, uint64_t call_base, int pack,
                          void *__restrict__ agg_out, int agg_fmt, float *__restrict__ deq_out, float deq_div)
{
    const int64_t v = v0 + (int64_t)blockIdx.x * kFusedBlock + threadIdx.x;
    const int64_t nfull = d >> 2;
    const int nvalid = v >= vend ? 0 : (v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0));
    if (!LEVELS && nvalid == 0) return;          // with LEVELS the sign-plane exchange needs whole waves

    const float nrm = *norm;
    const Scale sc = make_scale<SCHEME>(nrm, s);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c_lo, c_hi;
    if (UNIFORM_HI) {
        const uint64_t first = call_base + (uint64_t)v0;                      // scalar
        c_hi = (uint32_t)(first >> 32);
        c_lo = (uint32_t)first + (uint32_t)(blockIdx.x * kFusedBlock + threadIdx.x);   // no carry (host)
    } else {
        const uint64_t call = call_base + (uint64_t)v;
        c_lo = (uint32_t)call;
        c_hi = (uint32_t)(call >> 32);
    }
    const int Kc = KT > 0 ? KT : K;

    Acc<SCHEME> acc;
    auto one_worker = [&](int w, const f32x4 &g) {
        const Words4 r = philox4x32_10(c_lo, c_hi, worker0 + (uint32_t)w, 0u, k0, k1);
        const float f0 = Round<SCHEME>::value(g.x, sc, r.w[0]);
        const float f1 = Round<SCHEME>::value(g.y, sc, r.w[1]);
        const float f2 = Round<SCHEME>::value(g.z, sc, r.w[2]);
        const float f3 = Round<SCHEME>::value(g.w, sc, r.w[3]);
        acc.add(f0, f1, f2, f3);
        if (LEVELS) {
            store_codes(L.lv[w], L.sp[w], pack, v, nvalid, d, Round<SCHEME>::code_of_value(f0),
                        Round<SCHEME>::code_of_value(f1), Round<SCHEME>::code_of_value(f2),
                        Round<SCHEME>::code_of_value(f3));
        }
    };
    if (KT > 0) {
        constexpr int kInFlight = KT > 16 ? 16 : (KT > 0 ? KT : 1);   // loads issued before the first is consumed
#pragma unroll
        for (int w0 = 0; w0 < KT; w0 += kInFlight) {
            f32x4 g[kInFlight];
            if (nvalid == 4) {                       // one branch per batch, not per worker
#pragma unroll
                for (int j = 0; j < kInFlight; j++)
                    g[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w0 + j]) + v);
            } else {
#pragma unroll
                for (int j = 0; j < kInFlight; j++) g[j] = load_coords(P.x[w0 + j], v, nvalid);
            }
#pragma unroll
            for (int j = 0; j < kInFlight; j++) one_worker(w0 + j, g[j]);
        }
    } else {
        int w = 0;
        for (; w + 4 <= Kc; w += 4) {
            const f32x4 g0 = load_coords(P.x[w], v, nvalid), g1 = load_coords(P.x[w + 1], v, nvalid);
            const f32x4 g2 = load_coords(P.x[w + 2], v, nvalid), g3 = load_coords(P.x[w + 3], v, nvalid);
            one_worker(w, g0); one_worker(w + 1, g1); one_worker(w + 2, g2); one_worker(w + 3, g3);
        }
        for (; w < Kc; w++) one_worker(w, load_coords(P.x[w], v, nvalid));
    }
    if (nvalid == 0) return;

    const i32x4 a = acc.get();
    if (agg_out) {
        if (agg_fmt == GQ_AGG_I32) {
            if (nvalid == 4) {
                __builtin_nontemporal_store(a, reinterpret_cast<i32x4 *>(agg_out) + v);
            } else {
                int *o = reinterpret_cast<int *>(agg_out) + (v << 2);
                o[0] = a.x;
                if (nvalid > 1) o[1] = a.y;
                if (nvalid > 2) o[2] = a.z;
            }
        } else {
            if (nvalid == 4) {
                const i16x4 o = {(short)a.x, (short)a.y, (short)a.z, (short)a.w};
                __builtin_nontemporal_store(o, reinterpret_cast<i16x4 *>(agg_out) + v);
            } else {
                short *o = reinterpret_cast<short *>(agg_out) + (v << 2);
                o[0] = (short)a.x;
                if (nvalid > 1) o[1] = (short)a.y;
                if (nvalid > 2) o[2] = (short)a.z;
            }
        }
    }
    if (deq_out) {
        const float c = sc.scale != 0.0f ? nrm / deq_div : 0.0f;     // Eq. (1): norm / (n * unit)
        if (nvalid == 4) {
            const f32x4 o = {(float)a.x * c, (float)a.y * c, (float)a.z * c, (float)a.w * c};
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(deq_out) + v);
        } else {
            float *o = deq_out + (v << 2);
            o[0] = (float)a.x * c;
            if (nvalid > 1) o[1] = (float)a.y * c;
            if (nvalid > 2) o[2] = (float)a.z * c;
        }
    }
}

// =============================================================================================
// Algorithm 1 lines 2-5 for one worker with the codes stored: a lane owns kQuantVec vectors of four
// coordinates, kQuantBlock vectors apart, and issues all its loads before the first Philox call.
// =============================================================================================
constexpr int kQuantBlock = 128;
constexpr int kQuantVec = 4;

template <int SCHEME, bool UNIFORM_HI>
__global__ void __launch_bounds__(kQuantBlock)
quantize_kernel(const float *__restrict__ x, void *__restrict__ lv, uint32_t *__restrict__ sp, int64_t d,
                const float *__restrict__ norm, int s, uint64_t seed, uint32_t worker, uint64_t call_base, int pack)
{
    const int64_t nfull = d >> 2;
    const int64_t base = (int64_t)blockIdx.x * (kQuantBlock * kQuantVec) + threadIdx.x;
    const Scale sc = make_scale<SCHEME>(*norm, s);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    f32x4 g[kQuantVec];
    int nvalid[kQuantVec];
#pragma unroll
    for (int j = 0; j < kQuantVec; j++) {
        const int64_t v = base + (int64_t)j * kQuantBlock;
        nvalid[j] = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
        g[j] = load_coords(x, v, nvalid[j]);
    }
#pragma unroll
    for (int j = 0; j < kQuantVec; j++) {            // no lane leaves early: the sign-plane exchange needs whole waves
        const int64_t v = base + (int64_t)j * kQuantBlock;
        uint32_t c_lo, c_hi;
        if (UNIFORM_HI) {                             // host: call_base + v stays below the next multiple of 2^32
            c_hi = (uint32_t)(call_base >> 32);
            c_lo = (uint32_t)call_base + (uint32_t)v;
        } else {
            const uint64_t call = call_base + (uint64_t)v;
            c_lo = (uint32_t)call;
            c_hi = (uint32_t)(call >> 32);
        }
        const Words4 r = philox4x32_10(c_lo, c_hi, worker, 0u, k0, k1);
        store_codes(lv, sp, pack, v, nvalid[j], d,
                    Round<SCHEME>::code_of_value(Round<SCHEME>::value(g[j].x, sc, r.w[0])),
                    Round<SCHEME>::code_of_value(Round<SCHEME>::value(g[j].y, sc, r.w[1])),
                    Round<SCHEME>::code_of_value(Round<SCHEME>::value(g[j].z, sc, r.w[2])),
                    Round<SCHEME>::code_of_value(Round<SCHEME>::value(g[j].w, sc, r.w[3])));
    }
}

// =============================================================================================
// Algorithm 1 line 9 on stored codes.  Same ownership as the fused kernel: a lane owns four
// coordinates, i.e. one 32-bit (8-bit codes) or 16-bit (4-bit codes) word of every worker's level
// buffer and a nibble of its sign words; loads and the 128-bit stores of a wave are contiguous.
// =============================================================================================
constexpr int kAggBlock = 128;

template <int SCHEME, int PACK>
__global__ void __launch_bounds__(kAggBlock)
int_aggregate_kernel(LevelCPtrs L, int K, int64_t d, void *__restrict__ agg_out, int agg_fmt)
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
    const int64_t v = (int64_t)blockIdx.x * kAggBlock + threadIdx.x;
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
// Algorithm 2 (Section 4.3): the paper's own aggregation for the exponential grid.  Codes are moved
// to the prescaled representation sign * 2^-e, e = s - k + 1 + log2(n'), and reduced pairwise in
// tree order; every node rounds its sum to a neighbouring power of two with the random integer
// k, P(k > b) = 2^-b.  A lane owns four coordinates and walks the tree depth first with a stack of
// log2(n') + 1 partial results, so the K code words are consumed as they arrive.
// One signed int holds a pair: se = sign * e (0 for zero).
// =============================================================================================
constexpr int kReduceBlock = 128;

__device__ __forceinline__ int alg2_pair(int se1, int se2, uint32_t r)
{
    const int k = __clz((int)r) + 1;                       // P(k > b) = 2^-b; 33 for r = 0
    const int e1 = abs(se1), e2 = abs(se2);
    const bool both = (e1 > 0) && (e2 > 0);
    const bool opposite = both && ((se1 ^ se2) < 0);        // sign12 = -1
    const bool same = both && ((se1 ^ se2) >= 0);           // sign12 = +1
    const int diff = abs(e1 - e2) - (opposite ? 1 : 0);
    const bool smaller = (e1 > 0) && (e1 <= e2 || e2 == 0); // operand 1 has the larger magnitude
    const bool nonzero = !(opposite && e1 == e2);
    const int sel = smaller ? se1 : se2;
    const int e_sel = smaller ? e1 : e2;
    const int adj = (k > diff) ? (same ? -1 : (opposite ? 1 : 0)) : 0;
    const int e = nonzero ? e_sel + adj : 0;
    return sel < 0 ? -e : e;
}

template <int NPAD, bool UNIFORM_HI>
__global__ void __launch_bounds__(kReduceBlock)
exp_reduce_kernel(LevelCPtrs Lv, int K, int64_t d, int s, uint64_t seed, uint64_t call_base,
                  const float *__restrict__ norm, void *__restrict__ reduced_out, float *__restrict__ deq_out)
{
    constexpr int L = NPAD == 1 ? 0 : NPAD == 2 ? 1 : NPAD == 4 ? 2 : NPAD == 8 ? 3 : NPAD == 16 ? 4 : NPAD == 32 ? 5 : 6;
    const int64_t v = (int64_t)blockIdx.x * kReduceBlock + threadIdx.x;
    const int64_t nfull = d >> 2;
    const int nvalid = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
    if (nvalid == 0) return;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c_lo, c_hi;
    if (UNIFORM_HI) {
        c_hi = (uint32_t)(call_base >> 32);
        c_lo = (uint32_t)call_base + (uint32_t)v;           // no carry (host)
    } else {
        const uint64_t call = call_base + (uint64_t)v;
        c_lo = (uint32_t)call;
        c_hi = (uint32_t)(call >> 32);
    }
    auto fetch = [&](int w) -> uint32_t {
        if (w >= K) return 0u;                              // missing workers are zero leaves
        if (nvalid == 4) return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(Lv.lv[w]) + v);
        const uint8_t *b = reinterpret_cast<const uint8_t *>(Lv.lv[w]) + (v << 2);
        uint32_t t = 0;
        for (int i = 0; i < nvalid; i++) t |= (uint32_t)b[i] << (8 * i);
        return t;
    };
    // code k >= 1 of the exponential grid -> e = s - k + 1 + L; 0 stays 0
    auto leaf = [&](uint32_t word, int i) -> int {
        const int q = (int)(int8_t)(word >> (8 * i));
        const int e = q ? s + 1 + L - abs(q) : 0;
        return q < 0 ? -e : e;
    };
    int st[L + 1][4];                                       // the stack of partial results
    constexpr int kBatch = NPAD < 8 ? NPAD : 8;
#pragma unroll
    for (int w0 = 0; w0 < NPAD; w0 += kBatch) {
        uint32_t words[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; j++) words[j] = fetch(w0 + j);
#pragma unroll
        for (int j = 0; j < kBatch; j++) {
            const int i = w0 + j;                            // leaf index; the stack depth is popcount(i)
            int top = __builtin_popcount((unsigned)i);
#pragma unroll
            for (int c = 0; c < 4; c++) st[top][c] = leaf(words[j], c);
#pragma unroll
            for (int lvl = 1; lvl <= L; lvl++) {
                if (((i + 1) & ((1 << lvl) - 1)) == 0) {     // a subtree of 2^lvl leaves is complete
                    const uint32_t node = (uint32_t)((NPAD >> lvl) + (i >> lvl));   // heap numbering
                    const Words4 r = philox4x32_10(c_lo, c_hi, node, 1u, k0, k1);
#pragma unroll
                    for (int c = 0; c < 4; c++) st[top - 1][c] = alg2_pair(st[top - 1][c], st[top][c], r.w[c]);
                    top--;
                }
            }
        }
    }
    if (reduced_out) {
        const uint32_t wout = (uint32_t)(st[0][0] & 255) | ((uint32_t)(st[0][1] & 255) << 8) |
                              ((uint32_t)(st[0][2] & 255) << 16) | ((uint32_t)(st[0][3] & 255) << 24);
        if (nvalid == 4) {
            __builtin_nontemporal_store(wout, reinterpret_cast<uint32_t *>(reduced_out) + v);
        } else {
            uint8_t *b = reinterpret_cast<uint8_t *>(reduced_out) + (v << 2);
            for (int i = 0; i < nvalid; i++) b[i] = (uint8_t)(wout >> (8 * i));
        }
    }
    if (deq_out) {
        // the mean the pair stands for: sign * 2^-e * (2 n') * norm / K
        const float nrm = *norm;
        const float c = (nrm > 0.0f && nrm <= 3.402823466e+38f) ? nrm / (float)K : 0.0f;
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int se = st[0][i], e = abs(se);
            const float p2 = __uint_as_float((uint32_t)(127 + 1 + L - e) << 23);     // 2^(1+L-e), e <= s+L <= 37
            o[i] = e ? (se < 0 ? -(c * p2) : c * p2) : 0.0f;
        }
        if (nvalid == 4) {
            const f32x4 t = {o[0], o[1], o[2], o[3]};
            __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(deq_out) + v);
        } else {
            for (int i = 0; i < nvalid; i++) deq_out[(v << 2) + i] = o[i];
        }
    }
}

// =============================================================================================
// Section 7: low-bit linear codes averaged inside every reduce step, so that they never leave their
// b bits.  Same tree walk as exp_reduce_kernel; a node holds round((a + b) / 2), an odd sum going
// up iff its coin is set.  The coins of up to 32 nodes are the bits of ONE Philox word per
// coordinate (stream 2, counter word 2 = node / 32), so the kernel stays memory-bound.
// =============================================================================================
template <int NPAD, bool NIBBLE, bool UNIFORM_HI>
__global__ void __launch_bounds__(kReduceBlock)
avg_reduce_kernel(LevelCPtrs Lv, int K, int64_t d, uint64_t seed, uint64_t call_base,
                  const float *__restrict__ norm, float deq_div, void *__restrict__ reduced_out,
                  float *__restrict__ deq_out)
{
    constexpr int L = NPAD == 1 ? 0 : NPAD == 2 ? 1 : NPAD == 4 ? 2 : NPAD == 8 ? 3 : NPAD == 16 ? 4 : NPAD == 32 ? 5 : 6;
    const int64_t v = (int64_t)blockIdx.x * kReduceBlock + threadIdx.x;
    const int64_t nfull = d >> 2;
    const int nvalid = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
    if (nvalid == 0) return;
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    uint32_t c_lo, c_hi;
    if (UNIFORM_HI) {
        c_hi = (uint32_t)(call_base >> 32);
        c_lo = (uint32_t)call_base + (uint32_t)v;           // no carry (host)
    } else {
        const uint64_t call = call_base + (uint64_t)v;
        c_lo = (uint32_t)call;
        c_hi = (uint32_t)(call >> 32);
    }
    const Words4 coins0 = philox4x32_10(c_lo, c_hi, 0u, 2u, k0, k1);      // nodes 1..31
    Words4 coins1 = coins0;
    if (NPAD == 64) coins1 = philox4x32_10(c_lo, c_hi, 1u, 2u, k0, k1);   // nodes 32..63
    auto fetch = [&](int w) -> uint32_t {
        if (w >= K) return 0u;                              // missing workers are zero leaves
        if (!NIBBLE) {
            if (nvalid == 4) return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(Lv.lv[w]) + v);
            const uint8_t *b = reinterpret_cast<const uint8_t *>(Lv.lv[w]) + (v << 2);
            uint32_t t = 0;
            for (int i = 0; i < nvalid; i++) t |= (uint32_t)b[i] << (8 * i);
            return t;
        }
        if (nvalid == 4) return __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(Lv.lv[w]) + v);
        const uint8_t *b = reinterpret_cast<const uint8_t *>(Lv.lv[w]) + (v << 1);
        uint32_t t = b[0];
        if (nvalid == 3) t |= (uint32_t)b[1] << 8;
        return t;
    };
    auto leaf = [&](uint32_t word, int i) -> int {
        return NIBBLE ? ((int)(word << (28 - 4 * i))) >> 28 : (int)(int8_t)(word >> (8 * i));
    };
    int st[L + 1][4];
    constexpr int kBatch = NPAD < 8 ? NPAD : 8;
#pragma unroll
    for (int w0 = 0; w0 < NPAD; w0 += kBatch) {
        uint32_t words[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; j++) words[j] = fetch(w0 + j);
#pragma unroll
        for (int j = 0; j < kBatch; j++) {
            const int i = w0 + j;
            int top = __builtin_popcount((unsigned)i);
#pragma unroll
            for (int c = 0; c < 4; c++) st[top][c] = leaf(words[j], c);
#pragma unroll
            for (int lvl = 1; lvl <= L; lvl++) {
                if (((i + 1) & ((1 << lvl) - 1)) == 0) {
                    const int node = (NPAD >> lvl) + (i >> lvl);
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const uint32_t word = node < 32 ? coins0.w[c] : coins1.w[c];
                        const int coin = (int)((word >> (node & 31)) & 1u);
                        st[top - 1][c] = (st[top - 1][c] + st[top][c] + coin) >> 1;   // floor or ceil of the average
                    }
                    top--;
                }
            }
        }
    }
    if (reduced_out) {
        if (!NIBBLE) {
            const uint32_t wout = (uint32_t)(st[0][0] & 255) | ((uint32_t)(st[0][1] & 255) << 8) |
                                  ((uint32_t)(st[0][2] & 255) << 16) | ((uint32_t)(st[0][3] & 255) << 24);
            if (nvalid == 4) {
                __builtin_nontemporal_store(wout, reinterpret_cast<uint32_t *>(reduced_out) + v);
            } else {
                uint8_t *b = reinterpret_cast<uint8_t *>(reduced_out) + (v << 2);
                for (int i = 0; i < nvalid; i++) b[i] = (uint8_t)(wout >> (8 * i));
            }
        } else {
            uint32_t wout = (uint32_t)(st[0][0] & 15);
            if (nvalid > 1) wout |= (uint32_t)(st[0][1] & 15) << 4;
            if (nvalid > 2) wout |= (uint32_t)(st[0][2] & 15) << 8;
            if (nvalid > 3) wout |= (uint32_t)(st[0][3] & 15) << 12;
            if (nvalid == 4) {
                __builtin_nontemporal_store((uint16_t)wout, reinterpret_cast<uint16_t *>(reduced_out) + v);
            } else {
                uint8_t *b = reinterpret_cast<uint8_t *>(reduced_out) + (v << 1);
                b[0] = (uint8_t)wout;
                if (nvalid == 3) b[1] = (uint8_t)(wout >> 8);
            }
        }
    }
    if (deq_out) {
        const float nrm = *norm;
        const float c = (nrm > 0.0f && nrm <= 3.402823466e+38f) ? nrm / deq_div : 0.0f;   // norm * n' / (K s)
        if (nvalid == 4) {
            const f32x4 t = {(float)st[0][0] * c, (float)st[0][1] * c, (float)st[0][2] * c, (float)st[0][3] * c};
            __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(deq_out) + v);
        } else {
            for (int i = 0; i < nvalid; i++) deq_out[(v << 2) + i] = (float)st[0][i] * c;
        }
    }
}

// =============================================================================================
// Algorithm 1 lines 6-8, the sparse branch.  Sender side: the (index, code) pairs of a worker's
// non-zero int8 codes in increasing index order, by a count pass, a one-block scan of the block
// counts and a write pass that ranks the non-zeros inside a block with wave scans.  Receiver side:
// the K lists are added into a dense int32 sum with integer atomics (exact, order-free).
// =============================================================================================
constexpr int kCompactBlock = 256;
constexpr int kCompactTile = kCompactBlock * 16;        // codes per block: one 128-bit load per thread
constexpr int kScanBlock = 1024;

__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t x)    // 0x80 in every byte of x that is not zero
{
    return (x | ((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu)) & 0x80808080u;
}

// the 16 codes of unit t (bytes 16t .. 16t+15), zeros past the end of the buffer
__device__ __forceinline__ u32x4 load_code_unit(const uint8_t *lv, int64_t t, int64_t d)
{
    const int64_t first = t << 4;
    if (first + 16 <= d) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(lv) + t);
    uint32_t q[4] = {0u, 0u, 0u, 0u};
    for (int i = 0; i < 16 && first + i < d; i++) q[i >> 2] |= (uint32_t)lv[first + i] << (8 * (i & 3));
    return u32x4{q[0], q[1], q[2], q[3]};
}

__device__ __forceinline__ uint32_t count_unit(const u32x4 &c)
{
    return (uint32_t)(__builtin_popcount(nonzero_bytes(c.x)) + __builtin_popcount(nonzero_bytes(c.y)) +
                      __builtin_popcount(nonzero_bytes(c.z)) + __builtin_popcount(nonzero_bytes(c.w)));
}

// Exclusive prefix sum of one value per thread over the block; every thread must call it.
// `total` receives the block's sum.  sh must hold BLOCK/64 words.
template <int BLOCK>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *sh, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = (uint32_t)__shfl_up((int)incl, off, 64);
        if (lane >= off) incl += t;
    }
    if (lane == 63) sh[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
    for (int i = 0; i < BLOCK / 64; i++) {
        if (i < wave) base += sh[i];
        sum += sh[i];
    }
    __syncthreads();
    *total = sum;
    return base + incl - v;
}

__global__ void __launch_bounds__(kCompactBlock)
compact_count_kernel(const uint8_t *__restrict__ lv, int64_t d, uint32_t *__restrict__ block_counts)
{
    __shared__ uint32_t sh[kCompactBlock / 64];
    const int64_t t = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x;
    const uint32_t c = count_unit(load_code_unit(lv, t, d));
    uint32_t total;
    block_exclusive_scan<kCompactBlock>(c, sh, &total);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

// One block: counts[0..n) -> exclusive offsets in place; the grand total goes to *total_out.
__global__ void __launch_bounds__(kScanBlock)
compact_scan_kernel(uint32_t *__restrict__ counts, int64_t n, uint64_t *__restrict__ total_out)
{
    __shared__ uint32_t sh[kScanBlock / 64];
    const int64_t per = (n + kScanBlock - 1) / kScanBlock;
    const int64_t lo = (int64_t)threadIdx.x * per, hi = lo + per < n ? lo + per : n;
    uint32_t mine = 0;
    for (int64_t i = lo; i < hi; i++) mine += counts[i];
    uint32_t total;
    uint32_t run = block_exclusive_scan<kScanBlock>(mine, sh, &total);
    for (int64_t i = lo; i < hi; i++) {
        const uint32_t c = counts[i];
        counts[i] = run;
        run += c;
    }
    if (threadIdx.x == 0) *total_out = (uint64_t)total;
}

__global__ void __launch_bounds__(kCompactBlock)
compact_write_kernel(const uint8_t *__restrict__ lv, int64_t d, const uint32_t *__restrict__ block_offsets,
                     uint32_t *__restrict__ indices_out, int8_t *__restrict__ values_out, int64_t capacity)
{
    __shared__ uint32_t sh[kCompactBlock / 64];
    const int64_t t = (int64_t)blockIdx.x * kCompactBlock + threadIdx.x;
    const u32x4 c = load_code_unit(lv, t, d);
    uint32_t total;
    const uint32_t rank = block_exclusive_scan<kCompactBlock>(count_unit(c), sh, &total);
    int64_t pos = (int64_t)block_offsets[blockIdx.x] + rank;
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const uint32_t b = (w[i >> 2] >> (8 * (i & 3))) & 255u;
        if (b != 0u) {
            if (pos < capacity) {
                indices_out[pos] = (uint32_t)((t << 4) + i);
                values_out[pos] = (int8_t)b;
            }
            pos++;
        }
    }
}

__global__ void __launch_bounds__(kBlock) fill_zero_kernel(int *__restrict__ p, int64_t n)
{
    const int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t nfull = n >> 2;
    if (v < nfull) {
        const i32x4 z = {0, 0, 0, 0};
        reinterpret_cast<i32x4 *>(p)[v] = z;
    } else if (v == nfull) {
        for (int64_t i = nfull << 2; i < n; i++) p[i] = 0;
    }
}

struct SparseLists {
    const uint32_t *idx[kMaxWorkers];
    const int8_t *val[kMaxWorkers];
    const uint64_t *cnt[kMaxWorkers];
    int64_t cap[kMaxWorkers];
};

template <int SCHEME>
__global__ void __launch_bounds__(kBlock) sparse_scatter_kernel(SparseLists S, int64_t d, int *__restrict__ agg)
{
    const int w = blockIdx.y;
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint64_t have = *S.cnt[w];
    const int64_t n = have < (uint64_t)S.cap[w] ? (int64_t)have : S.cap[w];
    if (i >= n) return;
    const uint32_t j = S.idx[w][i];
    if ((int64_t)j >= d) return;                            // an index outside the buffer is ignored
    const int q = S.val[w][i];
    int val = q;
    if (SCHEME == 1) {
        const int mag = (int)((1u << abs(q)) >> 1);
        val = q < 0 ? -mag : mag;
    }
    atomicAdd(agg + j, val);
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

// =============================================================================================
// Host side: argument checks and launches.
// =============================================================================================
static inline bool aligned(const void *p, size_t a) { return p != nullptr && ((uintptr_t)p % a) == 0; }

static gq_status check_params(const gq_params *p, bool uses_pack, bool uses_agg)
{
    if (!p) return GQ_ERR_INVALID_ARG;
    if (p->scheme != GQ_LINEAR && p->scheme != GQ_EXP) return GQ_ERR_INVALID_ARG;
    if (p->s < 1) return GQ_ERR_INVALID_ARG;
    if (p->scheme == GQ_LINEAR && p->s > 32767) return GQ_ERR_UNSUPPORTED;
    if (p->scheme == GQ_EXP && p->s > 31) return GQ_ERR_UNSUPPORTED;
    if (uses_pack) {
        if (p->pack < GQ_PACK_I8 || p->pack > GQ_PACK_U4_SIGNPLANE) return GQ_ERR_INVALID_ARG;
        const int lim = p->pack == GQ_PACK_I8 ? 127 : p->pack == GQ_PACK_I4 ? 7 : p->pack == GQ_PACK_U8_SIGNPLANE ? 255 : 15;
        if (p->s > lim) return GQ_ERR_UNSUPPORTED;
    }
    if (uses_agg && p->agg != GQ_AGG_I32 && p->agg != GQ_AGG_I16) return GQ_ERR_INVALID_ARG;
    return GQ_OK;
}

static int64_t max_aggregate(const gq_params *p, int K)
{
    return p->scheme == GQ_LINEAR ? (int64_t)K * p->s : (int64_t)K * ((int64_t)1 << (p->s - 1));
}

static float dequant_divisor(const gq_params *p, int K)
{
    // n * (1/unit): K*s or K*2^(s-1); both are exact in binary32 for the supported ranges
    return p->scheme == GQ_LINEAR ? (float)((int64_t)K * p->s) : (float)K * (float)((int64_t)1 << (p->s - 1));
}

static inline gq_status launched()
{
    return hipGetLastError() == hipSuccess ? GQ_OK : GQ_ERR_DEVICE;
}

static inline bool grid_fits(int64_t blocks) { return blocks >= 0 && blocks <= 0x7FFFFFFF; }

template <int SCHEME>
static gq_status launch_quantize_aggregate(const GradPtrs &P, const LevelPtrs &L, bool levels, int K, int64_t d,
                                           const float *norm, const gq_params *p, uint32_t worker0,
                                           int64_t index_base, void *agg_out, float *deq_out, hipStream_t st)
{
    const int64_t nvec = (d + 3) / 4;
    const uint64_t call_base = (uint64_t)index_base / 4u;
    const float div = dequant_divisor(p, K);
    const dim3 block(kFusedBlock);
#define GQ_LAUNCH(KT, LV, UH, V0, COUNT)                                                                      \
    do {                                                                                                      \
        const int64_t blocks_ = ((COUNT) + kFusedBlock - 1) / kFusedBlock;                                    \
        if (!grid_fits(blocks_)) return GQ_ERR_INVALID_ARG;                                                   \
        hipLaunchKernelGGL((quantize_aggregate_kernel<SCHEME, KT, LV, UH>), dim3((unsigned)blocks_), block, 0, st, \
                           P, L, K, d, (int64_t)(V0), (int64_t)(V0) + (int64_t)(COUNT), norm, p->s, p->seed, worker0, call_base, p->pack,       \
                           agg_out, p->agg, deq_out, div);                                                    \
    } while (0)
    if (levels) {
        // storing codes: one launch; the scalar high word is used when the bucket does not cross 2^34
        const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)nvec) <= ((uint64_t)1 << 32);
        if (one_stretch) GQ_LAUNCH(0, true, true, 0, nvec);
        else GQ_LAUNCH(0, true, false, 0, nvec);
        return launched();
    }
    // One launch per stretch of vectors whose Philox call index shares its high 32 bits (a second
    // stretch exists only if the bucket crosses a multiple of 2^34 coordinates).
    int64_t v0 = 0;
    while (v0 < nvec) {
        const uint64_t first = call_base + (uint64_t)v0;
        const uint64_t room = ((uint64_t)1 << 32) - (first & 0xFFFFFFFFull);
        const int64_t count = (uint64_t)(nvec - v0) < room ? (nvec - v0) : (int64_t)room;
        if (K == 4) GQ_LAUNCH(4, false, true, v0, count);
        else if (K == 8) GQ_LAUNCH(8, false, true, v0, count);
        else if (K == 16) GQ_LAUNCH(16, false, true, v0, count);
        else if (K == 32) GQ_LAUNCH(32, false, true, v0, count);
        else GQ_LAUNCH(0, false, true, v0, count);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
        v0 += count;
    }
#undef GQ_LAUNCH
    return GQ_OK;
}

}  // namespace gq

using namespace gq;

extern "C" {

int gq_version(void) { return 1000; }

const char *gq_status_string(gq_status st)
{
    switch (st) {
    case GQ_OK: return "GQ_OK";
    case GQ_ERR_INVALID_ARG: return "GQ_ERR_INVALID_ARG";
    case GQ_ERR_UNSUPPORTED: return "GQ_ERR_UNSUPPORTED";
    case GQ_ERR_OVERFLOW: return "GQ_ERR_OVERFLOW";
    case GQ_ERR_WORKSPACE: return "GQ_ERR_WORKSPACE";
    case GQ_ERR_DEVICE: return "GQ_ERR_DEVICE";
    }
    return "GQ_ERR_UNKNOWN";
}

gq_status gq_check_width(const gq_params *p, int K)
{
    const gq_status st = check_params(p, false, true);
    if (st != GQ_OK) return st;
    if (K < 1 || K > GQ_MAX_WORKERS) return GQ_ERR_INVALID_ARG;
    const int64_t lim = p->agg == GQ_AGG_I32 ? 2147483647LL : 32767LL;
    return max_aggregate(p, K) <= lim ? GQ_OK : GQ_ERR_OVERFLOW;
}

size_t gq_norm_workspace_bytes(int K, int64_t d)
{
    if (K < 1 || K > GQ_MAX_WORKERS || d < 0) return 0;
    int64_t blocks, tpb;
    norm_tile_shape(d, &blocks, &tpb);
    const size_t per_worker = (size_t)K * (size_t)norm_blocks_per_worker(d);
    return (per_worker > (size_t)blocks ? per_worker : (size_t)blocks) * sizeof(uint64_t);
}

gq_status gq_global_norm(const float *const *x, int K, int64_t d, gq_norm_kind kind, float *norm_out,
                         uint32_t *status_flags, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!x || K < 1 || K > GQ_MAX_WORKERS || d < 0) return GQ_ERR_INVALID_ARG;
    if (kind != GQ_NORM_LINF && kind != GQ_NORM_L2 && kind != GQ_NORM_L2_MAX) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm_out, 4) || (status_flags && !aligned(status_flags, 4))) return GQ_ERR_INVALID_ARG;
    GradPtrs P;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(x[i], 16)) return GQ_ERR_INVALID_ARG;
        P.x[i] = x[i];
    }
    if (!workspace || workspace_bytes < gq_norm_workspace_bytes(K, d)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GQ_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    uint64_t *partial = reinterpret_cast<uint64_t *>(workspace);
    int groups = 1;
    int64_t per_group = 0;
    if (d > 0 && kind == GQ_NORM_L2_MAX) {
        const int bpw = norm_blocks_per_worker(d);
        hipLaunchKernelGGL(norm_partial_kernel<false>, dim3((unsigned)(K * bpw)), dim3(kBlock), 0, st, P, d, bpw, partial);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
        groups = K;
        per_group = bpw;
    } else if (d > 0) {
        int64_t blocks, tpb;
        norm_tile_shape(d, &blocks, &tpb);
        const dim3 grid((unsigned)blocks), block(kNormTileBlock);
#define GQ_NORM(MX, KT) hipLaunchKernelGGL((norm_tile_kernel<MX, KT>), grid, block, 0, st, P, K, d, tpb, partial)
        if (kind == GQ_NORM_LINF) {
            if (K == 16) GQ_NORM(true, 16); else if (K == 8) GQ_NORM(true, 8); else if (K == 32) GQ_NORM(true, 32);
            else if (K == 4) GQ_NORM(true, 4); else GQ_NORM(true, 0);
        } else {
            if (K == 16) GQ_NORM(false, 16); else if (K == 8) GQ_NORM(false, 8); else if (K == 32) GQ_NORM(false, 32);
            else if (K == 4) GQ_NORM(false, 4); else GQ_NORM(false, 0);
        }
#undef GQ_NORM
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
        per_group = blocks;
    }
    hipLaunchKernelGGL(norm_final_kernel, dim3(1), dim3(kNormFinalBlock), 0, st, partial, groups, per_group, (int)kind,
                       norm_out, status_flags);
    return launched();
}

gq_status gq_quantize(const float *x, int64_t d, const float *norm, const gq_params *p, uint32_t worker,
                      int64_t index_base, void *levels_out, uint32_t *signplane_out, void *hip_stream)
{
    const gq_status st = check_params(p, true, false);
    if (st != GQ_OK) return st;
    if (d < 0 || index_base < 0 || (index_base & 3) != 0) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    const bool plane = p->pack >= GQ_PACK_U8_SIGNPLANE;
    if (d > 0 && (!aligned(x, 16) || !aligned(levels_out, 16))) return GQ_ERR_INVALID_ARG;
    if (d > 0 && plane && !aligned(signplane_out, 4)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    const int64_t nvec = (d + 3) / 4;
    const int64_t per_block = (int64_t)kQuantBlock * kQuantVec;
    const int64_t blocks = (nvec + per_block - 1) / per_block;
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kQuantBlock);
    const uint64_t call_base = (uint64_t)index_base / 4u;
    // the high counter word is a scalar unless the bucket (rounded up to whole blocks) crosses 2^34
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * per_block)) <= ((uint64_t)1 << 32);
    uint32_t *sp = plane ? signplane_out : nullptr;
    hipStream_t st2 = (hipStream_t)hip_stream;
#define GQ_QUANT(SC, UH) hipLaunchKernelGGL((quantize_kernel<SC, UH>), grid, block, 0, st2, x, levels_out, sp, d, norm, \
                                            p->s, p->seed, worker, call_base, p->pack)
    if (p->scheme == GQ_LINEAR) { if (one_stretch) GQ_QUANT(0, true); else GQ_QUANT(0, false); }
    else                        { if (one_stretch) GQ_QUANT(1, true); else GQ_QUANT(1, false); }
#undef GQ_QUANT
    return launched();
}

gq_status gq_fused_quantize_aggregate(const float *const *x, int K, int64_t d, const float *norm, const gq_params *p,
                                      int64_t index_base, void *agg_out, float *dequant_out,
                                      void *const *levels_out, uint32_t *const *signplanes_out, void *hip_stream)
{
    const bool levels = levels_out != nullptr;
    gq_status st = check_params(p, levels, agg_out != nullptr);
    if (st != GQ_OK) return st;
    if (!x || K < 1 || K > GQ_MAX_WORKERS || d < 0 || index_base < 0 || (index_base & 3) != 0) return GQ_ERR_INVALID_ARG;
    if (!agg_out && !dequant_out) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    // the sum is formed in 32-bit registers whatever is stored; a 16-bit store must also hold it
    const int64_t lim = (agg_out && p->agg == GQ_AGG_I16) ? 32767LL : 2147483647LL;
    if (max_aggregate(p, K) > lim) return GQ_ERR_OVERFLOW;
    const bool plane = levels && p->pack >= GQ_PACK_U8_SIGNPLANE;
    if (plane && !signplanes_out) return GQ_ERR_INVALID_ARG;
    GradPtrs P;
    LevelPtrs L;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(x[i], 16)) return GQ_ERR_INVALID_ARG;
        P.x[i] = x[i];
        L.lv[i] = nullptr;
        L.sp[i] = nullptr;
        if (levels) {
            if (d > 0 && !aligned(levels_out[i], 16)) return GQ_ERR_INVALID_ARG;
            L.lv[i] = levels_out[i];
            if (plane) {
                if (d > 0 && !aligned(signplanes_out[i], 4)) return GQ_ERR_INVALID_ARG;
                L.sp[i] = signplanes_out[i];
            }
        }
    }
    if (d > 0 && ((agg_out && !aligned(agg_out, 16)) || (dequant_out && !aligned(dequant_out, 16)))) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    if (p->scheme == GQ_LINEAR)
        return launch_quantize_aggregate<0>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, (hipStream_t)hip_stream);
    return launch_quantize_aggregate<1>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, (hipStream_t)hip_stream);
}

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
    const int64_t nvec = (d + 3) / 4;
    const int64_t blocks = (nvec + kAggBlock - 1) / kAggBlock;
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kAggBlock);
    hipStream_t s = (hipStream_t)hip_stream;
#define GQ_AGG(SC, PK) hipLaunchKernelGGL((int_aggregate_kernel<SC, PK>), grid, block, 0, s, L, K, d, agg_out, p->agg)
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

gq_status gq_exp_reduce(const void *const *levels, int K, int64_t d, const gq_params *p, int64_t index_base,
                        const float *norm, void *reduced_out, float *dequant_out, void *hip_stream)
{
    gq_status st = check_params(p, false, false);
    if (st != GQ_OK) return st;
    if (p->scheme != GQ_EXP) return GQ_ERR_UNSUPPORTED;
    if (!levels || K < 1 || K > GQ_MAX_WORKERS || d < 0 || index_base < 0 || (index_base & 3) != 0) return GQ_ERR_INVALID_ARG;
    if (!reduced_out && !dequant_out) return GQ_ERR_INVALID_ARG;
    if (dequant_out && !aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    LevelCPtrs Lv;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(levels[i], 16)) return GQ_ERR_INVALID_ARG;
        Lv.lv[i] = levels[i];
        Lv.sp[i] = nullptr;
    }
    if (d > 0 && ((reduced_out && !aligned(reduced_out, 16)) || (dequant_out && !aligned(dequant_out, 16)))) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    const int64_t nvec = (d + 3) / 4;
    const int64_t blocks = (nvec + kReduceBlock - 1) / kReduceBlock;
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kReduceBlock);
    const uint64_t call_base = (uint64_t)index_base / 4u;
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * kReduceBlock)) <= ((uint64_t)1 << 32);
    hipStream_t s = (hipStream_t)hip_stream;
    int npad = 1;
    while (npad < K) npad <<= 1;
#define GQ_RED(N)                                                                                              \
    do {                                                                                                       \
        if (one_stretch) hipLaunchKernelGGL((exp_reduce_kernel<N, true>), grid, block, 0, s, Lv, K, d, p->s, p->seed, \
                                            call_base, norm, reduced_out, dequant_out);                        \
        else hipLaunchKernelGGL((exp_reduce_kernel<N, false>), grid, block, 0, s, Lv, K, d, p->s, p->seed,       \
                                call_base, norm, reduced_out, dequant_out);                                    \
    } while (0)
    switch (npad) {
    case 1: GQ_RED(1); break;
    case 2: GQ_RED(2); break;
    case 4: GQ_RED(4); break;
    case 8: GQ_RED(8); break;
    case 16: GQ_RED(16); break;
    case 32: GQ_RED(32); break;
    default: GQ_RED(64); break;
    }
#undef GQ_RED
    return launched();
}

gq_status gq_avg_reduce(const void *const *levels, int K, int64_t d, const gq_params *p, int64_t index_base,
                        const float *norm, void *reduced_out, float *dequant_out, void *hip_stream)
{
    gq_status st = check_params(p, true, false);
    if (st != GQ_OK) return st;
    if (p->scheme != GQ_LINEAR || (p->pack != GQ_PACK_I8 && p->pack != GQ_PACK_I4)) return GQ_ERR_UNSUPPORTED;
    if (!levels || K < 1 || K > GQ_MAX_WORKERS || d < 0 || index_base < 0 || (index_base & 3) != 0) return GQ_ERR_INVALID_ARG;
    if (!reduced_out && !dequant_out) return GQ_ERR_INVALID_ARG;
    if (dequant_out && !aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    LevelCPtrs Lv;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(levels[i], 16)) return GQ_ERR_INVALID_ARG;
        Lv.lv[i] = levels[i];
        Lv.sp[i] = nullptr;
    }
    if (d > 0 && ((reduced_out && !aligned(reduced_out, 16)) || (dequant_out && !aligned(dequant_out, 16)))) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    const int64_t nvec = (d + 3) / 4;
    const int64_t blocks = (nvec + kReduceBlock - 1) / kReduceBlock;
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kReduceBlock);
    const uint64_t call_base = (uint64_t)index_base / 4u;
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * kReduceBlock)) <= ((uint64_t)1 << 32);
    hipStream_t s = (hipStream_t)hip_stream;
    int npad = 1;
    while (npad < K) npad <<= 1;
    const float div = (float)((int64_t)K * p->s) / (float)npad;          // exact: a power-of-two division
    const bool nib = p->pack == GQ_PACK_I4;
#define GQ_AVG3(N, NB, UH) hipLaunchKernelGGL((avg_reduce_kernel<N, NB, UH>), grid, block, 0, s, Lv, K, d, p->seed, \
                                              call_base, norm, div, reduced_out, dequant_out)
#define GQ_AVG(N)                                                                              \
    do {                                                                                       \
        if (nib) { if (one_stretch) GQ_AVG3(N, true, true); else GQ_AVG3(N, true, false); }    \
        else     { if (one_stretch) GQ_AVG3(N, false, true); else GQ_AVG3(N, false, false); }  \
    } while (0)
    switch (npad) {
    case 1: GQ_AVG(1); break;
    case 2: GQ_AVG(2); break;
    case 4: GQ_AVG(4); break;
    case 8: GQ_AVG(8); break;
    case 16: GQ_AVG(16); break;
    case 32: GQ_AVG(32); break;
    default: GQ_AVG(64); break;
    }
#undef GQ_AVG
#undef GQ_AVG3
    return launched();
}

size_t gq_compact_workspace_bytes(int64_t d)
{
    if (d < 0 || d > 0xFFFFFFFFLL) return 0;
    const int64_t blocks = (d + kCompactTile - 1) / kCompactTile;
    return (size_t)(blocks > 0 ? blocks : 1) * sizeof(uint32_t);
}

gq_status gq_compact(const void *levels, int64_t d, const gq_params *p, uint32_t *indices_out, int8_t *values_out,
                     int64_t capacity, uint64_t *count_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const gq_status st = check_params(p, true, false);
    if (st != GQ_OK) return st;
    if (p->pack != GQ_PACK_I8) return GQ_ERR_UNSUPPORTED;
    if (d < 0 || d > 0xFFFFFFFFLL || capacity < 0) return GQ_ERR_INVALID_ARG;
    if (!aligned(count_out, 8)) return GQ_ERR_INVALID_ARG;
    if (d > 0 && !aligned(levels, 16)) return GQ_ERR_INVALID_ARG;
    if (capacity > 0 && (!aligned(indices_out, 4) || !values_out)) return GQ_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < gq_compact_workspace_bytes(d)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 4)) return GQ_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    uint32_t *counts = reinterpret_cast<uint32_t *>(workspace);
    const int64_t blocks = (d + kCompactTile - 1) / kCompactTile;
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
    const uint8_t *lv = reinterpret_cast<const uint8_t *>(levels);
    if (blocks > 0) {
        hipLaunchKernelGGL(compact_count_kernel, dim3((unsigned)blocks), dim3(kCompactBlock), 0, s, lv, d, counts);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    }
    hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(kScanBlock), 0, s, counts, blocks, count_out);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    if (blocks > 0) {
        hipLaunchKernelGGL(compact_write_kernel, dim3((unsigned)blocks), dim3(kCompactBlock), 0, s, lv, d, counts,
                           indices_out, values_out, capacity);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    }
    return GQ_OK;
}

gq_status gq_sparse_aggregate(const uint32_t *const *indices, const int8_t *const *values,
                              const uint64_t *const *counts, const int64_t *capacities, int K, int64_t d,
                              const gq_params *p, void *agg_out, void *hip_stream)
{
    gq_status st = check_params(p, false, true);
    if (st != GQ_OK) return st;
    if (p->agg != GQ_AGG_I32) return GQ_ERR_UNSUPPORTED;
    if (!indices || !values || !counts || !capacities || K < 1 || K > GQ_MAX_WORKERS || d < 0 || d > 0xFFFFFFFFLL)
        return GQ_ERR_INVALID_ARG;
    st = gq_check_width(p, K);
    if (st != GQ_OK) return st;
    SparseLists S;
    int64_t maxcap = 0;
    for (int i = 0; i < K; i++) {
        if (capacities[i] < 0 || !aligned(counts[i], 8)) return GQ_ERR_INVALID_ARG;
        if (capacities[i] > 0 && (!aligned(indices[i], 4) || !values[i])) return GQ_ERR_INVALID_ARG;
        S.idx[i] = indices[i];
        S.val[i] = values[i];
        S.cnt[i] = counts[i];
        S.cap[i] = capacities[i];
        if (capacities[i] > maxcap) maxcap = capacities[i];
    }
    if (d > 0 && !aligned(agg_out, 16)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t zblocks = ((d + 3) / 4 + kBlock - 1) / kBlock;
    const int64_t sblocks = (maxcap + kBlock - 1) / kBlock;
    if (!grid_fits(zblocks) || !grid_fits(sblocks)) return GQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)zblocks), dim3(kBlock), 0, s, (int *)agg_out, d);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    if (sblocks > 0) {
        const dim3 grid((unsigned)sblocks, (unsigned)K);
        if (p->scheme == GQ_LINEAR) hipLaunchKernelGGL(sparse_scatter_kernel<0>, grid, dim3(kBlock), 0, s, S, d, (int *)agg_out);
        else hipLaunchKernelGGL(sparse_scatter_kernel<1>, grid, dim3(kBlock), 0, s, S, d, (int *)agg_out);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    }
    return GQ_OK;
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
    if (!grid_fits(blocks)) return GQ_ERR_INVALID_ARG;
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
