// Algorithm 1's norm step on MI355X (gfx950): the global norm of K resident gradients.
// The contract of the entry points is stated in include/gqsgd.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <mutex>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 1's norm step: global norm.  Pass 1 reduces the gradients to 8-byte partials (a uint32 bit
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
    // block `blk` of a worker takes a contiguous stretch of its vectors, eight 128-bit loads in flight per lane
    const int64_t per_block = (((nvec + bpw - 1) / bpw) + kBlock - 1) / kBlock * kBlock;
    const int64_t end = (blk + 1) * per_block < nvec ? (blk + 1) * per_block : nvec;
    int64_t v = (int64_t)blk * per_block + threadIdx.x;
    NormAcc<MAXNORM> acc;
    for (; v + 7 * kBlock < end; v += 8 * kBlock) {
        f32x4 b[8];
#pragma unroll
        for (int j = 0; j < 8; j++) b[j] = __builtin_nontemporal_load(xv + v + j * kBlock);
#pragma unroll
        for (int j = 0; j < 8; j++) acc.take(b[j]);
    }
    for (; v < end; v += kBlock) acc.take(__builtin_nontemporal_load(xv + v));
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

// The launches of gq_global_norm, shared by both entry points: `partial` holds at least
// gq_norm_workspace_bytes(K, d) bytes.  Arguments other than `partial` have been checked.
static gq_status launch_global_norm(const GradPtrs &P, int K, int64_t d, gq_norm_kind kind, float *norm_out,
                                    uint32_t *status_flags, uint64_t *partial, hipStream_t st)
{
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

static gq_status check_global_norm_args(const float *const *x, int K, int64_t d, gq_norm_kind kind, const float *norm_out,
                                        const uint32_t *status_flags, GradPtrs *P)
{
    if (!x || K < 1 || K > GQ_MAX_WORKERS || d < 0) return GQ_ERR_INVALID_ARG;
    if (kind != GQ_NORM_LINF && kind != GQ_NORM_L2 && kind != GQ_NORM_L2_MAX) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm_out, 4) || (status_flags && !aligned(status_flags, 4))) return GQ_ERR_INVALID_ARG;
    for (int i = 0; i < K; i++) {
        if (d > 0 && !aligned(x[i], 16)) return GQ_ERR_INVALID_ARG;
        P->x[i] = x[i];
    }
    return GQ_OK;
}


// ---------------------------------------------------------------------------------------------
// Scratch of gq_global_norm_static: the block partials live in a file-scope device array instead of a
// caller-provided workspace, for callers that cannot allocate.  65536 partials of 8 bytes cover every
// (K, d) the library accepts (at most 2^16 tile partials, at most 64 * 1024 per-worker partials).
// In host code the array's name is only a handle; its device address is looked up once per device.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchWords = (size_t)1 << 16;
static __device__ __align__(256) uint64_t scratch[kStaticScratchWords];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static uint64_t *scratch_ptr[kMaxDevices];       // device address of `scratch` on each device, once resolved

// The address of the current device's copy of `scratch`, or nullptr if the runtime refuses.
static uint64_t *static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_ptr[dev] = reinterpret_cast<uint64_t *>(p);
    }
    return scratch_ptr[dev];
}

}  // namespace gq

using namespace gq;

extern "C" {

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
    GradPtrs P;
    const gq_status st = check_global_norm_args(x, K, d, kind, norm_out, status_flags, &P);
    if (st != GQ_OK) return st;
    if (!workspace || workspace_bytes < gq_norm_workspace_bytes(K, d)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GQ_ERR_INVALID_ARG;
    return launch_global_norm(P, K, d, kind, norm_out, status_flags, reinterpret_cast<uint64_t *>(workspace),
                              (hipStream_t)hip_stream);
}

gq_status gq_global_norm_static(const float *const *x, int K, int64_t d, gq_norm_kind kind, float *norm_out,
                                uint32_t *status_flags, void *hip_stream)
{
    GradPtrs P;
    const gq_status st = check_global_norm_args(x, K, d, kind, norm_out, status_flags, &P);
    if (st != GQ_OK) return st;
    if (gq_norm_workspace_bytes(K, d) > kStaticScratchWords * sizeof(uint64_t)) return GQ_ERR_WORKSPACE;
    uint64_t *partial = static_scratch_of_current_device();
    if (!partial) return GQ_ERR_DEVICE;
    // every partial the final kernel reads is written by this call's first kernel, so nothing needs clearing
    return launch_global_norm(P, K, d, kind, norm_out, status_flags, partial, (hipStream_t)hip_stream);
}

}  // extern "C"
