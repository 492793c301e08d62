// Algorithm 1 lines 2-5 (and line 9 fused in) on MI355X (gfx950): stochastic rounding of the gradients
// to integer codes, for one worker with the codes stored, or for all K workers with the integer sum
// formed in registers.  The contract of the entry points is stated in include/gqsgd.h.
//
// Data layout.  Every buffer is a flat array in HBM.  A lane always owns four consecutive
// coordinates of a gradient (one 128-bit load per worker), which are also the four words of one
// Philox call, so that a wave reads 1 KiB of contiguous gradient per worker and load.  All traffic is
// streaming with no reuse: nothing is staged through LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 1 lines 2-5 and 9 fused: quantize the K workers' coordinates in registers, add the
// integer values, write the sum (and/or its dequantised mean, Eq. (1), and/or the packed codes).
//   SCHEME      0 linear, 1 exponential
//   KT          compile-time worker count (fully unrolled, K loads in flight), 0 = run-time K
//   LEVELS      also store every worker's packed codes
//   UNIFORM_HI  the high word of the Philox call index is the same for the whole launch
//   WINDOWS     keep few loads in flight per lane and store the sum only inside chip-wide time
//               windows (see below)
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
    __device__ __forceinline__ void pin() { asm volatile("" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : : "memory"); }
};
template <> struct Acc<1> {
    int a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    __device__ __forceinline__ void add(float f0, float f1, float f2, float f3) { a0 += (int)f0; a1 += (int)f1; a2 += (int)f2; a3 += (int)f3; }
    __device__ __forceinline__ i32x4 get() const { return i32x4{a0, a1, a2, a3}; }
    __device__ __forceinline__ void pin() { asm volatile("" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : : "memory"); }
};

// Write windows.  The kernel reads 4K bytes and writes 4 bytes per coordinate.  With every wave storing
// whenever it happens to finish, HBM sees writes sprinkled evenly into the read stream and pays a bus
// turnaround for each; measured on MI355X this mix runs at 5.8-6.1 TB/s while the same reads alone
// reach 7 TB/s.  With WINDOWS a wave that has finished its sum waits (sleeping) until the constant
// 100 MHz counter, which all compute units share, enters the first tenth of a period of
// kWindowTicksPerWorker * K ticks, and stores then: the chip alternates between a long stretch of pure
// reads and a short burst of writes (6.3-6.5 TB/s for K >= 12).  The period is the time one
// generation of resident waves needs for its K loads, so a wave waits for about one window, not more.
// The wait is bounded (at most 4096 polls) and touches no memory, so it changes timing only.  For this
// to work the loads of a lane must really stay few in flight: the accumulators are pinned after each
// batch of four workers, which stops the compiler from hoisting all K loads to the top (it would
// otherwise, and with every load issued up front the windows were measured to gain nothing).
constexpr uint32_t kWindowTicksPerWorker = 62;    // ticks of the 100 MHz counter per worker and period
constexpr int kWindowMinWorkers = 8;
constexpr double kWindowMinLoads = 2.5e8;         // K * d from which the windows win (measured)

// The launch covers the 4-coordinate vectors v0 <= v < vend of the buffers.  With UNIFORM_HI the
// host guarantees that the Philox call index (call_base + v) does not cross a multiple of 2^32 inside
// the launch, so the high counter word is a scalar: the first round and half of the second are then
// shared by all lanes or all workers and leave the vector ALU.
template <int SCHEME, int KT, bool LEVELS, bool UNIFORM_HI, bool WINDOWS>
__global__ void __launch_bounds__(kFusedBlock)
quantize_aggregate_kernel(GradPtrs P, LevelPtrs L, int K, int64_t d, int64_t v0, int64_t vend, const float *__restrict__ norm, int s,
                          uint64_t seed, uint32_t worker0, uint64_t call_base, int pack,
                          void *__restrict__ agg_out, int agg_fmt, float *__restrict__ deq_out, float deq_div,
                          uint32_t win_period, uint32_t win_open)
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
        constexpr int kInFlight = WINDOWS ? (KT > 4 ? 4 : (KT > 0 ? KT : 1)) : (KT > 16 ? 16 : (KT > 0 ? KT : 1));   // loads issued before the first is consumed
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
            if (WINDOWS) acc.pin();
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

    if (WINDOWS) {
        for (int it = 0; it < 4096; it++) {
            const uint32_t t = (uint32_t)__builtin_amdgcn_s_memrealtime();
            if ((t % win_period) < win_open) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
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

template <int SCHEME>
static gq_status launch_quantize_aggregate(const GradPtrs &P, const LevelPtrs &L, bool levels, int K, int64_t d,
                                           const float *norm, const gq_params *p, uint32_t worker0,
                                           int64_t index_base, void *agg_out, float *deq_out, hipStream_t st)
{
    const int64_t nvec = (d + 3) / 4;
    const uint64_t call_base = (uint64_t)index_base / 4u;
    const float div = dequant_divisor(p, K);
    const dim3 block(kFusedBlock);
    // Write windows pay once a launch lasts many periods and a wave's K loads span about one period;
    // below these sizes the wait for the next window costs more than the cleaner read/write mix gains.
    const bool win = !levels && K >= kWindowMinWorkers && (double)K * (double)d >= kWindowMinLoads;
    const uint32_t win_period = kWindowTicksPerWorker * (uint32_t)K;
    const uint32_t win_open = win_period / 10u;
#define GQ_LAUNCH(KT, LV, UH, WIN, V0, COUNT)                                                                      \
    do {                                                                                                      \
        const int64_t blocks_ = ((COUNT) + kFusedBlock - 1) / kFusedBlock;                                    \
        if (!grid_fits(blocks_)) return GQ_ERR_INVALID_ARG;                                                   \
        hipLaunchKernelGGL((quantize_aggregate_kernel<SCHEME, KT, LV, UH, WIN>), dim3((unsigned)blocks_), block, 0, st, \
                           P, L, K, d, (int64_t)(V0), (int64_t)(V0) + (int64_t)(COUNT), norm, p->s, p->seed, worker0, call_base, p->pack,       \
                           agg_out, p->agg, deq_out, div, win_period, win_open);                                                    \
    } while (0)
    if (levels) {
        // storing codes: one launch; the scalar high word is used when the bucket does not cross 2^34
        const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)nvec) <= ((uint64_t)1 << 32);
        if (one_stretch) GQ_LAUNCH(0, true, true, false, 0, nvec);
        else GQ_LAUNCH(0, true, false, false, 0, nvec);
        return launched();
    }
    // One launch per stretch of vectors whose Philox call index shares its high 32 bits (a second
    // stretch exists only if the bucket crosses a multiple of 2^34 coordinates).
    int64_t v0 = 0;
    while (v0 < nvec) {
        const uint64_t first = call_base + (uint64_t)v0;
        const uint64_t room = ((uint64_t)1 << 32) - (first & 0xFFFFFFFFull);
        const int64_t count = (uint64_t)(nvec - v0) < room ? (nvec - v0) : (int64_t)room;
        if (win) {
            if (K == 4) GQ_LAUNCH(4, false, true, true, v0, count);
            else if (K == 8) GQ_LAUNCH(8, false, true, true, v0, count);
            else if (K == 16) GQ_LAUNCH(16, false, true, true, v0, count);
            else if (K == 32) GQ_LAUNCH(32, false, true, true, v0, count);
            else GQ_LAUNCH(0, false, true, true, v0, count);
        } else {
            if (K == 4) GQ_LAUNCH(4, false, true, false, v0, count);
            else if (K == 8) GQ_LAUNCH(8, false, true, false, v0, count);
            else if (K == 16) GQ_LAUNCH(16, false, true, false, v0, count);
            else if (K == 32) GQ_LAUNCH(32, false, true, false, v0, count);
            else GQ_LAUNCH(0, false, true, false, v0, count);
        }
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
        v0 += count;
    }
#undef GQ_LAUNCH
    return GQ_OK;
}

}  // namespace gq

using namespace gq;

extern "C" {

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

}  // extern "C"
