// Algorithm 1's quantisation loop (with its aggregation step fused in) on MI355X (gfx950): stochastic rounding of the gradients
// to integer codes, for one worker with the codes stored, or for all K workers with the integer sum
// formed in registers.  The contract of the entry points is stated in include/gqsgd.h.
//
// Data layout.  Every buffer is a flat array in HBM.  A lane owns vectors of four consecutive
// coordinates of a gradient (one 128-bit load per worker and vector), so that a wave reads 1 KiB of
// contiguous gradient per load.  With full draws (32 random bits per coordinate) a lane owns one
// vector, whose coordinates take the four words of one Philox call; with short draws (16 bits) it owns
// two vectors 64 apart and shares the words of its call with its neighbour lane.  All traffic is
// streaming with no reuse: nothing is staged through LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 1's quantisation loop and aggregation step fused: quantize the K workers' coordinates in registers, add the
// integer values, write the sum (and/or its dequantised mean, Eq. (1), and/or the packed codes).
//   SCHEME      0 linear, 1 exponential
//   KT          compile-time worker count (fully unrolled, K loads in flight), 0 = run-time K
//   LEVELS      also store every worker's packed codes
//   UNIFORM_HI  the high word of the Philox call index is the same for the whole launch
//   WINDOWS     keep few loads in flight per lane and store the sum only inside chip-wide time
//               windows (see below)
//   HALF        short draws: 16 random bits per coordinate, one Philox call per eight coordinates
// =============================================================================================
// OR over the 8 lanes that share one 32-bit sign word.  Every lane of the wave must be active.
__device__ __forceinline__ uint32_t or_over_8_lanes(uint32_t v)
{
    v |= dpp32<kDppQuadXor1>(v);
    v |= dpp32<kDppQuadXor2>(v);
    v |= dpp32<kDppHalfMirror>(v);
    return v;
}

// The four sign bits of a lane's codes; the codes are replaced by their magnitudes.
__device__ __forceinline__ uint32_t sign_nibble(int *q)
{
    uint32_t nib = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        nib |= (uint32_t)(q[i] < 0) << i;
        q[i] = abs(q[i]);
    }
    return nib;
}
__device__ __forceinline__ uint32_t pack_nibbles(const int *q)
{
    return (uint32_t)(q[0] & 15) | ((uint32_t)(q[1] & 15) << 4) | ((uint32_t)(q[2] & 15) << 8) | ((uint32_t)(q[3] & 15) << 12);
}

// Store the codes q[0..3] of vector v (nvalid of its coordinates exist).  The lanes of a wave must hold
// consecutive vectors, lane 0 a multiple of 8, and all be active (the sign words are assembled across lanes).
__device__ __forceinline__ void store_codes(void *lv, uint32_t *sp, int pack, int64_t v, int nvalid, int64_t d, int *q)
{
    if (pack >= 2) {
        const uint32_t word = or_over_8_lanes(sign_nibble(q) << (4 * (threadIdx.x & 7)));
        if ((threadIdx.x & 7) == 0 && ((v & ~(int64_t)7) << 2) < d) sp[v >> 3] = word;
    }
    if (nvalid == 0) return;
    if (pack == GQ_PACK_I8 || pack == GQ_PACK_U8_SIGNPLANE) {
        const uint32_t w = pack_bytes(q);
        if (nvalid == 4) {
            __builtin_nontemporal_store(w, reinterpret_cast<uint32_t *>(lv) + v);
        } else {
            uint8_t *b = reinterpret_cast<uint8_t *>(lv) + (v << 2);
            for (int i = 0; i < nvalid; i++) b[i] = (uint8_t)(w >> (8 * i));
        }
    } else {
        const uint32_t w = pack_nibbles(q);
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
// grain, which measurably helps the HBM read/write mix of this kernel (128 and 64 alike, 256 slower on MI355X).
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
// The wait is bounded (at most kWindowMaxPolls polls, a few periods even at K = 64) and touches no memory, so it
// changes timing only: if the counter did not advance, a wave would lose about 0.25 ms and go on.  For this
// to work the loads of a lane must really stay few in flight: the accumulators are pinned after each
// batch of four workers, which stops the compiler from hoisting all K loads to the top (it would
// otherwise, and with every load issued up front the windows were measured to gain nothing).
constexpr uint32_t kWindowTicksPerWorker = 62;    // ticks of the 100 MHz counter per worker and period
constexpr int kWindowMinWorkers = 8;
constexpr double kWindowMinLoads = 2.5e8;         // K * d from which the windows win (measured)
constexpr int kWindowMaxPolls = 1024;             // polls of about 0.2 us each: the longest period (K = 64, short draws) is 79 us

// The launch covers the vectors v0 <= v < vend of the buffers (HALF: v0 = 0).  With UNIFORM_HI the host
// guarantees that the Philox call index does not cross a multiple of 2^32 inside the launch, so the high
// counter word is a scalar: the first round and half of the second are then shared by all lanes or all
// workers and leave the vector ALU.
template <int SCHEME, int KT, bool LEVELS, bool UNIFORM_HI, bool WINDOWS, bool HALF>
__global__ void __launch_bounds__(kFusedBlock)
quantize_aggregate_kernel(GradPtrs P, LevelPtrs L, int K, int64_t d, int64_t v0, int64_t vend, const float *__restrict__ norm, int s,
                          uint64_t seed, uint32_t worker0, uint64_t call_base, int pack,
                          void *__restrict__ agg_out, int agg_fmt, float *__restrict__ deq_out, float deq_div,
                          uint32_t win_period, uint32_t win_open)
{
    constexpr int NV = HALF ? 2 : 1;             // vectors per lane
    const int64_t nfull = d >> 2;
    const int lane = (int)(threadIdx.x & 63u);
    int64_t v[NV];
    uint64_t local_call;                         // call index of this lane relative to the launch's first
    if (HALF) {
        const uint64_t chunk = (uint64_t)blockIdx.x * (kFusedBlock / 64) + (threadIdx.x >> 6);   // 128 vectors per wave
        v[0] = v0 + (int64_t)(chunk * 128u) + lane;
        v[NV - 1] = v[0] + 64;
        local_call = chunk * 64u + (uint64_t)(lane >> 1) + (uint64_t)(lane & 1) * 32u;
    } else {
        local_call = (uint64_t)blockIdx.x * kFusedBlock + threadIdx.x;
        v[0] = v0 + (int64_t)local_call;
    }
    int nvalid[NV];
#pragma unroll
    for (int t = 0; t < NV; t++) nvalid[t] = v[t] >= vend ? 0 : (v[t] < nfull ? 4 : (v[t] == nfull ? (int)(d & 3) : 0));
    // whole waves are needed by the sign-plane exchange (LEVELS) and by the exchange of short draws
    if (!LEVELS && !HALF && nvalid[0] == 0) return;

    const float nrm = *norm;
    const Scale sc = make_scale<SCHEME>(nrm, s);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint64_t first = call_base + (uint64_t)(HALF ? (v0 >> 1) : v0);      // scalar
    uint32_t c_lo, c_hi;
    if (UNIFORM_HI) {
        c_hi = (uint32_t)(first >> 32);
        c_lo = (uint32_t)first + (uint32_t)local_call;                            // fits and no carry (host)
    } else {
        const uint64_t call = first + local_call;
        c_lo = (uint32_t)call;
        c_hi = (uint32_t)(call >> 32);
    }
    const int Kc = KT > 0 ? KT : K;
    const bool whole = nvalid[NV - 1] == 4;      // every coordinate of the lane exists

    struct Unit { f32x4 g[NV]; };
    auto fetch = [&](int w) {
        Unit x;
#pragma unroll
        for (int t = 0; t < NV; t++) x.g[t] = load_coords(P.x[w], v[t], nvalid[t]);
        return x;
    };
    auto fetch_whole = [&](int w) {
        Unit x;
#pragma unroll
        for (int t = 0; t < NV; t++) x.g[t] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(P.x[w]) + v[t]);
        return x;
    };
    Acc<SCHEME> acc[NV];
    auto one_worker = [&](int w, const Unit &x) {
        const Words4 r = philox4x32_10(c_lo, c_hi, worker0 + (uint32_t)w, 0u, k0, k1);
        uint32_t draw[NV][4];
        if (HALF) {
            const ShortDraws sd = share_short_draws(r, (lane & 1) != 0);
#pragma unroll
            for (int j = 0; j < 4; j++) { draw[0][j] = short_draw(sd.a, j); draw[NV - 1][j] = short_draw(sd.b, j); }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++) draw[0][j] = r.w[j];
        }
#pragma unroll
        for (int t = 0; t < NV; t++) {
            const float f0 = Round<SCHEME>::value(x.g[t].x, sc, draw[t][0]);
            const float f1 = Round<SCHEME>::value(x.g[t].y, sc, draw[t][1]);
            const float f2 = Round<SCHEME>::value(x.g[t].z, sc, draw[t][2]);
            const float f3 = Round<SCHEME>::value(x.g[t].w, sc, draw[t][3]);
            acc[t].add(f0, f1, f2, f3);
            if (LEVELS) {
                int q[4] = {Round<SCHEME>::code_of_value(f0), Round<SCHEME>::code_of_value(f1),
                            Round<SCHEME>::code_of_value(f2), Round<SCHEME>::code_of_value(f3)};
                store_codes(L.lv[w], L.sp[w], pack, v[t], nvalid[t], d, q);
            }
        }
    };
    if (KT > 0) {
        // workers whose loads are issued before the first is consumed: few with WINDOWS, else up to 16
        // vectors; the bound is enforced (accumulators pinned) where the hoisted loads would not fit
        constexpr int kMost = WINDOWS ? 4 : 16 / NV;
        constexpr bool kPin = WINDOWS || HALF;
        constexpr int kInFlight = KT > kMost ? kMost : (KT > 0 ? KT : 1);
#pragma unroll
        for (int w0 = 0; w0 < KT; w0 += kInFlight) {
            Unit x[kInFlight];
            if (whole) {                             // one branch per batch, not per worker
#pragma unroll
                for (int j = 0; j < kInFlight; j++) x[j] = fetch_whole(w0 + j);
            } else {
#pragma unroll
                for (int j = 0; j < kInFlight; j++) x[j] = fetch(w0 + j);
            }
#pragma unroll
            for (int j = 0; j < kInFlight; j++) one_worker(w0 + j, x[j]);
            if (kPin) {
#pragma unroll
                for (int t = 0; t < NV; t++) acc[t].pin();
            }
        }
    } else {
        int w = 0;
        for (; w + 4 <= Kc; w += 4) {
            const Unit x0 = fetch(w), x1 = fetch(w + 1), x2 = fetch(w + 2), x3 = fetch(w + 3);
            one_worker(w, x0); one_worker(w + 1, x1); one_worker(w + 2, x2); one_worker(w + 3, x3);
        }
        for (; w < Kc; w++) one_worker(w, fetch(w));
    }
    if (nvalid[0] == 0) return;

    if (WINDOWS) {
        for (int it = 0; it < kWindowMaxPolls; it++) {
            const uint32_t t = (uint32_t)__builtin_amdgcn_s_memrealtime();
            if ((t % win_period) < win_open) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
    const float c = sc.scale != 0.0f ? nrm / deq_div : 0.0f;         // Eq. (1): norm / (n * unit)
#pragma unroll
    for (int t = 0; t < NV; t++) {
        const int nv = nvalid[t];
        if (nv == 0) break;
        const i32x4 a = acc[t].get();
        if (agg_out) {
            if (agg_fmt == GQ_AGG_I32) {
                if (nv == 4) {
                    __builtin_nontemporal_store(a, reinterpret_cast<i32x4 *>(agg_out) + v[t]);
                } else {
                    int *o = reinterpret_cast<int *>(agg_out) + (v[t] << 2);
                    o[0] = a.x;
                    if (nv > 1) o[1] = a.y;
                    if (nv > 2) o[2] = a.z;
                }
            } else {
                if (nv == 4) {
                    const i16x4 o = {(short)a.x, (short)a.y, (short)a.z, (short)a.w};
                    __builtin_nontemporal_store(o, reinterpret_cast<i16x4 *>(agg_out) + v[t]);
                } else {
                    short *o = reinterpret_cast<short *>(agg_out) + (v[t] << 2);
                    o[0] = (short)a.x;
                    if (nv > 1) o[1] = (short)a.y;
                    if (nv > 2) o[2] = (short)a.z;
                }
            }
        }
        if (deq_out) {
            if (nv == 4) {
                const f32x4 o = {(float)a.x * c, (float)a.y * c, (float)a.z * c, (float)a.w * c};
                __builtin_nontemporal_store(o, reinterpret_cast<f32x4 *>(deq_out) + v[t]);
            } else {
                float *o = deq_out + (v[t] << 2);
                o[0] = (float)a.x * c;
                if (nv > 1) o[1] = (float)a.y * c;
                if (nv > 2) o[2] = (float)a.z * c;
            }
        }
    }
}

// =============================================================================================
// Algorithm 1's quantisation loop for one worker with the codes stored: a lane owns kQuantVec vectors of four
// coordinates, kQuantBlock vectors apart (short draws: two pairs 64 apart, see share_short_draws), and
// issues all its loads before the first Philox call.
// =============================================================================================
constexpr int kQuantBlock = 128;
constexpr int kQuantVec = 4;

// The work of one workgroup.  WHOLE: its kQuantBlock * kQuantVec vectors all lie inside the buffer; the loads
// need no guards and the code words are staged in LDS and written out as one run, 16 (bytes) or 8 (nibbles)
// bytes per thread, instead of four narrow stores per thread.  Otherwise (the ragged last workgroup) every
// vector is guarded and stored on its own.
template <int SCHEME, bool UNIFORM_HI, bool HALF, bool WHOLE>
__device__ __forceinline__ void quantize_block(const float *__restrict__ x, void *__restrict__ lv, uint32_t *__restrict__ sp,
                                               int64_t d, const Scale &sc, uint64_t seed, uint32_t worker,
                                               uint64_t call_base, int pack, uint32_t *stage, uint32_t *stage_signs)
{
    constexpr int kBlockVecs = kQuantBlock * kQuantVec;
    const int64_t nfull = d >> 2;
    const int lane = (int)(threadIdx.x & 63u);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const int64_t vblock = (int64_t)blockIdx.x * kBlockVecs;          // scalar
    // vector j of this lane within the workgroup, and the Philox call (relative to the workgroup's first) that
    // it runs for vectors j, j+1 (short draws) or j (full draws)
    int li[kQuantVec];
    int lcall[kQuantVec];
#pragma unroll
    for (int j = 0; j < kQuantVec; j++) {
        if (HALF) {
            // the workgroup's 512 vectors are four chunks of 128; wave w takes chunks w and w + 2
            const int chunk = (int)(threadIdx.x >> 6) + 2 * (j >> 1);
            li[j] = chunk * 128 + 64 * (j & 1) + lane;
            lcall[j] = chunk * 64 + (lane >> 1) + (lane & 1) * 32;
        } else {
            li[j] = j * kQuantBlock + (int)threadIdx.x;
            lcall[j] = li[j];
        }
    }
    const float *xb = x + (vblock << 2);
    f32x4 g[kQuantVec];
    int nvalid[kQuantVec];
#pragma unroll
    for (int j = 0; j < kQuantVec; j++) {
        if (WHOLE) {
            nvalid[j] = 4;
            g[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(xb) + li[j]);
        } else {
            const int64_t v = vblock + li[j];
            nvalid[j] = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
            g[j] = load_coords(x, v, nvalid[j]);
        }
    }
    const uint64_t first = call_base + (uint64_t)(HALF ? (vblock >> 1) : vblock);    // scalar
    auto counter = [&](int c, uint32_t &c_lo, uint32_t &c_hi) {
        if (UNIFORM_HI) {                             // host: the launch stays below the next multiple of 2^32 calls
            c_hi = (uint32_t)(first >> 32);
            c_lo = (uint32_t)first + (uint32_t)c;
        } else {
            const uint64_t cc = first + (uint64_t)c;
            c_lo = (uint32_t)cc;
            c_hi = (uint32_t)(cc >> 32);
        }
    };
    const bool bytes = pack == GQ_PACK_I8 || pack == GQ_PACK_U8_SIGNPLANE;
    auto emit = [&](int j, const uint32_t *draw) {
        int q[4] = {Round<SCHEME>::code(g[j].x, sc, draw[0]), Round<SCHEME>::code(g[j].y, sc, draw[1]),
                    Round<SCHEME>::code(g[j].z, sc, draw[2]), Round<SCHEME>::code(g[j].w, sc, draw[3])};
        if (!WHOLE) {
            store_codes(lv, sp, pack, vblock + li[j], nvalid[j], d, q);
            return;
        }
        if (pack >= 2) {
            const uint32_t word = or_over_8_lanes(sign_nibble(q) << (4 * (threadIdx.x & 7)));
            if ((threadIdx.x & 7) == 0) stage_signs[li[j] >> 3] = word;
        }
        if (bytes) stage[li[j]] = pack_bytes(q);
        else reinterpret_cast<uint16_t *>(stage)[li[j]] = (uint16_t)pack_nibbles(q);
    };
    // no lane leaves early: the sign-plane exchange and the exchange of short draws need whole waves
    if (HALF) {
#pragma unroll
        for (int j = 0; j < kQuantVec; j += 2) {
            uint32_t c_lo, c_hi;
            counter(lcall[j], c_lo, c_hi);
            const ShortDraws sd = share_short_draws(philox4x32_10(c_lo, c_hi, worker, 0u, k0, k1), (lane & 1) != 0);
            uint32_t da[4], db[4];
#pragma unroll
            for (int i = 0; i < 4; i++) { da[i] = short_draw(sd.a, i); db[i] = short_draw(sd.b, i); }
            emit(j, da);
            emit(j + 1, db);
        }
    } else {
#pragma unroll
        for (int j = 0; j < kQuantVec; j++) {
            uint32_t c_lo, c_hi;
            counter(lcall[j], c_lo, c_hi);
            const Words4 r = philox4x32_10(c_lo, c_hi, worker, 0u, k0, k1);
            emit(j, r.w);
        }
    }
    if (WHOLE) {
        __syncthreads();
        const int t = (int)threadIdx.x;
        if (bytes) {
            const u32x4 w = *reinterpret_cast<const u32x4 *>(&stage[4 * t]);
            __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>(lv) + (vblock / 4 + t));
        } else {
            const uint64_t w = *reinterpret_cast<const uint64_t *>(reinterpret_cast<const uint16_t *>(stage) + 4 * t);
            __builtin_nontemporal_store(w, reinterpret_cast<uint64_t *>(lv) + (vblock / 4 + t));
        }
        if (pack >= 2 && t < kBlockVecs / 8) sp[vblock / 8 + t] = stage_signs[t];
    }
}

template <int SCHEME, bool UNIFORM_HI, bool HALF>
__global__ void __launch_bounds__(kQuantBlock)
quantize_kernel(const float *__restrict__ x, void *__restrict__ lv, uint32_t *__restrict__ sp, int64_t d,
                const float *__restrict__ norm, int s, uint64_t seed, uint32_t worker, uint64_t call_base, int pack)
{
    __shared__ uint32_t stage[kQuantBlock * kQuantVec];              // one code word per vector
    __shared__ uint32_t stage_signs[kQuantBlock * kQuantVec / 8];    // one sign word per 8 vectors
    const Scale sc = make_scale<SCHEME>(*norm, s);
    const bool whole = ((int64_t)blockIdx.x + 1) * (kQuantBlock * kQuantVec) <= (d >> 2);   // uniform over the workgroup
    if (whole) quantize_block<SCHEME, UNIFORM_HI, HALF, true>(x, lv, sp, d, sc, seed, worker, call_base, pack, stage, stage_signs);
    else quantize_block<SCHEME, UNIFORM_HI, HALF, false>(x, lv, sp, d, sc, seed, worker, call_base, pack, stage, stage_signs);
}

template <int SCHEME, bool HALF>
static gq_status launch_quantize_aggregate(const GradPtrs &P, const LevelPtrs &L, bool levels, int K, int64_t d,
                                           const float *norm, const gq_params *p, uint32_t worker0,
                                           int64_t index_base, void *agg_out, float *deq_out, hipStream_t st)
{
    constexpr int kLaneVecs = HALF ? 2 : 1;              // vectors per lane = vectors per Philox call
    const int64_t nvec = (d + 3) / 4;
    const uint64_t call_base = (uint64_t)index_base / (uint64_t)(4 * kLaneVecs);
    const float div = dequant_divisor(p, K);
    const dim3 block(kFusedBlock);
    // Write windows pay once a launch lasts many periods and a wave's K loads span about one period;
    // below these sizes the wait for the next window costs more than the cleaner read/write mix gains.
    // The caller may override the policy either way (gq_params.flags).
    const bool by_policy = K >= kWindowMinWorkers && (double)K * (double)d >= kWindowMinLoads;
    const bool win = !levels && !(p->flags & GQ_FLAG_WRITE_WINDOWS_OFF) && (by_policy || (p->flags & GQ_FLAG_WRITE_WINDOWS_ON));
    const uint32_t win_period = kWindowTicksPerWorker * (uint32_t)K * (uint32_t)kLaneVecs;   // a wave loads kLaneVecs KiB per worker
    const uint32_t win_open = win_period / 10u;
#define GQ_LAUNCH(KT, LV, UH, WIN, V0, COUNT)                                                                  \
    do {                                                                                                      \
        const int64_t blocks_ = ((COUNT) + kFusedBlock * kLaneVecs - 1) / (kFusedBlock * kLaneVecs);          \
        if (!grid_fits(blocks_, kFusedBlock)) return GQ_ERR_INVALID_ARG;                                                   \
        hipLaunchKernelGGL((quantize_aggregate_kernel<SCHEME, KT, LV, UH, WIN, HALF>), dim3((unsigned)blocks_), block, 0, st, \
                           P, L, K, d, (int64_t)(V0), (int64_t)(V0) + (int64_t)(COUNT), norm, p->s, p->seed, worker0,  \
                           call_base, p->pack, agg_out, p->agg, deq_out, div, win_period, win_open);          \
    } while (0)
#define GQ_LAUNCH_K(UH, WIN, V0, COUNT)                                                                        \
    do {                                                                                                      \
        if (K == 4) GQ_LAUNCH(4, false, UH, WIN, V0, COUNT);                                                  \
        else if (K == 8) GQ_LAUNCH(8, false, UH, WIN, V0, COUNT);                                             \
        else if (K == 16) GQ_LAUNCH(16, false, UH, WIN, V0, COUNT);                                           \
        else if (K == 32) GQ_LAUNCH(32, false, UH, WIN, V0, COUNT);                                           \
        else GQ_LAUNCH(0, false, UH, WIN, V0, COUNT);                                                         \
    } while (0)
    // calls of the launch, counting the lanes past the end of whole workgroups
    const uint64_t calls_padded = (uint64_t)((nvec + kFusedBlock * kLaneVecs - 1) / (kFusedBlock * kLaneVecs)) * kFusedBlock;
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + calls_padded) <= ((uint64_t)1 << 32);
    if (levels) {
        // storing codes: one launch; the scalar high word is used when the bucket does not cross 2^32 calls
        if (one_stretch) GQ_LAUNCH(0, true, true, false, 0, nvec);
        else GQ_LAUNCH(0, true, false, false, 0, nvec);
        return launched();
    }
    if (HALF) {
        // short draws pair the lanes of a wave, so the launch is not cut: a bucket that crosses a multiple
        // of 2^32 calls (2^35 coordinates) runs with the high counter word per lane
        if (one_stretch) { if (win) GQ_LAUNCH_K(true, true, 0, nvec); else GQ_LAUNCH_K(true, false, 0, nvec); }
        else             { if (win) GQ_LAUNCH_K(false, true, 0, nvec); else GQ_LAUNCH_K(false, false, 0, nvec); }
        return launched();
    }
    constexpr int64_t kMaxLaunchVecs = (int64_t)1 << 31;
    // One launch per stretch of vectors whose Philox call index shares its high 32 bits (a second
    // stretch exists only if the bucket crosses a multiple of 2^34 coordinates).
    int64_t v0 = 0;
    while (v0 < nvec) {
        const uint64_t first = call_base + (uint64_t)v0;
        const uint64_t room = ((uint64_t)1 << 32) - (first & 0xFFFFFFFFull);
        int64_t count = (uint64_t)(nvec - v0) < room ? (nvec - v0) : (int64_t)room;
        if (count > kMaxLaunchVecs) count = kMaxLaunchVecs;       // and no launch beyond HIP's limit of 2^32 - 1 threads
        if (win) GQ_LAUNCH_K(true, true, v0, count);
        else GQ_LAUNCH_K(true, false, v0, count);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
        v0 += count;
    }
#undef GQ_LAUNCH_K
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
    const bool half = short_draws(p);
    if (d < 0 || index_base < 0 || (index_base & (half ? 7 : 3)) != 0) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm, 4)) return GQ_ERR_INVALID_ARG;
    const bool plane = p->pack >= GQ_PACK_U8_SIGNPLANE;
    if (d > 0 && (!aligned(x, 16) || !aligned(levels_out, 16))) return GQ_ERR_INVALID_ARG;
    if (d > 0 && plane && !aligned(signplane_out, 4)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    const int64_t nvec = (d + 3) / 4;
    const int64_t per_block = (int64_t)kQuantBlock * kQuantVec;          // vectors per workgroup, either mode
    const int64_t blocks = (nvec + per_block - 1) / per_block;
    if (!grid_fits(blocks, kQuantBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kQuantBlock);
    const int lane_vecs = half ? 2 : 1;                                  // vectors per Philox call
    const uint64_t call_base = (uint64_t)index_base / (uint64_t)(4 * lane_vecs);
    // the high counter word is a scalar unless the bucket (rounded up to whole blocks) crosses 2^32 calls
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * per_block / lane_vecs)) <= ((uint64_t)1 << 32);
    uint32_t *sp = plane ? signplane_out : nullptr;
    hipStream_t st2 = (hipStream_t)hip_stream;
#define GQ_QUANT(SC, UH, HF) hipLaunchKernelGGL((quantize_kernel<SC, UH, HF>), grid, block, 0, st2, x, levels_out, sp, d, norm, \
                                                p->s, p->seed, worker, call_base, p->pack)
#define GQ_QUANT2(SC, UH) do { if (half) GQ_QUANT(SC, UH, true); else GQ_QUANT(SC, UH, false); } while (0)
    if (p->scheme == GQ_LINEAR) { if (one_stretch) GQ_QUANT2(0, true); else GQ_QUANT2(0, false); }
    else                        { if (one_stretch) GQ_QUANT2(1, true); else GQ_QUANT2(1, false); }
#undef GQ_QUANT2
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
    const bool half = short_draws(p);
    if (!x || K < 1 || K > GQ_MAX_WORKERS || d < 0 || index_base < 0 || (index_base & (half ? 7 : 3)) != 0) return GQ_ERR_INVALID_ARG;
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
    hipStream_t hs = (hipStream_t)hip_stream;
    if (p->scheme == GQ_LINEAR) {
        if (half) return launch_quantize_aggregate<0, true>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, hs);
        return launch_quantize_aggregate<0, false>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, hs);
    }
    if (half) return launch_quantize_aggregate<1, true>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, hs);
    return launch_quantize_aggregate<1, false>(P, L, levels, K, d, norm, p, 0u, index_base, agg_out, dequant_out, hs);
}

}  // extern "C"
