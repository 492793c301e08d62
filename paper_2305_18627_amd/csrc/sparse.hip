// Algorithm 1's sparse branch on MI355X (gfx950): compaction of non-zero codes and the sum of the K lists.
// Contracts: include/gqsgd.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 1's sparse branch, the sparse branch.  Sender side: the (index, code) pairs of a worker's
// non-zero int8 codes in increasing index order, by a count pass, a one-block scan of the block
// counts and a write pass that ranks the non-zeros inside a block with wave scans.  Receiver side:
// the K sorted lists are merged tile by tile into the dense int32 sum.
// =============================================================================================
constexpr int kCompactBlock = 256;
constexpr int kCompactTile = kCompactBlock * 16;        // codes per tile: one 128-bit load per thread
constexpr int kCompactTiles = 4;                        // consecutive tiles per block: fewer, larger block counts to scan
constexpr int kCompactSpan = kCompactTile * kCompactTiles;
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
    const int64_t t0 = (int64_t)blockIdx.x * (kCompactBlock * kCompactTiles) + threadIdx.x;
    u32x4 c[kCompactTiles];
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) c[j] = load_code_unit(lv, t0 + (int64_t)j * kCompactBlock, d);
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) mine += count_unit(c[j]);
    uint32_t total;
    block_exclusive_scan<kCompactBlock>(mine, sh, &total);
    if (threadIdx.x == 0) block_counts[blockIdx.x] = total;
}

// One block: counts[0..n) -> exclusive offsets in place; the grand total goes to *total_out.
// The counts are taken kScanBlock at a time with consecutive lanes on consecutive words; the running
// total is carried from one round to the next.
__global__ void __launch_bounds__(kScanBlock)
compact_scan_kernel(uint32_t *__restrict__ counts, int64_t n, uint64_t *__restrict__ total_out)
{
    __shared__ uint32_t sh[kScanBlock / 64];
    uint32_t carry = 0;
    for (int64_t base = 0; base < n; base += kScanBlock) {
        const int64_t i = base + threadIdx.x;
        const uint32_t c = i < n ? counts[i] : 0u;
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<kScanBlock>(c, sh, &total);
        if (i < n) counts[i] = carry + excl;
        carry += total;
    }
    if (threadIdx.x == 0) *total_out = (uint64_t)carry;
}

// A block takes its kCompactTiles tiles one after the other.  The pairs of a tile are first ranked into LDS (a
// tile never holds more than kCompactTile of them) and then copied out with consecutive lanes writing
// consecutive list entries; the list position runs on from tile to tile.
__global__ void __launch_bounds__(kCompactBlock)
compact_write_kernel(const uint8_t *__restrict__ lv, int64_t d, const uint32_t *__restrict__ block_offsets,
                     uint32_t *__restrict__ indices_out, int8_t *__restrict__ values_out, int64_t capacity)
{
    __shared__ uint32_t sh[kCompactBlock / 64];
    __shared__ uint32_t s_idx[kCompactTile];
    __shared__ int8_t s_val[kCompactTile];
    const int64_t t0 = (int64_t)blockIdx.x * (kCompactBlock * kCompactTiles) + threadIdx.x;
    u32x4 c[kCompactTiles];
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) c[j] = load_code_unit(lv, t0 + (int64_t)j * kCompactBlock, d);
    int64_t base = (int64_t)block_offsets[blockIdx.x];
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) {
        const int64_t t = t0 + (int64_t)j * kCompactBlock;
        uint32_t total;
        uint32_t rank = block_exclusive_scan<kCompactBlock>(count_unit(c[j]), sh, &total);
        const uint32_t w[4] = {c[j].x, c[j].y, c[j].z, c[j].w};
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const uint32_t b = (w[i >> 2] >> (8 * (i & 3))) & 255u;
            if (b != 0u) {
                s_idx[rank] = (uint32_t)((t << 4) + i);
                s_val[rank] = (int8_t)b;
                rank++;
            }
        }
        __syncthreads();
        for (uint32_t e = threadIdx.x; e < total; e += kCompactBlock) {
            if (base + e < capacity) {
                indices_out[base + e] = s_idx[e];
                values_out[base + e] = s_val[e];
            }
        }
        base += total;
        __syncthreads();                                 // the staging area is reused by the next tile
    }
}

struct SparseLists {
    const uint32_t *idx[kMaxWorkers];
    const int8_t *val[kMaxWorkers];
    const uint64_t *cnt[kMaxWorkers];
    int64_t cap[kMaxWorkers];
};

// Receiver side.  A block owns kSparseTiles consecutive tiles of kSparseTile coordinates.  It first finds, by
// binary search in every worker's sorted index list, where each of its tile boundaries falls (all
// K * (kSparseTiles + 1) searches run side by side, one per thread, so the block pays the latency of one
// search).  Then, tile by tile, the workers' entries are added into an LDS copy of the tile (LDS atomics), the
// threads being split evenly over the workers so that short lists are walked in parallel, and the tile is
// written with 128-bit stores.  No global atomics and no separate zero fill: every output word is written
// exactly once.
constexpr int kSparseTile = 4096;
constexpr int kSparseTiles = 4;

template <int SCHEME>
__global__ void __launch_bounds__(kBlock)
sparse_tile_kernel(SparseLists S, int K, int lanes_per_worker, int64_t d, int *__restrict__ agg)
{
    __shared__ int tile[kSparseTile];
    __shared__ int64_t bound[kMaxWorkers * (kSparseTiles + 1)];
    const int64_t lo0 = (int64_t)blockIdx.x * (kSparseTile * kSparseTiles);
    for (int b = threadIdx.x; b < K * (kSparseTiles + 1); b += kBlock) {
        const int w = b / (kSparseTiles + 1), t = b - w * (kSparseTiles + 1);
        const int64_t edge = lo0 + (int64_t)t * kSparseTile;
        const int64_t key = edge < d ? edge : d;
        const uint64_t have = *S.cnt[w];
        const int64_t n = have < (uint64_t)S.cap[w] ? (int64_t)have : S.cap[w];
        int64_t a = 0, e = n;                                  // first entry whose index is >= key
        while (a < e) {
            const int64_t mid = (a + e) >> 1;
            if ((int64_t)S.idx[w][mid] < key) a = mid + 1; else e = mid;
        }
        bound[b] = a;
    }
    const int w = (int)threadIdx.x / lanes_per_worker;         // this thread's worker (if w < K) and its slot
    const int slot = (int)threadIdx.x - w * lanes_per_worker;
#pragma unroll 1
    for (int t = 0; t < kSparseTiles; t++) {
        const int64_t lo = lo0 + (int64_t)t * kSparseTile;
        if (lo >= d) break;                                     // uniform over the block
        for (int i = threadIdx.x; i < kSparseTile; i += kBlock) tile[i] = 0;
        __syncthreads();                                        // also orders the searches before their first use
        auto add_entry = [&](int ww, int64_t e) {
            const int64_t j = (int64_t)S.idx[ww][e] - lo;
            const int q = S.val[ww][e];
            int val = q;
            if (SCHEME == 1) {
                const int mag = (int)((1u << abs(q)) >> 1);
                val = q < 0 ? -mag : mag;
            }
            if (j >= 0 && j < kSparseTile) atomicAdd(&tile[j], val);   // always true for a sorted list
        };
        // long lists: the whole block walks one worker's entries at a time (1 KiB contiguous per wave and load);
        // short lists: the threads are split over the workers, which are then walked side by side
        int64_t entries = 0;
        for (int ww = 0; ww < K; ww++) entries += bound[ww * (kSparseTiles + 1) + t + 1] - bound[ww * (kSparseTiles + 1) + t];
        if (entries >= (int64_t)K * (kBlock / 2)) {             // uniform over the block
            for (int ww = 0; ww < K; ww++) {
                const int64_t end = bound[ww * (kSparseTiles + 1) + t + 1];
                for (int64_t e = bound[ww * (kSparseTiles + 1) + t] + threadIdx.x; e < end; e += kBlock) add_entry(ww, e);
            }
        } else if (w < K) {
            const int64_t end = bound[w * (kSparseTiles + 1) + t + 1];
            for (int64_t e = bound[w * (kSparseTiles + 1) + t] + slot; e < end; e += lanes_per_worker) add_entry(w, e);
        }
        __syncthreads();
        for (int i = threadIdx.x * 4; i < kSparseTile; i += kBlock * 4) {
            const int64_t c = lo + i;
            if (c + 4 <= d) {
                const i32x4 o = {tile[i], tile[i + 1], tile[i + 2], tile[i + 3]};
                __builtin_nontemporal_store(o, reinterpret_cast<i32x4 *>(agg + c));
            } else {
                for (int u = 0; u < 4 && c + u < d; u++) agg[c + u] = tile[i + u];
            }
        }
        __syncthreads();                                        // the tile is cleared again by the next round
    }
}

}  // namespace gq

using namespace gq;

extern "C" {

size_t gq_compact_workspace_bytes(int64_t d)
{
    if (d < 0 || d > 0xFFFFFFFFLL) return 0;
    const int64_t blocks = (d + kCompactSpan - 1) / kCompactSpan;
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
    const int64_t blocks = (d + kCompactSpan - 1) / kCompactSpan;
    if (!grid_fits(blocks, kCompactBlock)) return GQ_ERR_INVALID_ARG;
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
    for (int i = 0; i < K; i++) {
        if (capacities[i] < 0 || !aligned(counts[i], 8)) return GQ_ERR_INVALID_ARG;
        if (capacities[i] > 0 && (!aligned(indices[i], 4) || !values[i])) return GQ_ERR_INVALID_ARG;
        S.idx[i] = indices[i];
        S.val[i] = values[i];
        S.cnt[i] = counts[i];
        S.cap[i] = capacities[i];
    }
    if (d > 0 && !aligned(agg_out, 16)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t span = (int64_t)kSparseTile * kSparseTiles;
    const int64_t blocks = (d + span - 1) / span;
    if (!grid_fits(blocks, kBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks);
    int kpad = 1;
    while (kpad < K) kpad <<= 1;
    const int lanes = kBlock / kpad;                            // threads per worker: 256 for K = 1 ... 4 for K = 64
    if (p->scheme == GQ_LINEAR) hipLaunchKernelGGL(sparse_tile_kernel<0>, grid, dim3(kBlock), 0, s, S, K, lanes, d, (int *)agg_out);
    else hipLaunchKernelGGL(sparse_tile_kernel<1>, grid, dim3(kBlock), 0, s, S, K, lanes, d, (int *)agg_out);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    return GQ_OK;
}

}  // extern "C"
