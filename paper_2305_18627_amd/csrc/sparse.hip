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
// Algorithm 1's sparse branch.  Sender side: the (index, code) pairs of a worker's non-zero int8 codes in
// increasing index order, in one pass over the codes (every workgroup learns its place in the list from the
// counts the workgroups before it publish; the non-zeros inside a workgroup's span are ranked with wave scans).
// Receiver side: the K sorted lists are added span by span into the dense int32 sum.
// =============================================================================================
constexpr int kCompactBlock = 256;
constexpr int kCompactTile = kCompactBlock * 16;        // codes per tile: one 128-bit load per thread
constexpr int kCompactTiles = 8;                        // consecutive tiles per span: 32 KiB of codes
constexpr int kCompactSpan = kCompactTile * kCompactTiles;

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

// ---------------------------------------------------------------------------------------------------------
// Sender side in ONE pass over the codes: a block counts the non-zeros of its span, learns how many lie before
// the span from the counts the blocks before it have published, and writes its pairs.  The codes are read once
// and nothing but the list is written: d + 5 * nnz bytes, the method's own traffic.
//
// Spans of kCompactSpan codes are grouped by 64.  One word per span and one word per group (plain stores and loads, no
// read-modify-write atomics: those serialise chip-wide on one address, measured at about 20 ns each):
//   span word    bits 31..0 the count of the span, bit 32 set once it is published
//   group word   bits 39..0 the sum of the counts of the group's 64 spans, bit 40 set once it is published
// A block publishes its count as soon as it has counted, before it waits for anybody.  What lies before block b
// is the sum of all earlier groups plus the counts of the earlier blocks of its own group; the last block of a
// group, which has just added up its 63 predecessors for itself, publishes the group's word.  No block waits for
// another block's prefix, so the waits do not chain: a few hundred words are read once or twice per block.
//
// Why every wait ends.  One workgroup per span.  Workgroups of a one-dimensional grid are handed to the eight XCDs
// in turn and each XCD starts its share in increasing order.  Let m be the smallest span not yet finished: every
// workgroup of m's XCD before m has finished, so m has a free slot and has started; it publishes its count after a
// bounded amount of work of its own (loads, a count, a block scan) and waits for nothing before that.  A span waits
// only for counts of earlier spans and for sums of earlier groups, whose writers wait only for counts of their own
// group: every word m waits for is there, m finishes, and the argument repeats.  The wait is bounded all the same
// (kPrefixMaxPolls polls of about a microsecond): a workgroup that gives up writes nothing and raises count_out to
// 2^64 - 1, which no real count reaches.
// ---------------------------------------------------------------------------------------------------------
constexpr int kGroupBlocks = 64;
constexpr uint64_t kPublished = 1ull << 32;
constexpr uint64_t kGroupPublished = 1ull << 40;
constexpr int kPrefixMaxPolls = 1 << 21;

// `empty_starts`: the one entry of the table of tile starts of an empty gradient, or nullptr
__global__ void __launch_bounds__(kBlock) compact_clear_kernel(uint64_t *__restrict__ state, int64_t words, uint64_t *__restrict__ count_out,
                                                               uint32_t *__restrict__ empty_starts)
{
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < words) state[i] = 0;
    if (i == 0) *count_out = 0;
    if (i == 0 && empty_starts) empty_starts[0] = 0;
}

__device__ __forceinline__ uint64_t state_load(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off, 64), hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), off, 64);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

// Number of non-zero codes before span `span`: the counts of the earlier spans of its own group plus the sums of
// the earlier groups.  Run by one whole wave; the result is uniform.  Both kinds of word are asked for in the same
// round trip (a poll queues behind the bulk reads of the whole chip, so trips are what costs).  *in_group receives the
// own group's part as soon as it is complete and *in_group_ready is set (the caller then publishes the group's sum
// if it is the group's last span, and calls again for the rest).  Returns true once everything is there, false
// after an unsuccessful poll; the caller counts those.
struct Before { uint64_t in_group, groups; bool in_group_ready, groups_ready; int64_t next_group; };

__device__ __forceinline__ void poll_before(const uint64_t *span_words, const uint64_t *group_words, int64_t span, Before *st)
{
    const int lane = (int)(threadIdx.x & 63u);
    const int64_t group = span / kGroupBlocks;
    const int member = (int)(span - group * kGroupBlocks);
    uint64_t w_in = kPublished, w_gr = kGroupPublished;
    if (!st->in_group_ready && lane < member) w_in = state_load(span_words + group * kGroupBlocks + lane);
    if (!st->groups_ready && st->next_group + lane < group) w_gr = state_load(group_words + st->next_group + lane);
    if (!st->in_group_ready && __ballot((w_in & kPublished) == 0) == 0ull) {
        st->in_group = wave_sum_u64(w_in & 0xFFFFFFFFull);
        st->in_group_ready = true;
    }
    if (!st->groups_ready && __ballot((w_gr & kGroupPublished) == 0) == 0ull) {
        st->groups += wave_sum_u64(w_gr & (kGroupPublished - 1ull));
        st->next_group += 64;
        if (st->next_group >= group) st->groups_ready = true;
    }
}

// Exclusive prefix sums over the block of kCompactTiles counts per thread at once.  Two counts share a 32-bit
// word (a thread counts at most 16 non-zeros per tile and a tile holds at most 4096, so 16 bits each never
// carry into each other), which halves the shuffles, and all tiles share the two barriers.
// rank[j] receives the number of non-zeros of tile j held by the threads before this one, total[j] the tile's count.
// sh must hold (kCompactBlock / 64) * (kCompactTiles / 2) words.  Every thread must call it.
__device__ __forceinline__ void block_scan_tiles(const uint32_t *cnt, uint32_t *sh, uint32_t *rank, uint32_t *total)
{
    constexpr int kPairs = kCompactTiles / 2, kWaves = kCompactBlock / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl[kPairs];
#pragma unroll
    for (int q = 0; q < kPairs; q++) incl[q] = cnt[2 * q] | (cnt[2 * q + 1] << 16);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
        for (int q = 0; q < kPairs; q++) {
            const uint32_t t = (uint32_t)__shfl_up((int)incl[q], off, 64);
            if (lane >= off) incl[q] += t;
        }
    }
    if (lane == 63) {
#pragma unroll
        for (int q = 0; q < kPairs; q++) sh[wave * kPairs + q] = incl[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kPairs; q++) {
        uint32_t before = 0, sum = 0;
#pragma unroll
        for (int i = 0; i < kWaves; i++) {
            const uint32_t w = sh[i * kPairs + q];
            if (i < wave) before += w;
            sum += w;
        }
        const uint32_t excl = before + incl[q] - (cnt[2 * q] | (cnt[2 * q + 1] << 16));
        rank[2 * q] = excl & 0xFFFFu;       rank[2 * q + 1] = excl >> 16;
        total[2 * q] = sum & 0xFFFFu;       total[2 * q + 1] = sum >> 16;
    }
    __syncthreads();
}

// The list entries of one span, given its codes: c[j] holds the 16 codes of unit threadIdx.x of tile j of the span
// (zeros past the end of the buffer).  Every thread of the workgroup must call it.
__device__ __forceinline__ void emit_span(const u32x4 (&c)[kCompactTiles], int64_t d, uint64_t *__restrict__ state, int64_t nspans,
                                          uint32_t *__restrict__ indices_out, int8_t *__restrict__ values_out, int64_t capacity,
                                          uint64_t *__restrict__ count_out, uint32_t *__restrict__ tile_starts_out)
{
    __shared__ uint32_t sh[(kCompactBlock / 64) * (kCompactTiles / 2)];
    __shared__ uint32_t s_idx[kCompactTile];
    __shared__ int8_t s_val[kCompactTile];
    __shared__ int64_t s_base;
    uint64_t *span_words = state + 2;
    uint64_t *group_words = span_words + nspans;
    const int64_t span = blockIdx.x;
    const int64_t t0 = span * (kCompactBlock * kCompactTiles) + threadIdx.x;
    uint32_t cnt[kCompactTiles], rank[kCompactTiles], total[kCompactTiles];
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) cnt[j] = count_unit(c[j]);
    block_scan_tiles(cnt, sh, rank, total);
    uint32_t span_total = 0;
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) span_total += total[j];
    // the span's count is what the other workgroups wait for: out with it before anything else
    if (threadIdx.x == 0) __hip_atomic_store(span_words + span, kPublished | span_total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // The pairs of a tile are ranked into LDS (a tile never holds more than kCompactTile of them) and then copied
    // out with consecutive lanes writing consecutive list entries; the list position runs on from tile to tile.
    // The first tile is ranked while the published count travels; only then does wave 0 ask what lies before.
    int64_t base = 0;
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) {
        if (j > 0 && total[j] == 0) continue;                // uniform over the block: nothing to rank or to copy
        const int64_t t = t0 + (int64_t)j * kCompactBlock;
        if (cnt[j] != 0) {
            uint32_t r = rank[j];
            const uint32_t w[4] = {c[j].x, c[j].y, c[j].z, c[j].w};
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const uint32_t b = (w[i >> 2] >> (8 * (i & 3))) & 255u;
                if (b != 0u) {
                    s_idx[r] = (uint32_t)((t << 4) + i);
                    s_val[r] = (int8_t)b;
                    r++;
                }
            }
        }
        if (j == 0) {
            if (threadIdx.x < 64) {                          // wave 0
                Before st = {0, 0, false, span / kGroupBlocks == 0, 0};
                bool group_sum_out = span % kGroupBlocks != kGroupBlocks - 1;     // only a group's last span owes one
                int polls = 0;
                bool gave_up = false;
                for (;;) {
                    poll_before(span_words, group_words, span, &st);
                    // the group's last span publishes the group's sum as soon as it has it, before it waits on
                    if (st.in_group_ready && !group_sum_out) {
                        if (threadIdx.x == 0)
                            __hip_atomic_store(group_words + span / kGroupBlocks, kGroupPublished | (st.in_group + span_total),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        group_sum_out = true;
                    }
                    if (st.in_group_ready && st.groups_ready) break;
                    if (++polls > kPrefixMaxPolls) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(4);
                }
                if (threadIdx.x == 0) {
                    const uint64_t before = st.in_group + st.groups;
                    if (gave_up) {
                        atomicMax(reinterpret_cast<unsigned long long *>(count_out), ~0ull);
                        s_base = -1;
                    } else {
                        if (span == nspans - 1)
                            atomicMax(reinterpret_cast<unsigned long long *>(count_out), (unsigned long long)(before + span_total));
                        s_base = (int64_t)before;
                    }
                }
            }
            __syncthreads();
            base = s_base;
            if (base < 0) return;                            // uniform over the block
            if (tile_starts_out) {
                // where each tile of the span begins in the list (what the receiver would otherwise search for),
                // and behind the last tile the end of the list
                const int64_t ntiles = (d + kCompactTile - 1) / kCompactTile;
                if (threadIdx.x < kCompactTiles) {
                    uint32_t start = (uint32_t)base;
#pragma unroll
                    for (int jj = 0; jj < kCompactTiles; jj++) if (jj < (int)threadIdx.x) start += total[jj];
                    const int64_t tile = span * kCompactTiles + threadIdx.x;
                    if (tile < ntiles) tile_starts_out[tile] = start;
                }
                if (span == nspans - 1 && threadIdx.x == 0) tile_starts_out[ntiles] = (uint32_t)(base + span_total);
            }
        } else {
            __syncthreads();
        }
        for (uint32_t e = threadIdx.x; e < total[j]; e += kCompactBlock) {
            if (base + e < capacity) {
                indices_out[base + e] = s_idx[e];
                values_out[base + e] = s_val[e];
            }
        }
        base += total[j];
        __syncthreads();                                     // the staging area is reused by the next tile
    }
}


__global__ void __launch_bounds__(kCompactBlock)
compact_onepass_kernel(const uint8_t *__restrict__ lv, int64_t d, uint64_t *__restrict__ state, int64_t nspans,
                       uint32_t *__restrict__ indices_out, int8_t *__restrict__ values_out, int64_t capacity,
                       uint64_t *__restrict__ count_out, uint32_t *__restrict__ tile_starts_out)
{
    const int64_t t0 = (int64_t)blockIdx.x * (kCompactBlock * kCompactTiles) + threadIdx.x;
    u32x4 c[kCompactTiles];
#pragma unroll
    for (int j = 0; j < kCompactTiles; j++) c[j] = load_code_unit(lv, t0 + (int64_t)j * kCompactBlock, d);
    emit_span(c, d, state, nspans, indices_out, values_out, capacity, count_out, tile_starts_out);
}

// ---------------------------------------------------------------------------------------------------------
// Sender side without the dense codes: Algorithm 1's quantisation loop for one worker feeding the list directly.
// A workgroup quantises its span tile by tile (the same rounding, random stream and call indices as gq_quantize),
// passes the code words of a tile through LDS so that every thread ends up with 16 consecutive codes, and hands the
// span to emit_span: 4 d bytes read, 5 nnz written, and the codes never reach memory.
//   full draws   a thread owns vectors t, t + 256, t + 512, t + 768 of a tile (a wave reads 1 KiB per load)
//   short draws  a lane owns vectors l and 64 + l of two chunks of 128 vectors and shares its Philox words with its
//                neighbour lane (one call per eight coordinates, every load contiguous over the wave)
// The loads of the next tile are issued before the current tile is rounded.
// ---------------------------------------------------------------------------------------------------------
template <int SCHEME, bool UNIFORM_HI, bool HALF, bool WHOLE>
__device__ __forceinline__ void quantize_span(const float *__restrict__ x, int64_t d, const Scale &sc, uint64_t seed, uint32_t worker,
                                              uint64_t call_base, uint32_t (*stage)[kCompactTile / 4], u32x4 (&c)[kCompactTiles])
{
    constexpr int kTileVecs = kCompactTile / 4;
    constexpr int kVecs = kTileVecs / kCompactBlock;                  // vectors per thread and tile: 4
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const int64_t nfull = d >> 2;
    const int64_t vspan = (int64_t)blockIdx.x * (kCompactSpan / 4);  // scalar
    const int t = (int)threadIdx.x;
    int li[kVecs];
#pragma unroll
    for (int i = 0; i < kVecs; i++) {
        // short draws: a wave takes chunks of 128 consecutive vectors, lane l owns vectors l and 64 + l of a chunk
        // (see share_short_draws); wave w takes chunks w and w + 4 of the tile's eight
        const int chunk = (t >> 6) + (kCompactBlock / 64) * (i >> 1);
        li[i] = HALF ? chunk * 128 + 64 * (i & 1) + (t & 63) : i * kCompactBlock + t;
    }
    auto load_tile = [&](int j, f32x4 *g) {
#pragma unroll
        for (int i = 0; i < kVecs; i++) {
            const int64_t v = vspan + (int64_t)j * kTileVecs + li[i];
            if (WHOLE) g[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(x) + v);
            else g[i] = load_coords(x, v, v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0));
        }
    };
    f32x4 g[kVecs], gn[kVecs];
    load_tile(0, g);
    static_for<0, kCompactTiles>([&](auto jj) {
        constexpr int j = decltype(jj)::value;
        if constexpr (j + 1 < kCompactTiles) load_tile(j + 1, gn);
        uint32_t *st = stage[j & 1];
        const int64_t vt = vspan + (int64_t)j * kTileVecs;           // scalar
        const uint64_t first = call_base + (uint64_t)(HALF ? (vt >> 1) : vt);
        auto counter = [&](int local, uint32_t &c_lo, uint32_t &c_hi) {
            if (UNIFORM_HI) {                                         // host: the launch stays below the next multiple of 2^32 calls
                c_hi = (uint32_t)(first >> 32);
                c_lo = (uint32_t)first + (uint32_t)local;
            } else {
                const uint64_t cc = first + (uint64_t)local;
                c_lo = (uint32_t)cc;
                c_hi = (uint32_t)(cc >> 32);
            }
        };
        auto emit = [&](int i, const uint32_t *draw) {
            const int q[4] = {Round<SCHEME>::code(g[i].x, sc, draw[0]), Round<SCHEME>::code(g[i].y, sc, draw[1]),
                              Round<SCHEME>::code(g[i].z, sc, draw[2]), Round<SCHEME>::code(g[i].w, sc, draw[3])};
            uint32_t w = pack_bytes(q);
            if (!WHOLE) {                                             // no entries for coordinates past the end
                const int64_t v = vt + li[i];
                const int nv = v < nfull ? 4 : (v == nfull ? (int)(d & 3) : 0);
                if (nv < 4) w &= (1u << (8 * nv)) - 1u;
            }
            st[li[i]] = w;
        };
        if (HALF) {
#pragma unroll
            for (int h = 0; h < kVecs / 2; h++) {
                uint32_t c_lo, c_hi;
                const int chunk = (t >> 6) + (kCompactBlock / 64) * h, lane = t & 63;
                counter(chunk * 64 + (lane >> 1) + (lane & 1) * 32, c_lo, c_hi);
                const ShortDraws sd = share_short_draws(philox4x32_10(c_lo, c_hi, worker, 0u, k0, k1), (lane & 1) != 0);
                uint32_t da[4], db[4];
#pragma unroll
                for (int i = 0; i < 4; i++) { da[i] = short_draw(sd.a, i); db[i] = short_draw(sd.b, i); }
                emit(2 * h, da);
                emit(2 * h + 1, db);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kVecs; i++) {
                uint32_t c_lo, c_hi;
                counter(li[i], c_lo, c_hi);
                const Words4 r = philox4x32_10(c_lo, c_hi, worker, 0u, k0, k1);
                emit(i, r.w);
            }
        }
        __syncthreads();
        // two staging buffers in turn: the barrier of the next tile separates these reads from the writes of the tile after
        c[j] = *reinterpret_cast<const u32x4 *>(&st[4 * t]);
        if constexpr (j + 1 < kCompactTiles) {
#pragma unroll
            for (int i = 0; i < kVecs; i++) g[i] = gn[i];
        }
    });
}

template <int SCHEME, bool UNIFORM_HI, bool HALF>
__global__ void __launch_bounds__(kCompactBlock)
quantize_compact_kernel(const float *__restrict__ x, int64_t d, const float *__restrict__ norm, int s, uint64_t seed, uint32_t worker,
                        uint64_t call_base, uint64_t *__restrict__ state, int64_t nspans, uint32_t *__restrict__ indices_out,
                        int8_t *__restrict__ values_out, int64_t capacity, uint64_t *__restrict__ count_out,
                        uint32_t *__restrict__ tile_starts_out)
{
    __shared__ __attribute__((aligned(16))) uint32_t stage[2][kCompactTile / 4];
    const Scale sc = make_scale<SCHEME>(*norm, s);
    const bool whole = ((int64_t)blockIdx.x + 1) * kCompactSpan <= (d & ~(int64_t)3);     // uniform over the workgroup
    u32x4 c[kCompactTiles];
    if (whole) quantize_span<SCHEME, UNIFORM_HI, HALF, true>(x, d, sc, seed, worker, call_base, stage, c);
    else quantize_span<SCHEME, UNIFORM_HI, HALF, false>(x, d, sc, seed, worker, call_base, stage, c);
    emit_span(c, d, state, nspans, indices_out, values_out, capacity, count_out, tile_starts_out);
}

struct SparseLists {
    const uint32_t *idx[kMaxWorkers];
    const int8_t *val[kMaxWorkers];
    const uint64_t *cnt[kMaxWorkers];
    const uint32_t *starts[kMaxWorkers];     // where every tile of kSparseTile coordinates begins in the list, or nullptr
    int64_t cap[kMaxWorkers];
};

// Receiver side.  A workgroup of 512 threads owns a span of 8192 coordinates, held as an int32 array in LDS.
// The threads are split evenly over the K workers (512 / K' lanes each, K' = K rounded up to a power of two), so
// that all K list segments of the span are walked side by side: every lane learns where its worker's segment begins
// and ends -- from the table of tile starts that gq_compact wrote beside the list, or, if the sender gave none, by
// binary search in the sorted index list -- and adds its share of the entries into the LDS array (LDS atomics),
// four loads in flight per lane.  The span is then written once with 128-bit stores.  No global atomics and no
// separate zero fill: every output word is written exactly once.
constexpr int kSparseBlock = 512;
constexpr int kSparseSpan = 2 * kCompactTile;            // two tiles of the sender's table of tile starts

template <int SCHEME>
__global__ void __launch_bounds__(kSparseBlock)
sparse_span_kernel(SparseLists S, int K, int lanes_per_worker, int64_t d, int *__restrict__ agg)
{
    __shared__ int span[kSparseSpan];
    __shared__ int64_t s_begin[kMaxWorkers], s_end[kMaxWorkers];
    const int64_t lo = (int64_t)blockIdx.x * kSparseSpan;
    const int64_t hi = lo + kSparseSpan < d ? lo + kSparseSpan : d;
    const int w = (int)threadIdx.x / lanes_per_worker;         // this thread's worker (if w < K) and its slot
    const int slot = (int)threadIdx.x - w * lanes_per_worker;
    // the worker's entries with lo <= index < hi lie at [begin, end) of its list: lane 0 of the worker's lanes looks up
    // begin, lane 1 end (there are at least eight lanes per worker)
    if (w < K && slot < 2) {
        const uint64_t have = *S.cnt[w];
        const int64_t n = have < (uint64_t)S.cap[w] ? (int64_t)have : S.cap[w];
        const int64_t key = slot == 0 ? lo : hi;
        int64_t at;
        if (S.starts[w]) {
            const int64_t ntiles = (d + kCompactTile - 1) / kCompactTile;
            const int64_t t = (key + kCompactTile - 1) / kCompactTile;     // key is a multiple of the tile size, or d
            at = (int64_t)S.starts[w][t < ntiles ? t : ntiles];
            at = at < n ? at : n;                              // a list cut short by its capacity ends at n
        } else {
            int64_t a = 0, e = n;                              // first entry whose index is >= key
            while (a < e) {
                const int64_t mid = (a + e) >> 1;
                if ((int64_t)S.idx[w][mid] < key) a = mid + 1; else e = mid;
            }
            at = a;
        }
        if (slot == 0) s_begin[w] = at; else s_end[w] = at;
    }
    for (int i = threadIdx.x * 4; i < kSparseSpan; i += kSparseBlock * 4) *reinterpret_cast<i32x4 *>(&span[i]) = i32x4{0, 0, 0, 0};
    __syncthreads();
    if (w < K) {
        const int64_t begin = s_begin[w], end = s_end[w];
        const uint32_t *idx = S.idx[w];
        const int8_t *val = S.val[w];
        auto add_entry = [&](uint32_t index, int q) {
            int v = q;
            if (SCHEME == 1) {
                const int mag = (int)((1u << abs(q)) >> 1);
                v = q < 0 ? -mag : mag;
            }
            const int64_t j = (int64_t)index - lo;
            if (j >= 0 && j < kSparseSpan) atomicAdd(&span[j], v);     // always true for a sorted list
        };
        int64_t e = begin + slot;
        const int64_t step = lanes_per_worker;
        for (; e + 3 * step < end; e += 4 * step) {            // four entries in flight per lane
            const uint32_t i0 = idx[e], i1 = idx[e + step], i2 = idx[e + 2 * step], i3 = idx[e + 3 * step];
            const int q0 = val[e], q1 = val[e + step], q2 = val[e + 2 * step], q3 = val[e + 3 * step];
            add_entry(i0, q0); add_entry(i1, q1); add_entry(i2, q2); add_entry(i3, q3);
        }
        for (; e < end; e += step) add_entry(idx[e], val[e]);
    }
    __syncthreads();
    for (int i = threadIdx.x * 4; i < kSparseSpan; i += kSparseBlock * 4) {
        const int64_t c = lo + i;
        if (c + 4 <= d) {
            __builtin_nontemporal_store(*reinterpret_cast<const i32x4 *>(&span[i]), reinterpret_cast<i32x4 *>(agg + c));
        } else {
            for (int u = 0; u < 4 && c + u < d; u++) agg[c + u] = span[i + u];
        }
    }
}

}  // namespace gq

using namespace gq;

extern "C" {

size_t gq_compact_workspace_bytes(int64_t d)
{
    if (d < 0 || d > 0xFFFFFFFFLL) return 0;
    const int64_t blocks = (d + kCompactSpan - 1) / kCompactSpan;
    const int64_t groups = (blocks + kGroupBlocks - 1) / kGroupBlocks;
    return (size_t)(2 + blocks + groups) * sizeof(uint64_t); // two spare words, a word per block and per group of 64
}

int64_t gq_tile_starts_len(int64_t d)
{
    if (d < 0 || d > 0xFFFFFFFFLL) return 0;
    return (d + kCompactTile - 1) / kCompactTile + 1;
}

gq_status gq_compact(const void *levels, int64_t d, const gq_params *p, uint32_t *indices_out, int8_t *values_out,
                     int64_t capacity, uint64_t *count_out, uint32_t *tile_starts_out, void *workspace, size_t workspace_bytes,
                     void *hip_stream)
{
    const gq_status st = check_params(p, true, false);
    if (st != GQ_OK) return st;
    if (p->pack != GQ_PACK_I8) return GQ_ERR_UNSUPPORTED;
    if (d < 0 || d > 0xFFFFFFFFLL || capacity < 0) return GQ_ERR_INVALID_ARG;
    if (!aligned(count_out, 8)) return GQ_ERR_INVALID_ARG;
    if (d > 0 && !aligned(levels, 16)) return GQ_ERR_INVALID_ARG;
    if (capacity > 0 && (!aligned(indices_out, 4) || !values_out)) return GQ_ERR_INVALID_ARG;
    if (tile_starts_out && !aligned(tile_starts_out, 4)) return GQ_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < gq_compact_workspace_bytes(d)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GQ_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    uint64_t *state = reinterpret_cast<uint64_t *>(workspace);
    const int64_t blocks = (d + kCompactSpan - 1) / kCompactSpan;
    if (!grid_fits(blocks, kCompactBlock)) return GQ_ERR_INVALID_ARG;
    const uint8_t *lv = reinterpret_cast<const uint8_t *>(levels);
    // the scan's words and the count start from zero (a fill kernel, so that the call can be captured in a graph)
    const int64_t words = 2 + blocks + (blocks + kGroupBlocks - 1) / kGroupBlocks;
    hipLaunchKernelGGL(compact_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, state, words, count_out,
                       blocks == 0 ? tile_starts_out : nullptr);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    if (blocks > 0) {
        hipLaunchKernelGGL(compact_onepass_kernel, dim3((unsigned)blocks), dim3(kCompactBlock), 0, s, lv, d, state, blocks,
                           indices_out, values_out, capacity, count_out, tile_starts_out);
        if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    }
    return GQ_OK;
}

gq_status gq_quantize_compact(const float *x, int64_t d, const float *norm, const gq_params *p, uint32_t worker, int64_t index_base,
                              uint32_t *indices_out, int8_t *values_out, int64_t capacity, uint64_t *count_out,
                              uint32_t *tile_starts_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const gq_status st = check_params(p, true, false);
    if (st != GQ_OK) return st;
    if (p->pack != GQ_PACK_I8) return GQ_ERR_UNSUPPORTED;
    const bool half = short_draws(p);
    if (d < 0 || d > 0xFFFFFFFFLL || capacity < 0 || index_base < 0 || (index_base & (half ? 7 : 3)) != 0) return GQ_ERR_INVALID_ARG;
    if (!aligned(norm, 4) || !aligned(count_out, 8)) return GQ_ERR_INVALID_ARG;
    if (d > 0 && !aligned(x, 16)) return GQ_ERR_INVALID_ARG;
    if (capacity > 0 && (!aligned(indices_out, 4) || !values_out)) return GQ_ERR_INVALID_ARG;
    if (tile_starts_out && !aligned(tile_starts_out, 4)) return GQ_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < gq_compact_workspace_bytes(d)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GQ_ERR_INVALID_ARG;
    hipStream_t hs = (hipStream_t)hip_stream;
    uint64_t *state = reinterpret_cast<uint64_t *>(workspace);
    const int64_t blocks = (d + kCompactSpan - 1) / kCompactSpan;
    if (!grid_fits(blocks, kCompactBlock)) return GQ_ERR_INVALID_ARG;
    const int64_t words = 2 + blocks + (blocks + kGroupBlocks - 1) / kGroupBlocks;
    hipLaunchKernelGGL(compact_clear_kernel, dim3((unsigned)((words + kBlock - 1) / kBlock)), dim3(kBlock), 0, hs, state, words, count_out,
                       blocks == 0 ? tile_starts_out : nullptr);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    if (blocks == 0) return GQ_OK;
    const int lane_vecs = half ? 2 : 1;                                  // vectors per Philox call
    const uint64_t call_base = (uint64_t)index_base / (uint64_t)(4 * lane_vecs);
    // the high counter word is a scalar unless the gradient (rounded up to whole spans) crosses 2^32 calls
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * (kCompactSpan / 4) / lane_vecs)) <= ((uint64_t)1 << 32);
#define GQ_QC(SC, UH, HF) hipLaunchKernelGGL((quantize_compact_kernel<SC, UH, HF>), dim3((unsigned)blocks), dim3(kCompactBlock), 0, hs, x, d, \
                                             norm, p->s, p->seed, worker, call_base, state, blocks, indices_out, values_out, capacity, \
                                             count_out, tile_starts_out)
#define GQ_QC2(SC, UH) do { if (half) GQ_QC(SC, UH, true); else GQ_QC(SC, UH, false); } while (0)
    if (p->scheme == GQ_LINEAR) { if (one_stretch) GQ_QC2(0, true); else GQ_QC2(0, false); }
    else                        { if (one_stretch) GQ_QC2(1, true); else GQ_QC2(1, false); }
#undef GQ_QC2
#undef GQ_QC
    return launched();
}

gq_status gq_sparse_aggregate(const uint32_t *const *indices, const int8_t *const *values,
                              const uint64_t *const *counts, const int64_t *capacities,
                              const uint32_t *const *tile_starts, int K, int64_t d,
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
        S.starts[i] = tile_starts ? tile_starts[i] : nullptr;
        if (S.starts[i] && !aligned(S.starts[i], 4)) return GQ_ERR_INVALID_ARG;
    }
    if (d > 0 && !aligned(agg_out, 16)) return GQ_ERR_INVALID_ARG;
    if (d == 0) return GQ_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t blocks = (d + kSparseSpan - 1) / kSparseSpan;
    if (!grid_fits(blocks, kSparseBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks);
    int kpad = 1;
    while (kpad < K) kpad <<= 1;
    const int lanes = kSparseBlock / kpad;                      // threads per worker: 512 for K = 1 ... 8 for K = 64
    if (p->scheme == GQ_LINEAR) hipLaunchKernelGGL(sparse_span_kernel<0>, grid, dim3(kSparseBlock), 0, s, S, K, lanes, d, (int *)agg_out);
    else hipLaunchKernelGGL(sparse_span_kernel<1>, grid, dim3(kSparseBlock), 0, s, S, K, lanes, d, (int *)agg_out);
    if (launched() != GQ_OK) return GQ_ERR_DEVICE;
    return GQ_OK;
}

}  // extern "C"
