// Tree reductions of stored codes on MI355X (gfx950): Algorithm 2 for the exponential grid and the
// in-step averaging of the Implementation section for low-bit linear codes.  Contracts: include/gqsgd.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

namespace gq {

// =============================================================================================
// Algorithm 2 (Section 4.3): the paper's own aggregation for the exponential grid.  Codes are moved
// to the prescaled representation sign * 2^-e, e = s - k + 1 + log2(n'), and reduced pairwise in
// tree order; every node rounds its sum to a neighbouring power of two with the random integer
// k = -floor(log2(max(p, 2^-m))), m = s + 1, p = r / 2^s for the node's s random bits r.  A lane owns four
// coordinates and walks the tree depth first with a stack of log2(n') + 1 partial results, so the K code
// words are consumed as they arrive.  A node's bits are the top s bits of a field of W = 8, 16 or 32 bits
// (s <= 8, 16, 31) of the Philox call of its group of 32 / W nodes, so one call serves 4, 2 or 1 nodes.
//
// Three arithmetic paths give the same results.  For s <= 16 a partial result is held as the floating-point
// number sign * 2^j it stands for (scaled by 2^(s + log2(n') + 1), so j = s + log2(n') + 1 - e >= 1, zero is 0):
// the sum of two of them is exact (or rounds to the larger operand where the cap on k forbids any move anyway),
// and the random rounding to a neighbouring power of two is an integer add on its mantissa followed by a mask,
// as in the exponential quantiser.  s <= 8 (8-bit fields) runs on packed binary16 pairs, two coordinates per
// instruction (exp_reduce_f16_kernel); 8 < s <= 16 on binary32; for s > 16 (32-bit fields) the integer form
// of the listing is kept.
// =============================================================================================
constexpr int kReduceBlock = 128;

// ---- binary32 path ----------------------------------------------------------------------------------------
// x1, x2: sign * 2^j or 0.  A = (2^s - 1 - r) << (23 - s) for the node's s random bits r.
//   same signs      mantissa of the sum is 2^(23-gap); adding A carries into the exponent iff r < 2^(s-gap),
//                   i.e. iff k > gap: up to the next power of two, never for gap > s (the cap k <= m)
//   opposite signs  the sum 2^ja - 2^jb has exponent ja - 1 and mantissa 2^23 - 2^(24-gap); adding
//                   B = A ^ 0x7FFFFF = (r << (23-s)) | (2^(23-s) - 1) carries iff r >= 2^(s+1-gap), i.e. iff NOT k > gap - 1:
//                   the result stays at 2^ja, else goes down to 2^(ja-1); always stays for gap > s + 1 (the cap)
//   a zero operand  leaves a zero mantissa: no carry, the other operand passes unchanged; x - x = +0
__device__ __forceinline__ float alg2_pair_f32(float x1, float x2, uint32_t A)
{
    const float sum = x1 + x2;
    const uint32_t opposite = (uint32_t)((int)(__float_as_uint(x1) ^ __float_as_uint(x2)) >> 31);   // all ones iff the signs differ
    const uint32_t R = A ^ (opposite & 0x7FFFFFu);
    return __uint_as_float((__float_as_uint(sum) + R) & 0xFF800000u);
}

// ---- packed binary16 path (8-bit fields, s <= 8) -------------------------------------------------------------
// Two coordinates per register: x1, x2 hold two binary16 numbers sign * 2^j or 0 (j <= s + log2(n') + 1 <= 15).
// The same construction on the 10-bit mantissa: A = (2^s - 1 - r) << (10 - s) in each half.  The binary16 sum is
// exact up to a gap of 10 (same signs) or 11 (opposite signs); beyond that it rounds to the larger operand,
// which is what the cap k <= m = s + 1 <= 9 asks for at those gaps anyway (the result never moves there).
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f16x2 alg2_pair_f16x2(f16x2 x1, f16x2 x2, uint32_t A)
{
    const f16x2 sum = x1 + x2;
    const uint32_t differ = __builtin_bit_cast(uint32_t, x1) ^ __builtin_bit_cast(uint32_t, x2);
    const i16x2 opposite = __builtin_bit_cast(i16x2, differ) >> (i16x2){15, 15};                     // all ones per half iff the signs differ
    const uint32_t R = A ^ (__builtin_bit_cast(uint32_t, opposite) & 0x03FF03FFu);
    const u16x2 rounded = __builtin_bit_cast(u16x2, sum) + __builtin_bit_cast(u16x2, R);             // no carry between the halves
    return __builtin_bit_cast(f16x2, __builtin_bit_cast(uint32_t, rounded) & 0xFC00FC00u);
}

// ---- integer path (32-bit fields) -------------------------------------------------------------------------
// A partial result: sg carries the sign in its top bit (its other bits are free), e is the exponent of 2^-e,
// and ZERO is stood for by any e >= kZeroE / 2.  With zero as a huge exponent the listing's special cases for
// zero operands disappear: 2^-e + "2^-huge" never rounds away from 2^-e, because k is at most m <= 32.
constexpr int kZeroE = 1 << 20;
struct Pow2 { int sg; int e; };

// One node: a = the operand with the smaller exponent (operand 1 on a tie), diff = e_b - e_a.
//   same signs      2^-ea + 2^-eb lies in [2^-ea, 2^-(ea-1)]: up to 2^-(ea-1) iff k > diff
//   opposite signs  2^-ea - 2^-eb lies in [2^-(ea+1), 2^-ea]: down to 2^-(ea+1) iff k > diff - 1; 0 if diff = 0
// with k = 1 + min(leading zeros of the 32-bit field, s), so k > t iff that minimum is >= t.
__device__ __forceinline__ Pow2 alg2_pair_int(const Pow2 &x1, const Pow2 &x2, uint32_t r, int s)
{
    const int lead = min(__clz((int)r), s);                          // k - 1; the cap m = s + 1 on k
    const bool first = x1.e <= x2.e;
    const int ea = min(x1.e, x2.e), eb = max(x1.e, x2.e);
    const int opp = (int)((uint32_t)(x1.sg ^ x2.sg) >> 31);          // 1 iff the signs differ
    const int t = (eb - ea) - opp;                                   // -1: equal magnitudes, opposite signs
    const int step = (lead >= t) ? (opp ? 1 : -1) : 0;
    Pow2 o;
    o.sg = first ? x1.sg : x2.sg;
    o.e = t < 0 ? kZeroE : ea + step;
    return o;
}

// Was `node` the first of its group of PER nodes to be visited by the depth-first walk?  Nodes of one tree
// level are visited in increasing order and a group lies inside one level, except the group of nodes 1..PER-1,
// whose first visited member is node 2 (node 1 in a tree of two leaves).
template <int NPAD, int PER> __device__ __forceinline__ constexpr bool first_of_group(int node)
{
    if (node % PER == 0) return true;
    if (node >= PER) return false;
    return NPAD == 2 ? node == 1 : (PER == 2 ? node == 1 : node == 2);
}

// leaf w0 + j as a compile-time constant
template <int W0, int J> using jj_leaf = std::integral_constant<int, W0 + J>;

template <int NPAD, bool UNIFORM_HI, int W>
__global__ void __launch_bounds__(kReduceBlock)
exp_reduce_kernel(LevelCPtrs Lv, int K, int64_t d, int s, uint64_t seed, uint64_t call_base,
                  const float *__restrict__ norm, void *__restrict__ reduced_out, float *__restrict__ deq_out)
{
    constexpr int L = NPAD == 1 ? 0 : NPAD == 2 ? 1 : NPAD == 4 ? 2 : NPAD == 8 ? 3 : NPAD == 16 ? 4 : NPAD == 32 ? 5 : 6;
    constexpr bool kFloat = W < 32;
    constexpr int PER = 32 / W;                              // tree nodes served by one Philox call
    // binary32 path: the value sign * 2^min(|q|, s) of every code byte q (0 for q = 0)
    __shared__ float leaf_value[kFloat ? 256 : 1];
    if (kFloat) {
        for (int b = threadIdx.x; b < 256; b += kReduceBlock) {
            const int q = (int)(int8_t)b;
            const float v = q ? __uint_as_float((uint32_t)(127 + min(abs(q), s)) << 23) : 0.0f;
            leaf_value[b] = q < 0 ? -v : v;
        }
        __syncthreads();
    }
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
    // the stack of partial results: binary32 values, or (sign carrier, exponent) pairs
    float st_f[kFloat ? L + 1 : 1][4];
    int st_sg[kFloat ? 1 : L + 1][4], st_e[kFloat ? 1 : L + 1][4];
    // the Philox words of the node groups in use, one slot per tree level; the binary32 path keeps them complemented
    uint32_t grp[L + 1][4];
    constexpr int kBatch = NPAD < 8 ? NPAD : 8;
    constexpr int kBatchL = NPAD < 8 ? L : 3;                // tree levels inside a batch of leaves
    // the node above the subtree of 2^lvl leaves that ends with leaf i
    auto fold = [&](auto leaf, auto level) {
        constexpr int i = decltype(leaf)::value, lvl = decltype(level)::value;
        if constexpr (((i + 1) & ((1 << lvl) - 1)) == 0) {               // the subtree is complete
            constexpr int top = __builtin_popcount((unsigned)i) - (lvl - 1);   // one partial result was folded per level below
            constexpr int node = (NPAD >> lvl) + (i >> lvl);             // heap numbering
            // the root shares its group with nodes 2 and 3 (one level down) when a call serves four nodes
            constexpr int slot = (PER == 4 && node == 1 && NPAD >= 4) ? lvl - 1 : lvl;
            if constexpr (first_of_group<NPAD, PER>(node)) {
                const Words4 r = philox4x32_10(c_lo, c_hi, (uint32_t)(node / PER), 1u, k0, k1);
#pragma unroll
                for (int c = 0; c < 4; c++) grp[slot][c] = kFloat ? ~r.w[c] : r.w[c];
            }
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if constexpr (kFloat) {
                    // the top s bits of the node's complemented field, moved to the top of the mantissa
                    const uint32_t A = __builtin_amdgcn_ubfe(grp[slot][c], (uint32_t)(W * (node % PER) + W - s), (uint32_t)s)
                                       << (23 - s);
                    st_f[top - 1][c] = alg2_pair_f32(st_f[top - 1][c], st_f[top][c], A);
                } else {
                    const Pow2 o = alg2_pair_int(Pow2{st_sg[top - 1][c], st_e[top - 1][c]}, Pow2{st_sg[top][c], st_e[top][c]},
                                                 grp[slot][c], s);
                    st_sg[top - 1][c] = o.sg; st_e[top - 1][c] = o.e;
                }
            }
        }
    };
    static_for<0, NPAD / kBatch>([&](auto batch) {
        constexpr int w0 = decltype(batch)::value * kBatch;
        // A batch of leaves beyond the last worker is a zero subtree: its root is set, not computed (K > NPAD / 2, so
        // only batches of the second half can be empty; the draws of their inner nodes are needed by nobody else).
        if (2 * w0 < NPAD || w0 < K) {
            uint32_t words[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; j++) words[j] = fetch(w0 + j);
            static_for<0, kBatch>([&](auto jj) {
                constexpr int j = decltype(jj)::value;
                constexpr int i = w0 + j;                    // leaf index; the stack depth is popcount(i)
                constexpr int top0 = __builtin_popcount((unsigned)i);
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    if constexpr (kFloat) {
                        st_f[top0][c] = leaf_value[(words[j] >> (8 * c)) & 255u];
                    } else {
                        // code k >= 1 of the exponential grid -> e = s - k + 1 + L; code 0 is zero
                        const int q = (int)(int8_t)(words[j] >> (8 * c));
                        st_sg[top0][c] = q;
                        st_e[top0][c] = q ? s + 1 + L - abs(q) : kZeroE;
                    }
                }
                static_for<1, kBatchL + 1>([&](auto ll) { fold(jj_leaf<w0, j>(), ll); });
            });
        } else {
            constexpr int top0 = __builtin_popcount((unsigned)w0);
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if constexpr (kFloat) {
                    st_f[top0][c] = 0.0f;
                } else {
                    st_sg[top0][c] = 0;
                    st_e[top0][c] = kZeroE;
                }
            }
        }
        // the batch's result is pinned: without this the compiler issues the loads of all NPAD workers before the first
        // node (one register each), and trees of 64 leaves run with two waves per SIMD
        if constexpr (NPAD > kBatch) {
            constexpr int t0 = __builtin_popcount((unsigned)w0);
            if constexpr (kFloat) asm volatile("" : "+v"(st_f[t0][0]), "+v"(st_f[t0][1]), "+v"(st_f[t0][2]), "+v"(st_f[t0][3]) : : "memory");
            else asm volatile("" : "+v"(st_e[t0][0]), "+v"(st_e[t0][1]), "+v"(st_e[t0][2]), "+v"(st_e[t0][3]),
                                   "+v"(st_sg[t0][0]), "+v"(st_sg[t0][1]), "+v"(st_sg[t0][2]), "+v"(st_sg[t0][3]) : : "memory");
        }
        static_for<kBatchL + 1, L + 1>([&](auto ll) { fold(jj_leaf<w0, kBatch - 1>(), ll); });
    });
    int root[4];                                            // sign * e of the root, 0 for zero
#pragma unroll
    for (int c = 0; c < 4; c++) {
        if (kFloat) {
            const uint32_t b = __float_as_uint(st_f[0][c]);
            const int j = (int)((b >> 23) & 255u) - 127;    // the root stands for 2^j, j = s + L + 1 - e
            const int e = (b & 0x7F800000u) ? s + L + 1 - j : 0;
            root[c] = (b >> 31) ? -e : e;
        } else {
            const int e = st_e[0][c] >= kZeroE / 2 ? 0 : st_e[0][c];
            root[c] = st_sg[0][c] < 0 ? -e : e;
        }
    }
    if (reduced_out) {
        const uint32_t wout = (uint32_t)(root[0] & 255) | ((uint32_t)(root[1] & 255) << 8) |
                              ((uint32_t)(root[2] & 255) << 16) | ((uint32_t)(root[3] & 255) << 24);
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
            const int se = root[i], e = abs(se);
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

// Algorithm 2 for s <= 8 on packed binary16 pairs: the same walk as exp_reduce_kernel with two coordinates per
// register, which halves the instructions of the pair reductions (they dominate the kernel's time).
template <int NPAD, bool UNIFORM_HI>
__global__ void __launch_bounds__(kReduceBlock)
exp_reduce_f16_kernel(LevelCPtrs Lv, int K, int64_t d, int s, uint64_t seed, uint64_t call_base,
                      const float *__restrict__ norm, void *__restrict__ reduced_out, float *__restrict__ deq_out)
{
    constexpr int L = NPAD == 1 ? 0 : NPAD == 2 ? 1 : NPAD == 4 ? 2 : NPAD == 8 ? 3 : NPAD == 16 ? 4 : NPAD == 32 ? 5 : 6;
    constexpr int PER = 4;                                   // tree nodes served by one Philox call (8-bit fields)
    // the binary16 value sign * 2^min(|q|, s) of every code byte q (0 for q = 0)
    __shared__ _Float16 leaf_value[256];
    for (int b = threadIdx.x; b < 256; b += kReduceBlock) {
        const int q = (int)(int8_t)b;
        const uint16_t bits = q ? (uint16_t)(((15 + min(abs(q), s)) << 10) | (q < 0 ? 0x8000 : 0)) : (uint16_t)0;
        leaf_value[b] = __builtin_bit_cast(_Float16, bits);
    }
    __syncthreads();
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
    // every byte of a complemented Philox word keeps its top s bits only: byte << 2 is then A of its half
    const uint32_t keep = 0x01010101u * ((0xFFu << (8 - s)) & 0xFFu);
    f16x2 st[L + 1][2];                                      // the stack: coordinates (0,1) and (2,3) of every partial result
    uint32_t grp[L + 1][4];                                  // masked complemented Philox words of the node groups in use
    constexpr int kBatch = NPAD < 8 ? NPAD : 8;
    constexpr int kBatchL = NPAD < 8 ? L : 3;                // tree levels inside a batch of leaves
    // the node above the subtree of 2^lvl leaves that ends with leaf i
    auto fold = [&](auto leaf, auto level) {
        constexpr int i = decltype(leaf)::value, lvl = decltype(level)::value;
        if constexpr (((i + 1) & ((1 << lvl) - 1)) == 0) {               // the subtree is complete
            constexpr int top = __builtin_popcount((unsigned)i) - (lvl - 1);   // one partial result was folded per level below
            constexpr int node = (NPAD >> lvl) + (i >> lvl);             // heap numbering
            constexpr int slot = (node == 1 && NPAD >= 4) ? lvl - 1 : lvl;     // the root shares its group with nodes 2 and 3
            if constexpr (first_of_group<NPAD, PER>(node)) {
                const Words4 r = philox4x32_10(c_lo, c_hi, (uint32_t)(node / PER), 1u, k0, k1);
#pragma unroll
                for (int c = 0; c < 4; c++) grp[slot][c] = ~r.w[c] & keep;
            }
            // byte `node % 4` of the words of coordinates (0,1) resp. (2,3) into the low bytes of the two halves
            constexpr uint32_t kZero = 0x0Cu;                // v_perm_b32 selector of a zero byte
            constexpr uint32_t sel = (kZero << 24) | ((uint32_t)(4 + node % PER) << 16) | (kZero << 8) | (uint32_t)(node % PER);
            const uint32_t A01 = __builtin_amdgcn_perm(grp[slot][1], grp[slot][0], sel) << 2;
            const uint32_t A23 = __builtin_amdgcn_perm(grp[slot][3], grp[slot][2], sel) << 2;
            st[top - 1][0] = alg2_pair_f16x2(st[top - 1][0], st[top][0], A01);
            st[top - 1][1] = alg2_pair_f16x2(st[top - 1][1], st[top][1], A23);
        }
    };
    static_for<0, NPAD / kBatch>([&](auto batch) {
        constexpr int w0 = decltype(batch)::value * kBatch;
        // A batch of leaves beyond the last worker is a zero subtree: its root is set, not computed (K > NPAD / 2, so
        // only batches of the second half can be empty; the draws of their inner nodes are needed by nobody else).
        if (2 * w0 < NPAD || w0 < K) {
            uint32_t words[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; j++) words[j] = fetch(w0 + j);
            static_for<0, kBatch>([&](auto jj) {
                constexpr int j = decltype(jj)::value;
                constexpr int top0 = __builtin_popcount((unsigned)(w0 + j));     // leaf w0 + j; the stack depth is popcount of it
                st[top0][0] = (f16x2){leaf_value[words[j] & 255u], leaf_value[(words[j] >> 8) & 255u]};
                st[top0][1] = (f16x2){leaf_value[(words[j] >> 16) & 255u], leaf_value[words[j] >> 24]};
                static_for<1, kBatchL + 1>([&](auto ll) { fold(jj_leaf<w0, j>(), ll); });
            });
        } else {
            constexpr int top0 = __builtin_popcount((unsigned)w0);
            st[top0][0] = (f16x2){(_Float16)0, (_Float16)0};
            st[top0][1] = (f16x2){(_Float16)0, (_Float16)0};
        }
        // the batch's result is pinned: without this the compiler issues the loads of all NPAD workers before the first
        // node (one register each), and trees of 64 leaves run with two waves per SIMD
        if constexpr (NPAD > kBatch) {
            constexpr int t0 = __builtin_popcount((unsigned)w0);
            asm volatile("" : "+v"(st[t0][0]), "+v"(st[t0][1]) : : "memory");
        }
        static_for<kBatchL + 1, L + 1>([&](auto ll) { fold(jj_leaf<w0, kBatch - 1>(), ll); });
    });
    int root[4];                                            // sign * e of the root, 0 for zero
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const uint32_t b = (__builtin_bit_cast(uint32_t, st[0][c >> 1]) >> (16 * (c & 1))) & 0xFFFFu;
        const int j = (int)((b >> 10) & 31u) - 15;          // the root stands for 2^j, j = s + L + 1 - e
        const int e = (b & 0x7C00u) ? s + L + 1 - j : 0;
        root[c] = (b & 0x8000u) ? -e : e;
    }
    if (reduced_out) {
        const uint32_t wout = (uint32_t)(root[0] & 255) | ((uint32_t)(root[1] & 255) << 8) |
                              ((uint32_t)(root[2] & 255) << 16) | ((uint32_t)(root[3] & 255) << 24);
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
            const int se = root[i], e = abs(se);
            const float p2 = __uint_as_float((uint32_t)(127 + 1 + L - e) << 23);     // 2^(1+L-e)
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
// Implementation section: low-bit linear codes averaged inside every reduce step, so that they never leave their
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

}  // namespace gq

using namespace gq;

extern "C" {

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
    if (!grid_fits(blocks, kReduceBlock)) return GQ_ERR_INVALID_ARG;
    const dim3 grid((unsigned)blocks), block(kReduceBlock);
    const uint64_t call_base = (uint64_t)index_base / 4u;
    const bool one_stretch = ((call_base & 0xFFFFFFFFull) + (uint64_t)(blocks * kReduceBlock)) <= ((uint64_t)1 << 32);
    hipStream_t s = (hipStream_t)hip_stream;
    int npad = 1;
    while (npad < K) npad <<= 1;
    // width of the field a node's s random bits are the top of
    const int field_bits = p->s <= 8 ? 8 : (p->s <= 16 ? 16 : 32);
#define GQ_RED3(N, UH, FB) hipLaunchKernelGGL((exp_reduce_kernel<N, UH, FB>), grid, block, 0, s, Lv, K, d, p->s, p->seed, \
                                              call_base, norm, reduced_out, dequant_out)
#define GQ_RED16(N, UH) hipLaunchKernelGGL((exp_reduce_f16_kernel<N, UH>), grid, block, 0, s, Lv, K, d, p->s, p->seed, \
                                           call_base, norm, reduced_out, dequant_out)
#define GQ_RED2(N, UH) do { if (field_bits == 8) GQ_RED16(N, UH); else if (field_bits == 16) GQ_RED3(N, UH, 16); else GQ_RED3(N, UH, 32); } while (0)
#define GQ_RED(N) do { if (one_stretch) GQ_RED2(N, true); else GQ_RED2(N, false); } while (0)
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
#undef GQ_RED2
#undef GQ_RED3
#undef GQ_RED16
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
    if (!grid_fits(blocks, kReduceBlock)) return GQ_ERR_INVALID_ARG;
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

}  // extern "C"
