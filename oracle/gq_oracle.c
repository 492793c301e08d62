/*
 * gq_oracle.c -- plain CPU reference ("oracle") for the Global-QSGD data-parallel hot path.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may load this file.  It shares no code, header, table or helper with the HIP
 * library; the HIP library never calls it.  Everything is scalar C, one coordinate at a time, in
 * the order the paper states the steps, so that it can be checked against the paper by eye.
 *
 * What it follows (arXiv 2305.18627):
 *   Algorithm 1, norm step  global norm of the concatenation [x_1 .. x_n]          -> gqo_global_norm
 *   Algorithm 1, loop body, y = |x| / norm, z = sign(x) o xi(y) with the random
 *   Definition 1, Eq. (2)   rounding xi to one of the two neighbouring levels      -> gqo_linear_code, gqo_exp_code
 *   Section 4.2             linear grid l_i = (s-i)/s; exponential grid 0 and 2^-j -> same two functions
 *   Sec. 4.2, Implementation 8-bit and packed 4-bit storage of the level integers   -> gqo_pack, gqo_unpack
 *   Algorithm 1, last step  aggregation = plain sum of the level integers          -> gqo_aggregate
 *   Section 4.2             headroom rule for the sum at a given integer width     -> gqo_check_width, gqo_fits_width
 *   Eq. (1)                 norm * (1/n) * sum                                     -> gqo_dequantize
 *   Algorithm 2, Sec. 4.3   reduce function on (sign, exponent) pairs, tree order  -> gqo_alg2_k, gqo_exp_reduce_pair,
 *                                                                                     gqo_exp_tree_reduce, gqo_exp_reduce_dequantize
 *   Implementation section  low-bit linear codes averaged inside every reduce step -> gqo_avg_pair, gqo_avg_tree_reduce,
 *                                                                                     gqo_avg_reduce_dequantize
 *   Algorithm 1, sparse branch: only the non-zero codes are exchanged              -> gqo_compact, gqo_sparse_aggregate
 *   Theorem 1, sparsity statement (in the form Eq. (2) implies)                      -> gqo_sparse_nnz_bound
 *
 * Stored level integer ("code").  The paper numbers levels downwards, l_0 = 1 > ... > l_s = 0.
 * The integer that is stored and summed is k = s - u for level l_u, so k = 0 is the zero level:
 *   linear:       k in 0..s  stands for k/s                      integer value  V(k) = k
 *   exponential:  k = 0 stands for 0, k in 1..s for 2^(k-s)      integer value  V(k) = 2^(k-1)
 *                                                                (in units of the smallest level 2^-(s-1))
 * The signed code is q = sign(x) * k.
 *
 * Readings of the paper taken here (the paper is silent or inconsistent on these):
 *   - exponential grid: printed as l_i = 1/2^(s-i), which contradicts l_0 = 1; the proof of
 *     Theorem 1 says the segment next to zero has length 2^-(s-1).  Grid used: {0} u {2^-j, j=0..s-1}.
 *   - "global L2 norm" is the (2,2) mixed norm = L2 norm of the concatenation; "global max norm"
 *     is (inf,inf).  (2,inf) = max of per-worker L2 norms (the norm step read literally) is offered as well.
 *   - exponential aggregation is the exact integer sum of V(k) (Algorithm 2's stochastic
 *     re-rounding is a different wire format and is not part of this path).
 *   - random numbers: Eq. (2) only fixes probabilities.  The draw is 32 bits r per (worker,
 *     coordinate) from Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) with
 *     counter = (lo32(g/4), hi32(g/4), worker, 0), key = (lo32(seed), hi32(seed)), word g mod 4,
 *     g = index_base + j the global coordinate index.
 *       linear:  U' = fl32(fl32(r) * c), c = 2^-32 - 2^-56 the largest binary32 below 2^-32, so that
 *                0 <= U' < 1 with the relative resolution of binary32 near 0;
 *                v = fl32(|x| * scale - U') with ONE rounding (fused multiply-add),
 *                scale = fl32(s / norm);  k = min(ceil(v), s).
 *                So k = h+1 exactly when U' < frac part, which has probability y*s - h as Eq. (2)
 *                asks, up to the binary32 granularity of U' and of v (a coordinate that sits on
 *                level k stays there with probability >= 1 - k*2^-23, with certainty for k <= 1).
 *                |x| >= norm (y = 1, the coordinate the max norm is taken from) is the top level with
 *                certainty: Eq. (2) keeps a value that sits on a level, and y = 1 is the one non-zero level
 *                that binary32 can recognise exactly, since |x| * fl32(s/norm) need not equal s.
 *       exp:     z = fl32(|x| * scale), scale = fl32(2^(s-1) / norm), clamped to 2^(s-1);  R = r >> 9.
 *                z >= 1: z = 2^e * (1 + m/2^23); round up iff m + R >= 2^23: probability m/2^23 =
 *                (z - 2^e)/2^e exactly as Eq. (2) asks.   z < 1: m = z*2^23 rounded to nearest
 *                integer (ties to even); round up to the smallest level iff m + R >= 2^23.
 *   - short draws (rng_bits = 16): the number of random bits per coordinate is a free choice under Eq. (2),
 *     which fixes probabilities only.  With 16 bits per coordinate one Philox call serves the eight
 *     coordinates 8c .. 8c+7: counter (lo32(g/8), hi32(g/8), worker, 0), word (g mod 8) / 2, low half for
 *     even g, high half for odd g.  The 16 bits r16 take the place of the TOP half of the 32-bit word
 *     (r = r16 * 2^16), and the two rules above are applied unchanged: P(up) is then met to 2^-16
 *     (linear: count of r16 giving "up" is ceil(frac * 2^16) up to the binary32 rounding of U' and v;
 *     exponential between two levels: floor(m / 2^7) of the 2^16 values).
 *   - Algorithm 2 (the paper's own aggregation for the exponential grid, kept beside the integer sum):
 *     values are prescaled by 1/(2 n'), n' = n rounded up to a power of two, so that a code k >= 1 of the
 *     exponential grid becomes the exponent e = s - k + 1 + log2(n') of sign * 2^-e, and e = 0 is zero
 *     (Section 4.3).  The listing takes p and m without defining them; the text has p ~ U[0,1], m = s + 1 and
 *     k = -floor(log2(2^-m + [p - 2^-m]_+)) = -floor(log2 p) capped at m.  p is drawn with s bits (p = r / 2^s),
 *     the resolution at which that law is exact: P(k > b) = 2^-b for b < m, P(k = m) = 2^-(m-1).  The cap has a
 *     consequence the paper does not mention: exponents differ by up to s - 1 between leaves but by up to
 *     s + log2(n') - 1 between inner nodes, and a pair whose gap reaches m (same signs) or m + 1 (opposite
 *     signs) is never rounded towards its smaller operand, which is then dropped: a relative error of at
 *     most 2^-(s+1) of that node's sum, instead of exact unbiasedness.  Below those gaps the pair reduction
 *     is exactly unbiased.  One field of W bits per (tree node, coordinate), W = 8, 16 or 32 for s <= 8, 16, 31,
 *     whose top s bits are r: Philox counter (lo32(g/4), hi32(g/4), node / (32/W), 1), word g mod 4, field
 *     node mod (32/W); nodes are numbered as a binary heap (root 1, children 2h and 2h+1, worker i is
 *     leaf n' + i, missing workers are zeros); operand 1 of a node is its child 2h.
 *     In the second-sign case the probability is printed as 2^(e2-e1-1); the text's equivalent form
 *     "k > e2 - e1 - 1" and unbiasedness both give 2^-(e2-e1-1), which is what the listing computes.
 *   - averaging inside each reduce step (the Implementation section says only that the average replaces the sum in every
 *     step and that each step rounds): a node holds round((a + b) / 2) of its two children, an odd sum
 *     being rounded up or down with probability 1/2 each, which keeps the result unbiased and inside the
 *     range of the inputs.  Same tree as above (heap numbering, n' leaves, missing workers are zeros); the
 *     coin of node h at coordinate g is bit h mod 32 of the Philox word with counter
 *     (lo32(g/4), hi32(g/4), h / 32, 2), word g mod 4.  The root stands for the mean over n' leaves.
 *   - sparse branch (Algorithm 1 says only that the non-zero values are all-gathered): a worker's message
 *     is the list of (coordinate index, signed code) of its non-zero codes in increasing index order, and the
 *     receiver adds the integer values of all K lists into a dense sum, which equals the dense aggregate.
 *   - top of the range: |x| >= norm is the top level (both grids); below it the code is clamped to s.
 *   - norm == 0, norm not finite, or scale not finite: every code is 0.
 *
 * Floating point: the two decisions that turn a float into an integer (ceil(v), the carry out of
 * m + R) are taken in IEEE binary32 exactly as written, because that is the precision the method
 * runs in; compile with -ffp-contract=off so that nothing else is fused.  Norm and dequantised
 * values are computed in binary64.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#include <math.h>
#include <float.h>

enum { GQO_LINEAR = 0, GQO_EXP = 1 };
enum { GQO_NORM_LINF = 0, GQO_NORM_L2 = 1, GQO_NORM_L2_MAX = 2 };
enum { GQO_PACK_I8 = 0, GQO_PACK_I4 = 1, GQO_PACK_U8_SIGNPLANE = 2, GQO_PACK_U4_SIGNPLANE = 3 };

/* ------------------------------------------------------------------------------------------
 * Philox4x32 with `rounds` rounds (Salmon et al., SC'11, Section 3.3 / Table 2 constants).
 * One round: two 32x32->64 products, the high halves are xored with the other two counter
 * words and the round key, the low halves pass through; the key is bumped between rounds.
 * ------------------------------------------------------------------------------------------ */
void gqo_philox4x32(int rounds, const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;   /* multipliers */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;   /* Weyl key increments */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; r++) {
        if (r > 0) { k0 += W0; k1 += W1; }
        uint64_t p0 = (uint64_t)M0 * (uint64_t)c0;
        uint64_t p1 = (uint64_t)M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32 random bits of (seed, worker, global coordinate index g). */
uint32_t gqo_random_word(uint64_t seed, uint32_t worker, uint64_t g)
{
    uint64_t call = g / 4u;
    uint32_t ctr[4] = { (uint32_t)call, (uint32_t)(call >> 32), worker, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    gqo_philox4x32(10, ctr, key, out);
    return out[g % 4u];
}

/* Short draws: the 16 random bits of (seed, worker, g), returned in the top half of a 32-bit word
 * (r16 * 2^16) so that the rounding rules below apply unchanged.  One Philox call per 8 coordinates. */
uint32_t gqo_random_word16(uint64_t seed, uint32_t worker, uint64_t g)
{
    uint64_t call = g / 8u;
    uint32_t ctr[4] = { (uint32_t)call, (uint32_t)(call >> 32), worker, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    gqo_philox4x32(10, ctr, key, out);
    uint32_t word = out[(g % 8u) / 2u];
    uint32_t r16 = (g % 2u) ? (word >> 16) : (word & 0xFFFFu);
    return r16 << 16;
}

/* The word that decides the rounding of coordinate g: rng_bits = 32 or 16 (anything else reads as 32). */
uint32_t gqo_random_word_bits(uint64_t seed, uint32_t worker, uint64_t g, int rng_bits)
{
    return rng_bits == 16 ? gqo_random_word16(seed, worker, g) : gqo_random_word(seed, worker, g);
}

void gqo_random_words(uint64_t seed, uint32_t worker, uint64_t index_base, int64_t d, int rng_bits, uint32_t *r)
{
    for (int64_t j = 0; j < d; j++) r[j] = gqo_random_word_bits(seed, worker, index_base + (uint64_t)j, rng_bits);
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1's norm step: the global norm.  Returns flag bits: 1 = norm not finite, 2 = norm zero.
 * ------------------------------------------------------------------------------------------ */
int gqo_global_norm(const float *const *x, int K, int64_t d, int kind, double *norm_exact, float *norm_f32)
{
    double result = 0.0;
    if (kind == GQO_NORM_LINF) {
        for (int i = 0; i < K; i++)
            for (int64_t j = 0; j < d; j++) {
                double a = fabs((double)x[i][j]);
                if (a != a) result = a;                       /* NaN is sticky */
                else if (!(result != result) && a > result) result = a;
            }
    } else if (kind == GQO_NORM_L2) {
        double acc = 0.0;
        for (int i = 0; i < K; i++)
            for (int64_t j = 0; j < d; j++) acc += (double)x[i][j] * (double)x[i][j];
        result = sqrt(acc);
    } else {                                                  /* (2,inf): max over workers of ||x_i||_2 */
        for (int i = 0; i < K; i++) {
            double acc = 0.0;
            for (int64_t j = 0; j < d; j++) acc += (double)x[i][j] * (double)x[i][j];
            double ni = sqrt(acc);
            if (ni != ni) result = ni;
            else if (!(result != result) && ni > result) result = ni;
        }
    }
    *norm_exact = result;
    *norm_f32 = (float)result;
    int flags = 0;
    if (!(fabs((double)*norm_f32) <= FLT_MAX)) flags |= 1;
    if (*norm_f32 == 0.0f) flags |= 2;
    return flags;
}

/* ------------------------------------------------------------------------------------------
 * Eq. (2) on the linear grid l_u = (s-u)/s.  With t = y*s, the neighbours of y are h/s and
 * (h+1)/s, h = floor(t), and the upper one is taken with probability t - h.
 * ------------------------------------------------------------------------------------------ */
int32_t gqo_linear_code(float x, float norm, int s, uint32_t r)
{
    if (!(norm > 0.0f) || !(norm <= FLT_MAX)) return 0;  /* zero, negative, NaN or infinite norm: every code is 0 */
    float scale = (float)s / norm;
    if (!(scale <= FLT_MAX)) return 0;
    if (fabsf(x) >= norm) return (x < 0.0f) ? -s : s;   /* y = 1 = l_0: Eq. (2) leaves a value on a level there */
    float u = (float)r * 0x1.fffffep-33f;          /* U' in [0,1): fl32(r) times the largest float below 2^-32 */
    float v = fmaf(fabsf(x), scale, -u);           /* t - U' with one rounding */
    if (v != v) return 0;
    float c = ceilf(v);                            /* = h+1 iff U' < t-h, else h; never negative as U' < 1 */
    if (c > (float)s) c = (float)s;
    int32_t k = (int32_t)c;
    return (x < 0.0f) ? -k : k;
}

/* ------------------------------------------------------------------------------------------
 * Eq. (2) on the exponential grid {0} u {2^-j : j = 0..s-1}.  z = y * 2^(s-1) measures y in
 * units of the smallest non-zero level, so the grid in z is 0, 1, 2, 4, .., 2^(s-1).
 * ------------------------------------------------------------------------------------------ */
int32_t gqo_exp_code(float x, float norm, int s, uint32_t r)
{
    if (!(norm > 0.0f) || !(norm <= FLT_MAX)) return 0;  /* zero, negative, NaN or infinite norm: every code is 0 */
    float top = ldexpf(1.0f, s - 1);
    float scale = top / norm;
    if (!(scale <= FLT_MAX)) return 0;
    float z = fabsf(x) * scale;
    if (z != z) return 0;
    if (z > top || fabsf(x) >= norm) z = top;     /* y = 1 = l_0 is on the grid whatever the rounding of the scale */
    uint32_t R = r >> 9;                            /* 23 dither bits */
    int32_t k;
    if (z >= 1.0f) {
        /* 2^e <= z < 2^(e+1): lower level code e+1, upper e+2, P(up) = (z-2^e)/2^e = m/2^23 */
        uint32_t bits; memcpy(&bits, &z, 4);
        int32_t e = (int32_t)(bits >> 23) - 127;
        uint32_t m = bits & 0x7FFFFFu;
        k = e + 1 + (int32_t)((m + R) >> 23);
    } else {
        /* 0 <= z < 1: lower level 0, upper level code 1, P(up) = z, resolved to 2^-23 */
        uint32_t m = (uint32_t)lrintf(z * 0x1p23f);   /* nearest, ties to even; at most 2^23 */
        k = (int32_t)((m + R) >> 23);
    }
    if (k > s) k = s;
    return (x < 0.0f) ? -k : k;
}

int32_t gqo_code(int scheme, float x, float norm, int s, uint32_t r)
{
    return scheme == GQO_LINEAR ? gqo_linear_code(x, norm, s, r) : gqo_exp_code(x, norm, s, r);
}

/* Codes for given random words (the words are an input: used by the rounding-law tests). */
void gqo_quantize_with_words(const float *x, const uint32_t *r, int64_t d, float norm,
                             int scheme, int s, int32_t *q)
{
    for (int64_t j = 0; j < d; j++) q[j] = gqo_code(scheme, x[j], norm, s, r[j]);
}

/* Algorithm 1's quantisation loop for one worker. */
void gqo_quantize(const float *x, int64_t d, float norm, int scheme, int s,
                  uint64_t seed, uint32_t worker, uint64_t index_base, int rng_bits, int32_t *q)
{
    for (int64_t j = 0; j < d; j++)
        q[j] = gqo_code(scheme, x[j], norm, s, gqo_random_word_bits(seed, worker, index_base + (uint64_t)j, rng_bits));
}

/* Signed integer value that a signed code contributes to the sum. */
int64_t gqo_code_value(int scheme, int32_t q)
{
    if (scheme == GQO_LINEAR || q == 0) return (int64_t)q;
    int32_t k = q < 0 ? -q : q;
    int64_t v = (int64_t)1 << (k - 1);
    return q < 0 ? -v : v;
}

/* Algorithm 1's aggregation step: A_j = sum_i V(q_ij), accumulated in 64 bits. */
void gqo_aggregate(const int32_t *const *q, int K, int64_t d, int scheme, int64_t *A)
{
    for (int64_t j = 0; j < d; j++) {
        int64_t acc = 0;
        for (int i = 0; i < K; i++) acc += gqo_code_value(scheme, q[i][j]);
        A[j] = acc;
    }
}

/* Largest magnitude the sum of K codes can reach: linear K*s, exponential K*2^(s-1). */
int64_t gqo_max_aggregate(int scheme, int s, int K)
{
    if (scheme == GQO_LINEAR) return (int64_t)K * s;
    if (s > 55) return INT64_MAX;
    return (int64_t)K * ((int64_t)1 << (s - 1));
}

/* Largest value of a signed integer of `bits` bits, 2^(bits-1) - 1 (Section 4.2 counts one bit for the sign);
 * widths of 64 and more are limited by the int64 the sums are held in here. */
static int64_t width_limit(int bits)
{
    if (bits < 1) return -1;
    if (bits >= 64) return INT64_MAX;
    return (int64_t)(((uint64_t)1 << (bits - 1)) - 1u);
}

/* 1 if a signed integer of `bits` bits always holds the sum, else 0. */
int gqo_check_width(int scheme, int s, int K, int bits)
{
    return gqo_max_aggregate(scheme, s, K) <= width_limit(bits);
}

/* 1 if every A_j fits a signed integer of `bits` bits. */
int gqo_fits_width(const int64_t *A, int64_t d, int bits)
{
    int64_t lim = width_limit(bits);
    for (int64_t j = 0; j < d; j++) if (A[j] > lim || A[j] < -lim - 1) return 0;
    return 1;
}

/* Eq. (1): norm * (1/n) * sum, with the grid's unit (1/s or 2^-(s-1)) put back. */
void gqo_dequantize(const int64_t *A, int64_t d, double norm, int scheme, int s, int K, double *out)
{
    double unit = scheme == GQO_LINEAR ? 1.0 / (double)s : ldexp(1.0, -(s - 1));
    for (int64_t j = 0; j < d; j++) out[j] = norm * ((double)A[j] * unit) / (double)K;
}

/* ------------------------------------------------------------------------------------------
 * Storage of signed codes.
 *   I8            byte j = q_j as two's complement                                  (s <= 127)
 *   I4            byte b = (q_2b & 15) | (q_2b+1 & 15) << 4, two's complement nibbles (s <= 7);
 *                 an odd d leaves the last high nibble 0
 *   U8_SIGNPLANE  byte j = |q_j| (s <= 255); sign word w bit t = 1 iff q_(32w+t) < 0
 *   U4_SIGNPLANE  nibbles as I4 but holding |q| (s <= 15); same sign words
 * Returns 0, or -1 if a code does not fit the format.
 * ------------------------------------------------------------------------------------------ */
int64_t gqo_levels_bytes(int64_t d, int pack)
{
    return (pack == GQO_PACK_I8 || pack == GQO_PACK_U8_SIGNPLANE) ? d : (d + 1) / 2;
}
int64_t gqo_signplane_words(int64_t d) { return (d + 31) / 32; }

int gqo_pack(const int32_t *q, int64_t d, int pack, uint8_t *levels, uint32_t *signplane)
{
    int has_plane = (pack == GQO_PACK_U8_SIGNPLANE || pack == GQO_PACK_U4_SIGNPLANE);
    int nib = (pack == GQO_PACK_I4 || pack == GQO_PACK_U4_SIGNPLANE);
    memset(levels, 0, (size_t)gqo_levels_bytes(d, pack));
    if (has_plane) memset(signplane, 0, (size_t)gqo_signplane_words(d) * 4);
    for (int64_t j = 0; j < d; j++) {
        int32_t v = q[j], mag = v < 0 ? -v : v;
        int32_t lim = pack == GQO_PACK_I8 ? 127 : pack == GQO_PACK_I4 ? 7 : pack == GQO_PACK_U8_SIGNPLANE ? 255 : 15;
        if (mag > lim) return -1;
        uint32_t field = has_plane ? (uint32_t)mag : (uint32_t)v;
        if (nib) levels[j / 2] |= (uint8_t)((field & 15u) << (4 * (j % 2)));
        else     levels[j] = (uint8_t)(field & 255u);
        if (has_plane && v < 0) signplane[j / 32] |= (uint32_t)1 << (j % 32);
    }
    return 0;
}

void gqo_unpack(const uint8_t *levels, const uint32_t *signplane, int64_t d, int pack, int32_t *q)
{
    for (int64_t j = 0; j < d; j++) {
        int32_t v;
        if (pack == GQO_PACK_I8) v = (int8_t)levels[j];
        else if (pack == GQO_PACK_U8_SIGNPLANE) v = levels[j];
        else {
            uint32_t n = (levels[j / 2] >> (4 * (j % 2))) & 15u;
            v = (pack == GQO_PACK_I4 && n >= 8) ? (int32_t)n - 16 : (int32_t)n;
        }
        if ((pack == GQO_PACK_U8_SIGNPLANE || pack == GQO_PACK_U4_SIGNPLANE) &&
            ((signplane[j / 32] >> (j % 32)) & 1u)) v = -v;
        q[j] = v;
    }
}

/* ------------------------------------------------------------------------------------------
 * The whole path for K workers, as the composition of the steps above (no fusion here):
 * quantize each worker, sum.  Used for parity of the fused GPU call and for the CPU timing.
 * Returns 0, or -1 if memory for the K code vectors could not be had.
 * ------------------------------------------------------------------------------------------ */
int gqo_quantize_aggregate(const float *const *x, int K, int64_t d, float norm, int scheme, int s,
                           uint64_t seed, uint64_t index_base, int rng_bits, int64_t *A)
{
    int32_t **q = (int32_t **)calloc((size_t)K, sizeof(int32_t *));
    if (!q) return -1;
    int rc = 0;
    for (int i = 0; i < K; i++) {
        q[i] = (int32_t *)malloc((size_t)(d > 0 ? d : 1) * sizeof(int32_t));
        if (!q[i]) { rc = -1; break; }
        gqo_quantize(x[i], d, norm, scheme, s, seed, (uint32_t)i, index_base, rng_bits, q[i]);
    }
    if (rc == 0) gqo_aggregate((const int32_t *const *)q, K, d, scheme, A);
    for (int i = 0; i < K; i++) free(q[i]);
    free(q);
    return rc;
}

/* ==========================================================================================
 * Algorithm 2: the reduce function for exponential dithering (Section 4.3).
 * A pair (sign, e), sign in {-1,+1}, e >= 0, stands for 0 if e = 0 and for sign * 2^-e otherwise.
 * ========================================================================================== */

/* The random integer k of Algorithm 2 (its first statement, derived in Section 4.3):
 *     k = -floor(log2(2^-m + [p - 2^-m]_+)),   m = s + 1,   p uniform on [0, 1).
 * Since 2^-m + [p - 2^-m]_+ = max(p, 2^-m), k = -floor(log2 p) capped at m: its support is 1..m,
 * P(k > b) = P(p < 2^-b) = 2^-b for b = 0..m-1, and P(k = m) = 2^-(m-1).
 * p is drawn with s bits, p = r / 2^s for a uniform s-bit integer r: that is the resolution at which the
 * law above holds exactly (r = 0 is the one value with p < 2^-m, and it has probability 2^-s = 2^-(m-1)). */
int gqo_alg2_k(uint32_t r, int s)
{
    int m = s + 1;
    if (r == 0u) return m;                       /* max(p, 2^-m) = 2^-m */
    int floor_log2_r = 0;
    while ((r >> (floor_log2_r + 1)) != 0u) floor_log2_r++;
    return s - floor_log2_r;                     /* -floor(log2(r / 2^s)) */
}

/* Algorithm 2, the reduction of one pair (Section 4.3): x1 + x2 for x = sign * 2^-e (e = 0: zero), rounded at
 * random to a neighbouring power of two so that the expectation is the exact sum.  k is the random integer
 * above.  Written out case by case from the derivation in the text:
 *   - a zero operand leaves the other one unchanged;
 *   - otherwise let a be the operand of larger magnitude (smaller exponent, operand 1 on a tie), b the
 *     other, and gap = e_b - e_a >= 0;
 *   - equal signs: |x1 + x2| = 2^-e_a (1 + 2^-gap) lies a fraction 2^-gap of the way from 2^-e_a up to
 *     2^-(e_a - 1), so it goes up with probability 2^-gap = P(k > gap);
 *   - opposite signs: gap = 0 cancels exactly; else |x1 + x2| = 2^-e_a (1 - 2^-gap) lies a fraction
 *     2^-(gap-1) of the way from 2^-e_a down to 2^-(e_a + 1), so it goes down with probability P(k > gap - 1);
 *   - the sign is that of a. */
void gqo_exp_reduce_pair(int sign1, int e1, int sign2, int e2, int k, int *sign_result, int *e_result)
{
    if (e1 == 0) { *sign_result = sign2; *e_result = e2; return; }
    if (e2 == 0) { *sign_result = sign1; *e_result = e1; return; }
    int first_is_a = e1 <= e2;
    int sign_a = first_is_a ? sign1 : sign2;
    int e_a = first_is_a ? e1 : e2;
    int e_b = first_is_a ? e2 : e1;
    int gap = e_b - e_a;
    *sign_result = sign_a;
    if (sign1 == sign2) {
        *e_result = (k > gap) ? e_a - 1 : e_a;
    } else if (gap == 0) {
        *e_result = 0;
    } else {
        *e_result = (k > gap - 1) ? e_a + 1 : e_a;
    }
}

static int ceil_log2_int(int n) { int l = 0; while ((1 << l) < n) l++; return l; }

uint32_t gqo_random_word_of(uint64_t seed, uint32_t word2, uint32_t word3, uint64_t g)
{
    uint64_t call = g / 4u;
    uint32_t ctr[4] = { (uint32_t)call, (uint32_t)(call >> 32), word2, word3 };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    gqo_philox4x32(10, ctr, key, out);
    return out[g % 4u];
}

/* The s random bits r of tree node `node` at coordinate g (p = r / 2^s in gqo_alg2_k).  A node's bits are the top
 * s bits of a field of W bits, W = 8 for s <= 8, 16 for s <= 16, else 32, so that one Philox call serves the
 * four coordinates 4c .. 4c+3 of 32 / W nodes: counter (lo32(g/4), hi32(g/4), node / (32/W), 1), word g mod 4,
 * field number node mod (32/W) counted from the low end of the word. */
int gqo_alg2_field_bits(int s) { return s <= 8 ? 8 : (s <= 16 ? 16 : 32); }

uint32_t gqo_alg2_draw(uint64_t seed, uint32_t node, uint64_t g, int s)
{
    int W = gqo_alg2_field_bits(s);
    uint32_t per_word = 32u / (uint32_t)W;
    uint32_t word = gqo_random_word_of(seed, node / per_word, 1u, g);
    uint32_t field = W == 32 ? word : ((word >> ((uint32_t)W * (node % per_word))) & ((1u << W) - 1u));
    return field >> (W - s);
}

/* Tree reduction of K workers' signed exponential-grid codes with Algorithm 2.
 * out[j] = sign * e of the root (0 for zero), for the prescale 1/(2 n'), n' = 2^ceil(log2 K). */
void gqo_exp_tree_reduce(const int32_t *const *q, int K, int64_t d, int s, uint64_t seed, uint64_t index_base,
                         int32_t *out)
{
    int L = ceil_log2_int(K), npad = 1 << L;
    int sg[2 * 64], ex[2 * 64];
    for (int64_t j = 0; j < d; j++) {
        for (int i = 0; i < npad; i++) {
            int code = i < K ? q[i][j] : 0;
            int k = code < 0 ? -code : code;
            sg[npad + i] = code < 0 ? -1 : 1;
            ex[npad + i] = k ? s - k + 1 + L : 0;           /* 2^(k-s) / (2 n') = 2^-(s-k+1+L) */
        }
        for (int h = npad - 1; h >= 1; h--) {
            uint32_t r = gqo_alg2_draw(seed, (uint32_t)h, index_base + (uint64_t)j, s);
            gqo_exp_reduce_pair(sg[2 * h], ex[2 * h], sg[2 * h + 1], ex[2 * h + 1], gqo_alg2_k(r, s), &sg[h], &ex[h]);
        }
        out[j] = ex[1] ? sg[1] * ex[1] : 0;
    }
}

/* The mean the reduced pair stands for: sign * 2^-e * (2 n') * norm / K. */
void gqo_exp_reduce_dequantize(const int32_t *se, int64_t d, double norm, int K, double *out)
{
    int L = ceil_log2_int(K);
    for (int64_t j = 0; j < d; j++) {
        int e = se[j] < 0 ? -se[j] : se[j];
        double v = e ? ldexp(1.0, 1 + L - e) : 0.0;
        out[j] = (se[j] < 0 ? -v : v) * norm / (double)K;
    }
}

/* ==========================================================================================
 * Implementation section: for low-bit linear dithering the paper averages inside every reduce step instead of
 * summing until the end, so that the codes never leave their b bits.
 * ========================================================================================== */

/* One step: the average of two codes, an odd sum rounded down (coin = 0) or up (coin = 1). */
int32_t gqo_avg_pair(int32_t a, int32_t b, int coin)
{
    int32_t m = a + b;
    int32_t half = (m - (((m % 2) + 2) % 2)) / 2;          /* floor(m / 2), exact for negative m too */
    return (m % 2 != 0 && coin) ? half + 1 : half;
}

/* Tree reduction of K workers' linear codes with in-step averaging: the root's code. */
void gqo_avg_tree_reduce(const int32_t *const *q, int K, int64_t d, uint64_t seed, uint64_t index_base, int32_t *out)
{
    int L = ceil_log2_int(K), npad = 1 << L;
    int32_t node[2 * 64];
    for (int64_t j = 0; j < d; j++) {
        for (int i = 0; i < npad; i++) node[npad + i] = i < K ? q[i][j] : 0;
        for (int h = npad - 1; h >= 1; h--) {
            uint32_t r = gqo_random_word_of(seed, (uint32_t)(h / 32), 2u, index_base + (uint64_t)j);
            node[h] = gqo_avg_pair(node[2 * h], node[2 * h + 1], (int)((r >> (h % 32)) & 1u));
        }
        out[j] = node[1];
    }
}

/* The mean over the K workers that the root code stands for: norm * code/s * n'/K. */
void gqo_avg_reduce_dequantize(const int32_t *code, int64_t d, double norm, int s, int K, double *out)
{
    int npad = 1 << ceil_log2_int(K);
    for (int64_t j = 0; j < d; j++) out[j] = norm * ((double)code[j] / (double)s) * (double)npad / (double)K;
}

/* ==========================================================================================
 * Algorithm 1's sparse branch.  What a worker sends is the list of its non-zero
 * codes with their coordinate indices, in increasing index order; what every receiver forms from
 * the K lists is the same integer sum as the dense aggregate.
 * ========================================================================================== */

/* Theorem 1's sparsity statement under the (2,2) norm, in the form that follows from Eq. (2).  Let top = s (linear grid)
 * or 2^(s-1) (exponential grid), so that 1/top is the smallest non-zero level.  Since the squares of all K d values of y sum
 * to at most 1, at most top^2 coordinates have y >= 1/top; every other coordinate is non-zero with probability top * y; and
 * the sum of all y is at most sqrt(K d).  Hence
 *     E[number of non-zero codes over all K workers]  <=  top^2 + top * sqrt(K d),
 * and never more than K d.  (The statement as printed has sqrt(nd) without the factor top.)  Returns -1 for arguments
 * outside the grids' ranges. */
double gqo_sparse_nnz_bound(int scheme, int s, int K, int64_t d)
{
    if ((scheme != 0 && scheme != 1) || s < 1 || K < 1 || d < 0) return -1.0;
    if (scheme == 1 && s > 31) return -1.0;
    double top = scheme == 0 ? (double)s : ldexp(1.0, s - 1);
    double all = (double)K * (double)d;
    double bound = top * top + top * sqrt(all);
    return bound < all ? bound : all;
}

/* Returns the number of non-zero codes; writes at most `capacity` (index, code) pairs. */
int64_t gqo_compact(const int32_t *q, int64_t d, int64_t capacity, uint32_t *index_out, int32_t *code_out)
{
    int64_t n = 0;
    for (int64_t j = 0; j < d; j++) {
        if (q[j] != 0) {
            if (n < capacity) { index_out[n] = (uint32_t)j; code_out[n] = q[j]; }
            n++;
        }
    }
    return n;
}

/* A_j = sum over workers and over their list entries with index j of the integer value of the code. */
void gqo_sparse_aggregate(const uint32_t *const *index, const int32_t *const *code, const int64_t *count,
                          int K, int64_t d, int scheme, int64_t *A)
{
    for (int64_t j = 0; j < d; j++) A[j] = 0;
    for (int i = 0; i < K; i++)
        for (int64_t t = 0; t < count[i]; t++) A[index[i][t]] += gqo_code_value(scheme, code[i][t]);
}
