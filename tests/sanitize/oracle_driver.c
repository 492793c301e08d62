/*
 * Calls every function of oracle/gq_oracle.c on small ragged inputs.  Built together with the oracle under
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py and run as a subprocess: any read or write out
 * of bounds, signed overflow, bad shift or misaligned access in the oracle ends the run with a non-zero status.
 * The buffers are heap blocks of exactly the size each call is entitled to, so that one byte too far is caught.
 * Values are also sanity-checked so that the calls cannot be optimised away.  Test infrastructure only.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

void gqo_philox4x32(int rounds, const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t gqo_random_word(uint64_t seed, uint32_t worker, uint64_t g);
uint32_t gqo_random_word16(uint64_t seed, uint32_t worker, uint64_t g);
uint32_t gqo_random_word_bits(uint64_t seed, uint32_t worker, uint64_t g, int rng_bits);
void gqo_random_words(uint64_t seed, uint32_t worker, uint64_t index_base, int64_t d, int rng_bits, uint32_t *r);
int gqo_global_norm(const float *const *x, int K, int64_t d, int kind, double *norm_exact, float *norm_f32);
int32_t gqo_linear_code(float x, float norm, int s, uint32_t r);
int32_t gqo_exp_code(float x, float norm, int s, uint32_t r);
int32_t gqo_code(int scheme, float x, float norm, int s, uint32_t r);
void gqo_quantize_with_words(const float *x, const uint32_t *r, int64_t d, float norm, int scheme, int s, int32_t *q);
void gqo_quantize(const float *x, int64_t d, float norm, int scheme, int s, uint64_t seed, uint32_t worker,
                  uint64_t index_base, int rng_bits, int32_t *q);
int64_t gqo_code_value(int scheme, int32_t q);
void gqo_aggregate(const int32_t *const *q, int K, int64_t d, int scheme, int64_t *A);
int64_t gqo_max_aggregate(int scheme, int s, int K);
int gqo_check_width(int scheme, int s, int K, int bits);
int gqo_fits_width(const int64_t *A, int64_t d, int bits);
void gqo_dequantize(const int64_t *A, int64_t d, double norm, int scheme, int s, int K, double *out);
int64_t gqo_levels_bytes(int64_t d, int pack);
int64_t gqo_signplane_words(int64_t d);
int gqo_pack(const int32_t *q, int64_t d, int pack, uint8_t *levels, uint32_t *signplane);
void gqo_unpack(const uint8_t *levels, const uint32_t *signplane, int64_t d, int pack, int32_t *q);
int gqo_quantize_aggregate(const float *const *x, int K, int64_t d, float norm, int scheme, int s, uint64_t seed,
                           uint64_t index_base, int rng_bits, int64_t *A);
int gqo_alg2_k(uint32_t r, int s);
uint32_t gqo_alg2_draw(uint64_t seed, uint32_t node, uint64_t g, int s);
int gqo_alg2_field_bits(int s);
void gqo_exp_reduce_pair(int sign1, int e1, int sign2, int e2, int k, int *sign_result, int *e_result);
uint32_t gqo_random_word_of(uint64_t seed, uint32_t word2, uint32_t word3, uint64_t g);
void gqo_exp_tree_reduce(const int32_t *const *q, int K, int64_t d, int s, uint64_t seed, uint64_t index_base, int32_t *out);
void gqo_exp_reduce_dequantize(const int32_t *se, int64_t d, double norm, int K, double *out);
int32_t gqo_avg_pair(int32_t a, int32_t b, int coin);
void gqo_avg_tree_reduce(const int32_t *const *q, int K, int64_t d, uint64_t seed, uint64_t index_base, int32_t *out);
void gqo_avg_reduce_dequantize(const int32_t *code, int64_t d, double norm, int s, int K, double *out);
int64_t gqo_compact(const int32_t *q, int64_t d, int64_t capacity, uint32_t *index_out, int32_t *code_out);
void gqo_sparse_aggregate(const uint32_t *const *index, const int32_t *const *code, const int64_t *count, int K,
                          int64_t d, int scheme, int64_t *A);
double gqo_sparse_nnz_bound(int scheme, int s, int K, int64_t d);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed line %d: %s\n", __LINE__, #cond); failures++; } } while (0)

/* exact-size heap block (size 0 still gives a valid pointer) */
static void *block(size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (!p) { perror("malloc"); exit(2); } return p; }

static const int64_t SIZES[] = { 0, 1, 2, 3, 4, 5, 7, 8, 9, 31, 32, 33, 63, 64, 65, 1021 };
static const uint64_t BASES[] = { 0u, 8u * 12345u, ((uint64_t)1 << 34) - 8u, ((uint64_t)1 << 34) + 8u, ((uint64_t)1 << 36) };
enum { NSIZES = sizeof(SIZES) / sizeof(SIZES[0]), NBASES = sizeof(BASES) / sizeof(BASES[0]) };

static void fill(float *x, int64_t d, uint32_t salt, float scale)
{
    for (int64_t j = 0; j < d; j++) {
        uint32_t r = gqo_random_word(0x1234u + salt, 7u, (uint64_t)j);
        x[j] = scale * ((float)(int32_t)r * 0x1p-31f);
    }
}

static void one_case(int K, int64_t d, int scheme, int s, int pack, uint64_t base, int rng_bits)
{
    float **x = (float **)block((size_t)K * sizeof(float *));
    int32_t **q = (int32_t **)block((size_t)K * sizeof(int32_t *));
    for (int i = 0; i < K; i++) {
        x[i] = (float *)block((size_t)d * sizeof(float));
        q[i] = (int32_t *)block((size_t)d * sizeof(int32_t));
        fill(x[i], d, (uint32_t)i, 3e-3f);
    }
    if (d > 2) { x[0][1] = -0.0f; x[K - 1][d - 1] = 1e-42f; }            /* a negative zero and a denormal */
    for (int kind = 0; kind < 3; kind++) {
        double ne; float nf;
        int fl = gqo_global_norm((const float *const *)x, K, d, kind, &ne, &nf);
        CHECK(d == 0 ? (fl == 2) : (fl == 0));
        float norm = nf;
        int64_t *A = (int64_t *)block((size_t)d * sizeof(int64_t));
        for (int i = 0; i < K; i++) {
            gqo_quantize(x[i], d, norm, scheme, s, 99u, (uint32_t)i, base, rng_bits, q[i]);
            for (int64_t j = 0; j < d; j++) CHECK(q[i][j] >= -s && q[i][j] <= s);
            /* words given from outside must reproduce the same codes */
            uint32_t *r = (uint32_t *)block((size_t)d * sizeof(uint32_t));
            int32_t *q2 = (int32_t *)block((size_t)d * sizeof(int32_t));
            gqo_random_words(99u, (uint32_t)i, base, d, rng_bits, r);
            gqo_quantize_with_words(x[i], r, d, norm, scheme, s, q2);
            CHECK(memcmp(q2, q[i], (size_t)d * sizeof(int32_t)) == 0);
            free(r); free(q2);
            /* storage round trip in exactly sized buffers */
            uint8_t *lv = (uint8_t *)block((size_t)gqo_levels_bytes(d, pack));
            uint32_t *sp = (uint32_t *)block((size_t)gqo_signplane_words(d) * 4u);
            int32_t *back = (int32_t *)block((size_t)d * sizeof(int32_t));
            CHECK(gqo_pack(q[i], d, pack, lv, sp) == 0);
            gqo_unpack(lv, sp, d, pack, back);
            CHECK(memcmp(back, q[i], (size_t)d * sizeof(int32_t)) == 0);
            free(lv); free(sp); free(back);
        }
        gqo_aggregate((const int32_t *const *)q, K, d, scheme, A);
        CHECK(gqo_fits_width(A, d, 64 - 1) == 1);
        for (int64_t j = 0; j < d; j++) CHECK(llabs((long long)A[j]) <= gqo_max_aggregate(scheme, s, K));
        int64_t *A2 = (int64_t *)block((size_t)d * sizeof(int64_t));
        CHECK(gqo_quantize_aggregate((const float *const *)x, K, d, norm, scheme, s, 99u, base, rng_bits, A2) == 0);
        CHECK(memcmp(A, A2, (size_t)d * sizeof(int64_t)) == 0);
        double *out = (double *)block((size_t)d * sizeof(double));
        gqo_dequantize(A, d, (double)norm, scheme, s, K, out);
        for (int64_t j = 0; j < d; j++) CHECK(fabs(out[j]) <= (double)norm * 1.0000001);
        free(out); free(A2);
        /* sparse branch: full capacity, a short buffer, no buffer at all */
        {
            uint32_t **idx = (uint32_t **)block((size_t)K * sizeof(uint32_t *));
            int32_t **val = (int32_t **)block((size_t)K * sizeof(int32_t *));
            int64_t *cnt = (int64_t *)block((size_t)K * sizeof(int64_t));
            for (int i = 0; i < K; i++) {
                int64_t n = gqo_compact(q[i], d, 0, NULL, NULL);
                idx[i] = (uint32_t *)block((size_t)n * sizeof(uint32_t));
                val[i] = (int32_t *)block((size_t)n * sizeof(int32_t));
                CHECK(gqo_compact(q[i], d, n, idx[i], val[i]) == n);
                if (n > 1) {
                    uint32_t *si = (uint32_t *)block((size_t)(n - 1) * sizeof(uint32_t));
                    int32_t *sv = (int32_t *)block((size_t)(n - 1) * sizeof(int32_t));
                    CHECK(gqo_compact(q[i], d, n - 1, si, sv) == n);
                    CHECK(memcmp(si, idx[i], (size_t)(n - 1) * sizeof(uint32_t)) == 0);
                    free(si); free(sv);
                }
                cnt[i] = n;
            }
            int64_t *A3 = (int64_t *)block((size_t)d * sizeof(int64_t));
            gqo_sparse_aggregate((const uint32_t *const *)idx, (const int32_t *const *)val, cnt, K, d, scheme, A3);
            CHECK(memcmp(A, A3, (size_t)d * sizeof(int64_t)) == 0);
            for (int i = 0; i < K; i++) { free(idx[i]); free(val[i]); }
            free(idx); free(val); free(cnt); free(A3);
        }
        /* tree reductions */
        {
            int32_t *red = (int32_t *)block((size_t)d * sizeof(int32_t));
            double *m = (double *)block((size_t)d * sizeof(double));
            if (scheme == 1) {
                gqo_exp_tree_reduce((const int32_t *const *)q, K, d, s, 5u, base, red);
                gqo_exp_reduce_dequantize(red, d, (double)norm, K, m);
                for (int64_t j = 0; j < d; j++) CHECK(abs(red[j]) <= s + 6);
            } else {
                gqo_avg_tree_reduce((const int32_t *const *)q, K, d, 5u, base, red);
                gqo_avg_reduce_dequantize(red, d, (double)norm, s, K, m);
                for (int64_t j = 0; j < d; j++) CHECK(abs(red[j]) <= s);
            }
            free(red); free(m);
        }
        free(A);
    }
    for (int i = 0; i < K; i++) { free(x[i]); free(q[i]); }
    free(x); free(q);
}

int main(void)
{
    /* the block function and the word selectors at the ends of their ranges */
    uint32_t ctr[4] = { 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu }, key[2] = { 0xFFFFFFFFu, 0xFFFFFFFFu }, out[4];
    gqo_philox4x32(10, ctr, key, out);
    gqo_philox4x32(0, ctr, key, out);
    CHECK(out[0] == 0xFFFFFFFFu);
    (void)gqo_random_word(~(uint64_t)0, 0xFFFFFFFFu, ~(uint64_t)0);
    (void)gqo_random_word16(~(uint64_t)0, 0xFFFFFFFFu, ~(uint64_t)0);
    (void)gqo_random_word_bits(1u, 2u, 3u, 16);
    (void)gqo_random_word_of(~(uint64_t)0, 63u, 2u, ~(uint64_t)0);

    /* single codes at the edges: every random word extreme, top of the range, beyond it, unusable norms */
    const uint32_t words[] = { 0u, 1u, 0x1FFu, 0x200u, 0x7FFFFFFFu, 0x80000000u, 0xFFFFFE00u, 0xFFFFFFFFu };
    const float xsv[] = { 0.0f, -0.0f, 1e-45f, -1e-38f, 1e-3f, -0.999999f, 1.0f, -1.0f, 1.0000001f, 3e38f, INFINITY, -INFINITY, NAN };
    const float norms[] = { 1.0f, 1e-45f, 1e-38f, 3e38f, 0.0f, -0.0f, -1.0f, INFINITY, NAN, 1e-3f };
    for (size_t a = 0; a < sizeof(words) / 4; a++)
        for (size_t b = 0; b < sizeof(xsv) / 4; b++)
            for (size_t c = 0; c < sizeof(norms) / 4; c++) {
                const int ls[] = { 1, 2, 7, 15, 127, 255, 32767 };
                for (size_t t = 0; t < sizeof(ls) / sizeof(int); t++) {
                    int32_t k = gqo_linear_code(xsv[b], norms[c], ls[t], words[a]);
                    CHECK(k >= -ls[t] && k <= ls[t]);
                    CHECK(gqo_code(0, xsv[b], norms[c], ls[t], words[a]) == k);
                }
                const int es[] = { 1, 2, 7, 16, 31 };
                for (size_t t = 0; t < sizeof(es) / sizeof(int); t++) {
                    int32_t k = gqo_exp_code(xsv[b], norms[c], es[t], words[a]);
                    CHECK(k >= -es[t] && k <= es[t]);
                    CHECK(gqo_code(1, xsv[b], norms[c], es[t], words[a]) == k);
                    CHECK(llabs((long long)gqo_code_value(1, k)) <= ((long long)1 << (es[t] - 1)));
                }
            }
    CHECK(gqo_code_value(1, 31) == ((int64_t)1 << 30) && gqo_code_value(1, -31) == -((int64_t)1 << 30));
    CHECK(gqo_code_value(0, -32767) == -32767 && gqo_code_value(1, 0) == 0);

    /* the sparsity bound at the ends of its ranges */
    CHECK(gqo_sparse_nnz_bound(0, 32767, 64, ((int64_t)1 << 40)) > 0.0 && gqo_sparse_nnz_bound(1, 31, 64, ((int64_t)1 << 40)) > 0.0);
    CHECK(gqo_sparse_nnz_bound(0, 1, 1, 0) == 0.0 && gqo_sparse_nnz_bound(1, 32, 1, 1) == -1.0 && gqo_sparse_nnz_bound(0, 0, 1, 1) == -1.0);
    CHECK(gqo_sparse_nnz_bound(0, 4, 4, 1024) == 272.0 && gqo_sparse_nnz_bound(0, 1, 1, -1) == -1.0);

    /* headroom rule at the ends */
    CHECK(gqo_max_aggregate(0, 32767, 64) == 64 * 32767 && gqo_max_aggregate(1, 31, 64) == (int64_t)64 << 30);
    CHECK(gqo_max_aggregate(1, 60, 64) > 0);
    CHECK(gqo_check_width(0, 127, 16, 32) == 1 && gqo_check_width(1, 15, 32, 16) == 0 && gqo_check_width(1, 31, 64, 64) == 1);
    CHECK(gqo_check_width(0, 1, 1, 2) == 1 && gqo_check_width(0, 2, 1, 2) == 0);
    { int64_t edge[4] = { 32767, -32768, 32768, -32769 };
      CHECK(gqo_fits_width(edge, 2, 16) == 1 && gqo_fits_width(edge, 3, 16) == 0 && gqo_fits_width(edge + 3, 1, 16) == 0);
      CHECK(gqo_fits_width(edge, 0, 16) == 1); }

    /* codes that do not fit a format are refused, not written */
    { int32_t big[3] = { 1, -128, 3 }; uint8_t lv[3]; uint32_t sp[1];
      CHECK(gqo_pack(big, 3, 0, lv, sp) == -1 && gqo_pack(big, 3, 1, lv, sp) == -1 && gqo_pack(big, 3, 3, lv, sp) == -1);
      CHECK(gqo_pack(big, 3, 2, lv, sp) == 0 && sp[0] == 2u); }

    /* Algorithm 2: every k, every pair of small exponents and signs, zero operands */
    for (int s = 1; s <= 31; s++) {
        uint32_t top = (s == 31 ? 0x7FFFFFFFu : ((1u << s) - 1u));
        CHECK(gqo_alg2_k(0u, s) == s + 1 && gqo_alg2_k(top, s) == 1 && gqo_alg2_k(1u, s) == s);
        CHECK(gqo_alg2_field_bits(s) == (s <= 8 ? 8 : s <= 16 ? 16 : 32));
        for (uint32_t node = 1; node < 64; node += 7) {
            uint32_t r = gqo_alg2_draw(~(uint64_t)0, node, ~(uint64_t)0 - node, s);
            CHECK(r <= top);
            int k = gqo_alg2_k(r, s);
            CHECK(k >= 1 && k <= s + 1);
        }
    }
    for (int k = 1; k <= 33; k++)
        for (int e1 = 0; e1 <= 40; e1++)
            for (int e2 = 0; e2 <= 40; e2++)
                for (int sg = 0; sg < 4; sg++) {
                    int sr = 0, er = -1;
                    gqo_exp_reduce_pair((sg & 1) ? -1 : 1, e1, (sg & 2) ? -1 : 1, e2, k, &sr, &er);
                    CHECK((sr == 1 || sr == -1) && er >= 0 && er <= 41);
                }
    /* in-step averaging at the ends of int32-safe inputs */
    CHECK(gqo_avg_pair(127, 127, 1) == 127 && gqo_avg_pair(-128, -127, 0) == -128 && gqo_avg_pair(-128, -127, 1) == -127);
    CHECK(gqo_avg_pair(-1, 0, 0) == -1 && gqo_avg_pair(-1, 0, 1) == 0 && gqo_avg_pair(32767, -32767, 1) == 0);

    /* whole-path cases: ragged sizes, K = 1 .. 64, s at each format's limit, bases past 2^34, both draw widths */
    struct { int scheme, s, pack; } fmts[] = { {0, 127, 0}, {0, 7, 1}, {0, 255, 2}, {0, 15, 3}, {0, 1, 1},
                                               {1, 31, 2}, {1, 7, 1}, {1, 15, 3}, {1, 16, 0}, {1, 1, 0} };
    const int Ks[] = { 1, 2, 3, 5, 64 };
    int cases = 0;
    for (size_t f = 0; f < sizeof(fmts) / sizeof(fmts[0]); f++)
        for (size_t k = 0; k < sizeof(Ks) / sizeof(int); k++)
            for (int si = 0; si < NSIZES; si++) {
                int64_t d = SIZES[si];
                if (Ks[k] == 64 && d > 65) continue;                    /* keep the run short */
                uint64_t base = BASES[(f + k + (size_t)si) % NBASES];
                one_case(Ks[k], d, fmts[f].scheme, fmts[f].s, fmts[f].pack, base, ((f + (size_t)si) & 1) ? 16 : 32);
                cases++;
            }
    printf("oracle driver: %d whole-path cases, %d failed checks\n", cases, failures);
    return failures ? 1 : 0;
}
