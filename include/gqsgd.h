/*
 * gqsgd.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of Global-QSGD
 * (arXiv 2305.18627): global norm -> stochastic rounding to integer levels -> integer sum over
 * workers -> dequantisation, plus the fused quantize+aggregate call.
 *
 * One GPU, one process.  The n = K workers of the paper's Algorithm 1 are K gradient buffers
 * resident on the same device.
 *
 * Conventions that hold for every call
 *   pointers   Every data pointer is a DEVICE pointer unless its comment says "host".  Arrays of
 *              per-worker pointers (x, levels, ...) are HOST arrays of K DEVICE pointers; they are
 *              read during the call only.  The caller owns every buffer; the library allocates
 *              nothing and keeps no pointer after a call returns.
 *   alignment  Gradient, level, aggregate and output buffers must be 16-byte aligned, sign planes
 *              and the norm 4-byte aligned, the norm workspace 8-byte aligned.
 *   stream     `hip_stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue work
 *              and never synchronise; the norm stays on the device so that the norm pass and the
 *              quantisation pass need no host round trip.
 *   errors     Argument errors are returned synchronously and nothing is enqueued.  A launch
 *              failure is returned as GQ_ERR_DEVICE.  Conditions that depend on the data are
 *              reported through the device word `status_flags` of gq_global_norm.
 *   sizes      1 <= K <= GQ_MAX_WORKERS, d >= 0 (d = 0 is a valid no-op), any d (ragged tails are
 *              handled inside), index_base >= 0 and a multiple of 4 (of 8 with rng_bits = 16).
 *              gq_fused_quantize_aggregate with rng_bits = 32 and no stored codes takes any d.  Every
 *              other call accepts any d up to 2^34 - 1024 coordinates (the sparse branch: 2^32 - 1) and
 *              answers GQ_ERR_INVALID_ARG beyond what one launch can cover: cut longer gradients into
 *              buckets and pass their offsets as index_base.
 *
 * The stored integer ("code").  The paper numbers levels downwards, l_0 = 1 > ... > l_s = 0
 * (Definition 1).  The integer stored and summed is k = s - u for level l_u, signed with sign(x):
 *   linear grid       k in 0..s stands for k/s                   adds  k         to the sum
 *   exponential grid  k = 0 stands for 0, k in 1..s for 2^(k-s)  adds  2^(k-1)   to the sum
 * (Section 4.2; the exponential grid is read as {0} u {2^-j, j = 0..s-1}).
 *
 * Random rounding.  Eq. (2) fixes probabilities only.  Every (worker, coordinate) draws 32 bits r
 * from Philox4x32-10 (Salmon et al., SC'11): counter (lo32(g/4), hi32(g/4), worker, 0), key
 * (lo32(seed), hi32(seed)), word g mod 4, where g = index_base + j is the global coordinate index.
 *   linear       U' = fl32(fl32(r) * (2^-32 - 2^-56));  v = fma(|x|, fl32(s/norm), -U');  k = min(ceil(v), s)
 *   exponential  z = min(fl32(|x| * fl32(2^(s-1)/norm)), 2^(s-1));  R = r >> 9;
 *                z >= 1: round the binary32 z up to the next power of two iff mantissa + R >= 2^23;
 *                z <  1: k = 1 iff rne(z * 2^23) + R >= 2^23, else 0
 *   both grids   |x| >= norm (y = 1, e.g. the coordinate a max norm is taken from) is the top level k = s with certainty
 * Short draws (rng_bits = 16): one Philox call serves the eight coordinates 8c .. 8c+7, counter
 * (lo32(g/8), hi32(g/8), worker, 0); coordinate g takes the low (g even) or high (g odd) half of word
 * (g mod 8) / 2 as the TOP half of r, zeros below, and the two rules apply unchanged: the probability
 * of Eq. (2) is then met to 2^-16 and the generator costs half as much per coordinate.  index_base
 * must then be a multiple of 8.  Only gq_quantize, gq_quantize_compact and gq_fused_quantize_aggregate (and the
 * per-bucket schedule built on it) draw from this stream; the other calls ignore rng_bits.
 * A norm that is zero, negative or not finite (or so small that the scale overflows) gives all-zero codes, also at
 * NaN or Inf coordinates.  Under a usable norm a NaN coordinate gives code 0 and |x| > norm the top level.
 */
#ifndef GQSGD_H
#define GQSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GQ_MAX_WORKERS 64

typedef enum {
    GQ_OK = 0,
    GQ_ERR_INVALID_ARG = 1,  /* NULL / misaligned pointer, K or d or index_base out of range, bad enum */
    GQ_ERR_UNSUPPORTED = 2,  /* s does not fit the pack format, or a combination that is not built   */
    GQ_ERR_OVERFLOW = 3,     /* the integer sum of K codes can exceed the aggregate width            */
    GQ_ERR_WORKSPACE = 4,    /* workspace NULL or smaller than gq_norm_workspace_bytes               */
    GQ_ERR_DEVICE = 5        /* the HIP runtime reported an error at launch                          */
} gq_status;

/* Mixed norms ||[x_1..x_n]||_{q,p} of Section 4.1 that Algorithm 1's norm step may use. */
typedef enum {
    GQ_NORM_LINF = 0,   /* (inf,inf): max |x_ij| over all workers and coordinates (the paper's default) */
    GQ_NORM_L2 = 1,     /* (2,2):     L2 norm of the concatenation                                      */
    GQ_NORM_L2_MAX = 2  /* (2,inf):   max over workers of ||x_i||_2 (the norm step read literally)             */
} gq_norm_kind;

typedef enum { GQ_LINEAR = 0, GQ_EXP = 1 } gq_scheme;           /* level grid, Section 4.2 */

/* Storage of the signed codes of one worker (Section 4.2: 8-bit levels; Implementation section: two 4-bit values packed into a byte).
 *   I8            byte j = q_j, two's complement                                       needs s <= 127
 *   I4            byte b = (q_2b & 15) | (q_2b+1 & 15) << 4, two's complement nibbles   needs s <= 7
 *                 (an odd d leaves the last high nibble 0)
 *   U8_SIGNPLANE  byte j = |q_j|; sign word w, bit t = 1 iff q_(32w+t) < 0              needs s <= 255
 *   U4_SIGNPLANE  nibbles as I4 holding |q|; same sign words                            needs s <= 15
 * Level buffers hold d (8-bit) or ceil(d/2) (4-bit) bytes, sign planes ceil(d/32) uint32 words;
 * pad bits are written as 0. */
typedef enum { GQ_PACK_I8 = 0, GQ_PACK_I4 = 1, GQ_PACK_U8_SIGNPLANE = 2, GQ_PACK_U4_SIGNPLANE = 3 } gq_pack;

typedef enum { GQ_AGG_I32 = 0, GQ_AGG_I16 = 1 } gq_agg;         /* width of the integer sum */

typedef struct {
    int32_t scheme;   /* gq_scheme                                                        */
    int32_t s;        /* number of non-zero levels, s >= 1 (exponential: s <= 31)          */
    int32_t pack;     /* gq_pack: format of level buffers (ignored where none is touched) */
    int32_t agg;      /* gq_agg: format of the integer sum (ignored where none is touched) */
    int32_t rng_bits; /* random bits per coordinate of the quantisation draw: 32 (0 reads as 32) or 16 */
    int32_t flags;    /* 0, or one of the GQ_FLAG_* bits below; any other bit: GQ_ERR_INVALID_ARG   */
    uint64_t seed;    /* Philox key                                                       */
} gq_params;

/* gq_params.flags.  The fused call stores its sums either as each wave finishes or, in large launches, only
 * inside short chip-wide time windows (all waves watch the same 100 MHz counter), which separates the
 * write bursts from the read stream in HBM.  The windows change timing only, never a result.  By default the
 * library uses them where they were measured to pay (K >= 8 and K * d >= 2.5e8, no codes stored).  The two
 * bits override that policy: OFF never waits, ON waits in every launch that stores no codes.  Both
 * bits at once: GQ_ERR_INVALID_ARG.  Every call other than gq_fused_quantize_aggregate (and the bucketed
 * schedule built on it) ignores them. */
#define GQ_FLAG_WRITE_WINDOWS_OFF 1
#define GQ_FLAG_WRITE_WINDOWS_ON 2

/* Library version (major * 1000 + minor). */
int gq_version(void);

/* Static, human-readable name of a status code. */
const char *gq_status_string(gq_status st);

/* Section 4.2, integer headroom: GQ_OK if a signed integer of p->agg's width always holds the sum
 * of K codes, i.e. K*s (linear) or K*2^(s-1) (exponential) <= 2^(A-1)-1; GQ_ERR_OVERFLOW if not;
 * GQ_ERR_INVALID_ARG for bad parameters.  Host only, touches no device. */
gq_status gq_check_width(const gq_params *p /* host */, int K);

/* Theorem 1's sparsity statement, in the form that follows from Eq. (2): an upper bound on the EXPECTED number of
 * non-zero codes over all K workers of d coordinates when the norm is the (2,2) norm (GQ_NORM_L2),
 *     unit^2 + unit * sqrt(K d),   unit = s (linear) or 2^(s-1) (exponential), never more than K d
 * (at most unit^2 coordinates reach the smallest non-zero level 1/unit; every other one is non-zero with probability
 * unit * y; the y of all coordinates sum to at most sqrt(K d)).  What a caller sizes the lists of the sparse branch by
 * before the first call; the count returned by gq_compact / gq_quantize_compact says whether a list was large enough.
 * Under the other norms no such bound holds.  Host only; -1 for bad parameters. */
double gq_sparse_nnz_bound(const gq_params *p /* host */, int K, int64_t d);

/* Bytes of device workspace gq_global_norm needs for (K, d); 0 if K or d is out of range. */
size_t gq_norm_workspace_bytes(int K, int64_t d);

/* Algorithm 1's norm step: the global norm of K gradients of d coordinates each.
 *   x             host array of K device pointers to fp32[d]
 *   norm_out      device fp32[1]: the norm, rounded once from a binary64 reduction (LINF is exact)
 *   status_flags  device uint32[1] or NULL: overwritten with bit0 = norm is not finite (a NaN or
 *                 Inf somewhere in x, or overflow), bit1 = norm is zero (every code will be 0)
 *   workspace     device scratch of at least gq_norm_workspace_bytes(K, d) bytes; contents are
 *                 overwritten; must not be shared by calls that may run concurrently
 * The result does not depend on scheduling (no atomics): equal inputs give equal bits. */
gq_status gq_global_norm(const float *const *x /* host */, int K, int64_t d, gq_norm_kind kind,
                         float *norm_out, uint32_t *status_flags,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* gq_global_norm for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same kernels, same
 * bits in norm_out and status_flags.  The block partials go to a 512 KiB array that is part of the
 * library's device image (one copy per GPU, held until the process ends), which covers every (K, d)
 * gq_global_norm accepts; a size whose partials would not fit is answered with GQ_ERR_WORKSPACE.  The
 * call allocates nothing and synchronises nothing.  Its first call on a device looks up the array's
 * address (not an allocation; make that call before a capture begins); GQ_ERR_DEVICE if the runtime
 * cannot give it.  All calls on one GPU share the array: calls that may overlap on one GPU (different
 * streams) race and must be ordered by the caller; nothing needs clearing between calls. */
gq_status gq_global_norm_static(const float *const *x /* host */, int K, int64_t d, gq_norm_kind kind,
                                float *norm_out, uint32_t *status_flags, void *hip_stream);

/* Algorithm 1's quantisation loop for ONE worker: y = |x|/norm, code = sign(x) * xi(y) (Definition 1, Eq. (2)).
 *   x              device fp32[d]
 *   norm           device fp32[1] (as written by gq_global_norm)
 *   worker         the worker word of the random stream (distinct workers round independently)
 *   index_base     global index of x[0]; a gradient cut into buckets gives the same codes as the
 *                  whole when each bucket passes its offset
 *   levels_out     device buffer in p->pack format
 *   signplane_out  device uint32[ceil(d/32)] for the *_SIGNPLANE formats, else NULL */
gq_status gq_quantize(const float *x, int64_t d, const float *norm, const gq_params *p /* host */,
                      uint32_t worker, int64_t index_base,
                      void *levels_out, uint32_t *signplane_out, void *hip_stream);

/* Algorithm 1's aggregation step on one device: A_j = sum over the K workers of the integer value of the code.
 *   levels      host array of K device pointers to level buffers in p->pack format
 *   signplanes  host array of K device pointers (the *_SIGNPLANE formats), else NULL
 *   agg_out     device int32[d] or int16[d] according to p->agg
 * Returns GQ_ERR_OVERFLOW (and enqueues nothing) if gq_check_width(p, K) fails. */
gq_status gq_int_aggregate(const void *const *levels /* host */, const uint32_t *const *signplanes /* host */,
                           int K, int64_t d, const gq_params *p /* host */, void *agg_out, void *hip_stream);

/* Eq. (1): out_j = norm * A_j / (K*s) (linear) or norm * A_j / (K*2^(s-1)) (exponential): the MEAN
 * of the workers' quantised gradients.
 *   agg   device int32[d] or int16[d] according to p->agg
 *   out   device fp32[d]; computed as fl32(fl32(A_j) * fl32(norm / (K*unit))) */
gq_status gq_dequantize(const void *agg, int64_t d, const float *norm, const gq_params *p /* host */,
                        int K, float *out, void *hip_stream);

/* The fused call: gq_quantize for all K workers (worker word = position in x) and the integer sum,
 * in registers, in one pass over the gradients.  Outputs are optional but at least one of agg_out
 * and dequant_out must be given:
 *   agg_out         device int32[d] / int16[d] (p->agg), or NULL
 *   dequant_out     device fp32[d] as gq_dequantize would write it, or NULL
 *   levels_out      host array of K device level buffers (p->pack) to also store the codes, or NULL
 *   signplanes_out  host array of K device sign planes (the *_SIGNPLANE formats with levels_out), else NULL
 * Results equal those of the separate calls bit for bit. */
gq_status gq_fused_quantize_aggregate(const float *const *x /* host */, int K, int64_t d, const float *norm,
                                      const gq_params *p /* host */, int64_t index_base,
                                      void *agg_out, float *dequant_out,
                                      void *const *levels_out /* host */, uint32_t *const *signplanes_out /* host */,
                                      void *hip_stream);

/* The per-bucket schedule: what a communication hook that is called once per gradient bucket runs
 * (Implementation section), with the pipelining the paper leaves open (Algorithm 1's remark that the norm
 * exchange can be hidden behind the preceding round; Evaluation section, "Limitations").  The gradient
 * is cut into buckets of `bucket` coordinates (a multiple of 8; the last one may be shorter); bucket b gets
 * its OWN norm, norms_out[b] = gq_global_norm of the K slices, and is quantised and summed with it by
 * gq_fused_quantize_aggregate with index_base = b * bucket -- the same kernels, so the same bits as those
 * two calls made bucket by bucket.
 *   norms_out      device fp32[ceil(d / bucket)]; status_flags device uint32[ceil(d / bucket)] or NULL
 *   agg_out        device int32[d] / int16[d] (p->agg) or NULL; dequant_out device fp32[d] or NULL (one is needed):
 *                  slice b holds the sum / the mean of bucket b under norm b
 *   workspace      device scratch of at least gq_bucketed_workspace_bytes(K, d, bucket) bytes
 *   hip_stream     carries every fused call (and every norm if side_stream is NULL: the serial schedule)
 *   side_stream    a second hipStream_t of the same priority, or NULL.  If given, the norm of bucket b + 1 runs on
 *                  it beside the fused call of bucket b; the call forks it from hip_stream on entry and joins
 *                  it back before returning (HIP events created and destroyed inside the call), so the caller
 *                  orders nothing itself and work enqueued on hip_stream afterwards sees every result.
 * Results do not depend on the schedule.  On one GPU both kernels draw on the same HBM, so the second
 * stream hides nothing (measured: it is slower); it is there for callers whose norm step has something to
 * hide behind.  Errors as in the two calls; at most 65536 buckets. */
size_t gq_bucketed_workspace_bytes(int K, int64_t d, int64_t bucket);
gq_status gq_bucketed_quantize_aggregate(const float *const *x /* host */, int K, int64_t d, int64_t bucket,
                                         gq_norm_kind kind, const gq_params *p /* host */, float *norms_out,
                                         uint32_t *status_flags, void *agg_out, float *dequant_out,
                                         void *workspace, size_t workspace_bytes, void *hip_stream, void *side_stream);

/* Algorithm 2 (Section 4.3): the paper's own aggregation for the exponential grid, kept beside the
 * exact integer sum of gq_int_aggregate.  The K workers' codes (written by gq_quantize with GQ_EXP and
 * GQ_PACK_I8) are moved to the prescaled representation sign * 2^-e, e = s - k + 1 + log2(n'), n' = K
 * rounded up to a power of two (the paper's division by 2n keeps every partial sum within 1/2), and
 * reduced pairwise in tree order: nodes numbered as a binary heap (root 1, children 2h and 2h+1, worker i
 * is leaf n'+i, missing workers are zeros, operand 1 is child 2h); every node rounds its sum to a
 * neighbouring power of two, upwards iff k > diff as in the listing.  k follows the listing's first statement
 * with m = s + 1 and p = r / 2^s for an s-bit random integer r: k = s - floor(log2 r), and k = m for r = 0, so
 * that P(k > b) = 2^-b for b < m.  The s bits of node h at coordinate g are the top s bits of field h mod (32/W)
 * (counted from the low end) of word g mod 4 of the Philox call with counter (lo32(g/4), hi32(g/4), h / (32/W), 1),
 * W = 8 for s <= 8, 16 for s <= 16, else 32: one call serves the four coordinates of 32/W nodes.
 *   levels       host array of K device int8[d] code buffers
 *   reduced_out  device int8[d]: sign * e of the root (0 for zero), or NULL
 *   dequant_out  device fp32[d]: the mean it stands for, sign * 2^-e * 2n' * norm / K, or NULL
 *   norm         device fp32[1]; read only if dequant_out is given
 * p->pack and p->agg are ignored; p->scheme must be GQ_EXP (else GQ_ERR_UNSUPPORTED).  The result is
 * unbiased for the exact sum wherever no pair of operands is further apart than the cap on k reaches (gap < m
 * for equal signs; beyond it the smaller operand, at most 2^-(s+1) of the larger, is dropped), and adds at most a
 * factor 9/8 of second moment per tree level. */
gq_status gq_exp_reduce(const void *const *levels /* host */, int K, int64_t d, const gq_params *p /* host */,
                        int64_t index_base, const float *norm, void *reduced_out, float *dequant_out,
                        void *hip_stream);

/* Implementation section, low-bit linear dithering: the average is taken inside every reduce step instead of summing
 * until the end, so the codes never leave their b bits (a 4-bit sum over 4 workers would leave one value
 * bit).  Same tree as gq_exp_reduce (n' = K rounded up to a power of two, heap numbering, missing workers
 * are zeros).  A node holds round((a + b) / 2); an odd sum is rounded up iff its coin is set, the coin of
 * node h at coordinate g being bit h mod 32 of the Philox word with counter (lo32(g/4), hi32(g/4), h / 32, 2),
 * word g mod 4: unbiased, and never outside the range of the inputs.
 *   levels       host array of K device code buffers in p->pack format (GQ_PACK_I8 or GQ_PACK_I4,
 *                linear grid; other formats: GQ_ERR_UNSUPPORTED)
 *   reduced_out  device buffer in the same format: the root's code, which stands for the mean over n' leaves, or NULL
 *   dequant_out  device fp32[d]: the mean over the K workers, norm * code * n' / (K * s), or NULL
 *   norm         device fp32[1]; read only if dequant_out is given */
gq_status gq_avg_reduce(const void *const *levels /* host */, int K, int64_t d, const gq_params *p /* host */,
                        int64_t index_base, const float *norm, void *reduced_out, float *dequant_out,
                        void *hip_stream);

/* Algorithm 1's sparse branch: only the non-zero codes are exchanged (Theorem 1 bounds their
 * number under the (2,2) norm).  Sender side: the (coordinate index, signed code) pairs of the non-zero int8
 * codes of ONE worker, in increasing index order.
 *   levels           device int8[d] codes (p->pack must be GQ_PACK_I8; d <= 2^32 - 1, indices are 32-bit)
 *   indices_out      device uint32[capacity]; values_out device int8[capacity]
 *   count_out        device uint64[1]: the TRUE number of non-zero codes; if it exceeds `capacity` only the
 *                    first `capacity` pairs were written and the caller must retry with larger buffers
 *   tile_starts_out  device uint32[gq_tile_starts_len(d)] or NULL: entry t = the number of non-zero codes with index
 *                    below 4096 * t, i.e. where coordinates 4096 t .. 4096 t + 4095 begin in the list; the last
 *                    entry (t = ceil(d / 4096)) is the count.  A small table (4 bytes per 4096 coordinates) that
 *                    travels with the list and spares the receiver every search.
 *   workspace        device scratch of at least gq_compact_workspace_bytes(d) bytes, 8-byte aligned, overwritten (the
 *                    words of a scan over spans of 32768 codes); not to be shared by calls that may overlap
 * The codes are read once and only the list is written.  The result is unique (sorted by index) and does not
 * depend on scheduling.  count_out = 2^64 - 1 reports that the scan over the blocks gave up waiting (it cannot
 * in a working launch: every block waits only for blocks that started before it); the lists are then incomplete. */
size_t gq_compact_workspace_bytes(int64_t d);
int64_t gq_tile_starts_len(int64_t d);          /* ceil(d / 4096) + 1; 0 if d is out of range */
gq_status gq_compact(const void *levels, int64_t d, const gq_params *p /* host */, uint32_t *indices_out,
                     int8_t *values_out, int64_t capacity, uint64_t *count_out, uint32_t *tile_starts_out,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* The sender side in one call (Algorithm 1: the quantisation loop followed by the sparse branch's selection of
 * the non-zero codes): what gq_quantize (int8 codes) followed by gq_compact writes -- the same list, count and tile
 * starts, bit for bit, from the same rounding rule and random stream -- without the dense codes ever reaching
 * memory: 4 d bytes read, 5 bytes per non-zero written.
 *   x, norm, worker, index_base   as for gq_quantize (p->pack must be GQ_PACK_I8; both settings of p->rng_bits)
 *   the other arguments           as for gq_compact; indices count from x[0]; d <= 2^32 - 1 */
gq_status gq_quantize_compact(const float *x, int64_t d, const float *norm, const gq_params *p /* host */,
                              uint32_t worker, int64_t index_base, uint32_t *indices_out, int8_t *values_out,
                              int64_t capacity, uint64_t *count_out, uint32_t *tile_starts_out,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Receiver side of the sparse branch: the dense integer sum A_j of the K workers' lists, equal to what
 * gq_int_aggregate forms from the dense codes.
 *   indices, values  host arrays of K device lists as written by gq_compact (indices strictly increasing)
 *   counts           host array of K device uint64[1] (read on the device; min(count, capacity) entries are used)
 *   capacities       host array of K list capacities
 *   tile_starts      host array of K device tables as written by gq_compact for the same d, or NULL (the array, or
 *                    single entries of it): without a table the receiver locates its tiles by binary search
 *   agg_out          device int32[d] (p->agg must be GQ_AGG_I32), fully overwritten
 * Entries whose index is not below d are ignored.  Returns GQ_ERR_OVERFLOW if gq_check_width(p, K) fails. */
gq_status gq_sparse_aggregate(const uint32_t *const *indices /* host */, const int8_t *const *values /* host */,
                              const uint64_t *const *counts /* host */, const int64_t *capacities /* host */,
                              const uint32_t *const *tile_starts /* host */, int K, int64_t d,
                              const gq_params *p /* host */, void *agg_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GQSGD_H */
