// Per-bucket schedule of Algorithm 1 on MI355X (gfx950): for every bucket of a long gradient its own norm
// step and its own fused quantize+aggregate, optionally with the norm step of the next bucket on a second
// stream beside the fused call of the current one.  Contract: include/gqsgd.h.
//
// The paper calls its hook once per gradient bucket (Implementation section), remarks that the norm exchange
// of one round can be hidden behind the preceding round (Algorithm 1, the remark on its norm step) and
// names the missing pipelining as a limitation (Evaluation section, "Limitations").  This file is that
// pipeline for one GPU: host code only, the kernels are those of gq_global_norm and gq_fused_quantize_aggregate.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>

#include "gqsgd.h"
#include "gq_host.hpp"

using namespace gq;

namespace {

constexpr int64_t kMaxBuckets = 1 << 16;

// Events of one two-stream call; destroyed when the call returns (the runtime keeps what enqueued work still needs).
struct Events {
    std::vector<hipEvent_t> ev;
    ~Events() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); }
    hipEvent_t make()
    {
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        ev.push_back(e);
        return e;
    }
};

}  // namespace

extern "C" {

size_t gq_bucketed_workspace_bytes(int K, int64_t d, int64_t bucket)
{
    if (d < 0 || bucket < 8 || (bucket & 7) != 0) return 0;
    // the norm's need is not monotone in the length, so both lengths that occur are asked for
    const int64_t nb = (d + bucket - 1) / bucket;
    const int64_t last = nb > 0 ? d - (nb - 1) * bucket : 0;
    const size_t whole = gq_norm_workspace_bytes(K, d < bucket ? d : bucket), rest = gq_norm_workspace_bytes(K, last);
    return whole > rest ? whole : rest;
}

gq_status gq_bucketed_quantize_aggregate(const float *const *x, int K, int64_t d, int64_t bucket, gq_norm_kind kind,
                                         const gq_params *p, float *norms_out, uint32_t *status_flags, void *agg_out,
                                         float *dequant_out, void *workspace, size_t workspace_bytes, void *hip_stream,
                                         void *side_stream)
{
    gq_status st = check_params(p, false, agg_out != nullptr);
    if (st != GQ_OK) return st;
    if (!x || K < 1 || K > GQ_MAX_WORKERS || d < 0) return GQ_ERR_INVALID_ARG;
    if (bucket < 8 || (bucket & 7) != 0) return GQ_ERR_INVALID_ARG;     // slices stay 16-byte aligned in every format
    const int64_t nb = (d + bucket - 1) / bucket;
    if (nb > kMaxBuckets) return GQ_ERR_INVALID_ARG;
    if (!agg_out && !dequant_out) return GQ_ERR_INVALID_ARG;
    if (nb > 0 && (!aligned(norms_out, 4) || (status_flags && !aligned(status_flags, 4)))) return GQ_ERR_INVALID_ARG;
    for (int i = 0; i < K; i++)
        if (d > 0 && !aligned(x[i], 16)) return GQ_ERR_INVALID_ARG;
    if (d > 0 && ((agg_out && !aligned(agg_out, 16)) || (dequant_out && !aligned(dequant_out, 16)))) return GQ_ERR_INVALID_ARG;
    const int64_t lim = (agg_out && p->agg == GQ_AGG_I16) ? 32767LL : 2147483647LL;
    if (max_aggregate(p, K) > lim) return GQ_ERR_OVERFLOW;
    if (!workspace || workspace_bytes < gq_bucketed_workspace_bytes(K, d, bucket)) return GQ_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GQ_ERR_INVALID_ARG;
    if (side_stream && side_stream == hip_stream) return GQ_ERR_INVALID_ARG;
    if (nb == 0) return GQ_OK;

    hipStream_t main_st = (hipStream_t)hip_stream;
    hipStream_t side_st = (hipStream_t)side_stream;
    const bool two = side_stream != nullptr && nb > 1;
    const size_t agg_width = p->agg == GQ_AGG_I16 ? 2 : 4;
    const float *xb[GQ_MAX_WORKERS];

    Events events;
    std::vector<hipEvent_t> norm_done, fused_done;
    if (two) {
        // fork: the side stream starts behind everything already enqueued on the main stream
        hipEvent_t fork = events.make();
        if (!fork) return GQ_ERR_DEVICE;
        if (hipEventRecord(fork, main_st) != hipSuccess || hipStreamWaitEvent(side_st, fork, 0) != hipSuccess) return GQ_ERR_DEVICE;
        for (int64_t b = 0; b < nb; b++) {
            norm_done.push_back(events.make());
            fused_done.push_back(events.make());
            if (!norm_done.back() || !fused_done.back()) {
                // join before giving up: nothing but the fork wait has been enqueued on the side stream
                hipEvent_t join = events.make();
                if (join && hipEventRecord(join, side_st) == hipSuccess) (void)hipStreamWaitEvent(main_st, join, 0);
                return GQ_ERR_DEVICE;
            }
        }
    }
    gq_status result = GQ_OK;
    for (int64_t b = 0; b < nb && result == GQ_OK; b++) {
        const int64_t lo = b * bucket;
        const int64_t len = d - lo < bucket ? d - lo : bucket;
        for (int i = 0; i < K; i++) xb[i] = x[i] + lo;
        hipStream_t norm_st = two ? side_st : main_st;
        // the norm of bucket b may start once the fused call of bucket b - 2 has finished: it then runs
        // beside the fused call of bucket b - 1, and the side stream never runs further ahead than that
        if (two && b >= 2 && hipStreamWaitEvent(side_st, fused_done[b - 2], 0) != hipSuccess) { result = GQ_ERR_DEVICE; break; }
        result = gq_global_norm(xb, K, len, kind, norms_out + b, status_flags ? status_flags + b : nullptr, workspace,
                                workspace_bytes, norm_st);
        if (result != GQ_OK) break;
        if (two) {
            if (hipEventRecord(norm_done[b], side_st) != hipSuccess || hipStreamWaitEvent(main_st, norm_done[b], 0) != hipSuccess) {
                result = GQ_ERR_DEVICE;
                break;
            }
        }
        result = gq_fused_quantize_aggregate(xb, K, len, norms_out + b, p, lo,
                                             agg_out ? (void *)((char *)agg_out + (size_t)lo * agg_width) : nullptr,
                                             dequant_out ? dequant_out + lo : nullptr, nullptr, nullptr, main_st);
        if (result != GQ_OK) break;
        if (two && hipEventRecord(fused_done[b], main_st) != hipSuccess) { result = GQ_ERR_DEVICE; break; }
    }
    if (two) {
        // join: whatever the side stream still holds is ordered before the main stream's next work
        hipEvent_t join = events.make();
        if (!join || hipEventRecord(join, side_st) != hipSuccess || hipStreamWaitEvent(main_st, join, 0) != hipSuccess) {
            if (result == GQ_OK) result = GQ_ERR_DEVICE;
        }
    }
    return result;
}

}  // extern "C"
