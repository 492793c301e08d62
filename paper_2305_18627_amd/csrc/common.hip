// Entry points that touch no device: version, status names, the integer headroom rule of Section 4.2, the sparsity
// bound of Theorem 1.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <math.h>

#include "gqsgd.h"
#include "gq_device.hpp"
#include "gq_host.hpp"

using namespace gq;

extern "C" {

int gq_version(void) { return 1004; }

const char *gq_status_string(gq_status st)
{
    switch (st) {
    case GQ_OK: return "GQ_OK";
    case GQ_ERR_INVALID_ARG: return "GQ_ERR_INVALID_ARG";
    case GQ_ERR_UNSUPPORTED: return "GQ_ERR_UNSUPPORTED";
    case GQ_ERR_OVERFLOW: return "GQ_ERR_OVERFLOW";
    case GQ_ERR_WORKSPACE: return "GQ_ERR_WORKSPACE";
    case GQ_ERR_DEVICE: return "GQ_ERR_DEVICE";
    }
    return "GQ_ERR_UNKNOWN";
}

gq_status gq_check_width(const gq_params *p, int K)
{
    const gq_status st = check_params(p, false, true);
    if (st != GQ_OK) return st;
    if (K < 1 || K > GQ_MAX_WORKERS) return GQ_ERR_INVALID_ARG;
    const int64_t lim = p->agg == GQ_AGG_I32 ? 2147483647LL : 32767LL;
    return max_aggregate(p, K) <= lim ? GQ_OK : GQ_ERR_OVERFLOW;
}

double gq_sparse_nnz_bound(const gq_params *p, int K, int64_t d)
{
    if (check_params(p, false, false) != GQ_OK || K < 1 || K > GQ_MAX_WORKERS || d < 0) return -1.0;
    // the smallest non-zero level is 1 / unit: at most unit^2 coordinates reach it, the others are non-zero with
    // probability unit * y, and all y together sum to at most sqrt(K d)
    const double unit = p->scheme == GQ_LINEAR ? (double)p->s : (double)((int64_t)1 << (p->s - 1));
    const double coords = (double)K * (double)d;
    const double bound = unit * unit + unit * sqrt(coords);
    return bound < coords ? bound : coords;
}

}  // extern "C"
