// Host-side helpers shared by the entry points: argument checks and launch bookkeeping.
// Internal to the library; the public surface is include/gqsgd.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gqsgd.h"

namespace gq {

static inline bool aligned(const void *p, size_t a) { return p != nullptr && ((uintptr_t)p % a) == 0; }

static inline gq_status check_params(const gq_params *p, bool uses_pack, bool uses_agg)
{
    if (!p) return GQ_ERR_INVALID_ARG;
    if (p->scheme != GQ_LINEAR && p->scheme != GQ_EXP) return GQ_ERR_INVALID_ARG;
    if (p->s < 1) return GQ_ERR_INVALID_ARG;
    if (p->scheme == GQ_LINEAR && p->s > 32767) return GQ_ERR_UNSUPPORTED;
    if (p->scheme == GQ_EXP && p->s > 31) return GQ_ERR_UNSUPPORTED;
    if (uses_pack) {
        if (p->pack < GQ_PACK_I8 || p->pack > GQ_PACK_U4_SIGNPLANE) return GQ_ERR_INVALID_ARG;
        const int lim = p->pack == GQ_PACK_I8 ? 127 : p->pack == GQ_PACK_I4 ? 7 : p->pack == GQ_PACK_U8_SIGNPLANE ? 255 : 15;
        if (p->s > lim) return GQ_ERR_UNSUPPORTED;
    }
    if (uses_agg && p->agg != GQ_AGG_I32 && p->agg != GQ_AGG_I16) return GQ_ERR_INVALID_ARG;
    if (p->rng_bits != 0 && p->rng_bits != 16 && p->rng_bits != 32) return GQ_ERR_INVALID_ARG;
    const int32_t window_bits = GQ_FLAG_WRITE_WINDOWS_OFF | GQ_FLAG_WRITE_WINDOWS_ON;
    if ((p->flags & ~window_bits) != 0 || (p->flags & window_bits) == window_bits) return GQ_ERR_INVALID_ARG;
    return GQ_OK;
}

// 16 random bits per coordinate instead of 32 (one Philox call per eight coordinates)
static inline bool short_draws(const gq_params *p) { return p->rng_bits == 16; }

static inline int64_t max_aggregate(const gq_params *p, int K)
{
    return p->scheme == GQ_LINEAR ? (int64_t)K * p->s : (int64_t)K * ((int64_t)1 << (p->s - 1));
}

static inline float dequant_divisor(const gq_params *p, int K)
{
    // n * (1/unit): K*s or K*2^(s-1); both are exact in binary32 for the supported ranges
    return p->scheme == GQ_LINEAR ? (float)((int64_t)K * p->s) : (float)K * (float)((int64_t)1 << (p->s - 1));
}

static inline gq_status launched()
{
    return hipGetLastError() == hipSuccess ? GQ_OK : GQ_ERR_DEVICE;
}

// A launch may hold at most 2^32 - 1 threads in x (HIP's limit on gridDim.x * blockDim.x).
static inline bool grid_fits(int64_t blocks, int threads) { return blocks >= 0 && blocks * (int64_t)threads <= 0xFFFFFFFFLL; }

}  // namespace gq
