"""GPU parity at the full sizes of workloads c2, c4 and c5, in the launch shapes the library uses
for them.  The oracle cannot evaluate 10^10 coordinates, but the random stream is a function of
the coordinate index, so it evaluates windows exactly; what cannot be windowed (norms over the
whole input) is checked against torch's own reductions in binary64, and structural identities
(fused == separate calls, bucketed == whole) are checked over every coordinate on the device."""
import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import gq_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2305_18627_amd as gq
    DEV = torch.device("cuda:0")
else:
    gq = None
    DEV = None

RTOL = 1e-5


def host(t):
    return t.detach().cpu().numpy()


def spans(d, seed, edges=()):
    """The index ranges on which the oracle is evaluated at full size: the first and the last 2^20
    coordinates, 64 random windows of 2^16, and 4096 coordinates either side of every edge given
    (bucket or block boundaries).  Starts are multiples of 8 so that any draw mode can be replayed."""
    rng = np.random.default_rng(seed)
    out = [(0, min(d, 1 << 20)), (max(0, d - (1 << 20)) & ~7, d)]
    out += [(int(lo) & ~7, min(d, (int(lo) & ~7) + (1 << 16))) for lo in rng.integers(0, max(1, d - (1 << 16)), 64)]
    out += [(max(0, int(e) - 4096) & ~7, min(d, int(e) + 4096)) for e in edges]
    return sorted(set(out))


def torch_norm(xs, kind):
    if kind == "linf":
        return max(float(x.abs().max()) for x in xs)
    per = [float((x.double() * x.double()).sum()) for x in xs]
    return float(np.sqrt(sum(per))) if kind == "l2" else float(np.sqrt(max(per)))


def test_workload_c2_layer_blocks_exponential_int8():
    # d = 25.6e6, K = 8, 160 layer blocks with std in [1e-5, 1e-2], L2 norm, exponential s = 16, int8 codes, int32 sum
    cfg = SI.CONFIGS["c2"]
    K, d, s = cfg["K"], cfg["d"], cfg["s"]
    xs = SI.make_workers("c2", device=DEV)
    norm_t = torch.zeros(1, device=DEV)
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    gq.global_norm(xs, gq.GQ_NORM_L2, norm_t, flags)
    ne, nf, fl = O.global_norm([host(x) for x in xs], O.NORM_L2)               # the oracle in full
    assert abs(float(norm_t.item()) - ne) <= RTOL * ne and flags.item() == fl == 0
    norm_t.fill_(float(nf))                                                      # both sides use the oracle's norm
    p = gq.make_params(gq.GQ_EXP, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    assert gq.check_width(p, K) == gq.GQ_OK and O.check_width(O.EXP, s, K, 32)
    lvs = [torch.empty(d, dtype=torch.uint8, device=DEV) for _ in range(K)]
    for i in range(K):
        gq.quantize(xs[i], norm_t, p, i, 0, lvs[i])
    agg = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, agg)
    deq = torch.empty(d, device=DEV)
    gq.dequantize(agg, d, norm_t, p, K, deq)
    fagg = torch.empty(d, dtype=torch.int32, device=DEV)
    fdeq = torch.empty(d, device=DEV)
    flv = [torch.empty(d, dtype=torch.uint8, device=DEV) for _ in range(K)]
    gq.fused_quantize_aggregate(xs, norm_t, p, 0, fagg, fdeq, flv, None)
    torch.cuda.synchronize()
    assert torch.equal(agg, fagg) and torch.equal(deq, fdeq)
    assert all(torch.equal(a, b) for a, b in zip(lvs, flv))
    per_block = d // cfg["blocks"]
    for lo, hi in spans(d, 2, edges=[per_block * b for b in (1, 57, 159)]):
        xh = [host(x[lo:hi]) for x in xs]
        want = O.quantize_aggregate(xh, nf, O.EXP, s, SI.QUANT_SEED, lo)
        assert np.array_equal(host(agg[lo:hi]).astype(np.int64), want), lo
        wd = O.dequantize(want, float(nf), O.EXP, s, K)
        gd = host(deq[lo:hi]).astype(np.float64)
        assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)) and np.all(gd[want == 0] == 0.0)
        for i in (0, K - 1):
            q = O.quantize(xh[i], nf, O.EXP, s, SI.QUANT_SEED, i, lo)
            assert np.array_equal(host(lvs[i][lo:hi]).view(np.int8), q.astype(np.int8))
    assert int(agg.abs().max()) <= O.max_aggregate(O.EXP, s, K)


def test_workload_c4_student_t_exponential_int4_int16():
    # d = 350e6, K = 32, 1e-4 * t(3), max norm, exponential s = 7, packed int4 codes, int16 sum
    cfg = SI.CONFIGS["c4"]
    K, d, s = cfg["K"], cfg["d"], cfg["s"]
    xs = SI.make_workers("c4", device=DEV)
    norm_t = torch.zeros(1, device=DEV)
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    gq.global_norm(xs, gq.GQ_NORM_LINF, norm_t, flags)
    torch.cuda.synchronize()
    nf = np.float32(torch_norm(xs, "linf"))
    assert np.float32(norm_t.item()) == nf and flags.item() == 0                 # the max norm is exact
    p = gq.make_params(gq.GQ_EXP, s, gq.GQ_PACK_I4, gq.GQ_AGG_I16, seed=SI.QUANT_SEED)
    # Section 4.2 headroom at 16 bits: 32 * 2^6 = 2048 holds, s = 15 (32 * 2^14) must be refused
    assert gq.check_width(p, K) == gq.GQ_OK
    p15 = gq.make_params(gq.GQ_EXP, 15, gq.GQ_PACK_U4_SIGNPLANE, gq.GQ_AGG_I16, seed=SI.QUANT_SEED)
    assert gq.check_width(p15, K) == gq.GQ_ERR_OVERFLOW and not O.check_width(O.EXP, 15, K, 16)
    agg = torch.empty(d, dtype=torch.int16, device=DEV)
    with pytest.raises(gq.GQError) as e:
        gq.fused_quantize_aggregate(xs, norm_t, p15, 0, agg)
    assert e.value.status == gq.GQ_ERR_OVERFLOW
    nb = gq.levels_nbytes(d, gq.GQ_PACK_I4)
    lvs = [torch.empty(nb, dtype=torch.uint8, device=DEV) for _ in range(K)]
    for i in range(K):
        gq.quantize(xs[i], norm_t, p, i, 0, lvs[i])
    gq.int_aggregate(lvs, None, d, p, agg)
    fagg = torch.empty(d, dtype=torch.int16, device=DEV)
    gq.fused_quantize_aggregate(xs, norm_t, p, 0, fagg)
    torch.cuda.synchronize()
    assert torch.equal(agg, fagg)
    for lo, hi in spans(d, 4):
        xh = [host(x[lo:hi]) for x in xs]
        want = O.quantize_aggregate(xh, nf, O.EXP, s, SI.QUANT_SEED, lo)
        assert O.fits_width(want, 16)
        assert np.array_equal(host(agg[lo:hi]).astype(np.int64), want), lo
        for i in (0, 13, K - 1):
            wl, _ = O.pack(O.quantize(xh[i], nf, O.EXP, s, SI.QUANT_SEED, i, lo), O.PACK_I4)
            assert np.array_equal(host(lvs[i][lo // 2:hi // 2]), wl)
    assert int(agg.abs().max()) <= 2048


def test_workload_c5_bucketed_fused_quantize_aggregate_dequantize():
    # d = 1.5e9, K = 8, Gaussian mixture, L2 norm over the WHOLE input, then per 2^26-coordinate bucket
    # (22 full + 1 partial) linear s = 15 fused quantize+aggregate+dequantize -> fp32
    cfg = SI.CONFIGS["c5"]
    K, d, s, bucket = cfg["K"], cfg["d"], cfg["s"], cfg["bucket"]
    xs = SI.make_workers("c5", device=DEV)
    norm_t = torch.zeros(1, device=DEV)
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    gq.global_norm(xs, gq.GQ_NORM_L2, norm_t, flags)
    torch.cuda.synchronize()
    want_norm = torch_norm(xs, "l2")
    assert abs(float(norm_t.item()) - want_norm) <= RTOL * want_norm and flags.item() == 0
    nf = np.float32(want_norm)          # torch's binary64 norm rounded once: the norm both sides are given
    norm_t.fill_(float(nf))
    p = gq.make_params(gq.GQ_LINEAR, s, gq.GQ_PACK_U4_SIGNPLANE, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    out = torch.empty(d, device=DEV)
    nb = SI.num_buckets(d, bucket)
    assert nb == 23 and d - 22 * bucket == 23_604_992
    for b in range(nb):
        lo, hi = b * bucket, min(d, (b + 1) * bucket)
        gq.fused_quantize_aggregate([x[lo:hi] for x in xs], norm_t, p, lo, None, out[lo:hi])
    whole = torch.empty(d, device=DEV)
    gq.fused_quantize_aggregate(xs, norm_t, p, 0, None, whole)
    torch.cuda.synchronize()
    assert torch.equal(out, whole)                                               # bucketed == unbucketed
    del whole
    for lo, hi in spans(d, 5, edges=[b * bucket for b in range(1, nb)]):
        xh = [host(x[lo:hi]) for x in xs]
        A = O.quantize_aggregate(xh, nf, O.LINEAR, s, SI.QUANT_SEED, lo)
        wd = O.dequantize(A, float(nf), O.LINEAR, s, K)
        gd = host(out[lo:hi]).astype(np.float64)
        assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)), lo
        assert np.all(gd[A == 0] == 0.0)
    # the sparse regime of the L2 norm: almost every level is 0 or +-1, and the mean is unbiased:
    # sum_j out_j against sum_j xbar_j within 6 standard deviations of the rounding noise
    tot = float(out.double().sum())
    expect = sum(float(x.double().sum()) for x in xs) / K
    sd = float(nf) / (K * s) * np.sqrt(K * d * 0.25)
    assert abs(tot - expect) <= 6.0 * sd


def test_one_launch_across_two_to_the_34_coordinates():
    # a single worker of 2^34 + 2^20 + 5 coordinates (69 GB): the Philox call index crosses 2^32 INSIDE the call, which
    # the library handles by cutting the launch there; element indices pass 2^32 and byte offsets 2^36
    torch.cuda.empty_cache()
    d = (1 << 34) + (1 << 20) + 5
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * d + 2 * d + (8 << 30):
        pytest.skip("needs 110 GB of free device memory")
    x = torch.empty(d, dtype=torch.float32, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(2034)
    step = 1 << 28
    for lo in range(0, d, step):
        x[lo:lo + step].normal_(0.0, 1e-3, generator=g)
    nf = np.float32(4.5e-3)
    x.clamp_(-float(nf), float(nf))
    norm_t = torch.tensor([float(nf)], device=DEV)
    p = gq.make_params(gq.GQ_LINEAR, 127, gq.GQ_PACK_I8, gq.GQ_AGG_I16, seed=SI.QUANT_SEED)
    agg = torch.empty(d, dtype=torch.int16, device=DEV)
    gq.fused_quantize_aggregate([x], norm_t, p, 0, agg)
    torch.cuda.synchronize()
    edge = 1 << 34
    for lo, hi in [(0, 1 << 16), (edge - (1 << 16), edge + (1 << 16)), (d - (1 << 16) - 5, d), (3 * (1 << 32) + 8, 3 * (1 << 32) + 8 + (1 << 15))]:
        want = O.quantize_aggregate([host(x[lo:hi])], nf, O.LINEAR, 127, SI.QUANT_SEED, lo & ~3 if lo % 4 else lo)[0:hi - lo] \
            if lo % 4 == 0 else None
        if want is None:
            lo4 = lo & ~3
            want = O.quantize_aggregate([host(x[lo4:hi])], nf, O.LINEAR, 127, SI.QUANT_SEED, lo4)[lo - lo4:]
        assert np.array_equal(host(agg[lo:hi]).astype(np.int64), want), lo
    # the tail of the same gradient as a bucket with its offset
    lo = edge - (1 << 20)
    part = torch.empty(d - lo, dtype=torch.int16, device=DEV)
    gq.fused_quantize_aggregate([x[lo:]], norm_t, p, lo, part)
    torch.cuda.synchronize()
    assert torch.equal(part, agg[lo:])
    del x, agg, part
    torch.cuda.empty_cache()
