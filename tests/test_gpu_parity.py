"""GPU parity: every entry point of the C ABI (through the ctypes binding) against the CPU oracle,
element by element, on the same seeded inputs.

Bars: codes, packed bytes, sign words and integer sums are bit-exact; the max norm is bit-exact;
L2 norms and dequantised values agree to 1e-5 relative (the arithmetic gives ~1e-7: one binary64
reduction rounded once, resp. two binary32 roundings).  For bit parity both sides are given the
SAME binary32 norm, namely the oracle's, uploaded to the device.
"""
import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import gq_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2305_18627_amd as gq
    DEV = torch.device("cuda:0")
else:                                                  # collected but never run without a GPU
    gq = None
    DEV = None

SCHEMES = {"linear": 0, "exp": 1}
PACKS = {"i8": 0, "i4": 1, "u8s": 2, "u4s": 3}
NORMS = {"linf": 0, "l2": 1, "l2max": 2}
RTOL = 1e-5


def dev_scalar(v, dtype=torch.float32):
    return torch.tensor([v], dtype=dtype, device=DEV)


def host(t):
    return t.detach().cpu().numpy()


def gaussians(K, d, seed, std=1e-3):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return [(torch.randn(d, generator=g) * std).to(DEV) for _ in range(K)]


def oracle_norm(xs, kind):
    ne, nf, fl = O.global_norm([host(x) for x in xs], kind)
    return ne, nf, fl


def gpu_quantize(x, norm_t, params, worker, index_base):
    d = x.numel()
    lv = torch.full((max(gq.levels_nbytes(d, params.pack), 1) + 16,), 0xAB, dtype=torch.uint8, device=DEV)
    plane = params.pack >= 2
    sp = torch.full((gq.signplane_nwords(d) + 4,), -1, dtype=torch.int32, device=DEV) if plane else None
    gq.quantize(x, norm_t, params, worker, index_base, lv, sp)
    torch.cuda.synchronize()
    return lv, sp


# ------------------------------------------------------------------------------------ norm
@pytest.mark.parametrize("kind", ["linf", "l2", "l2max"])
@pytest.mark.parametrize("K,d", [(1, 1), (1, 3), (2, 4), (3, 5), (4, 1023), (3, 4096 + 7), (4, 1 << 20), (5, (1 << 21) + 3),
                                 (2, 9_000_001)])
def test_global_norm(kind, K, d):
    xs = gaussians(K, d, seed=K * 131 + d % 997, std=2e-3)
    out = dev_scalar(-1.0)
    flags = torch.tensor([77], dtype=torch.int32, device=DEV)
    gq.global_norm(xs, NORMS[kind], out, flags)
    torch.cuda.synchronize()
    ne, nf, fl = oracle_norm(xs, NORMS[kind])
    got = host(out)[0]
    if kind == "linf":
        assert got == nf
    else:
        assert abs(float(got) - ne) <= RTOL * ne
        assert abs(float(got) - ne) <= 2.0 ** -23 * ne          # what the arithmetic really gives
    assert int(host(flags)[0]) == fl == 0


def test_global_norm_flags_and_errors():
    out = dev_scalar(-1.0)
    flags = torch.tensor([77], dtype=torch.int32, device=DEV)
    for kind in NORMS.values():
        xs = [torch.zeros(1000, device=DEV), torch.zeros(1000, device=DEV)]
        xs[1][17] = -0.0
        gq.global_norm(xs, kind, out, flags)
        assert host(out)[0] == 0.0 and int(host(flags)[0]) == 2
        for bad in (float("nan"), float("inf"), float("-inf")):
            for pos in (0, 999, 998):
                xs = gaussians(2, 1000, seed=5)
                xs[1][pos] = bad
                gq.global_norm(xs, kind, out, flags)
                assert int(host(flags)[0]) & 1
                assert O.global_norm([host(x) for x in xs], kind)[2] & 1
        # squares overflow binary32, the norm does not
        xs = [torch.full((4,), 1e30, device=DEV)]
        gq.global_norm(xs, kind, out, flags)
        assert int(host(flags)[0]) == 0 and np.isfinite(host(out)[0])
    # d = 0: norm of nothing is 0
    gq.global_norm([torch.empty(0, device=DEV)], 0, out, flags)
    assert host(out)[0] == 0.0 and int(host(flags)[0]) == 2
    # errors: workspace too small, misaligned gradient, bad kind, too many workers
    xs = gaussians(2, 1 << 16, seed=1)
    with pytest.raises(gq.GQError) as e:
        gq.global_norm(xs, 0, out, flags, workspace=torch.empty(8, dtype=torch.uint8, device=DEV))
    assert e.value.status == gq.GQ_ERR_WORKSPACE
    with pytest.raises(gq.GQError) as e:
        gq.global_norm([xs[0][1:], xs[1][1:]], 0, out, flags)
    assert e.value.status == gq.GQ_ERR_INVALID_ARG
    with pytest.raises(gq.GQError):
        gq.global_norm(xs, 7, out, flags)
    with pytest.raises(gq.GQError):
        gq.global_norm([xs[0]] * 65, 0, out, flags)
    assert gq.norm_workspace_bytes(0, 10) == 0 and gq.norm_workspace_bytes(4, -1) == 0


# ------------------------------------------------------------------------------------ quantize
@pytest.mark.parametrize("scheme,s,pack", [("linear", 127, "i8"), ("linear", 7, "i4"), ("linear", 255, "u8s"),
                                           ("linear", 15, "u4s"), ("linear", 1, "i4"), ("exp", 16, "i8"),
                                           ("exp", 7, "i4"), ("exp", 31, "u8s"), ("exp", 15, "u4s")])
@pytest.mark.parametrize("d", [1, 2, 3, 4, 31, 32, 33, 255, 1021, 4099, 70_001])
def test_quantize_matches_oracle(scheme, s, pack, d):
    x = gaussians(1, d, seed=d + s)[0]
    xh = host(x)
    x[0] = float(np.abs(xh).max()) if d > 1 else x[0]           # one coordinate at the top of the range
    xh = host(x)
    _, nf, _ = oracle_norm([x], NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=SI.QUANT_SEED)
    for worker, base in [(0, 0), (3, 4 * 1234567), (17, 1 << 36)]:
        lv, sp = gpu_quantize(x, norm_t, params, worker, base)
        q = O.quantize(xh, nf, SCHEMES[scheme], s, SI.QUANT_SEED, worker, base)
        want_lv, want_sp = O.pack(q, PACKS[pack])
        n = want_lv.shape[0]
        got = host(lv)
        assert np.array_equal(got[:n], want_lv)
        assert np.all(got[n:] == 0xAB)                           # nothing written past the end
        if want_sp is not None:
            gs = host(sp).view(np.uint32)
            assert np.array_equal(gs[:want_sp.shape[0]], want_sp)
            assert np.all(gs[want_sp.shape[0]:] == 0xFFFFFFFF)


def test_quantize_special_norms_and_values():
    d = 5000
    x = gaussians(1, d, seed=2)[0]
    xh = host(x)
    for scheme, s, pack in [("linear", 127, "i8"), ("exp", 16, "i8")]:
        params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=9)
        # unusable norms: zero, negative zero, NaN, Inf, and one so small that s/norm overflows
        for bad in (0.0, -0.0, float("nan"), float("inf"), 1e-45):
            lv, _ = gpu_quantize(x, dev_scalar(bad), params, 0, 0)
            assert np.all(host(lv)[:d] == 0)
            assert np.all(O.quantize(xh, np.float32(bad), SCHEMES[scheme], s, 9, 0, 0) == 0)
        # assorted norms, including tiny and huge ones: the division and the scale must match bit for bit
        for nrm in (1e-3, 4.7e-3, 0.3333, 1.0, 123.456, 3e-30, 2.5e30, 1.1754944e-38):
            scale = nrm / 5e-3
            xs = (x * scale).contiguous()
            lv, _ = gpu_quantize(xs, dev_scalar(nrm), params, 1, 0)
            q = O.quantize(host(xs), np.float32(nrm), SCHEMES[scheme], s, 9, 1, 0)
            assert np.array_equal(host(lv)[:d].view(np.int8), np.clip(q, -128, 127).astype(np.int8))
    # denormal gradients with a denormal norm are not flushed
    xs = torch.full((d,), 2e-39, device=DEV)
    params = gq.make_params(0, 1, 0, 0, seed=4)
    lv, _ = gpu_quantize(xs, dev_scalar(4e-39), params, 0, 0)
    q = O.quantize(host(xs), np.float32(4e-39), 0, 1, 4, 0, 0)
    assert np.array_equal(host(lv)[:d].view(np.int8), q.astype(np.int8)) and 0.4 < q.mean() < 0.6


def test_binding_refuses_buffers_that_are_too_small():
    # the C ABI cannot see sizes; the binding checks them before anything is launched
    d = 4096
    xs = gaussians(2, d, seed=4)
    n = dev_scalar(1.0)
    P = gq.make_params
    ok_lv = torch.zeros(d, dtype=torch.uint8, device=DEV)
    ok_agg = torch.zeros(d, dtype=torch.int32, device=DEV)
    with pytest.raises(ValueError):
        gq.quantize(xs[0], n, P(0, 127), 0, 0, ok_lv[:d - 1])
    with pytest.raises(ValueError):
        gq.quantize(xs[0], n, P(0, 15, gq.GQ_PACK_U4_SIGNPLANE), 0, 0, ok_lv, torch.zeros(d // 32 - 1, dtype=torch.int32, device=DEV))
    with pytest.raises(ValueError):
        gq.quantize(xs[0].double(), n, P(0, 127), 0, 0, ok_lv)
    with pytest.raises(ValueError):
        gq.quantize(xs[0][::2], n, P(0, 127), 0, 0, ok_lv)                       # not contiguous
    with pytest.raises(ValueError):
        gq.fused_quantize_aggregate(xs, n, P(0, 127), 0, ok_agg[:d - 1])
    with pytest.raises(ValueError):
        gq.fused_quantize_aggregate([xs[0], xs[1][:d - 4]], n, P(0, 127), 0, ok_agg)
    with pytest.raises(ValueError):
        gq.fused_quantize_aggregate(xs, n, P(0, 127), 0, ok_agg, None, [ok_lv, ok_lv[:100]])
    with pytest.raises(ValueError):
        gq.int_aggregate([ok_lv, ok_lv], None, d, P(0, 127), ok_agg.short())       # int32 sum into 2-byte elements
    with pytest.raises(ValueError):
        gq.dequantize(ok_agg, d, n, P(0, 127), 2, torch.zeros(d - 1, device=DEV))
    with pytest.raises(ValueError):
        gq.global_norm(xs, 0, n.cpu())
    with pytest.raises(ValueError):
        gq.exp_reduce([ok_lv, ok_lv[:7]], d, P(1, 7), 0, n, ok_lv, None)
    # int16 sums need only two bytes per coordinate
    gq.fused_quantize_aggregate(xs, n, P(0, 127, 0, gq.GQ_AGG_I16), 0, torch.zeros(d, dtype=torch.int16, device=DEV))
    torch.cuda.synchronize()


def test_argument_errors():
    d = 1024
    x = gaussians(1, d + 4, seed=3)[0]
    n = dev_scalar(1.0)
    lv = torch.zeros(d + 16, dtype=torch.uint8, device=DEV)
    agg = torch.zeros(d + 16, dtype=torch.int32, device=DEV)
    P = gq.make_params

    def status(fn, *a, **k):
        with pytest.raises(gq.GQError) as e:
            fn(*a, **k)
        return e.value.status

    assert status(gq.quantize, x[1:d + 1], n, P(0, 127), 0, 0, lv) == gq.GQ_ERR_INVALID_ARG     # misaligned x
    assert status(gq.quantize, x[:d], n, P(0, 127), 0, 2, lv) == gq.GQ_ERR_INVALID_ARG          # index_base % 4
    assert status(gq.quantize, x[:d], n, P(0, 127), 0, -4, lv) == gq.GQ_ERR_INVALID_ARG
    assert status(gq.quantize, x[:d], n, P(0, 128), 0, 0, lv) == gq.GQ_ERR_UNSUPPORTED          # s > 127 in int8
    assert status(gq.quantize, x[:d], n, P(0, 8, gq.GQ_PACK_I4), 0, 0, lv) == gq.GQ_ERR_UNSUPPORTED
    assert status(gq.quantize, x[:d], n, P(1, 32, gq.GQ_PACK_U8_SIGNPLANE), 0, 0, lv) == gq.GQ_ERR_UNSUPPORTED
    assert status(gq.quantize, x[:d], n, P(0, 0), 0, 0, lv) == gq.GQ_ERR_INVALID_ARG
    assert status(gq.quantize, x[:d], n, P(5, 3), 0, 0, lv) == gq.GQ_ERR_INVALID_ARG
    assert status(gq.quantize, x[:d], n, P(0, 15, gq.GQ_PACK_U4_SIGNPLANE), 0, 0, lv, None) == gq.GQ_ERR_INVALID_ARG
    xs = [x[:d]] * 32
    # Section 4.2 headroom: 32 workers, exponential s = 15 cannot be summed in 16 bits; s = 7 can
    assert gq.check_width(P(1, 15, 3, gq.GQ_AGG_I16), 32) == gq.GQ_ERR_OVERFLOW
    assert gq.check_width(P(1, 7, 1, gq.GQ_AGG_I16), 32) == gq.GQ_OK
    assert status(gq.fused_quantize_aggregate, xs, n, P(1, 15, 3, gq.GQ_AGG_I16), 0, agg) == gq.GQ_ERR_OVERFLOW
    assert status(gq.int_aggregate, [lv] * 32, [agg] * 32, d, P(1, 15, 3, gq.GQ_AGG_I16), agg) == gq.GQ_ERR_OVERFLOW
    assert status(gq.fused_quantize_aggregate, xs, n, P(0, 127), 0, None, None) == gq.GQ_ERR_INVALID_ARG
    assert status(gq.fused_quantize_aggregate, xs, n, P(0, 127), 0, agg[1:]) == gq.GQ_ERR_INVALID_ARG
    assert status(gq.dequantize, agg, d, n, P(0, 127), 0, x[:d]) == gq.GQ_ERR_INVALID_ARG       # K = 0
    # d = 0 is a valid no-op everywhere
    e = torch.empty(0, device=DEV)
    gq.quantize(e, n, P(0, 127), 0, 0, lv)
    gq.fused_quantize_aggregate([e, e], n, P(0, 127), 0, agg)
    gq.int_aggregate([lv, lv], None, 0, P(0, 127), agg)
    gq.dequantize(agg, 0, n, P(0, 127), 2, x)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------ aggregate
@pytest.mark.parametrize("scheme,s,pack,agg", [("linear", 127, "i8", 0), ("linear", 7, "i4", 1), ("linear", 255, "u8s", 0),
                                               ("linear", 15, "u4s", 1), ("exp", 16, "i8", 0), ("exp", 7, "i4", 1),
                                               ("exp", 9, "u8s", 1), ("exp", 15, "u4s", 0)])
@pytest.mark.parametrize("K,d", [(1, 1), (2, 15), (3, 16), (4, 17), (5, 31), (16, 32), (7, 33), (32, 4097), (6, 65_537)])
def test_int_aggregate_matches_oracle(scheme, s, pack, agg, K, d):
    check_int_aggregate(scheme, s, pack, agg, K, d)


# packed 4-bit codes: workgroups of 1024 coordinates take the eight-coordinates-per-lane kernel, the rest
# the general one; both widths of the sum, every split of K into batches of 8, 4, 2, 1
@pytest.mark.parametrize("scheme,s,pack", [("linear", 7, "i4"), ("exp", 7, "i4"), ("exp", 3, "i4"), ("linear", 15, "u4s"),
                                           ("linear", 1, "u4s"), ("exp", 15, "u4s")])
@pytest.mark.parametrize("agg", [0, 1])
@pytest.mark.parametrize("K,d", [(1, 1024), (2, 1025), (7, 6143), (13, 2048), (15, 70_001), (64, 3073), (33, 1023 + 4096)])
def test_int_aggregate_packed_nibbles(scheme, s, pack, agg, K, d):
    check_int_aggregate(scheme, s, pack, agg, K, d)


def check_int_aggregate(scheme, s, pack, agg, K, d):
    rng = np.random.default_rng(K * 1000 + d + s)
    qs = [rng.integers(-s, s + 1, d).astype(np.int32) for _ in range(K)]
    qs[0][:] = s                                                 # a worker stuck at the top level
    if K > 1:
        qs[1][:] = np.where(np.arange(d) % 2 == 0, s, -s)
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], agg, seed=0)
    want = O.aggregate(qs, SCHEMES[scheme])
    if gq.check_width(params, K) != gq.GQ_OK:
        assert not O.check_width(SCHEMES[scheme], s, K, 16 if agg else 32)
        with pytest.raises(gq.GQError):
            gq.int_aggregate([torch.zeros(d + 16, dtype=torch.uint8, device=DEV)] * K, None, d, params,
                             torch.zeros(d + 16, dtype=torch.int32, device=DEV))
        return
    assert O.check_width(SCHEMES[scheme], s, K, 16 if agg else 32) and O.fits_width(want, 16 if agg else 32)
    lvs, sps = [], []
    for q in qs:
        lv, sp = O.pack(q, PACKS[pack])
        lvs.append(torch.from_numpy(np.concatenate([lv, np.full(16, 0xFF, np.uint8)])).to(DEV)[:lv.shape[0]])
        sps.append(torch.from_numpy(sp.view(np.int32)).to(DEV) if sp is not None else None)
    out = torch.full((d + 8,), 0x5A5A, dtype=torch.int16 if agg else torch.int32, device=DEV)
    gq.int_aggregate(lvs, sps if sps[0] is not None else None, d, params, out)
    torch.cuda.synchronize()
    got = host(out)
    assert np.array_equal(got[:d].astype(np.int64), want)
    assert np.all(got[d:] == 0x5A5A)


# ------------------------------------------------------------------------------------ dequantize
@pytest.mark.parametrize("scheme,s,agg", [("linear", 127, 0), ("linear", 15, 1), ("exp", 16, 0), ("exp", 7, 1)])
@pytest.mark.parametrize("K,d", [(4, 1), (16, 1023), (8, 100_003)])
def test_dequantize_matches_oracle(scheme, s, agg, K, d):
    rng = np.random.default_rng(d + s)
    lim = min(O.max_aggregate(SCHEMES[scheme], s, K), 32767 if agg else 2 ** 31 - 1)
    A = rng.integers(-lim, lim + 1, d)
    A[rng.random(d) < 0.3] = 0
    params = gq.make_params(SCHEMES[scheme], s, 0, agg, seed=0)
    a = torch.from_numpy(A.astype(np.int16 if agg else np.int32)).to(DEV)
    out = torch.full((d + 8,), 7.0, device=DEV)
    for nrm in (3.7e-3, 1.0, 2.5e-30):
        gq.dequantize(a, d, dev_scalar(nrm), params, K, out)
        torch.cuda.synchronize()
        want = O.dequantize(A, float(np.float32(nrm)), SCHEMES[scheme], s, K)
        got = host(out).astype(np.float64)
        assert np.all(np.abs(got[:d] - want) <= RTOL * np.abs(want))
        assert np.all(got[:d][A == 0] == 0.0) and np.all(got[d:] == 7.0)
    for bad in (0.0, float("nan"), float("inf")):               # unusable norm: the output is all zero
        gq.dequantize(a, d, dev_scalar(bad), params, K, out)
        assert np.all(host(out)[:d] == 0.0)


# ------------------------------------------------------------------------------------ fused
def run_fused(xs, norm_t, params, base, want_levels, agg=True, deq=True):
    K, d = len(xs), xs[0].numel()
    agg_out = torch.full((d + 8,), 0x5A5A, dtype=torch.int16 if params.agg else torch.int32, device=DEV) if agg else None
    deq_out = torch.full((d + 8,), 7.0, device=DEV) if deq else None
    lvs = sps = None
    if want_levels:
        lvs = [torch.full((gq.levels_nbytes(d, params.pack) + 16,), 0xAB, dtype=torch.uint8, device=DEV) for _ in range(K)]
        if params.pack >= 2:
            sps = [torch.full((gq.signplane_nwords(d) + 4,), -1, dtype=torch.int32, device=DEV) for _ in range(K)]
    gq.fused_quantize_aggregate(xs, norm_t, params, base, agg_out, deq_out, lvs, sps)
    torch.cuda.synchronize()
    return agg_out, deq_out, lvs, sps


@pytest.mark.parametrize("scheme,s,pack,agg", [("linear", 127, "i8", 0), ("linear", 15, "u4s", 0), ("linear", 7, "i4", 1),
                                               ("exp", 16, "i8", 0), ("exp", 7, "i4", 1), ("exp", 9, "u8s", 1)])
@pytest.mark.parametrize("K,d", [(1, 4099), (2, 3), (3, 70_001), (4, 70_002), (5, 1021), (8, 70_003), (16, 70_000),
                                 (32, 8191), (33, 513), (64, 1000)])
def test_fused_matches_oracle(scheme, s, pack, agg, K, d):
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], agg, seed=SI.QUANT_SEED + K)
    if gq.check_width(params, K) != gq.GQ_OK:
        pytest.skip("sum does not fit the width (covered by the error tests)")
    xs = gaussians(K, d, seed=K * 7 + d)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    base = 4 * 98765
    want = O.quantize_aggregate(xh, nf, SCHEMES[scheme], s, params.seed, base)
    want_deq = O.dequantize(want, float(nf), SCHEMES[scheme], s, K)
    for with_levels in (False, True):
        agg_out, deq_out, lvs, sps = run_fused(xs, norm_t, params, base, with_levels)
        got = host(agg_out)
        assert np.array_equal(got[:d].astype(np.int64), want) and np.all(got[d:] == 0x5A5A)
        gd = host(deq_out).astype(np.float64)
        assert np.all(np.abs(gd[:d] - want_deq) <= RTOL * np.abs(want_deq))
        assert np.all(gd[:d][want == 0] == 0.0) and np.all(gd[d:] == 7.0)
        if with_levels:
            for i in range(K):
                q = O.quantize(xh[i], nf, SCHEMES[scheme], s, params.seed, i, base)
                wl, ws = O.pack(q, PACKS[pack])
                gl = host(lvs[i])
                assert np.array_equal(gl[:wl.shape[0]], wl) and np.all(gl[wl.shape[0]:] == 0xAB)
                if ws is not None:
                    gs = host(sps[i]).view(np.uint32)
                    assert np.array_equal(gs[:ws.shape[0]], ws) and np.all(gs[ws.shape[0]:] == 0xFFFFFFFF)
    # outputs are optional one by one
    a_only, _, _, _ = run_fused(xs, norm_t, params, base, False, agg=True, deq=False)
    _, d_only, _, _ = run_fused(xs, norm_t, params, base, False, agg=False, deq=True)
    assert np.array_equal(host(a_only)[:d].astype(np.int64), want)
    assert np.array_equal(host(d_only)[:d], host(deq_out)[:d])


@pytest.mark.parametrize("rng_bits", [32, 16])
def test_fused_degenerate_inputs(rng_bits):
    # the degenerate cases of the method: an all-zero gradient (norm 0), unusable norms, identical workers,
    # one non-zero coordinate sitting on the norm
    K, d = 4, 10_007
    for scheme, s in ((0, 127), (1, 16)):
        p = gq.make_params(scheme, s, 0, 0, seed=3, rng_bits=rng_bits)
        zeros = [torch.zeros(d, device=DEV) for _ in range(K)]
        norm_t = dev_scalar(-1.0)
        flags = torch.zeros(1, dtype=torch.int32, device=DEV)
        gq.global_norm(zeros, NORMS["l2"], norm_t, flags)
        assert float(norm_t.item()) == 0.0 and int(flags.item()) == 2
        agg, deq, lvs, _ = run_fused(zeros, norm_t, p, 0, True)
        assert bool((agg[:d] == 0).all()) and bool((deq[:d] == 0).all()) and all(bool((l[:d] == 0).all()) for l in lvs)
        xs = gaussians(K, d, seed=8)
        for bad in (0.0, float("nan"), float("inf"), -1.0):
            agg, deq, lvs, _ = run_fused(xs, dev_scalar(bad), p, 0, True)
            assert bool((agg[:d] == 0).all()) and bool((deq[:d] == 0).all()) and all(bool((l[:d] == 0).all()) for l in lvs)
            assert np.all(O.quantize_aggregate([host(x) for x in xs], np.float32(bad), scheme, s, 3, 0, rng_bits=rng_bits) == 0)
        # identical workers still round independently (the worker word is part of the counter), and the sum of
        # the K copies equals the oracle's
        same = [xs[0]] * K
        _, nf, _ = oracle_norm(same, NORMS["linf"])
        agg, _, lvs, _ = run_fused(same, dev_scalar(float(nf)), p, 0, True)
        want = O.quantize_aggregate([host(xs[0])] * K, nf, scheme, s, 3, 0, rng_bits=rng_bits)
        assert np.array_equal(host(agg)[:d].astype(np.int64), want)
        assert not torch.equal(lvs[0][:d], lvs[1][:d])
        # a single non-zero coordinate: y = 1 there, the top level with certainty; everything else stays zero
        one = [torch.zeros(d, device=DEV) for _ in range(K)]
        one[2][4321] = -0.75
        gq.global_norm(one, NORMS["linf"], norm_t, flags)
        agg, deq, _, _ = run_fused(one, norm_t, p, 0, False)
        top = s if scheme == 0 else 2 ** (s - 1)
        assert int(agg[4321].item()) == -top and int(agg.abs()[:d].sum().item()) == top
        assert abs(float(deq[4321].item()) - (-0.75 / K)) <= RTOL * 0.75 / K


@pytest.mark.parametrize("rng_bits", [32, 16])
@pytest.mark.parametrize("scheme,s,pack", [("linear", 127, "i8"), ("linear", 15, "u4s"), ("exp", 16, "i8"), ("exp", 7, "i4")])
def test_nan_and_inf_coordinates_match_the_oracle(scheme, s, pack, rng_bits):
    # a gradient that holds a NaN or an Inf: the norm of gq_global_norm is then unusable and EVERY code is 0, also
    # at the NaN / Inf coordinates themselves (Inf * 0 and NaN * 0 are NaN, which must not turn into the top level);
    # with a finite norm given by the caller a NaN coordinate rounds to 0 and an Inf coordinate to the top level
    K, d = 4, 9_001
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=17, rng_bits=rng_bits)
    for bad in (float("nan"), float("inf"), float("-inf")):
        xs = gaussians(K, d, seed=3)
        for w, pos in ((0, 0), (1, 4097), (1, 4098), (3, d - 1), (2, 777)):
            xs[w][pos] = bad
        xh = [host(x) for x in xs]
        for kind in ("linf", "l2", "l2max", None):
            if kind is None:
                norm_t = dev_scalar(5e-3)                                 # a finite norm from the caller
            else:
                norm_t = dev_scalar(-1.0)
                flags = torch.zeros(1, dtype=torch.int32, device=DEV)
                gq.global_norm(xs, NORMS[kind], norm_t, flags)
                assert int(flags.item()) & 1
            nf = np.float32(norm_t.item())
            qs = [O.quantize(xh[i], nf, SCHEMES[scheme], s, 17, i, 0, rng_bits=rng_bits) for i in range(K)]
            want = O.aggregate(qs, SCHEMES[scheme])
            if kind is not None:
                assert not want.any() and not any(q.any() for q in qs)
            elif bad != bad:
                assert qs[1][4097] == 0 and qs[0][0] == 0
            else:
                assert abs(qs[1][4097]) == s
            agg, deq, lvs, sps = run_fused(xs, norm_t, params, 0, True)
            assert np.array_equal(host(agg)[:d].astype(np.int64), want)
            if kind is not None:
                assert bool((deq[:d] == 0).all())
            lone, spone = [], []
            for i in range(K):
                wl, ws = O.pack(qs[i], PACKS[pack])
                assert np.array_equal(host(lvs[i])[:wl.shape[0]], wl)
                lv, sp = gpu_quantize(xs[i], norm_t, params, i, 0)
                assert np.array_equal(host(lv)[:wl.shape[0]], wl)
                if ws is not None:
                    assert np.array_equal(host(sps[i]).view(np.uint32)[:ws.shape[0]], ws)
                    assert np.array_equal(host(sp).view(np.uint32)[:ws.shape[0]], ws)
                lone.append(lv); spone.append(sp)
            dense = torch.zeros(d, dtype=torch.int32, device=DEV)
            gq.int_aggregate(lone, spone if spone[0] is not None else None, d, params, dense)
            torch.cuda.synchronize()
            assert np.array_equal(host(dense).astype(np.int64), want)


def test_fused_equals_separate_calls_and_buckets_equal_whole():
    K, d = 8, 300_007
    xs = gaussians(K, d, seed=77)
    for scheme, s, pack, kind in [("linear", 127, "i8", "linf"), ("exp", 7, "i4", "l2"), ("linear", 15, "u4s", "l2max")]:
        params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=5)
        norm_t = dev_scalar(0.0)
        gq.global_norm(xs, NORMS[kind], norm_t)
        whole, whole_deq, _, _ = run_fused(xs, norm_t, params, 0, False)
        # (a) separate calls: quantize each worker, integer sum, dequantize
        lvs, sps = [], []
        for i in range(K):
            lv, sp = gpu_quantize(xs[i], norm_t, params, i, 0)
            lvs.append(lv); sps.append(sp)
        agg = torch.zeros(d, dtype=torch.int32, device=DEV)
        gq.int_aggregate(lvs, sps if sps[0] is not None else None, d, params, agg)
        deq = torch.zeros(d, device=DEV)
        gq.dequantize(agg, d, norm_t, params, K, deq)
        torch.cuda.synchronize()
        assert torch.equal(agg, whole[:d]) and torch.equal(deq, whole_deq[:d])
        # (b) buckets with their offsets reproduce the whole
        cut = [0, 4 * 10_001, 4 * 40_000, d]
        for lo, hi in zip(cut[:-1], cut[1:]):
            part, _, _, _ = run_fused([x[lo:hi] for x in xs], norm_t, params, lo, False)
            assert torch.equal(part[:hi - lo], whole[lo:hi])
        # (c) the order of the workers does not matter to the sum when each keeps its worker word:
        #     checked through the separate path, where the worker word is an argument
        agg2 = torch.zeros(d, dtype=torch.int32, device=DEV)
        gq.int_aggregate(lvs[::-1], sps[::-1] if sps[0] is not None else None, d, params, agg2)
        torch.cuda.synchronize()
        assert torch.equal(agg2, agg)


def test_fused_equals_separate_calls_on_random_shapes():
    # 120 seeded cases over worker counts 1..64 (the specialised 4, 8, 16, 32 and the run-time path), ragged lengths,
    # both grids, all four storage formats, both sum widths, both draw widths, bucket offsets, with and without stored
    # codes: the fused call writes the codes of gq_quantize, the sum of gq_int_aggregate and the mean of gq_dequantize,
    # bit for bit (each of which the tests above compare with the oracle at fixed shapes)
    rng = np.random.default_rng(11)
    g = torch.Generator(device=DEV).manual_seed(13)
    done = 0
    while done < 120:
        K = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 24, 32, 33, 48, 64]))
        d = int(rng.choice([rng.integers(1, 40), rng.integers(1, 5000), rng.integers(1, 200_000)]))
        scheme = int(rng.integers(0, 2))
        pack = int(rng.integers(0, 4))
        smax = (127, 7, 255, 15)[pack] if scheme == 0 else min((127, 7, 255, 15)[pack], 31)
        s = int(rng.integers(1, smax + 1))
        aggf = int(rng.integers(0, 2))
        bits = int(rng.choice([32, 16]))
        p = gq.make_params(scheme, s, pack, aggf, seed=int(rng.integers(0, 1 << 62)), rng_bits=bits)
        if gq.check_width(p, K) != gq.GQ_OK:
            continue                                                  # this sum does not fit this width: another draw
        done += 1
        base = int(rng.integers(0, 1 << 30)) * 8
        xs = [torch.randn(d, generator=g, device=DEV) * float(10 ** rng.uniform(-5, 0)) for _ in range(K)]
        norm_t = dev_scalar(0.0)
        gq.global_norm(xs, int(rng.integers(0, 3)), norm_t)
        case = (done, K, d, scheme, s, pack, aggf, bits, base)
        with_codes = bool(rng.integers(0, 2))
        agg_out, deq_out, lvs, sps = run_fused(xs, norm_t, p, base, with_codes)
        # separate calls
        qlv, qsp = [], []
        for i in range(K):
            lv, sp = gpu_quantize(xs[i], norm_t, p, i, base)
            qlv.append(lv); qsp.append(sp)
        agg = torch.full((d + 8,), 0x5A5A, dtype=torch.int16 if aggf else torch.int32, device=DEV)
        gq.int_aggregate(qlv, qsp if qsp[0] is not None else None, d, p, agg)          # the guard entries behind d must survive
        deq = torch.full((d + 8,), 7.0, device=DEV)
        gq.dequantize(agg, d, norm_t, p, K, deq)
        torch.cuda.synchronize()
        assert torch.equal(agg, agg_out) and torch.equal(deq, deq_out), case
        if with_codes:
            for i in range(K):
                assert torch.equal(lvs[i], qlv[i]), case
                if qsp[i] is not None:
                    assert torch.equal(sps[i], qsp[i]), case


@pytest.mark.parametrize("scheme,s,pack", [("linear", 127, "i8"), ("linear", 15, "u4s"), ("exp", 7, "i4"), ("exp", 16, "i8")])
@pytest.mark.parametrize("K,d,bucket", [(1, 8, 8), (3, 1000, 4096), (4, 4096, 1024), (5, 70_001, 8192), (8, 20_003, 20_000), (16, 33_000, 32_768)])
def test_per_bucket_schedule_matches_the_oracle_bucket_by_bucket(scheme, s, pack, K, d, bucket):
    # gq_bucketed_quantize_aggregate at small sizes: one bucket, whole buckets only, a last bucket of a few coordinates.
    # Every bucket's norm against the oracle's norm of the K slices; the sums against the oracle's quantisation under
    # that norm and the bucket's offset; the means to 1e-5; both schedules identical; guard entries untouched
    xs = gaussians(K, d, seed=K + d + s)
    xh = [host(x) for x in xs]
    nb = (d + bucket - 1) // bucket
    p = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=2025)
    side = torch.cuda.Stream()
    means = {}
    for kind in ("linf", "l2", "l2max"):
        got = []
        for two in (False, True):
            norms = torch.full((nb + 2,), -1.0, device=DEV)
            flags = torch.full((nb + 2,), 77, dtype=torch.int32, device=DEV)
            agg = torch.full((d + 8,), 0x5A5A, dtype=torch.int32, device=DEV)
            out = torch.full((d + 8,), 7.0, device=DEV)
            gq.bucketed_quantize_aggregate(xs, bucket, NORMS[kind], p, norms, flags, agg, out, side_stream=side if two else None)
            torch.cuda.synchronize()
            got.append((norms, flags, agg, out))
        for a, b in zip(got[0], got[1]):
            assert torch.equal(a, b)
        norms, flags, agg, out = got[0]
        means[kind] = out
        assert bool((norms[nb:] == -1.0).all()) and bool((flags[nb:] == 77).all()) and bool((flags[:nb] == 0).all())
        assert bool((agg[d:] == 0x5A5A).all()) and bool((out[d:] == 7.0).all())
        for b in range(nb):
            lo, hi = b * bucket, min(d, (b + 1) * bucket)
            _, nf, _ = O.global_norm([x[lo:hi] for x in xh], NORMS[kind])
            gn = np.float32(norms[b].item())
            if kind == "linf":
                assert gn == nf
            else:
                assert abs(float(gn) - float(nf)) <= RTOL * float(nf)
            # the codes are decided under the library's own norm of the bucket (one ulp of norm can move a code)
            A = O.quantize_aggregate([x[lo:hi] for x in xh], gn, SCHEMES[scheme], s, 2025, lo)
            assert np.array_equal(host(agg[lo:hi]).astype(np.int64), A), (kind, b)
            wd = O.dequantize(A, float(gn), SCHEMES[scheme], s, K)
            gd = host(out[lo:hi]).astype(np.float64)
            assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)) and np.all(gd[A == 0] == 0.0)
    # one output may be left out; neither is an error, and so are a bucket that is no multiple of 8 and a short workspace
    norms = torch.zeros(nb, device=DEV)
    only = torch.zeros(d, device=DEV)
    gq.bucketed_quantize_aggregate(xs, bucket, NORMS["linf"], p, norms, None, None, only)
    torch.cuda.synchronize()
    assert torch.equal(only, means["linf"][:d])
    for bad_call in (lambda: gq.bucketed_quantize_aggregate(xs, bucket, NORMS["linf"], p, norms, None, None, None),
                     lambda: gq.bucketed_quantize_aggregate(xs, bucket + 4, NORMS["linf"], p, norms, None, None, only),
                     lambda: gq.bucketed_quantize_aggregate(xs, 0, NORMS["linf"], p, norms, None, None, only)):
        with pytest.raises((gq.GQError, ValueError, ZeroDivisionError)):
            bad_call()
    if gq.bucketed_workspace_bytes(K, d, bucket) > 8:
        with pytest.raises(gq.GQError) as e:
            gq.bucketed_quantize_aggregate(xs, bucket, NORMS["linf"], p, norms, None, None, only,
                                           workspace=torch.zeros(8, dtype=torch.uint8, device=DEV))
        assert e.value.status == gq.GQ_ERR_WORKSPACE


def test_fused_across_the_2_to_34_index_boundary():
    # the Philox call index g/4 crosses a multiple of 2^32 inside the bucket: the high counter word changes
    K, d = 16, 70_001
    xs = gaussians(K, d, seed=99)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    for scheme, s in [("linear", 127), ("exp", 16)]:
        params = gq.make_params(SCHEMES[scheme], s, 0, 0, seed=31337)
        for base in ((1 << 34) - 4 * 1000, (1 << 34) - 4 * 129, (1 << 34) - 4, 1 << 34, 3 * (1 << 34) - 4 * 17_000):
            want = O.quantize_aggregate(xh, nf, SCHEMES[scheme], s, params.seed, base)
            for with_levels in (False, True):
                agg_out, _, _, _ = run_fused(xs, norm_t, params, base, with_levels)
                got = host(agg_out)
                assert np.array_equal(got[:d].astype(np.int64), want) and np.all(got[d:] == 0x5A5A)
    # and for a run-time worker count
    params = gq.make_params(0, 127, 0, 0, seed=31337)
    base = (1 << 34) - 4 * 777
    want = O.quantize_aggregate(xh[:5], nf, 0, 127, params.seed, base)
    agg_out, _, _, _ = run_fused(xs[:5], norm_t, params, base, False)
    assert np.array_equal(host(agg_out)[:d].astype(np.int64), want)


# ------------------------------------------------------------------------------------ short draws
# 16 random bits per coordinate, one Philox call per eight coordinates: a lane owns two vectors.
@pytest.mark.parametrize("scheme,s,pack", [("linear", 127, "i8"), ("linear", 7, "i4"), ("linear", 255, "u8s"),
                                           ("linear", 15, "u4s"), ("exp", 16, "i8"), ("exp", 7, "i4"),
                                           ("exp", 31, "u8s"), ("exp", 15, "u4s")])
@pytest.mark.parametrize("d", [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 13, 31, 32, 33, 63, 64, 65, 255, 1021, 4099, 70_001, 70_004])
def test_quantize_short_draws_matches_oracle(scheme, s, pack, d):
    x = gaussians(1, d, seed=d + s + 1)[0]
    xh = host(x)
    _, nf, _ = oracle_norm([x], NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=SI.QUANT_SEED, rng_bits=16)
    for worker, base in [(0, 0), (3, 8 * 1234567), (17, 1 << 37), (5, (1 << 35) - 8 * 100)]:
        lv, sp = gpu_quantize(x, norm_t, params, worker, base)
        q = O.quantize(xh, nf, SCHEMES[scheme], s, SI.QUANT_SEED, worker, base, rng_bits=16)
        want_lv, want_sp = O.pack(q, PACKS[pack])
        n = want_lv.shape[0]
        got = host(lv)
        assert np.array_equal(got[:n], want_lv)
        assert np.all(got[n:] == 0xAB)
        if want_sp is not None:
            gs = host(sp).view(np.uint32)
            assert np.array_equal(gs[:want_sp.shape[0]], want_sp)
            assert np.all(gs[want_sp.shape[0]:] == 0xFFFFFFFF)


@pytest.mark.parametrize("scheme,s,pack,agg", [("linear", 127, "i8", 0), ("linear", 15, "u4s", 0), ("linear", 7, "i4", 1),
                                               ("exp", 16, "i8", 0), ("exp", 7, "i4", 1), ("exp", 9, "u8s", 1)])
@pytest.mark.parametrize("K,d", [(1, 4099), (2, 3), (2, 5), (3, 70_001), (4, 70_006), (5, 1021), (8, 70_003), (16, 70_000),
                                 (32, 8191), (33, 513), (64, 1004)])
def test_fused_short_draws_matches_oracle(scheme, s, pack, agg, K, d):
    params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], agg, seed=SI.QUANT_SEED + K, rng_bits=16)
    if gq.check_width(params, K) != gq.GQ_OK:
        pytest.skip("sum does not fit the width (covered by the error tests)")
    xs = gaussians(K, d, seed=K * 11 + d)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    base = 8 * 98765
    want = O.quantize_aggregate(xh, nf, SCHEMES[scheme], s, params.seed, base, rng_bits=16)
    assert not np.array_equal(want, O.quantize_aggregate(xh, nf, SCHEMES[scheme], s, params.seed, base)) or d < 8
    want_deq = O.dequantize(want, float(nf), SCHEMES[scheme], s, K)
    for with_levels in (False, True):
        agg_out, deq_out, lvs, sps = run_fused(xs, norm_t, params, base, with_levels)
        got = host(agg_out)
        assert np.array_equal(got[:d].astype(np.int64), want) and np.all(got[d:] == 0x5A5A)
        gd = host(deq_out).astype(np.float64)
        assert np.all(np.abs(gd[:d] - want_deq) <= RTOL * np.abs(want_deq))
        assert np.all(gd[:d][want == 0] == 0.0) and np.all(gd[d:] == 7.0)
        if with_levels:
            for i in range(K):
                q = O.quantize(xh[i], nf, SCHEMES[scheme], s, params.seed, i, base, rng_bits=16)
                wl, ws = O.pack(q, PACKS[pack])
                gl = host(lvs[i])
                assert np.array_equal(gl[:wl.shape[0]], wl) and np.all(gl[wl.shape[0]:] == 0xAB)
                if ws is not None:
                    gs = host(sps[i]).view(np.uint32)
                    assert np.array_equal(gs[:ws.shape[0]], ws) and np.all(gs[ws.shape[0]:] == 0xFFFFFFFF)


def test_short_draws_buckets_boundary_and_separate_calls():
    K, d = 8, 300_011
    xs = gaussians(K, d, seed=78)
    xh = [host(x) for x in xs]
    for scheme, s, pack in [("linear", 127, "i8"), ("exp", 7, "i4"), ("linear", 15, "u4s")]:
        params = gq.make_params(SCHEMES[scheme], s, PACKS[pack], 0, seed=6, rng_bits=16)
        norm_t = dev_scalar(0.0)
        gq.global_norm(xs, NORMS["linf"], norm_t)
        whole, whole_deq, _, _ = run_fused(xs, norm_t, params, 0, False)
        lvs, sps = [], []
        for i in range(K):
            lv, sp = gpu_quantize(xs[i], norm_t, params, i, 0)
            lvs.append(lv); sps.append(sp)
        agg = torch.zeros(d, dtype=torch.int32, device=DEV)
        gq.int_aggregate(lvs, sps if sps[0] is not None else None, d, params, agg)
        torch.cuda.synchronize()
        assert torch.equal(agg, whole[:d])
        cut = [0, 8 * 10_001, 8 * 20_000, d]
        for lo, hi in zip(cut[:-1], cut[1:]):
            part, _, _, _ = run_fused([x[lo:hi] for x in xs], norm_t, params, lo, False)
            assert torch.equal(part[:hi - lo], whole[lo:hi])
    # the Philox call index g/8 crosses a multiple of 2^32 inside the bucket
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    d2 = 70_001
    params = gq.make_params(0, 127, 0, 0, seed=31337, rng_bits=16)
    for base in ((1 << 35) - 8 * 1000, (1 << 35) - 8 * 129, (1 << 35) - 8, 1 << 35, 3 * (1 << 35) - 8 * 8_000):
        want = O.quantize_aggregate([x[:d2] for x in xh], nf, 0, 127, params.seed, base, rng_bits=16)
        for with_levels in (False, True):
            agg_out, _, _, _ = run_fused([x[:d2] for x in xs], norm_t, params, base, with_levels)
            assert np.array_equal(host(agg_out)[:d2].astype(np.int64), want)
        want5 = O.quantize_aggregate([x[:d2] for x in xh[:5]], nf, 0, 127, params.seed, base, rng_bits=16)
        agg_out, _, _, _ = run_fused([x[:d2] for x in xs[:5]], norm_t, params, base, False)
        assert np.array_equal(host(agg_out)[:d2].astype(np.int64), want5)


# ------------------------------------------------------------------------------------ Algorithm 2
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 13, 16, 17, 24, 25, 32, 33, 41, 48, 56, 64])
@pytest.mark.parametrize("s,d", [(7, 70_003), (16, 4099), (31, 1021), (1, 255), (8, 4098), (9, 515)])
def test_exp_reduce_matches_oracle(K, s, d):
    # the paper's reduce function for exponential dithering, tree order: reduced (sign, e) bit-exact,
    # the mean it stands for to 1e-5
    xs = gaussians(K, d, seed=K * 31 + s, std=3e-3)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    params = gq.make_params(1, s, 0, 0, seed=SI.QUANT_SEED + s)
    for base in (0, 4 * 55_555, (1 << 34) - 4 * 100):
        lvs, qs = [], []
        for i in range(K):
            lv, _ = gpu_quantize(xs[i], norm_t, params, i, base)
            lvs.append(lv)
            qs.append(O.quantize(xh[i], nf, O.EXP, s, params.seed, i, base))
            assert np.array_equal(host(lv)[:d].view(np.int8), qs[i].astype(np.int8))
        red = torch.full((d + 16,), 0x5A, dtype=torch.int8, device=DEV)
        deq = torch.full((d + 8,), 7.0, device=DEV)
        gq.exp_reduce(lvs, d, params, base, norm_t, red, deq)
        torch.cuda.synchronize()
        want = O.exp_tree_reduce(qs, s, params.seed, base)
        got = host(red)
        assert np.array_equal(got[:d].astype(np.int32), want) and np.all(got[d:] == 0x5A)
        wd = O.exp_reduce_dequantize(want, float(nf), K)
        gd = host(deq).astype(np.float64)
        assert np.all(np.abs(gd[:d] - wd) <= RTOL * np.abs(wd))
        assert np.all(gd[:d][want == 0] == 0.0) and np.all(gd[d:] == 7.0)
        # outputs are optional one by one
        red2 = torch.zeros(d, dtype=torch.int8, device=DEV)
        gq.exp_reduce(lvs, d, params, base, None, red2, None)
        deq2 = torch.zeros(d, device=DEV)
        gq.exp_reduce(lvs, d, params, base, norm_t, None, deq2)
        torch.cuda.synchronize()
        assert torch.equal(red2, red[:d]) and torch.equal(deq2, deq[:d])
    with pytest.raises(gq.GQError) as e:
        gq.exp_reduce(lvs, d, gq.make_params(0, s if s <= 127 else 127), 0, norm_t, red, None)
    assert e.value.status == gq.GQ_ERR_UNSUPPORTED
    with pytest.raises(gq.GQError):
        gq.exp_reduce(lvs, d, params, 0, None, None, None)


def test_exp_reduce_is_unbiased_for_the_integer_sum_on_gpu():
    # E[Algorithm 2 result] = the exact sum that gq_int_aggregate forms, measured over seeds on the GPU
    K, d, s, T = 16, 4096, 7, 300
    xs = gaussians(K, d, seed=5, std=3e-3)
    norm_t = dev_scalar(0.0)
    gq.global_norm(xs, NORMS["linf"], norm_t)
    p = gq.make_params(1, s, 0, 0, seed=11)
    lvs = [gpu_quantize(xs[i], norm_t, p, i, 0)[0] for i in range(K)]
    agg = torch.zeros(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, agg)
    exact = torch.zeros(d, device=DEV)
    gq.dequantize(agg, d, norm_t, p, K, exact)
    acc = torch.zeros(d, dtype=torch.float64, device=DEV)
    out = torch.zeros(d, device=DEV)
    for t in range(T):
        gq.exp_reduce(lvs, d, gq.make_params(1, s, 0, 0, seed=2000 + t), 0, norm_t, None, out)
        acc += out.double()
    mean = host(acc) / T
    # the deviation of one result is bounded through its second moment, at most (9/8)^log2(n') times the square of
    # the mean of the workers' absolute values (the sample deviation cannot serve: rare large roundings hide from it)
    absmean = np.zeros(d)
    for lv in lvs:
        k = np.abs(host(lv)[:d].view(np.int8).astype(np.int64))
        absmean += np.where(k > 0, 2.0 ** (k - 1), 0.0)
    absmean *= float(norm_t.item()) / (K * 2.0 ** (s - 1))
    sd_bound = np.sqrt((9.0 / 8.0) ** 4) * absmean
    assert np.all(np.abs(mean - host(exact).astype(np.float64)) <= 5.0 * sd_bound / np.sqrt(T) + 1e-12)


# ------------------------------------------------------------------------------------ Implementation section: in-step averaging
@pytest.mark.parametrize("K", [1, 2, 3, 4, 7, 8, 16, 32, 33, 64])
@pytest.mark.parametrize("s,pack,d", [(7, "i4", 70_003), (7, "i4", 4098), (127, "i8", 4099), (1, "i4", 255), (15, "i8", 1021)])
def test_avg_reduce_matches_oracle(K, s, pack, d):
    xs = gaussians(K, d, seed=K * 17 + s, std=3e-3)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    params = gq.make_params(0, s, PACKS[pack], 0, seed=SI.QUANT_SEED + 3 * s)
    for base in (0, 4 * 31_337, (1 << 34) - 4 * 50):
        lvs = [gpu_quantize(xs[i], norm_t, params, i, base)[0] for i in range(K)]
        qs = [O.quantize(xh[i], nf, O.LINEAR, s, params.seed, i, base) for i in range(K)]
        nb = gq.levels_nbytes(d, PACKS[pack])
        red = torch.full((nb + 16,), 0x5A, dtype=torch.uint8, device=DEV)
        deq = torch.full((d + 8,), 7.0, device=DEV)
        gq.avg_reduce(lvs, d, params, base, norm_t, red, deq)
        torch.cuda.synchronize()
        want = O.avg_tree_reduce(qs, params.seed, base)
        wl, _ = O.pack(want, PACKS[pack])
        got = host(red)
        assert np.array_equal(got[:nb], wl) and np.all(got[nb:] == 0x5A)
        wd = O.avg_reduce_dequantize(want, float(nf), s, K)
        gd = host(deq).astype(np.float64)
        assert np.all(np.abs(gd[:d] - wd) <= RTOL * np.abs(wd))
        assert np.all(gd[:d][want == 0] == 0.0) and np.all(gd[d:] == 7.0)
    for bad in (gq.make_params(1, 7, PACKS["i4"]), gq.make_params(0, 15, PACKS["u4s"])):
        with pytest.raises(gq.GQError) as e:
            gq.avg_reduce(lvs, d, bad, 0, norm_t, red, None)
        assert e.value.status == gq.GQ_ERR_UNSUPPORTED


# ------------------------------------------------------------------------------------ sparse branch
@pytest.mark.parametrize("d", [1, 15, 16, 17, 4095, 4096, 4097, 70_001, (1 << 20) + 3])
@pytest.mark.parametrize("density", [0.0, 0.02, 0.5, 1.0])
def test_compact_matches_oracle(d, density):
    rng = np.random.default_rng(d % 1000 + int(density * 100))
    q = rng.integers(-127, 128, d).astype(np.int32)
    q[q == 0] = 1
    q[rng.random(d) >= density] = 0
    lv = torch.from_numpy(q.astype(np.int8)).to(DEV)
    n, widx, wval = O.compact(q)
    params = gq.make_params(0, 127, 0, 0, seed=0)
    cap = d + 5
    idx = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    val = torch.full((cap,), 0x5A, dtype=torch.int8, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    nts = gq.tile_starts_len(d)
    starts = torch.full((nts + 4,), -1, dtype=torch.int32, device=DEV)
    gq.compact(lv, d, params, idx, val, cnt, tile_starts_out=starts)
    torch.cuda.synchronize()
    assert int(cnt.item()) == n
    gi, gv = host(idx).view(np.uint32), host(val)
    assert np.array_equal(gi[:n], widx) and np.array_equal(gv[:n].astype(np.int32), wval)
    assert np.all(gi[n:] == 0xFFFFFFFF) and np.all(gv[n:] == 0x5A)          # nothing written past the count
    # the table of tile starts: entry t = how many of the oracle's indices lie below 4096 t; the last entry is the count
    gs = host(starts).view(np.uint32)
    assert nts == (d + 4095) // 4096 + 1
    assert np.array_equal(gs[:nts], np.searchsorted(widx.astype(np.int64), 4096 * np.arange(nts, dtype=np.int64)).astype(np.uint32))
    assert gs[nts - 1] == n and np.all(gs[nts:] == 0xFFFFFFFF)
    if n > 3:                                                                # a short buffer: true count, first entries
        idx2 = torch.full((3 + 4,), -1, dtype=torch.int32, device=DEV)[:3]
        val2 = torch.full((3 + 4,), 0x5A, dtype=torch.int8, device=DEV)[:3]
        gq.compact(lv, d, params, idx2, val2, cnt)
        torch.cuda.synchronize()
        assert int(cnt.item()) == n and np.array_equal(host(idx2).view(np.uint32), widx[:3])


def test_compact_errors():
    lv = torch.zeros(64, dtype=torch.int8, device=DEV)
    idx = torch.zeros(64, dtype=torch.int32, device=DEV)
    val = torch.zeros(64, dtype=torch.int8, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    with pytest.raises(gq.GQError) as e:
        gq.compact(lv, 64, gq.make_params(0, 7, PACKS["i4"]), idx, val, cnt)
    assert e.value.status == gq.GQ_ERR_UNSUPPORTED
    big = torch.zeros(1 << 20, dtype=torch.int8, device=DEV)
    with pytest.raises(gq.GQError) as e:
        gq.compact(big, 1 << 20, gq.make_params(0, 127), idx, val, cnt, workspace=torch.zeros(8, dtype=torch.uint8, device=DEV))
    assert e.value.status == gq.GQ_ERR_WORKSPACE
    assert gq.compact_workspace_bytes(-1) == 0 and gq.compact_workspace_bytes(1 << 33) == 0
    assert gq.compact_workspace_bytes(0) == 16 and gq.compact_workspace_bytes(32769) == 40
    gq.compact(lv, 0, gq.make_params(0, 127), idx, val, cnt)                # d = 0: count 0
    torch.cuda.synchronize()
    assert int(cnt.item()) == 0


def check_quantize_compact(x, xh, nf, norm_t, scheme, s, seed, worker, base, rng_bits):
    """gq_quantize_compact against the oracle's quantisation followed by its compaction: count, list, tile starts, guards."""
    d = x.numel()
    p = gq.make_params(SCHEMES[scheme], s, 0, 0, seed=seed, rng_bits=rng_bits)
    q = O.quantize(xh, nf, SCHEMES[scheme], s, seed, worker, base, rng_bits=rng_bits)
    n, widx, wval = O.compact(q)
    cap = n + 7
    idx = torch.full((cap,), -1, dtype=torch.int32, device=DEV)
    val = torch.full((cap,), 0x5A, dtype=torch.int8, device=DEV)
    cnt = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    nts = gq.tile_starts_len(d)
    starts = torch.full((nts + 4,), -1, dtype=torch.int32, device=DEV)
    gq.quantize_compact(x, norm_t, p, worker, base, idx, val, cnt, tile_starts_out=starts)
    torch.cuda.synchronize()
    assert int(cnt.item()) == n
    gi, gv = host(idx).view(np.uint32), host(val)
    assert np.array_equal(gi[:n], widx) and np.array_equal(gv[:n].astype(np.int32), wval)
    assert np.all(gi[n:] == 0xFFFFFFFF) and np.all(gv[n:] == 0x5A)
    gs = host(starts).view(np.uint32)
    assert np.array_equal(gs[:nts], np.searchsorted(widx.astype(np.int64), 4096 * np.arange(nts, dtype=np.int64)).astype(np.uint32))
    assert np.all(gs[nts:] == 0xFFFFFFFF)
    return n


@pytest.mark.parametrize("rng_bits", [32, 16])
@pytest.mark.parametrize("scheme,s,kind", [("linear", 127, "linf"), ("linear", 15, "l2"), ("exp", 7, "l2"), ("exp", 16, "linf")])
@pytest.mark.parametrize("d", [1, 5, 4095, 4097, 32_768, 32_771, 70_001, 1_048_579])
def test_quantize_compact_matches_oracle(scheme, s, kind, d, rng_bits):
    # the sender without dense codes: one span, a ragged span, many spans with a ragged tail; a bucket offset
    x = gaussians(1, d, seed=d + s)[0]
    xh = host(x)
    _, nf, _ = oracle_norm([x], NORMS[kind])
    norm_t = dev_scalar(float(nf))
    total = 0
    for worker, base in ((0, 0), (3, 8 * 12_345)):
        total += check_quantize_compact(x, xh, nf, norm_t, scheme, s, 777, worker, base, rng_bits)
    if d >= 4095:
        assert total > 0


def test_quantize_compact_bucket_offsets_unusable_norm_and_short_buffers():
    d = 100_003
    x = gaussians(1, d, seed=5)[0]
    xh = host(x)
    _, nf, _ = oracle_norm([x], NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    # the Philox call index crosses a multiple of 2^32 inside the gradient (full draws: 2^34 coordinates, short: 2^35)
    for rng_bits, top in ((32, 1 << 34), (16, 1 << 35)):
        for base in (top - 8 * 1000, top - 8, top, 3 * top - 8 * 9_000):
            check_quantize_compact(x, xh, nf, norm_t, "linear", 127, 31337, 2, base, rng_bits)
            check_quantize_compact(x, xh, nf, norm_t, "exp", 12, 31337, 2, base, rng_bits)
    # the same list as gq_quantize followed by gq_compact on the GPU
    p = gq.make_params(0, 127, 0, 0, seed=9)
    lv = gpu_quantize(x, norm_t, p, 1, 64)[0]
    n_max = d
    outs = []
    for call in ("two", "one"):
        idx = torch.zeros(n_max, dtype=torch.int32, device=DEV); val = torch.zeros(n_max, dtype=torch.int8, device=DEV)
        cnt = torch.zeros(1, dtype=torch.int64, device=DEV); st = torch.zeros(gq.tile_starts_len(d), dtype=torch.int32, device=DEV)
        if call == "two":
            gq.compact(lv, d, p, idx, val, cnt, tile_starts_out=st)
        else:
            gq.quantize_compact(x, norm_t, p, 1, 64, idx, val, cnt, tile_starts_out=st)
        outs.append((idx, val, cnt, st))
    torch.cuda.synchronize()
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    n = int(outs[0][2].item())
    # a list buffer that is too short: the true count, the first entries, nothing beyond
    idx2 = torch.full((3 + 4,), -1, dtype=torch.int32, device=DEV); val2 = torch.full((3 + 4,), 0x5A, dtype=torch.int8, device=DEV)
    cnt2 = torch.zeros(1, dtype=torch.int64, device=DEV)
    gq.quantize_compact(x, norm_t, p, 1, 64, idx2[:3], val2[:3], cnt2)
    torch.cuda.synchronize()
    assert int(cnt2.item()) == n and torch.equal(idx2[:3], outs[0][0][:3]) and bool((idx2[3:] == -1).all()) and bool((val2[3:] == 0x5A).all())
    # an unusable norm: no entries; NaN coordinates under a usable norm follow the oracle
    for bad in (0.0, float("nan"), float("inf")):
        cnt3 = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        gq.quantize_compact(x, dev_scalar(bad), p, 0, 0, idx2[:3], val2[:3], cnt3)
        torch.cuda.synchronize()
        assert int(cnt3.item()) == 0
    xn = x.clone(); xn[17] = float("nan"); xn[4099] = float("inf"); xn[d - 1] = float("-inf")
    check_quantize_compact(xn, host(xn), nf, norm_t, "linear", 127, 9, 0, 0, 32)
    check_quantize_compact(xn, host(xn), nf, norm_t, "exp", 7, 9, 0, 0, 16)
    # argument errors
    with pytest.raises(gq.GQError) as e:
        gq.quantize_compact(x, norm_t, gq.make_params(0, 7, PACKS["i4"]), 0, 0, idx2, val2, cnt2)
    assert e.value.status == gq.GQ_ERR_UNSUPPORTED
    with pytest.raises(gq.GQError) as e:
        gq.quantize_compact(x, norm_t, p, 0, 2, idx2, val2, cnt2)
    assert e.value.status == gq.GQ_ERR_INVALID_ARG
    with pytest.raises(gq.GQError) as e:
        gq.quantize_compact(x, norm_t, gq.make_params(0, 127, rng_bits=16), 0, 4, idx2, val2, cnt2)
    assert e.value.status == gq.GQ_ERR_INVALID_ARG
    with pytest.raises(gq.GQError) as e:
        gq.quantize_compact(x, norm_t, p, 0, 0, idx2, val2, cnt2, workspace=torch.zeros(8, dtype=torch.uint8, device=DEV))
    assert e.value.status == gq.GQ_ERR_WORKSPACE
    empty = torch.zeros(0, dtype=torch.float32, device=DEV)
    cnt4 = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    gq.quantize_compact(empty, norm_t, p, 0, 0, idx2, val2, cnt4)
    torch.cuda.synchronize()
    assert int(cnt4.item()) == 0


def test_quantize_compact_equals_the_two_calls_on_random_shapes():
    # 150 seeded cases over lengths (1 .. 3e6), both grids, every s, both draw widths, bucket offsets up to and across the
    # points where the Philox call index passes 2^32, scaled and zero-riddled gradients, norms above and below the largest
    # coordinate: list, count, table and guard entries are those of gq_quantize followed by gq_compact, bit for bit
    # (which the tests above compare with the oracle)
    rng = np.random.default_rng(7)
    g = torch.Generator(device=DEV).manual_seed(5)
    for it in range(150):
        d = int(rng.choice([rng.integers(1, 70), rng.integers(1, 40_000), rng.integers(1, 3_000_000)]))
        scheme = int(rng.integers(0, 2))
        s = int(rng.integers(1, 128)) if scheme == 0 else int(rng.integers(1, 32))
        bits = int(rng.choice([32, 16]))
        base = int(rng.integers(0, 1 << 33)) * 8
        if rng.random() < 0.2:
            base = max((1 << (34 if bits == 32 else 35)) - 8 * int(rng.integers(0, d // 8 + 2)), 0)
        worker = int(rng.integers(0, 64))
        x = torch.randn(d, generator=g, device=DEV) * float(10 ** rng.uniform(-6, 0))
        if rng.random() < 0.3:
            x[torch.rand(d, generator=g, device=DEV) < 0.9] = 0.0
        norm = torch.zeros(1, device=DEV)
        gq.global_norm([x], int(rng.integers(0, 2)), norm, torch.zeros(1, dtype=torch.int32, device=DEV))
        if rng.random() < 0.3:
            norm *= float(rng.uniform(0.3, 30))
        p = gq.make_params(scheme, s, 0, 0, seed=int(rng.integers(0, 1 << 62)), rng_bits=bits)
        lv = torch.empty(d, dtype=torch.uint8, device=DEV)
        gq.quantize(x, norm, p, worker, base, lv)
        outs = []
        for fused in (False, True):
            idx = torch.full((d + 3,), -1, dtype=torch.int32, device=DEV)
            val = torch.full((d + 3,), 0x5A, dtype=torch.int8, device=DEV)
            cnt = torch.full((1,), -1, dtype=torch.int64, device=DEV)
            tab = torch.full((gq.tile_starts_len(d) + 2,), -1, dtype=torch.int32, device=DEV)
            if fused:
                gq.quantize_compact(x, norm, p, worker, base, idx, val, cnt, tile_starts_out=tab)
            else:
                gq.compact(lv, d, p, idx, val, cnt, tile_starts_out=tab)
            outs.append((idx, val, cnt, tab))
        torch.cuda.synchronize()
        case = (it, d, scheme, s, bits, base, worker)
        assert all(torch.equal(a, b) for a, b in zip(outs[0], outs[1])), case
        assert int(outs[0][2].item()) == int(torch.count_nonzero(lv)), case


@pytest.mark.parametrize("scheme,s,kind", [("linear", 15, "l2"), ("linear", 127, "linf"), ("exp", 7, "l2")])
@pytest.mark.parametrize("K,d", [(1, 1000), (4, 70_001), (16, 300_000)])
def test_sparse_path_equals_dense_aggregate(scheme, s, kind, K, d):
    # quantize -> compact each worker -> add the K lists: the same integer sum as the dense path
    xs = gaussians(K, d, seed=K + d)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS[kind])
    norm_t = dev_scalar(float(nf))
    p = gq.make_params(SCHEMES[scheme], s, 0, 0, seed=4242)
    lvs = [gpu_quantize(xs[i], norm_t, p, i, 0)[0] for i in range(K)]
    dense = torch.zeros(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, dense)
    idxs, vals, cnts = [], [], []
    total = 0
    for i in range(K):
        q = O.quantize(xh[i], nf, SCHEMES[scheme], s, 4242, i, 0)
        n, widx, wval = O.compact(q)
        idx = torch.zeros(max(n, 1), dtype=torch.int32, device=DEV)
        val = torch.zeros(max(n, 1), dtype=torch.int8, device=DEV)
        cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
        gq.compact(lvs[i], d, p, idx, val, cnt)
        torch.cuda.synchronize()
        assert int(cnt.item()) == n
        assert np.array_equal(host(idx).view(np.uint32)[:n], widx) and np.array_equal(host(val)[:n].astype(np.int32), wval)
        idxs.append(idx); vals.append(val); cnts.append(cnt); total += n
    agg = torch.full((d + 8,), 0x5A5A, dtype=torch.int32, device=DEV)
    gq.sparse_aggregate(idxs, vals, cnts, d, p, agg)
    torch.cuda.synchronize()
    assert torch.equal(agg[:d], dense) and bool((agg[d:] == 0x5A5A).all())
    want = O.quantize_aggregate(xh, nf, SCHEMES[scheme], s, 4242, 0)
    assert np.array_equal(host(agg)[:d].astype(np.int64), want)
    # the same with the senders' tables of tile starts (no searches), and with a table for some workers only
    tabs = []
    for i in range(K):
        t = torch.zeros(gq.tile_starts_len(d), dtype=torch.int32, device=DEV)
        gq.compact(lvs[i], d, p, idxs[i], vals[i], cnts[i], tile_starts_out=t)
        tabs.append(t)
    for given in (tabs, [t if i % 2 == 0 else None for i, t in enumerate(tabs)]):
        agg2 = torch.full((d + 8,), 0x5A5A, dtype=torch.int32, device=DEV)
        gq.sparse_aggregate(idxs, vals, cnts, d, p, agg2, tile_starts=given)
        torch.cuda.synchronize()
        assert torch.equal(agg2, agg)
    # lists cut short by their capacity: what was written is summed, with or without the table
    if K > 1 and total > 8 * K:
        short = [idx[:max(int(c.item()) // 2, 1)] for idx, c in zip(idxs, cnts)]
        short_v = [v[:s_.numel()] for v, s_ in zip(vals, short)]
        a1 = torch.zeros(d, dtype=torch.int32, device=DEV); a2 = torch.zeros(d, dtype=torch.int32, device=DEV)
        gq.sparse_aggregate(short, short_v, cnts, d, p, a1)
        gq.sparse_aggregate(short, short_v, cnts, d, p, a2, tile_starts=tabs)
        torch.cuda.synchronize()
        wi = [host(s_).view(np.uint32) for s_ in short]
        wv = [host(v).astype(np.int32) for v in short_v]
        assert np.array_equal(host(a1).astype(np.int64), O.sparse_aggregate(wi, wv, d, SCHEMES[scheme]))
        assert torch.equal(a1, a2)
    if kind == "l2" and scheme == "linear" and K * d > 10000:
        # the sparse regime the paper's Theorem 1 speaks of: far fewer non-zeros than coordinates,
        # within the bound that follows from Eq. (2), s^2 + s*sqrt(nd)
        assert total <= 1.2 * (s * s + s * np.sqrt(K * d)) and total < 0.2 * K * d


def test_step_replays_from_a_hip_graph():
    # every call only enqueues on the given stream (no allocation, no synchronisation, no memset), so the
    # whole step can be captured once and replayed; each replay is compared with the eager result on fresh data
    K, d = 8, 300_001
    xs = gaussians(K, d, seed=21)
    p = gq.make_params(0, 127, 0, 0, seed=77)
    norm_t = dev_scalar(0.0)
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = torch.empty(gq.norm_workspace_bytes(K, d), dtype=torch.uint8, device=DEV)
    agg = torch.zeros(d, dtype=torch.int32, device=DEV)
    out = torch.zeros(d, device=DEV)
    cidx = torch.zeros(d, dtype=torch.int32, device=DEV)
    cval = torch.zeros(d, dtype=torch.int8, device=DEV)
    ccnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    cws = torch.empty(gq.compact_workspace_bytes(d), dtype=torch.uint8, device=DEV)
    lv0 = torch.zeros(d, dtype=torch.uint8, device=DEV)

    def step():
        gq.global_norm(xs, NORMS["l2"], norm_t, flags, ws)
        gq.fused_quantize_aggregate(xs, norm_t, p, 0, agg, None)
        gq.dequantize(agg, d, norm_t, p, K, out)
        gq.quantize(xs[0], norm_t, p, 0, 0, lv0)
        gq.compact(lv0, d, p, cidx, cval, ccnt, cws)

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cpu").manual_seed(5)
    for rep in range(4):
        for x in xs:                                     # new gradients in the captured buffers
            x.copy_((torch.randn(d, generator=gen) * (1e-3 * (rep + 1))).to(DEV))
        agg.fill_(-1); out.fill_(-1.0); norm_t.fill_(-1.0); ccnt.fill_(-1)
        g.replay()
        torch.cuda.synchronize()
        got = (norm_t.clone(), agg.clone(), out.clone(), ccnt.clone(), cidx.clone())
        agg.fill_(-2); out.fill_(-2.0); norm_t.fill_(-2.0); ccnt.fill_(-2)
        step()
        torch.cuda.synchronize()
        assert torch.equal(got[0], norm_t) and torch.equal(got[1], agg) and torch.equal(got[2], out)
        assert torch.equal(got[3], ccnt) and torch.equal(got[4][:int(ccnt.item())], cidx[:int(ccnt.item())])
        assert float(norm_t.item()) > 0 and int(agg.abs().max()) > 0


def test_unbiased_on_gpu_monte_carlo():
    # E[G(x)] = mean of the workers (Definition 3), measured on the GPU path alone over many seeds
    K, d, T = 4, 2048, 400
    xs = gaussians(K, d, seed=123, std=1e-3)
    xbar = np.mean(np.stack([host(x).astype(np.float64) for x in xs]), axis=0)
    norm_t = dev_scalar(0.0)
    gq.global_norm(xs, NORMS["linf"], norm_t)
    nrm = float(host(norm_t)[0])
    for scheme, s in [("linear", 15), ("exp", 7)]:
        acc = torch.zeros(d, dtype=torch.float64, device=DEV)
        out = torch.zeros(d, device=DEV)
        for t in range(T):
            params = gq.make_params(SCHEMES[scheme], s, 0, 0, seed=1000 + t)
            gq.fused_quantize_aggregate(xs, norm_t, params, 0, None, out)
            acc += out.double()
        mean = host(acc) / T
        step = nrm / s if scheme == "linear" else nrm       # a bound on the per-worker rounding error
        assert np.all(np.abs(mean - xbar) <= 5.0 * 0.5 * step / np.sqrt(K * T))


# ------------------------------------------------------------------------------------ workloads
def check_windows(xs, agg, nf, scheme, s, seed, windows, width, rng_bits=32):
    d = xs[0].numel()
    for lo in windows:
        lo = max(0, min(lo, d - width)) & ~7
        hi = min(d, lo + width)
        want = O.quantize_aggregate([host(x[lo:hi]) for x in xs], nf, scheme, s, seed, lo, rng_bits=rng_bits)
        assert np.array_equal(host(agg[lo:hi]).astype(np.int64), want), "window at %d" % lo


@pytest.mark.parametrize("scheme,s,agg_fmt,K,d,rng_bits", [(0, 127, 0, 12, 21_000_003, 32), (1, 7, 1, 24, 10_500_001, 32),
                                                           (0, 63, 0, 8, 31_300_002, 32), (1, 12, 0, 19, 13_200_001, 32),
                                                           (0, 127, 0, 16, 16_000_005, 16), (1, 7, 1, 32, 8_000_003, 16),
                                                           (0, 15, 0, 11, 23_000_001, 16)])
def test_fused_large_launches_equal_small_buckets_and_oracle(scheme, s, agg_fmt, K, d, rng_bits):
    # Launches with K * d >= 2.5e8 take the kernel variant that bounds its loads in flight and stores
    # inside time windows; the same gradient cut into buckets below that size takes the plain variant.
    # Both must give the same integers, and those of the oracle on sampled windows.
    g = torch.Generator(device=DEV).manual_seed(1000 * K + s)
    xs = [torch.randn(d, generator=g, device=DEV) * 1e-3 for _ in range(K)]
    mx = max(float(x.abs().max()) for x in xs)
    nf = np.float32(mx)
    norm_t = dev_scalar(float(nf))
    params = gq.make_params(scheme, s, 0, agg_fmt, seed=SI.QUANT_SEED + 1, rng_bits=rng_bits)
    adt = torch.int16 if agg_fmt == 1 else torch.int32
    whole = torch.full((d + 8,), 0x5A5A, dtype=adt, device=DEV)
    whole_deq = torch.full((d + 8,), 7.0, device=DEV)
    gq.fused_quantize_aggregate(xs, norm_t, params, 0, whole, whole_deq)
    parts = torch.empty(d, dtype=adt, device=DEV)
    parts_deq = torch.empty(d, device=DEV)
    step = (int(2.0e8 / K) // 16) * 16
    assert K * step < 2.5e8 <= K * d
    for lo in range(0, d, step):
        hi = min(d, lo + step)
        gq.fused_quantize_aggregate([x[lo:hi] for x in xs], norm_t, params, lo, parts[lo:hi], parts_deq[lo:hi])
    # and the same launch with the windows switched off by the caller
    off = gq.make_params(scheme, s, 0, agg_fmt, seed=SI.QUANT_SEED + 1, rng_bits=rng_bits, flags=gq.GQ_FLAG_WRITE_WINDOWS_OFF)
    plain = torch.empty(d, dtype=adt, device=DEV)
    gq.fused_quantize_aggregate(xs, norm_t, off, 0, plain, None)
    torch.cuda.synchronize()
    assert torch.equal(whole[:d], parts) and torch.equal(whole_deq[:d], parts_deq) and torch.equal(whole[:d], plain)
    assert bool((whole[d:] == 0x5A5A).all()) and bool((whole_deq[d:] == 7.0).all())
    rng = np.random.default_rng(K)
    wins = [0, d - (1 << 15)] + [int(v) for v in rng.integers(0, d - (1 << 15), 6)]
    check_windows(xs, whole[:d], nf, scheme, s, params.seed, wins, 1 << 15, rng_bits=rng_bits)


@pytest.mark.parametrize("rng_bits", [32, 16])
@pytest.mark.parametrize("scheme,s,agg_fmt", [(0, 127, 0), (1, 7, 1)])
@pytest.mark.parametrize("K,d", [(1, 4099), (3, 70_001), (4, 8_191), (8, 300_003), (16, 70_000), (33, 5_001), (64, 1_000)])
def test_write_windows_forced_on_and_off_change_no_result(scheme, s, agg_fmt, K, d, rng_bits):
    # gq_params.flags: the time windows in which the fused kernel stores its sums change timing only.  Forced on
    # in small launches (where the library would not use them, every worker count and the run-time-K path) and forced
    # off, the integers and the means are those of the default policy and of the oracle.
    xs = gaussians(K, d, seed=K + d)
    xh = [host(x) for x in xs]
    _, nf, _ = oracle_norm(xs, NORMS["linf"])
    norm_t = dev_scalar(float(nf))
    base = 8 * 4242
    want = O.quantize_aggregate(xh, nf, scheme, s, 77, base, rng_bits=rng_bits)
    outs = []
    for flags in (0, gq.GQ_FLAG_WRITE_WINDOWS_ON, gq.GQ_FLAG_WRITE_WINDOWS_OFF):
        params = gq.make_params(scheme, s, 0, agg_fmt, seed=77, rng_bits=rng_bits, flags=flags)
        agg_out, deq_out, _, _ = run_fused(xs, norm_t, params, base, False)
        got = host(agg_out)
        assert np.array_equal(got[:d].astype(np.int64), want) and np.all(got[d:] == 0x5A5A)
        outs.append((agg_out, deq_out))
    assert all(torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1]) for o in outs[1:])
    with pytest.raises(gq.GQError) as e:
        run_fused(xs, norm_t, gq.make_params(scheme, s, 0, agg_fmt, seed=77, flags=3), base, False)
    assert e.value.status == gq.GQ_ERR_INVALID_ARG


def test_workload_c1_full_parity():
    # d = 2^20, K = 4, L2 norm, linear s = 127, int8 codes, int32 sum: everything compared in full
    cfg = SI.CONFIGS["c1"]
    xs = SI.make_workers("c1", device=DEV)
    K, d = cfg["K"], cfg["d"]
    ne, nf, _ = oracle_norm(xs, NORMS["l2"])
    norm_gpu = dev_scalar(0.0)
    gq.global_norm(xs, NORMS["l2"], norm_gpu)
    assert abs(float(host(norm_gpu)[0]) - ne) <= RTOL * ne
    params = gq.make_params(0, 127, 0, 0, seed=SI.QUANT_SEED)
    norm_t = dev_scalar(float(nf))
    agg, deq, lvs, _ = run_fused(xs, norm_t, params, 0, True)
    want = O.quantize_aggregate([host(x) for x in xs], nf, 0, 127, SI.QUANT_SEED, 0)
    assert np.array_equal(host(agg)[:d].astype(np.int64), want)
    wd = O.dequantize(want, float(nf), 0, 127, K)
    assert np.all(np.abs(host(deq)[:d] - wd) <= RTOL * np.abs(wd))
    for i in range(K):
        q = O.quantize(host(xs[i]), nf, 0, 127, SI.QUANT_SEED, i, 0)
        assert np.array_equal(host(lvs[i])[:d].view(np.int8), q.astype(np.int8))


def test_workload_c3_sampled_parity_at_bench_shape():
    # the scored call: d = 110e6, K = 16, max norm, linear s = 127, int32 sum -- the launch the
    # benchmark times -- compared with the oracle on windows (the random stream is a function of the
    # coordinate index, so the oracle can evaluate any window on its own)
    cfg = SI.CONFIGS["c3"]
    K, d = cfg["K"], cfg["d"]
    xs = SI.make_workers("c3", device=DEV)
    norm_t = dev_scalar(0.0)
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)
    gq.global_norm(xs, NORMS["linf"], norm_t, flags)
    torch.cuda.synchronize()
    mx = max(float(x.abs().max()) for x in xs)
    assert float(host(norm_t)[0]) == mx and int(host(flags)[0]) == 0      # max norm is exact
    nf = np.float32(mx)
    params = gq.make_params(0, 127, 0, 0, seed=SI.QUANT_SEED)
    agg = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.fused_quantize_aggregate(xs, norm_t, params, 0, agg)
    torch.cuda.synchronize()
    # the oracle on the first and the last 2^20 coordinates and on 64 random windows of 2^16
    rng = np.random.default_rng(3)
    check_windows(xs, agg, nf, 0, 127, SI.QUANT_SEED, [0, d - (1 << 20)], 1 << 20)
    check_windows(xs, agg, nf, 0, 127, SI.QUANT_SEED, [int(v) for v in rng.integers(0, d - (1 << 16), 64)], 1 << 16)
    # properties that hold at any size: bound by n*s, sign pattern, and the sum of the sums against
    # the exact expectation s/norm * sum_i sum_j x_ij within 6 standard deviations
    assert int(agg.abs().max()) <= K * 127
    tot = float(agg.double().sum())
    expect = sum(float(x.double().sum()) for x in xs) * 127.0 / float(nf)
    assert abs(tot - expect) <= 6.0 * 0.5 * np.sqrt(K * d)
