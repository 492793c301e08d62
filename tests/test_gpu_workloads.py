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


# ------------------------------------------------------------------------------------ sparse branch at full size
def list_window(idx, lo, hi):
    """Positions [a, b) of the entries of the sorted device index list `idx` (int32 storage of uint32 values)
    whose coordinate lies in [lo, hi)."""
    wide = idx.to(torch.int64) & 0xFFFFFFFF
    edge = torch.tensor([lo, hi], dtype=torch.int64, device=idx.device)
    a, b = torch.searchsorted(wide, edge).tolist()
    return a, b


def compact_with_guard(lv, d, p, ws, starts=None):
    """gq_compact into buffers sized by a first counting call, with 8 guard entries behind them."""
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    probe_i = torch.empty(1, dtype=torch.int32, device=DEV)
    probe_v = torch.empty(1, dtype=torch.int8, device=DEV)
    gq.compact(lv, d, p, probe_i, probe_v, cnt, ws)
    torch.cuda.synchronize()
    n = int(cnt.item())
    idx = torch.full((n + 8,), -1, dtype=torch.int32, device=DEV)
    val = torch.full((n + 8,), 0x5A, dtype=torch.int8, device=DEV)
    cnt.fill_(-1)
    gq.compact(lv, d, p, idx, val, cnt, ws, tile_starts_out=starts)
    torch.cuda.synchronize()
    assert int(cnt.item()) == n
    assert bool((idx[n:] == -1).all()) and bool((val[n:] == 0x5A).all())       # nothing written past the count
    return n, idx, val, cnt


@pytest.mark.parametrize("kind", ["linf", "l2"])
def test_workload_c3_sparse_branch_at_full_size(kind):
    # Algorithm 1's sparse branch at the scored shape (d = 110e6, K = 16, linear s = 127, int8 codes): the block
    # scan runs over the 3357 spans of one worker, far more than are resident at once, which smaller inputs never reach.
    # Max norm: about 16 % of the codes are non-zero; L2 norm: about 0.05 % (the regime of Theorem 1).
    cfg = SI.CONFIGS["c3"]
    K, d, s = cfg["K"], cfg["d"], cfg["s"]
    xs = SI.make_workers("c3", device=DEV)
    nf = np.float32(torch_norm(xs, kind))
    norm_t = torch.tensor([float(nf)], device=DEV)
    p = gq.make_params(gq.GQ_LINEAR, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    lvs = [torch.empty(d, dtype=torch.uint8, device=DEV) for _ in range(K)]
    for i in range(K):
        gq.quantize(xs[i], norm_t, p, i, 0, lvs[i])
    dense = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, dense)
    ws = torch.empty(gq.compact_workspace_bytes(d), dtype=torch.uint8, device=DEV)
    assert gq.compact_workspace_bytes(d) == 8 * (2 + 3357 + 53)
    idxs, vals, cnts, total = [], [], [], 0
    windows = spans(d, 33, edges=[1024 * 16384 * r for r in range(1, 7)])
    tabs = []
    edges = torch.arange(gq.tile_starts_len(d), dtype=torch.int64, device=DEV) * 4096
    for i in range(K):
        tab = torch.full((gq.tile_starts_len(d),), -1, dtype=torch.int32, device=DEV)
        n, idx, val, cnt = compact_with_guard(lvs[i], d, p, ws, tab)
        idxs.append(idx[:n]); vals.append(val[:n]); cnts.append(cnt); tabs.append(tab); total += n
        assert n == int(torch.count_nonzero(lvs[i]))
        # the table of tile starts is the position of every multiple of 4096 in the (oracle-checked) index list
        assert torch.equal(tab.to(torch.int64) & 0xFFFFFFFF, torch.searchsorted(idx[:n].to(torch.int64) & 0xFFFFFFFF, edges))
        # the sender without stored codes: count, list (with guards behind it) and table, bit for bit those of the two calls
        idx1 = torch.full((n + 8,), -1, dtype=torch.int32, device=DEV)
        val1 = torch.full((n + 8,), 0x5A, dtype=torch.int8, device=DEV)
        cnt1 = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        tab1 = torch.full((gq.tile_starts_len(d),), -1, dtype=torch.int32, device=DEV)
        gq.quantize_compact(xs[i], norm_t, p, i, 0, idx1, val1, cnt1, ws, tile_starts_out=tab1)
        torch.cuda.synchronize()
        assert int(cnt1.item()) == n and torch.equal(idx1, idx) and torch.equal(val1, val) and torch.equal(tab1, tab), i
        del idx1, val1, tab1
        if i in (0, K - 1):
            # the sender in full against the oracle: its own codes from the same gradient, its own list
            q = O.quantize(host(xs[i]), nf, O.LINEAR, s, SI.QUANT_SEED, i, 0)
            assert np.array_equal(host(lvs[i]).view(np.int8), q.astype(np.int8))
            n_o, widx, wval = O.compact(q)
            assert n == n_o
            assert np.array_equal(host(idx[:n]).view(np.uint32), widx)
            assert np.array_equal(host(val[:n]).astype(np.int32), wval)
            del q, widx, wval
        else:
            # on windows: the list restricted to the window is the oracle's list of the window, and it sits at
            # the position given by the number of non-zero codes before the window
            for lo, hi in windows:
                q = O.quantize(host(xs[i][lo:hi]), nf, O.LINEAR, s, SI.QUANT_SEED, i, lo)
                n_w, widx, wval = O.compact(q)
                a, b = list_window(idx[:n], lo, hi)
                assert b - a == n_w and a == int(torch.count_nonzero(lvs[i][:lo])), (i, lo)
                assert np.array_equal(host(idx[a:b]).view(np.uint32).astype(np.int64), widx.astype(np.int64) + lo)
                assert np.array_equal(host(val[a:b]).astype(np.int32), wval)
    frac = total / (float(K) * d)
    assert (0.10 < frac < 0.25) if kind == "linf" else (0.0002 < frac < 0.002)      # about 16 % and 0.05 %
    if kind == "l2":
        assert total <= 1.2 * (s * s + s * np.sqrt(float(K) * d))               # the bound Eq. (2) implies
        assert gq.sparse_nnz_bound(p, K, d) == s * s + s * np.sqrt(float(K) * d)  # and what the library sizes lists by
    # the receiver: the K lists add up to the dense integer sum over every coordinate, and to the oracle's on windows
    agg = torch.full((d + 8,), 0x5A5A, dtype=torch.int32, device=DEV)
    gq.sparse_aggregate(idxs, vals, cnts, d, p, agg)
    torch.cuda.synchronize()
    assert torch.equal(agg[:d], dense) and bool((agg[d:] == 0x5A5A).all())
    agg_t = torch.full((d + 8,), 0x5A5A, dtype=torch.int32, device=DEV)
    gq.sparse_aggregate(idxs, vals, cnts, d, p, agg_t, tile_starts=tabs)           # with the senders' tables: no searches
    torch.cuda.synchronize()
    assert torch.equal(agg_t, agg)
    del agg_t
    for lo, hi in windows:
        want = O.quantize_aggregate([host(x[lo:hi]) for x in xs], nf, O.LINEAR, s, SI.QUANT_SEED, lo)
        assert np.array_equal(host(agg[lo:hi]).astype(np.int64), want), lo
        # and the oracle's own receiver on the window's part of the lists
        wi, wv = [], []
        for i in range(K):
            a, b = list_window(idxs[i], lo, hi)
            wi.append((host(idxs[i][a:b]).view(np.uint32).astype(np.int64) - lo).astype(np.uint32))
            wv.append(host(vals[i][a:b]).astype(np.int32))
        assert np.array_equal(O.sparse_aggregate(wi, wv, hi - lo, O.LINEAR), want)


def test_sparse_branch_with_32_bit_indices_up_to_the_limit():
    # d = 2^32 - 1, the largest gradient the sparse branch takes: coordinate indices use all 32 bits, the scan
    # runs over 131072 spans.  Two mostly-zero code vectors are built from seeded positions,
    # so the expected lists are the construction itself (sorted positions and their codes); the oracle's
    # compaction and receiver are run on windows of the same vectors.
    torch.cuda.empty_cache()
    d = (1 << 32) - 1
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * (1 << 30):
        pytest.skip("needs 60 GB of free device memory")
    assert gq.compact_workspace_bytes(d) == 8 * (2 + 131072 + 2048) and gq.compact_workspace_bytes(d + 1) == 0
    rng = np.random.default_rng(2032)
    half = 1 << 31
    special = np.array([0, 1, 15, 16, 16383, 16384, 65535, 65536, half - 1, half, half + 1, d - 2, d - 1,
                        16384 * 1024 - 1, 16384 * 1024, 255 * 16384 * 1024 + 5], dtype=np.int64)
    runs = np.concatenate([np.arange(half - 30_000, half + 30_000), np.arange(d - 40_000, d),
                           np.arange(7 * 16384 * 1024 - 5000, 7 * 16384 * 1024 + 5000)])
    p = gq.make_params(gq.GQ_LINEAR, 127, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=0)
    ws = torch.empty(gq.compact_workspace_bytes(d), dtype=torch.uint8, device=DEV)
    lvs, lists, pos_all, val_all = [], [], [], []
    for w in range(2):
        pos = np.unique(np.concatenate([rng.integers(0, d, 3_000_000), special, runs if w == 0 else runs[::3]]))
        val = rng.integers(1, 128, pos.shape[0]).astype(np.int8) * rng.choice(np.array([-1, 1], np.int8), pos.shape[0])
        lv = torch.zeros(d, dtype=torch.int8, device=DEV)
        lv[torch.from_numpy(pos).to(DEV)] = torch.from_numpy(val).to(DEV)
        tab = torch.full((gq.tile_starts_len(d),), -1, dtype=torch.int32, device=DEV)
        n, idx, vv, cnt = compact_with_guard(lv, d, p, ws, tab)
        assert n == pos.shape[0]
        assert np.array_equal(host(tab).view(np.uint32).astype(np.int64), np.searchsorted(pos, 4096 * np.arange(gq.tile_starts_len(d), dtype=np.int64)))
        assert np.array_equal(host(idx[:n]).view(np.uint32).astype(np.int64), pos)
        assert np.array_equal(host(vv[:n]), val)
        lvs.append(lv); lists.append((idx[:n], vv[:n], cnt, tab)); pos_all.append(pos); val_all.append(val)
        # the oracle's compaction on windows of the same vector
        for lo, hi in [(0, 1 << 20), (half - (1 << 19), half + (1 << 19)), (d - (1 << 20), d),
                       (255 * 16384 * 1024 - 4096, 255 * 16384 * 1024 + 4096)]:
            n_w, widx, wval = O.compact(host(lv[lo:hi]).astype(np.int32))
            a, b = np.searchsorted(pos, [lo, hi])
            assert n_w == b - a
            assert np.array_equal(host(idx[a:b]).view(np.uint32).astype(np.int64), widx.astype(np.int64) + lo)
            assert np.array_equal(host(vv[a:b]).astype(np.int32), wval)
    # a short buffer: the true count and the first entries
    short_i = torch.full((1000 + 8,), -1, dtype=torch.int32, device=DEV)
    short_v = torch.full((1000 + 8,), 0x5A, dtype=torch.int8, device=DEV)
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    gq.compact(lvs[0], d, p, short_i[:1000], short_v[:1000], cnt, ws)
    torch.cuda.synchronize()
    assert int(cnt.item()) == pos_all[0].shape[0] and torch.equal(short_i[:1000], lists[0][0][:1000])
    assert bool((short_i[1000:] == -1).all()) and bool((short_v[1000:] == 0x5A).all())
    # the receiver: both lists into the dense sum; against the dense path over every coordinate, against the
    # construction (scatter-add of the positions), and against the oracle's receiver on windows
    agg = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.sparse_aggregate([l[0] for l in lists], [l[1] for l in lists], [l[2] for l in lists], d, p, agg)
    agg_t = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.sparse_aggregate([l[0] for l in lists], [l[1] for l in lists], [l[2] for l in lists], d, p, agg_t, tile_starts=[l[3] for l in lists])
    torch.cuda.synchronize()
    assert torch.equal(agg_t, agg)
    del agg_t
    dense = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate([lv.view(torch.uint8) for lv in lvs], None, d, p, dense)
    torch.cuda.synchronize()
    assert torch.equal(agg, dense)
    del dense
    built = torch.zeros(d, dtype=torch.int32, device=DEV)
    for pos, val in zip(pos_all, val_all):
        built.index_add_(0, torch.from_numpy(pos).to(DEV), torch.from_numpy(val.astype(np.int32)).to(DEV))
    assert torch.equal(agg, built)
    del built
    for lo, hi in [(0, 1 << 16), (half - (1 << 15), half + (1 << 15)), (d - (1 << 16), d)]:
        wi, wv = [], []
        for pos, val in zip(pos_all, val_all):
            a, b = np.searchsorted(pos, [lo, hi])
            wi.append((pos[a:b] - lo).astype(np.uint32)); wv.append(val[a:b].astype(np.int32))
        assert np.array_equal(O.sparse_aggregate(wi, wv, hi - lo, O.LINEAR), host(agg[lo:hi]).astype(np.int64))
    del agg, lvs, lists
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------ tree reductions at full size
def test_workload_c4_algorithm_2_at_full_size():
    # Algorithm 2 (the paper's reduce function for exponential dithering) over K = 32 int8 code vectors of
    # d = 350e6 coordinates, the shape of workload c4: reduced (sign, e) codes bit-exact on windows, the mean they
    # stand for to 1e-5, and properties that hold everywhere
    cfg = SI.CONFIGS["c4"]
    K, d, s = cfg["K"], cfg["d"], cfg["s"]
    xs = SI.make_workers("c4", device=DEV)
    nf = np.float32(torch_norm(xs, "linf"))
    norm_t = torch.tensor([float(nf)], device=DEV)
    p = gq.make_params(gq.GQ_EXP, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    lvs = [torch.empty(d, dtype=torch.uint8, device=DEV) for _ in range(K)]
    for i in range(K):
        gq.quantize(xs[i], norm_t, p, i, 0, lvs[i])
    red = torch.empty(d, dtype=torch.int8, device=DEV)
    deq = torch.empty(d, device=DEV)
    gq.exp_reduce(lvs, d, p, 0, norm_t, red, deq)
    torch.cuda.synchronize()
    for lo, hi in spans(d, 44):
        qs = [O.quantize(host(xs[i][lo:hi]), nf, O.EXP, s, SI.QUANT_SEED, i, lo) for i in range(K)]
        for i in (0, 17, K - 1):
            assert np.array_equal(host(lvs[i][lo:hi]).view(np.int8), qs[i].astype(np.int8))
        want = O.exp_tree_reduce(qs, s, SI.QUANT_SEED, lo)
        assert np.array_equal(host(red[lo:hi]).astype(np.int32), want), lo
        wd = O.exp_reduce_dequantize(want, float(nf), K)
        gd = host(deq[lo:hi]).astype(np.float64)
        assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)) and np.all(gd[want == 0] == 0.0)
    # everywhere: exponents stay inside the prescaled range 1 .. s + log2(n'), and a coordinate whose codes
    # are all zero reduces to zero
    assert int(red.abs().max()) <= s + 5
    anyone = torch.zeros(d, dtype=torch.bool, device=DEV)
    for lv in lvs:
        anyone |= lv != 0
    assert not bool((red[~anyone] != 0).any())
    # unbiased for the exact integer sum (Section 4.3): summed over all coordinates along the sign of the exact
    # mean, the error stays within 6 standard deviations.  A node's second moment is at most 9/8 of its exact
    # sum's square, so by induction over the 5 tree levels Var(result_j) <= (9/8)^5 (sum_i |value_ij|)^2.
    agg = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, agg)
    exact = torch.empty(d, device=DEV)
    gq.dequantize(agg, d, norm_t, p, K, exact)
    absval = torch.zeros(d, device=DEV)
    for lv in lvs:
        k = lv.view(torch.int8).abs()
        absval += torch.where(k > 0, torch.exp2(k.float() - 1.0), torch.zeros((), device=DEV))
    absmean = absval.double() * (float(nf) / (K * 2.0 ** (s - 1)))
    torch.cuda.synchronize()
    diff = float(((deq.double() - exact.double()) * torch.sign(exact).double()).sum())
    assert abs(diff) <= 6.0 * np.sqrt((9.0 / 8.0) ** 5 * float((absmean * absmean).sum()))


@pytest.mark.parametrize("pack", ["i8", "i4"])
def test_workload_c3_in_step_averaging_at_full_size(pack):
    # the Implementation section's in-step averaging over K = 16 code vectors of d = 110e6 coordinates (workload c3's
    # shape): int8 codes with s = 127, and packed 4-bit codes with s = 7
    cfg = SI.CONFIGS["c3"]
    K, d = cfg["K"], cfg["d"]
    s = 127 if pack == "i8" else 7
    fmt = gq.GQ_PACK_I8 if pack == "i8" else gq.GQ_PACK_I4
    xs = SI.make_workers("c3", device=DEV)
    nf = np.float32(torch_norm(xs, "linf"))
    norm_t = torch.tensor([float(nf)], device=DEV)
    p = gq.make_params(gq.GQ_LINEAR, s, fmt, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    nb = gq.levels_nbytes(d, fmt)
    lvs = [torch.empty(nb, dtype=torch.uint8, device=DEV) for _ in range(K)]
    for i in range(K):
        gq.quantize(xs[i], norm_t, p, i, 0, lvs[i])
    red = torch.empty(nb, dtype=torch.uint8, device=DEV)
    deq = torch.empty(d, device=DEV)
    gq.avg_reduce(lvs, d, p, 0, norm_t, red, deq)
    torch.cuda.synchronize()
    per = 1 if pack == "i8" else 2
    for lo, hi in spans(d, 55):
        qs = [O.quantize(host(xs[i][lo:hi]), nf, O.LINEAR, s, SI.QUANT_SEED, i, lo) for i in range(K)]
        want = O.avg_tree_reduce(qs, SI.QUANT_SEED, lo)
        wl, _ = O.pack(want, O.PACK_I8 if pack == "i8" else O.PACK_I4)
        assert np.array_equal(host(red[lo // per:(hi + per - 1) // per]), wl), lo
        wd = O.avg_reduce_dequantize(want, float(nf), s, K)
        gd = host(deq[lo:hi]).astype(np.float64)
        assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)) and np.all(gd[want == 0] == 0.0)
    # everywhere: the averaged code never leaves the range of the inputs' codes, and, summed over all coordinates
    # along the sign of the exact mean, the result agrees with the exact mean of the codes within 6 standard
    # deviations of the coin noise (a node adds at most 1/4 of variance, halved in weight at every level above it:
    # less than 1/2 at the root, in units of one code)
    agg = torch.empty(d, dtype=torch.int32, device=DEV)
    gq.int_aggregate(lvs, None, d, p, agg)
    exact = torch.empty(d, device=DEV)
    gq.dequantize(agg, d, norm_t, p, K, exact)
    torch.cuda.synchronize()
    unit = float(nf) / s
    assert float(deq.abs().max()) <= float(nf) * (1 + 1e-6)
    diff = float(((deq.double() - exact.double()) * torch.sign(exact).double()).sum())
    assert abs(diff) <= 6.0 * unit * np.sqrt(d * 0.5)


# ------------------------------------------------------------------------------------ per-bucket schedule
def test_workload_c5_per_bucket_norms_two_streams_equal_the_serial_schedule():
    # c5's shape (d = 1.5e9, K = 8, 22 buckets of 2^26 and one of 23,604,992, linear s = 15) run the way a per-bucket
    # hook runs it: every bucket under its OWN norm.  The schedule with the next bucket's norm on a second stream
    # must give the bits of the serial schedule, which must give the bits of the two calls made bucket by bucket;
    # the oracle checks windows (max norm: exact, so every window; L2 norm: the buckets whose norm equals torch's
    # binary64 reduction rounded once, since one ulp of norm can move a code)
    cfg = SI.CONFIGS["c5"]
    K, d, s, bucket = cfg["K"], cfg["d"], cfg["s"], cfg["bucket"]
    xs = SI.make_workers("c5", device=DEV)
    nb = SI.num_buckets(d, bucket)
    p = gq.make_params(gq.GQ_LINEAR, s, gq.GQ_PACK_U4_SIGNPLANE, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    side = torch.cuda.Stream()
    ws = torch.empty(gq.bucketed_workspace_bytes(K, d, bucket), dtype=torch.uint8, device=DEV)
    for kind_name, kind in (("linf", gq.GQ_NORM_LINF), ("l2", gq.GQ_NORM_L2)):
        # serial schedule
        norms_s = torch.full((nb,), -1.0, device=DEV)
        flags_s = torch.full((nb,), 77, dtype=torch.int32, device=DEV)
        agg_s = torch.empty(d, dtype=torch.int32, device=DEV)
        out_s = torch.empty(d, device=DEV)
        gq.bucketed_quantize_aggregate(xs, bucket, kind, p, norms_s, flags_s, agg_s, out_s, ws)
        torch.cuda.synchronize()
        assert bool((flags_s == 0).all())
        # two streams, three times over buffers refilled with garbage; the result is read by work enqueued on the
        # main stream right behind the call, with no synchronisation in between
        for rep in range(3):
            norms_t = torch.full((nb,), -2.0, device=DEV)
            flags_t = torch.full((nb,), 78, dtype=torch.int32, device=DEV)
            agg_t = torch.full((d,), -7, dtype=torch.int32, device=DEV)
            out_t = torch.full((d,), -7.0, device=DEV)
            gq.bucketed_quantize_aggregate(xs, bucket, kind, p, norms_t, flags_t, agg_t, out_t, ws, side_stream=side)
            got = (norms_t.clone(), agg_t.clone(), out_t.clone(), flags_t.clone())
            torch.cuda.synchronize()
            assert torch.equal(got[0], norms_s) and torch.equal(got[1], agg_s) and torch.equal(got[2], out_s)
            assert torch.equal(got[3], flags_s)
            del norms_t, flags_t, agg_t, out_t, got
        # the two calls made bucket by bucket
        n1 = torch.zeros(1, device=DEV)
        part_a = torch.empty(bucket, dtype=torch.int32, device=DEV)
        part_o = torch.empty(bucket, device=DEV)
        want_norms = []
        for b in range(nb):
            lo, hi = b * bucket, min(d, (b + 1) * bucket)
            xb = [x[lo:hi] for x in xs]
            gq.global_norm(xb, kind, n1)
            gq.fused_quantize_aggregate(xb, n1, p, lo, part_a[:hi - lo], part_o[:hi - lo])
            torch.cuda.synchronize()
            assert float(n1.item()) == float(norms_s[b].item())
            assert torch.equal(part_a[:hi - lo], agg_s[lo:hi]) and torch.equal(part_o[:hi - lo], out_s[lo:hi])
            want_norms.append(torch_norm(xb, kind_name))
        got_norms = host(norms_s).astype(np.float64)
        assert np.all(np.abs(got_norms - np.array(want_norms)) <= RTOL * np.array(want_norms))
        if kind_name == "linf":
            assert np.array_equal(host(norms_s), np.array(want_norms, dtype=np.float32))
        # the oracle on windows, each under the norm of the bucket it lies in
        compared = 0
        for lo, hi in spans(d, 6, edges=[b * bucket for b in range(1, nb)]):
            for b in range(lo // bucket, (hi - 1) // bucket + 1):
                a, e = max(lo, b * bucket), min(hi, (b + 1) * bucket)
                nf = np.float32(want_norms[b])
                if np.float32(got_norms[b]) != nf:
                    continue
                xh = [host(x[a:e]) for x in xs]
                A = O.quantize_aggregate(xh, nf, O.LINEAR, s, SI.QUANT_SEED, a)
                assert np.array_equal(host(agg_s[a:e]).astype(np.int64), A), a
                wd = O.dequantize(A, float(nf), O.LINEAR, s, K)
                gd = host(out_s[a:e]).astype(np.float64)
                assert np.all(np.abs(gd - wd) <= RTOL * np.abs(wd)) and np.all(gd[A == 0] == 0.0)
                compared += 1
        assert compared >= (80 if kind_name == "linf" else 40)
        del agg_s, out_s
    # the short form: d below one bucket, and a single-bucket call with a side stream (nothing to overlap)
    small = [x[:100_003] for x in xs]
    norms = torch.zeros(1, device=DEV)
    o1 = torch.empty(100_003, device=DEV)
    o2 = torch.empty(100_003, device=DEV)
    gq.bucketed_quantize_aggregate(small, bucket, gq.GQ_NORM_LINF, p, norms, None, None, o1)
    gq.bucketed_quantize_aggregate(small, bucket, gq.GQ_NORM_LINF, p, norms, None, None, o2, side_stream=side)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and float(norms.item()) == max(float(x.abs().max()) for x in small)


def test_per_bucket_schedule_replays_from_a_hip_graph():
    # the two-stream schedule forks and joins its side stream with events inside the call, so the whole call can be
    # captured from the main stream and replayed; every replay is compared with the eager serial schedule on fresh data
    K, d, bucket, s = 8, 5 * (1 << 20) + 4099, 1 << 20, 15
    g0 = torch.Generator(device="cpu").manual_seed(77)
    xs = [(torch.randn(d, generator=g0) * 1e-3).to(DEV) for _ in range(K)]
    nb = SI.num_buckets(d, bucket)
    p = gq.make_params(gq.GQ_LINEAR, s, gq.GQ_PACK_I8, gq.GQ_AGG_I32, seed=SI.QUANT_SEED)
    ws = torch.empty(gq.bucketed_workspace_bytes(K, d, bucket), dtype=torch.uint8, device=DEV)
    norms = torch.zeros(nb, device=DEV)
    flags = torch.zeros(nb, dtype=torch.int32, device=DEV)
    agg = torch.zeros(d, dtype=torch.int32, device=DEV)
    out = torch.zeros(d, device=DEV)
    side = torch.cuda.Stream()

    def two_streams():
        gq.bucketed_quantize_aggregate(xs, bucket, gq.GQ_NORM_L2, p, norms, flags, agg, out, ws, side_stream=side)

    two_streams()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            two_streams()
    torch.cuda.current_stream().wait_stream(cap)
    torch.cuda.synchronize()
    for rep in range(4):
        for x in xs:
            x.copy_((torch.randn(d, generator=g0) * (1e-3 * (rep + 1))).to(DEV))
        norms.fill_(-1.0); agg.fill_(-1); out.fill_(-1.0); flags.fill_(9)
        graph.replay()
        torch.cuda.synchronize()
        got = (norms.clone(), agg.clone(), out.clone(), flags.clone())
        norms.fill_(-2.0); agg.fill_(-2); out.fill_(-2.0); flags.fill_(8)
        gq.bucketed_quantize_aggregate(xs, bucket, gq.GQ_NORM_L2, p, norms, flags, agg, out, ws)       # eager, serial
        torch.cuda.synchronize()
        assert torch.equal(got[0], norms) and torch.equal(got[1], agg) and torch.equal(got[2], out) and torch.equal(got[3], flags)
        assert float(norms.min()) > 0 and int(agg.abs().max()) > 0 and int(flags.max()) == 0
