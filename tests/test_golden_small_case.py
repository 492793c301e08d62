"""The stored small case (tests/golden/small_case.json, written by tests/golden/make_golden.py from the
oracle alone): the oracle must still reproduce it, and on a GPU the library must reproduce it too."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import gq_oracle as O

CASE = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "small_case.json")))
SCH = {"linear": 0, "exp": 1}
PK = {"i8": 0, "i4": 1, "u8s": 2, "u4s": 3}


def inputs():
    return [np.array(b, np.uint32).view(np.float32) for b in CASE["x_bits"]]


def test_oracle_reproduces_the_stored_case():
    xs = inputs()
    K, seed, base = CASE["K"], CASE["seed"], CASE["index_base"]
    for name, kind in (("linf", O.NORM_LINF), ("l2", O.NORM_L2), ("l2max", O.NORM_L2_MAX)):
        _, nf, fl = O.global_norm(xs, kind)
        assert int(np.float32(nf).view(np.uint32)) == CASE["norms"][name]["f32_bits"] and fl == CASE["norms"][name]["flags"]
    _, nf, _ = O.global_norm(xs, O.NORM_LINF)
    for run in CASE["runs"]:
        sc, s, pk = SCH[run["scheme"]], run["s"], PK[run["pack"]]
        qs = [O.quantize(xs[i], nf, sc, s, seed, i, base, rng_bits=run["rng_bits"]) for i in range(K)]
        assert [q.tolist() for q in qs] == run["codes"]
        for i, q in enumerate(qs):
            lv, sp = O.pack(q, pk)
            assert lv.tobytes().hex() == run["levels_hex"][i]
            assert (None if sp is None else [int(v) for v in sp]) == run["signplane"][i]
        A = O.aggregate(qs, sc)
        assert A.tolist() == run["aggregate"]
        assert np.allclose(O.dequantize(A, float(nf), sc, s, K), run["dequantized"], rtol=1e-15, atol=0)
        if "alg2_reduced" in run:
            assert O.exp_tree_reduce(qs, s, seed, base).tolist() == run["alg2_reduced"]
        if "avg_reduced" in run:
            assert O.avg_tree_reduce(qs, seed, base).tolist() == run["avg_reduced"]
        if "compact" in run:
            for q, c in zip(qs, run["compact"]):
                n, idx, val = O.compact(q)
                assert n == c["count"] and idx.tolist() == c["index"] and val.tolist() == c["code"]


@pytest.mark.gpu
def test_library_reproduces_the_stored_case():
    import paper_2305_18627_amd as gq
    dev = torch.device("cuda:0")
    K, d, seed, base = CASE["K"], CASE["d"], CASE["seed"], CASE["index_base"]
    xs = [torch.from_numpy(x.copy()).to(dev) for x in inputs()]
    norm = torch.zeros(1, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    for name, kind in (("linf", 0), ("l2", 1), ("l2max", 2)):
        gq.global_norm(xs, kind, norm, flags)
        want = np.array([CASE["norms"][name]["f32_bits"]], np.uint32).view(np.float32)[0]
        got = np.float32(norm.item())
        assert (got == want) if name == "linf" else (abs(float(got) - float(want)) <= 1e-5 * float(want))
        assert flags.item() == CASE["norms"][name]["flags"]
    gq.global_norm(xs, 0, norm, flags)
    for run in CASE["runs"]:
        sc, s, pk = SCH[run["scheme"]], run["s"], PK[run["pack"]]
        p = gq.make_params(sc, s, pk, gq.GQ_AGG_I32, seed=seed, rng_bits=run["rng_bits"])
        agg = torch.zeros(d, dtype=torch.int32, device=dev)
        deq = torch.zeros(d, device=dev)
        lvs = [torch.zeros(gq.levels_nbytes(d, pk), dtype=torch.uint8, device=dev) for _ in range(K)]
        sps = [torch.zeros(gq.signplane_nwords(d), dtype=torch.int32, device=dev) for _ in range(K)] if pk >= 2 else None
        gq.fused_quantize_aggregate(xs, norm, p, base, agg, deq, lvs, sps)
        torch.cuda.synchronize()
        assert agg.cpu().tolist() == run["aggregate"]
        want = np.array(run["dequantized"])
        assert np.all(np.abs(deq.cpu().numpy() - want) <= 1e-5 * np.abs(want))
        for i in range(K):
            assert lvs[i].cpu().numpy().tobytes().hex() == run["levels_hex"][i]
            if sps is not None:
                assert [int(v) for v in sps[i].cpu().numpy().view(np.uint32)] == run["signplane"][i]
        if "alg2_reduced" in run:
            red = torch.zeros(d, dtype=torch.int8, device=dev)
            gq.exp_reduce(lvs, d, p, base, norm, red, deq)
            torch.cuda.synchronize()
            assert red.cpu().tolist() == run["alg2_reduced"]
            want = np.array(run["alg2_mean"])
            assert np.all(np.abs(deq.cpu().numpy() - want) <= 1e-5 * np.abs(want))
        if "avg_reduced" in run:
            red = torch.zeros(gq.levels_nbytes(d, pk), dtype=torch.uint8, device=dev)
            gq.avg_reduce(lvs, d, p, base, norm, red, deq)
            torch.cuda.synchronize()
            assert red.cpu().numpy().tobytes().hex() == O.pack(np.array(run["avg_reduced"], np.int32), pk)[0].tobytes().hex()
            want = np.array(run["avg_mean"])
            assert np.all(np.abs(deq.cpu().numpy() - want) <= 1e-5 * np.abs(want))
        if "compact" in run:
            for i, c in enumerate(run["compact"]):
                idx = torch.zeros(d, dtype=torch.int32, device=dev)
                val = torch.zeros(d, dtype=torch.int8, device=dev)
                cnt = torch.zeros(1, dtype=torch.int64, device=dev)
                gq.compact(lvs[i], d, p, idx, val, cnt)
                torch.cuda.synchronize()
                n = int(cnt.item())
                assert n == c["count"] and idx.cpu().tolist()[:n] == c["index"] and val.cpu().tolist()[:n] == c["code"]
