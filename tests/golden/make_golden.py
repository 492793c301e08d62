"""Writes tests/golden/small_case.json: a small fixed input and what the CPU oracle computes from it.

Run from the repository root:  python tests/golden/make_golden.py
Only the oracle is called.  The inputs are stored in the file itself (as float32 bit patterns), so the
fixture does not depend on any random-number generator staying the same.  The file pins the oracle
against accidental change and gives the GPU tests a second, stored, expectation.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import gq_oracle as O  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "small_case.json")
SEED, K, D, BASE = 0xC0FFEE, 3, 37, 4 * 1000


def main():
    rng = np.random.default_rng(20230529)
    xs = [(rng.standard_normal(D) * 1e-3).astype(np.float32) for _ in range(K)]
    xs[0][3] = 0.0
    xs[1][5] = np.float32(-abs(xs[1]).max())
    case = {"seed": SEED, "K": K, "d": D, "index_base": BASE,
            "x_bits": [[int(v) for v in x.view(np.uint32)] for x in xs], "norms": {}, "runs": []}
    for kind, name in ((O.NORM_LINF, "linf"), (O.NORM_L2, "l2"), (O.NORM_L2_MAX, "l2max")):
        _, nf, fl = O.global_norm(xs, kind)
        case["norms"][name] = {"f32_bits": int(np.float32(nf).view(np.uint32)), "flags": fl}
    _, nf, _ = O.global_norm(xs, O.NORM_LINF)
    for scheme, sname, s, pack, pname, bits in ((O.LINEAR, "linear", 127, O.PACK_I8, "i8", 32), (O.LINEAR, "linear", 7, O.PACK_I4, "i4", 32),
                                                (O.LINEAR, "linear", 15, O.PACK_U4_SIGNPLANE, "u4s", 32),
                                                (O.EXP, "exp", 7, O.PACK_I4, "i4", 32), (O.EXP, "exp", 16, O.PACK_I8, "i8", 32),
                                                (O.LINEAR, "linear", 127, O.PACK_U8_SIGNPLANE, "u8s", 16),
                                                (O.EXP, "exp", 7, O.PACK_I4, "i4", 16)):
        qs = [O.quantize(xs[i], nf, scheme, s, SEED, i, BASE, rng_bits=bits) for i in range(K)]
        packed = [O.pack(q, pack) for q in qs]
        A = O.aggregate(qs, scheme)
        run = {"scheme": sname, "s": s, "pack": pname, "rng_bits": bits,
               "codes": [q.tolist() for q in qs],
               "levels_hex": [lv.tobytes().hex() for lv, _ in packed],
               "signplane": [None if sp is None else [int(v) for v in sp] for _, sp in packed],
               "aggregate": A.tolist(),
               "dequantized": [float(v) for v in O.dequantize(A, float(nf), scheme, s, K)]}
        if bits == 16:                       # the reduce calls below do not depend on how the codes were drawn
            case["runs"].append(run)
            continue
        if scheme == O.EXP and pack == O.PACK_I8:
            se = O.exp_tree_reduce(qs, s, SEED, BASE)
            run["alg2_reduced"] = se.tolist()
            run["alg2_mean"] = [float(v) for v in O.exp_reduce_dequantize(se, float(nf), K)]
        if scheme == O.LINEAR and pack in (O.PACK_I8, O.PACK_I4):
            av = O.avg_tree_reduce(qs, SEED, BASE)
            run["avg_reduced"] = av.tolist()
            run["avg_mean"] = [float(v) for v in O.avg_reduce_dequantize(av, float(nf), s, K)]
        if pack == O.PACK_I8:
            run["compact"] = [{"count": n, "index": idx.tolist(), "code": val.tolist()} for n, idx, val in map(O.compact, qs)]
        case["runs"].append(run)
    with open(OUT, "w") as f:
        json.dump(case, f, indent=0, separators=(",", ":"))
        f.write("\n")
    print("wrote", OUT, os.path.getsize(OUT), "bytes")


if __name__ == "__main__":
    main()
