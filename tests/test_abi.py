"""The C-ABI library loads (no GPU needed) and exports every function include/gqsgd.h declares;
the host-only entry points answer as the header says."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gqsgd.h")


@pytest.fixture(scope="module")
def gq():
    from paper_2305_18627_amd import build as B
    if B.is_stale():
        B.build()
    import paper_2305_18627_amd as gq
    return gq


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(gq):
    names = declared_functions()
    assert len(names) >= 9
    raw = ctypes.CDLL(os.path.join(ROOT, "paper_2305_18627_amd", "libgqsgd.so"))
    for n in names:
        assert hasattr(raw, n), n
    from paper_2305_18627_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_host_only_entry_points(gq):
    assert gq.version() >= 1000
    assert gq.status_string(gq.GQ_OK) == "GQ_OK" and gq.status_string(gq.GQ_ERR_OVERFLOW) == "GQ_ERR_OVERFLOW"
    P = gq.make_params
    # Section 4.2: n*s (linear) or n*2^(s-1) (exponential) must fit the signed aggregate width
    assert gq.check_width(P(gq.GQ_LINEAR, 127, agg=gq.GQ_AGG_I32), 16) == gq.GQ_OK
    assert gq.check_width(P(gq.GQ_LINEAR, 127, agg=gq.GQ_AGG_I16), 64) == gq.GQ_OK          # 8128
    assert gq.check_width(P(gq.GQ_LINEAR, 1024, agg=gq.GQ_AGG_I16), 32) == gq.GQ_ERR_OVERFLOW  # 32768
    assert gq.check_width(P(gq.GQ_LINEAR, 1023, agg=gq.GQ_AGG_I16), 32) == gq.GQ_OK         # 32736
    assert gq.check_width(P(gq.GQ_EXP, 7, agg=gq.GQ_AGG_I16), 32) == gq.GQ_OK               # 2048
    assert gq.check_width(P(gq.GQ_EXP, 15, agg=gq.GQ_AGG_I16), 32) == gq.GQ_ERR_OVERFLOW    # 2^19
    assert gq.check_width(P(gq.GQ_EXP, 16, agg=gq.GQ_AGG_I32), 8) == gq.GQ_OK
    assert gq.check_width(P(gq.GQ_EXP, 31, agg=gq.GQ_AGG_I32), 2) == gq.GQ_ERR_OVERFLOW     # 2^31
    assert gq.check_width(P(gq.GQ_EXP, 31, agg=gq.GQ_AGG_I32), 1) == gq.GQ_OK               # 2^30
    assert gq.check_width(P(gq.GQ_LINEAR, 0), 4) == gq.GQ_ERR_INVALID_ARG
    assert gq.check_width(P(gq.GQ_LINEAR, 5), 0) == gq.GQ_ERR_INVALID_ARG
    assert gq.check_width(P(gq.GQ_LINEAR, 5), 65) == gq.GQ_ERR_INVALID_ARG
    assert gq.check_width(P(gq.GQ_EXP, 32), 1) == gq.GQ_ERR_UNSUPPORTED
    # agreement with the oracle's rule over a grid of settings
    from oracle import gq_oracle as O
    for scheme in (0, 1):
        for s in (1, 2, 3, 7, 15, 16, 31):
            for K in (1, 2, 4, 16, 32, 64):
                for agg, bits in ((gq.GQ_AGG_I32, 32), (gq.GQ_AGG_I16, 16)):
                    ok = gq.check_width(P(scheme, s, agg=agg), K) == gq.GQ_OK
                    assert ok == O.check_width(scheme, s, K, bits)
    # workspace: 8 bytes per block partial, bounded (at most 2^16 tile partials or 1024 per worker),
    # 0 for bad arguments
    assert gq.norm_workspace_bytes(1, 1) == 8
    for K, d in ((1, 0), (4, 1 << 20), (16, 110_000_000), (32, 350_000_000), (8, 1_500_000_000), (64, 1 << 40)):
        b = gq.norm_workspace_bytes(K, d)
        assert b % 8 == 0 and 8 * K <= b <= 8 * max(1 << 16, 1024 * K)
    assert gq.norm_workspace_bytes(65, 10) == 0 and gq.norm_workspace_bytes(1, -1) == 0


def test_parameter_struct_layout_matches_the_header(gq):
    # gq_params as declared in include/gqsgd.h: six int32 then the 64-bit seed (32 bytes, seed at 24)
    import ctypes as C
    src = open(os.path.join(ROOT, "include", "gqsgd.h")).read()
    body = src[src.index("typedef struct {"):src.index("} gq_params;")]
    fields = re.findall(r"(int32_t|uint64_t)\s+(\w+);", body)
    assert [n for _, n in fields] == ["scheme", "s", "pack", "agg", "rng_bits", "flags", "seed"]
    assert [n for n, _ in gq.gq_params._fields_] == [n for _, n in fields]
    assert C.sizeof(gq.gq_params) == 32 and gq.gq_params.seed.offset == 24 and gq.gq_params.rng_bits.offset == 16
    p = gq.make_params(1, 7, 1, 1, seed=0x1122334455667788, rng_bits=16)
    assert (p.scheme, p.s, p.pack, p.agg, p.rng_bits, p.flags, p.seed) == (1, 7, 1, 1, 16, 0, 0x1122334455667788)
    assert gq.make_params(0, 5).rng_bits == 32


def test_argument_checks_need_no_device(gq):
    """Every entry point validates its arguments on the host before anything is enqueued, so the error
    paths can be exercised without a GPU (the pointers below are never dereferenced)."""
    import ctypes as C
    lib = gq.lib()
    P = gq.make_params
    fake = C.c_void_p(0x1000)                 # aligned, never touched
    odd = C.c_void_p(0x1004)                  # 4-byte but not 16-byte aligned
    arr = (C.c_void_p * 2)(0x1000, 0x2000)
    bad_arr = (C.c_void_p * 2)(0x1000, 0x2004)
    ok = P(gq.GQ_LINEAR, 127)
    I = gq.GQ_ERR_INVALID_ARG
    # gq_global_norm
    assert lib.gq_global_norm(arr, 0, 16, 0, fake, None, fake, 1 << 20, None) == I            # K = 0
    assert lib.gq_global_norm(arr, 2, -1, 0, fake, None, fake, 1 << 20, None) == I            # d < 0
    assert lib.gq_global_norm(arr, 2, 16, 9, fake, None, fake, 1 << 20, None) == I            # bad kind
    assert lib.gq_global_norm(bad_arr, 2, 16, 0, fake, None, fake, 1 << 20, None) == I        # misaligned gradient
    assert lib.gq_global_norm(arr, 2, 16, 0, None, None, fake, 1 << 20, None) == I            # no output
    assert lib.gq_global_norm(arr, 2, 1 << 20, 0, fake, None, fake, 8, None) == gq.GQ_ERR_WORKSPACE
    assert lib.gq_global_norm(arr, 2, 1 << 20, 0, fake, None, None, 1 << 20, None) == gq.GQ_ERR_WORKSPACE
    # gq_global_norm_static: the same checks without a workspace
    assert lib.gq_global_norm_static(arr, 0, 16, 0, fake, None, None) == I                    # K = 0
    assert lib.gq_global_norm_static(arr, 2, -1, 0, fake, None, None) == I                    # d < 0
    assert lib.gq_global_norm_static(arr, 2, 16, 9, fake, None, None) == I                    # bad kind
    assert lib.gq_global_norm_static(bad_arr, 2, 16, 0, fake, None, None) == I                # misaligned gradient
    assert lib.gq_global_norm_static(arr, 2, 16, 0, None, None, None) == I                    # no output
    assert lib.gq_global_norm_static(None, 2, 16, 0, fake, None, None) == I
    # gq_params.flags: only the two write-window bits, and not both
    for bad_flags in (3, 4, -1, 1 << 20):
        assert lib.gq_check_width(C.byref(P(gq.GQ_LINEAR, 127, flags=bad_flags)), 4) == I
    for good_flags in (0, gq.GQ_FLAG_WRITE_WINDOWS_OFF, gq.GQ_FLAG_WRITE_WINDOWS_ON):
        assert lib.gq_check_width(C.byref(P(gq.GQ_LINEAR, 127, flags=good_flags)), 4) == gq.GQ_OK
    # gq_bucketed_quantize_aggregate
    bk = lambda p=ok, x=arr, K=2, d=64, bucket=16, kind=0, norms=fake, agg=fake, deq=None, ws=fake, wsb=1 << 20, st=None, side=None: \
        lib.gq_bucketed_quantize_aggregate(x, K, d, bucket, kind, C.byref(p), norms, None, agg, deq, ws, wsb, st, side)
    assert bk(bucket=0) == I and bk(bucket=12) == I and bk(bucket=-8) == I and bk(d=-1) == I and bk(K=0) == I
    assert bk(x=bad_arr) == I and bk(norms=None) == I and bk(agg=None) == I and bk(agg=odd) == I and bk(kind=9) == I
    assert bk(d=1 << 40, bucket=8) == I                                                        # more than 65536 buckets
    assert bk(st=fake, side=fake) == I                                                         # one stream given twice
    assert bk(ws=None) == gq.GQ_ERR_WORKSPACE and bk(d=1 << 22, bucket=1 << 21, wsb=8) == gq.GQ_ERR_WORKSPACE
    assert bk(p=P(gq.GQ_EXP, 15, 0, gq.GQ_AGG_I16), K=2) == gq.GQ_ERR_OVERFLOW
    assert bk(d=0) == gq.GQ_OK                                                                 # nothing to do
    assert lib.gq_bucketed_workspace_bytes(2, 64, 12) == 0 and lib.gq_bucketed_workspace_bytes(2, -1, 16) == 0
    assert lib.gq_bucketed_workspace_bytes(4, 1 << 30, 1 << 26) == lib.gq_norm_workspace_bytes(4, 1 << 26)
    # gq_quantize
    q = lambda p, x=fake, d=16, base=0, lv=fake, sp=None: lib.gq_quantize(x, d, fake, C.byref(p), 0, base, lv, sp, None)
    assert q(ok, x=odd) == I and q(ok, lv=odd) == I and q(ok, base=2) == I and q(ok, base=-4) == I and q(ok, d=-1) == I
    assert q(P(gq.GQ_LINEAR, 128)) == gq.GQ_ERR_UNSUPPORTED and q(P(gq.GQ_LINEAR, 8, gq.GQ_PACK_I4)) == gq.GQ_ERR_UNSUPPORTED
    assert q(P(gq.GQ_LINEAR, 256, gq.GQ_PACK_U8_SIGNPLANE), sp=fake) == gq.GQ_ERR_UNSUPPORTED
    assert q(P(gq.GQ_EXP, 32, gq.GQ_PACK_U8_SIGNPLANE), sp=fake) == gq.GQ_ERR_UNSUPPORTED
    assert q(P(gq.GQ_LINEAR, 15, gq.GQ_PACK_U4_SIGNPLANE), sp=None) == I                       # sign plane missing
    assert q(P(2, 15)) == I and q(P(gq.GQ_LINEAR, 0)) == I and q(P(gq.GQ_LINEAR, 5, 9)) == I
    assert lib.gq_quantize(fake, 16, fake, None, 0, 0, fake, None, None) == I                 # no parameters
    # random bits per coordinate: 32 (0 reads as 32) or 16; 16 wants index_base to be a multiple of 8
    assert q(P(gq.GQ_LINEAR, 127, rng_bits=8)) == I and q(P(gq.GQ_LINEAR, 127, rng_bits=24)) == I
    assert q(P(gq.GQ_LINEAR, 127, rng_bits=16), base=4) == I and q(P(gq.GQ_LINEAR, 127, rng_bits=16), d=0, base=8) == gq.GQ_OK
    assert q(P(gq.GQ_LINEAR, 127, rng_bits=0), d=0, base=4) == gq.GQ_OK and q(P(gq.GQ_LINEAR, 127, rng_bits=32), d=0, base=4) == gq.GQ_OK
    # gq_fused_quantize_aggregate
    f = lambda p, K=2, x=arr, agg=fake, deq=None, base=0: lib.gq_fused_quantize_aggregate(
        x, K, 16, fake, C.byref(p), base, agg, deq, None, None, None)
    assert f(ok, agg=None) == I and f(ok, K=0) == I and f(ok, K=65) == I and f(ok, x=bad_arr) == I
    assert f(ok, agg=odd) == I and f(ok, base=6) == I
    assert f(P(gq.GQ_LINEAR, 127, rng_bits=16), base=12) == I and f(P(gq.GQ_LINEAR, 127, rng_bits=5)) == I
    assert f(P(gq.GQ_EXP, 15, agg=gq.GQ_AGG_I16), K=2, x=None) == I
    big = (C.c_void_p * 32)(*([0x1000] * 32))
    assert f(P(gq.GQ_EXP, 15, agg=gq.GQ_AGG_I16), K=32, x=big) == gq.GQ_ERR_OVERFLOW
    assert f(P(gq.GQ_LINEAR, 1024, agg=gq.GQ_AGG_I16), K=32, x=big) == gq.GQ_ERR_OVERFLOW
    # gq_int_aggregate / gq_dequantize / gq_exp_reduce
    assert lib.gq_int_aggregate(big, None, 32, 16, C.byref(P(gq.GQ_EXP, 15, gq.GQ_PACK_U4_SIGNPLANE, gq.GQ_AGG_I16)),
                                fake, None) == gq.GQ_ERR_OVERFLOW
    assert lib.gq_int_aggregate(arr, None, 2, 16, C.byref(P(gq.GQ_LINEAR, 15, gq.GQ_PACK_U4_SIGNPLANE)), fake, None) == I
    assert lib.gq_int_aggregate(bad_arr, None, 2, 16, C.byref(ok), fake, None) == I
    assert lib.gq_int_aggregate(arr, None, 2, 16, C.byref(ok), odd, None) == I
    # a launch holds at most 2^32 - 1 threads: sizes that one launch cannot cover are refused, not launched
    assert lib.gq_int_aggregate(arr, None, 2, 1 << 34, C.byref(ok), fake, None) == I
    assert lib.gq_dequantize(fake, 1 << 34, fake, C.byref(ok), 2, fake, None) == I
    assert lib.gq_fused_quantize_aggregate(arr, 2, 1 << 34, fake, C.byref(ok), 0, fake, None, arr, None, None) == I
    assert lib.gq_exp_reduce(arr, 2, 1 << 34, C.byref(P(gq.GQ_EXP, 7)), 0, fake, fake, None, None) == I
    assert lib.gq_dequantize(fake, 16, fake, C.byref(ok), 0, fake, None) == I
    assert lib.gq_dequantize(odd, 16, fake, C.byref(ok), 2, fake, None) == I
    assert lib.gq_exp_reduce(arr, 2, 16, C.byref(ok), 0, fake, fake, None, None) == gq.GQ_ERR_UNSUPPORTED   # not GQ_EXP
    ex = P(gq.GQ_EXP, 7)
    assert lib.gq_exp_reduce(arr, 2, 16, C.byref(ex), 0, fake, None, None, None) == I          # no output
    assert lib.gq_exp_reduce(arr, 2, 16, C.byref(ex), 2, fake, fake, None, None) == I          # index_base % 4
    assert lib.gq_exp_reduce(arr, 2, 16, C.byref(ex), 0, None, None, fake, None) == I          # mean without norm
    assert lib.gq_exp_reduce(bad_arr, 2, 16, C.byref(ex), 0, fake, fake, None, None) == I
    av = P(gq.GQ_LINEAR, 7, gq.GQ_PACK_I4)
    assert lib.gq_avg_reduce(arr, 2, 16, C.byref(ex), 0, fake, fake, None, None) == gq.GQ_ERR_UNSUPPORTED   # not linear
    assert lib.gq_avg_reduce(arr, 2, 16, C.byref(P(gq.GQ_LINEAR, 15, gq.GQ_PACK_U4_SIGNPLANE)), 0, fake, fake, None, None) \
        == gq.GQ_ERR_UNSUPPORTED
    assert lib.gq_avg_reduce(arr, 2, 16, C.byref(av), 0, fake, None, None, None) == I
    assert lib.gq_avg_reduce(arr, 2, 16, C.byref(av), 0, None, None, fake, None) == I
    assert lib.gq_avg_reduce(arr, 0, 16, C.byref(av), 0, fake, fake, None, None) == I
    assert lib.gq_avg_reduce(arr, 2, 16, C.byref(P(gq.GQ_LINEAR, 8, gq.GQ_PACK_I4)), 0, fake, fake, None, None) == gq.GQ_ERR_UNSUPPORTED
    # sparse branch
    assert gq.compact_workspace_bytes(-1) == 0 and gq.compact_workspace_bytes(1 << 33) == 0
    assert gq.compact_workspace_bytes(0) == 16 and gq.compact_workspace_bytes(32768) == 32 and gq.compact_workspace_bytes(32769) == 40
    assert gq.tile_starts_len(0) == 1 and gq.tile_starts_len(4096) == 2 and gq.tile_starts_len(4097) == 3
    assert gq.tile_starts_len(-1) == 0 and gq.tile_starts_len(1 << 33) == 0 and gq.tile_starts_len((1 << 32) - 1) == (1 << 20) + 1
    cp = lambda p, lv=fake, d=64, cap=16, cnt=fake, ws=fake, wsb=1024, ts=None: lib.gq_compact(lv, d, C.byref(p), fake, fake, cap, cnt, ts, ws, wsb, None)
    assert cp(av) == gq.GQ_ERR_UNSUPPORTED and cp(ok, lv=odd) == I and cp(ok, d=-1) == I and cp(ok, d=1 << 33) == I
    assert cp(ok, ts=C.c_void_p(0x1002)) == I
    assert cp(ok, cap=-1) == I and cp(ok, cnt=None) == I and cp(ok, cnt=odd) == I
    assert cp(ok, ws=None) == gq.GQ_ERR_WORKSPACE and cp(ok, d=1 << 20, wsb=8) == gq.GQ_ERR_WORKSPACE
    # the sender straight from the gradient: the argument checks of gq_quantize and of gq_compact together
    qc = lambda p, x=fake, d=64, norm=fake, base=0, cap=16, cnt=fake, ws=fake, wsb=1024, ts=None: \
        lib.gq_quantize_compact(x, d, norm, C.byref(p), 0, base, fake, fake, cap, cnt, ts, ws, wsb, None)
    assert qc(av) == gq.GQ_ERR_UNSUPPORTED and qc(ok, x=odd) == I and qc(ok, d=-1) == I and qc(ok, d=1 << 33) == I
    assert qc(ok, norm=None) == I and qc(ok, base=2) == I and qc(ok, base=-4) == I
    assert qc(P(gq.GQ_LINEAR, 127, rng_bits=16), base=4) == I                                   # short draws: multiples of 8
    assert qc(ok, ts=C.c_void_p(0x1002)) == I and qc(ok, cap=-1) == I and qc(ok, cnt=None) == I and qc(ok, cnt=odd) == I
    assert qc(ok, ws=None) == gq.GQ_ERR_WORKSPACE and qc(ok, d=1 << 20, wsb=8) == gq.GQ_ERR_WORKSPACE
    caps = (C.c_int64 * 2)(4, 4)
    sa = lambda p, K=2, idx=arr, d=64, agg=fake, ts=None: lib.gq_sparse_aggregate(idx, arr, arr, caps, ts, K, d, C.byref(p), agg, None)
    assert sa(ok, ts=(C.c_void_p * 2)(0x1000, 0x2002)) == I
    assert sa(P(gq.GQ_LINEAR, 127, agg=gq.GQ_AGG_I16)) == gq.GQ_ERR_UNSUPPORTED
    assert sa(ok, K=0) == I and sa(ok, idx=None) == I and sa(ok, agg=odd) == I and sa(ok, d=1 << 33) == I
    assert sa(ok, idx=(C.c_void_p * 2)(0x1000, 0x2002)) == I


def test_sparsity_bound_matches_the_oracle(gq):
    # host-only, like the headroom rule: the library's value against the oracle's over both grids and the ends of the ranges
    from oracle import gq_oracle as O
    for scheme, ss in ((gq.GQ_LINEAR, (1, 4, 15, 127, 255, 32767)), (gq.GQ_EXP, (1, 4, 7, 16, 31))):
        for s in ss:
            for K in (1, 3, 16, 64):
                for d in (0, 1, 100, 1 << 20, 110_000_000, (1 << 34) - 1024):
                    p = gq.make_params(scheme, s, gq.GQ_PACK_I8 if s <= 127 else gq.GQ_PACK_U8_SIGNPLANE)
                    assert gq.sparse_nnz_bound(p, K, d) == O.sparse_nnz_bound(scheme, s, K, d), (scheme, s, K, d)
    ok = gq.make_params(gq.GQ_LINEAR, 127)
    assert gq.sparse_nnz_bound(ok, 0, 10) == -1.0 and gq.sparse_nnz_bound(ok, 65, 10) == -1.0 and gq.sparse_nnz_bound(ok, 1, -1) == -1.0
    assert gq.sparse_nnz_bound(gq.make_params(gq.GQ_EXP, 32), 1, 10) == -1.0 and gq.sparse_nnz_bound(gq.make_params(2, 4), 1, 10) == -1.0
    assert gq.sparse_nnz_bound(gq.make_params(gq.GQ_LINEAR, 4), 4, 1024) == 272.0


def test_header_is_plain_c_and_cxx(tmp_path):
    # the boundary is a C ABI: include/gqsgd.h compiles on its own as C99 and as C++17, with no torch or HIP types
    import shutil
    import subprocess
    for compiler, std, ext in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "cpp")):
        exe = shutil.which(compiler)
        if exe is None:
            pytest.skip("no " + compiler)
        src = tmp_path / ("use_header." + ext)
        src.write_text('#include "gqsgd.h"\n'
                       'int use(void) { gq_params p; p.flags = GQ_FLAG_WRITE_WINDOWS_OFF; return (int)sizeof(p) + (int)GQ_OK + GQ_MAX_WORKERS; }\n')
        res = subprocess.run([exe, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", os.path.join(ROOT, "include"), str(src)],
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout
    text = open(HEADER).read()
    assert "torch" not in text and "#include <hip" not in text and "#include \"hip" not in text
