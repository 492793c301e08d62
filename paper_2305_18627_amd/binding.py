"""Thin ctypes binding of the C ABI in include/gqsgd.h.

Argument marshalling only: every step of the path runs in the HIP kernels of libgqsgd.so.
PyTorch is used for device memory (tensor.data_ptr()) and for the current HIP stream, nothing
else.  There is no CPU fallback: if the library has not been built, importing this module raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgqsgd.so")

GQ_MAX_WORKERS = 64
GQ_OK, GQ_ERR_INVALID_ARG, GQ_ERR_UNSUPPORTED, GQ_ERR_OVERFLOW, GQ_ERR_WORKSPACE, GQ_ERR_DEVICE = range(6)
GQ_NORM_LINF, GQ_NORM_L2, GQ_NORM_L2_MAX = 0, 1, 2
GQ_LINEAR, GQ_EXP = 0, 1
GQ_PACK_I8, GQ_PACK_I4, GQ_PACK_U8_SIGNPLANE, GQ_PACK_U4_SIGNPLANE = 0, 1, 2, 3
GQ_AGG_I32, GQ_AGG_I16 = 0, 1
GQ_FLAG_WRITE_WINDOWS_OFF, GQ_FLAG_WRITE_WINDOWS_ON = 1, 2

# every symbol include/gqsgd.h declares
EXPORTS = ("gq_version", "gq_status_string", "gq_check_width", "gq_sparse_nnz_bound", "gq_norm_workspace_bytes", "gq_global_norm",
           "gq_global_norm_static", "gq_bucketed_workspace_bytes", "gq_bucketed_quantize_aggregate",
           "gq_quantize", "gq_int_aggregate", "gq_dequantize", "gq_fused_quantize_aggregate", "gq_exp_reduce", "gq_avg_reduce", "gq_compact_workspace_bytes", "gq_tile_starts_len", "gq_compact",
           "gq_quantize_compact",
           "gq_sparse_aggregate")


class gq_params(C.Structure):
    _fields_ = [("scheme", C.c_int32), ("s", C.c_int32), ("pack", C.c_int32), ("agg", C.c_int32),
                ("rng_bits", C.c_int32), ("flags", C.c_int32), ("seed", C.c_uint64)]


class GQError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        name = _lib.gq_status_string(int(status)).decode() if _lib is not None else str(status)
        super().__init__("%s failed: %s" % (where, name))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                          "or python paper_2305_18627_amd/build.py); there is no fallback path" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i64, u32, i32, sz = C.c_void_p, C.c_int64, C.c_uint32, C.c_int, C.c_size_t
    pp = C.POINTER(gq_params)
    sigs = {
        "gq_version": (C.c_int, []),
        "gq_status_string": (C.c_char_p, [i32]),
        "gq_check_width": (i32, [pp, i32]),
        "gq_sparse_nnz_bound": (C.c_double, [pp, i32, i64]),
        "gq_norm_workspace_bytes": (sz, [i32, i64]),
        "gq_global_norm": (i32, [C.POINTER(vp), i32, i64, i32, vp, vp, vp, sz, vp]),
        "gq_global_norm_static": (i32, [C.POINTER(vp), i32, i64, i32, vp, vp, vp]),
        "gq_quantize": (i32, [vp, i64, vp, pp, u32, i64, vp, vp, vp]),
        "gq_int_aggregate": (i32, [C.POINTER(vp), C.POINTER(vp), i32, i64, pp, vp, vp]),
        "gq_dequantize": (i32, [vp, i64, vp, pp, i32, vp, vp]),
        "gq_bucketed_workspace_bytes": (sz, [i32, i64, i64]),
        "gq_bucketed_quantize_aggregate": (i32, [C.POINTER(vp), i32, i64, i64, i32, pp, vp, vp, vp, vp, vp, sz, vp, vp]),
        "gq_exp_reduce": (i32, [C.POINTER(vp), i32, i64, pp, i64, vp, vp, vp, vp]),
        "gq_avg_reduce": (i32, [C.POINTER(vp), i32, i64, pp, i64, vp, vp, vp, vp]),
        "gq_compact_workspace_bytes": (sz, [i64]),
        "gq_tile_starts_len": (i64, [i64]),
        "gq_compact": (i32, [vp, i64, pp, vp, vp, i64, vp, vp, vp, sz, vp]),
        "gq_quantize_compact": (i32, [vp, i64, vp, pp, u32, i64, vp, vp, i64, vp, vp, vp, sz, vp]),
        "gq_sparse_aggregate": (i32, [C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(i64), C.POINTER(vp), i32, i64, pp, vp, vp]),
        "gq_fused_quantize_aggregate": (i32, [C.POINTER(vp), i32, i64, vp, pp, i64, vp, vp, C.POINTER(vp),
                                               C.POINTER(vp), vp]),
    }
    for name, (res, args) in sigs.items():
        f = getattr(lib, name)
        f.restype = res
        f.argtypes = args
    return lib


_lib = None
_lib = _load()


def lib():
    """The loaded ctypes library (for tests that call the C ABI directly)."""
    return _lib


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)


def _ptr_array(ts):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    return arr


def _check(st, where):
    if st != GQ_OK:
        raise GQError(st, where)


# The C ABI takes raw pointers and cannot see buffer sizes; the checks below are the binding's part of the
# contract: a tensor that is too small, not contiguous or not on the GPU is refused here, before any launch.
def _need(t, nbytes, what):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous CUDA tensor" % what)
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise ValueError("%s holds %d bytes, the call needs %d" % (what, have, nbytes))


def _need_grads(xs):
    d = xs[0].numel() if xs else 0
    for x in xs:
        if x.dtype != torch.float32 or x.numel() != d:
            raise ValueError("gradients must be float32 tensors of equal length")
        _need(x, 4 * d, "gradient")
    return d


def _agg_bytes(params):
    return 2 if params.agg == GQ_AGG_I16 else 4


def _need_levels(levels, signplanes, d, params, what="levels"):
    if levels is None:
        return
    for t in levels:
        _need(t, levels_nbytes(d, params.pack), what)
    if params.pack >= GQ_PACK_U8_SIGNPLANE and signplanes is not None:
        for t in signplanes:
            _need(t, 4 * signplane_nwords(d), "sign plane")


def make_params(scheme, s, pack=GQ_PACK_I8, agg=GQ_AGG_I32, seed=0, rng_bits=32, flags=0):
    return gq_params(int(scheme), int(s), int(pack), int(agg), int(rng_bits), int(flags), int(seed))


def levels_nbytes(d, pack):
    return d if pack in (GQ_PACK_I8, GQ_PACK_U8_SIGNPLANE) else (d + 1) // 2


def signplane_nwords(d):
    return (d + 31) // 32


def status_string(st):
    return _lib.gq_status_string(int(st)).decode()


def version():
    return int(_lib.gq_version())


def check_width(params, K):
    """gq_check_width: the status code (GQ_OK / GQ_ERR_OVERFLOW / ...), not an exception."""
    return int(_lib.gq_check_width(C.byref(params), int(K)))


def sparse_nnz_bound(params, K, d):
    """gq_sparse_nnz_bound: the bound on the expected number of non-zero codes under the (2,2) norm; -1 for bad parameters."""
    return float(_lib.gq_sparse_nnz_bound(C.byref(params), int(K), int(d)))


def norm_workspace_bytes(K, d):
    return int(_lib.gq_norm_workspace_bytes(int(K), int(d)))


def global_norm(xs, kind, norm_out, status_flags=None, workspace=None, stream=None):
    """gq_global_norm over the K tensors xs (fp32, equal length).  Returns the workspace used."""
    K, d = len(xs), _need_grads(xs)
    _need(norm_out, 4, "norm_out"); _need(status_flags, 4, "status_flags")
    if workspace is None:
        workspace = torch.empty(max(norm_workspace_bytes(K, d), 8), dtype=torch.uint8, device=norm_out.device)
    st = _lib.gq_global_norm(_ptr_array(xs), K, d, int(kind), _ptr(norm_out), _ptr(status_flags),
                             _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "gq_global_norm")
    return workspace


def global_norm_static(xs, kind, norm_out, status_flags=None, stream=None):
    """gq_global_norm_static: the norm with the library's own static scratch; nothing is allocated."""
    K, d = len(xs), _need_grads(xs)
    _need(norm_out, 4, "norm_out"); _need(status_flags, 4, "status_flags")
    st = _lib.gq_global_norm_static(_ptr_array(xs), K, d, int(kind), _ptr(norm_out), _ptr(status_flags), _stream(stream))
    _check(st, "gq_global_norm_static")


def quantize(x, norm, params, worker, index_base, levels_out, signplane_out=None, stream=None):
    d = _need_grads([x])
    _need(norm, 4, "norm")
    _need_levels([levels_out], [signplane_out] if signplane_out is not None else None, d, params, "levels_out")
    st = _lib.gq_quantize(_ptr(x), x.numel(), _ptr(norm), C.byref(params), int(worker), int(index_base),
                          _ptr(levels_out), _ptr(signplane_out), _stream(stream))
    _check(st, "gq_quantize")


def int_aggregate(levels, signplanes, d, params, agg_out, stream=None):
    _need_levels(levels, signplanes, int(d), params)
    _need(agg_out, _agg_bytes(params) * int(d), "agg_out")
    st = _lib.gq_int_aggregate(_ptr_array(levels), _ptr_array(signplanes), len(levels), int(d),
                               C.byref(params), _ptr(agg_out), _stream(stream))
    _check(st, "gq_int_aggregate")


def dequantize(agg, d, norm, params, K, out, stream=None):
    _need(agg, _agg_bytes(params) * int(d), "agg"); _need(out, 4 * int(d), "out"); _need(norm, 4, "norm")
    st = _lib.gq_dequantize(_ptr(agg), int(d), _ptr(norm), C.byref(params), int(K), _ptr(out), _stream(stream))
    _check(st, "gq_dequantize")


def fused_quantize_aggregate(xs, norm, params, index_base=0, agg_out=None, dequant_out=None,
                             levels_out=None, signplanes_out=None, stream=None):
    K, d = len(xs), _need_grads(xs)
    _need(norm, 4, "norm"); _need(agg_out, _agg_bytes(params) * d, "agg_out"); _need(dequant_out, 4 * d, "dequant_out")
    _need_levels(levels_out, signplanes_out, d, params, "levels_out")
    st = _lib.gq_fused_quantize_aggregate(_ptr_array(xs), K, d, _ptr(norm), C.byref(params), int(index_base),
                                          _ptr(agg_out), _ptr(dequant_out), _ptr_array(levels_out),
                                          _ptr_array(signplanes_out), _stream(stream))
    _check(st, "gq_fused_quantize_aggregate")


def bucketed_workspace_bytes(K, d, bucket):
    return int(_lib.gq_bucketed_workspace_bytes(int(K), int(d), int(bucket)))


def bucketed_quantize_aggregate(xs, bucket, kind, params, norms_out, status_flags=None, agg_out=None, dequant_out=None,
                                workspace=None, stream=None, side_stream=None):
    """gq_bucketed_quantize_aggregate: per bucket its own norm and fused quantize+aggregate; with side_stream the
    norm of the next bucket runs beside the fused call of the current one.  Returns the workspace used."""
    K, d = len(xs), _need_grads(xs)
    nb = (d + int(bucket) - 1) // int(bucket) if bucket > 0 else 0
    _need(norms_out, 4 * nb, "norms_out"); _need(status_flags, 4 * nb, "status_flags")
    _need(agg_out, _agg_bytes(params) * d, "agg_out"); _need(dequant_out, 4 * d, "dequant_out")
    if workspace is None:
        workspace = torch.empty(max(bucketed_workspace_bytes(K, d, bucket), 8), dtype=torch.uint8, device=norms_out.device)
    side = _stream(side_stream) if side_stream is not None else C.c_void_p(None)
    st = _lib.gq_bucketed_quantize_aggregate(_ptr_array(xs), K, d, int(bucket), int(kind), C.byref(params), _ptr(norms_out),
                                             _ptr(status_flags), _ptr(agg_out), _ptr(dequant_out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream), side)
    _check(st, "gq_bucketed_quantize_aggregate")
    return workspace


def exp_reduce(levels, d, params, index_base=0, norm=None, reduced_out=None, dequant_out=None, stream=None):
    for t in levels:
        _need(t, int(d), "levels")                               # int8 codes
    _need(reduced_out, int(d), "reduced_out"); _need(dequant_out, 4 * int(d), "dequant_out"); _need(norm, 4, "norm")
    st = _lib.gq_exp_reduce(_ptr_array(levels), len(levels), int(d), C.byref(params), int(index_base), _ptr(norm),
                            _ptr(reduced_out), _ptr(dequant_out), _stream(stream))
    _check(st, "gq_exp_reduce")


def avg_reduce(levels, d, params, index_base=0, norm=None, reduced_out=None, dequant_out=None, stream=None):
    _need_levels(levels, None, int(d), params)
    _need(reduced_out, levels_nbytes(int(d), params.pack), "reduced_out"); _need(dequant_out, 4 * int(d), "dequant_out")
    _need(norm, 4, "norm")
    st = _lib.gq_avg_reduce(_ptr_array(levels), len(levels), int(d), C.byref(params), int(index_base), _ptr(norm),
                            _ptr(reduced_out), _ptr(dequant_out), _stream(stream))
    _check(st, "gq_avg_reduce")


def compact_workspace_bytes(d):
    return int(_lib.gq_compact_workspace_bytes(int(d)))


def tile_starts_len(d):
    return int(_lib.gq_tile_starts_len(int(d)))


def compact(levels, d, params, indices_out, values_out, count_out, workspace=None, stream=None, tile_starts_out=None):
    """gq_compact: the non-zero int8 codes of one worker as (index, code) pairs, and optionally the table of where
    every tile of 4096 coordinates begins in the list.  Returns the workspace used."""
    _need(levels, int(d), "levels"); _need(count_out, 8, "count_out")
    _need(values_out, indices_out.numel(), "values_out"); _need(indices_out, 0, "indices_out")
    _need(tile_starts_out, 4 * tile_starts_len(d), "tile_starts_out")
    if workspace is None:
        workspace = torch.empty(compact_workspace_bytes(d), dtype=torch.uint8, device=count_out.device)
    st = _lib.gq_compact(_ptr(levels), int(d), C.byref(params), _ptr(indices_out), _ptr(values_out),
                         indices_out.numel(), _ptr(count_out), _ptr(tile_starts_out), _ptr(workspace),
                         workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "gq_compact")
    return workspace


def quantize_compact(x, norm, params, worker, index_base, indices_out, values_out, count_out, workspace=None, stream=None,
                     tile_starts_out=None):
    """gq_quantize_compact: the list gq_quantize + gq_compact would write, straight from the gradient.  Returns the
    workspace used."""
    d = _need_grads([x])
    _need(norm, 4, "norm"); _need(count_out, 8, "count_out")
    _need(values_out, indices_out.numel(), "values_out"); _need(indices_out, 0, "indices_out")
    _need(tile_starts_out, 4 * tile_starts_len(d), "tile_starts_out")
    if workspace is None:
        workspace = torch.empty(compact_workspace_bytes(d), dtype=torch.uint8, device=count_out.device)
    st = _lib.gq_quantize_compact(_ptr(x), d, _ptr(norm), C.byref(params), int(worker), int(index_base), _ptr(indices_out),
                                  _ptr(values_out), indices_out.numel(), _ptr(count_out), _ptr(tile_starts_out), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "gq_quantize_compact")
    return workspace


def sparse_aggregate(indices, values, counts, d, params, agg_out, stream=None, tile_starts=None):
    for i, v, c in zip(indices, values, counts):
        _need(i, 0, "indices"); _need(v, i.numel(), "values"); _need(c, 8, "count")
    if tile_starts is not None:
        for t in tile_starts:
            _need(t, 4 * tile_starts_len(d), "tile_starts")
    _need(agg_out, 4 * int(d), "agg_out")
    caps = (C.c_int64 * len(indices))(*[t.numel() for t in indices])
    starts = None if tile_starts is None else (C.c_void_p * len(tile_starts))(*[t.data_ptr() if t is not None else None for t in tile_starts])
    st = _lib.gq_sparse_aggregate(_ptr_array(indices), _ptr_array(values), _ptr_array(counts), caps, starts, len(indices),
                                  int(d), C.byref(params), _ptr(agg_out), _stream(stream))
    _check(st, "gq_sparse_aggregate")
