"""ctypes/numpy face of the C oracle (oracle/gq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package imports it, and it imports nothing from the
product package.  Arrays in, arrays out; every function cites the passage of arXiv 2305.18627
that the C routine behind it follows.
"""
import ctypes as C
import numpy as np

from . import build_oracle

LINEAR, EXP = 0, 1
NORM_LINF, NORM_L2, NORM_L2_MAX = 0, 1, 2
PACK_I8, PACK_I4, PACK_U8_SIGNPLANE, PACK_U4_SIGNPLANE = 0, 1, 2, 3

_lib = C.CDLL(build_oracle.build())

_f32p = C.POINTER(C.c_float)
_u32p = C.POINTER(C.c_uint32)
_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)
_f64p = C.POINTER(C.c_double)
_u8p = C.POINTER(C.c_uint8)


def _sig(name, res, *args):
    f = getattr(_lib, name)
    f.restype = res
    f.argtypes = list(args)
    return f


_philox = _sig("gqo_philox4x32", None, C.c_int, _u32p, _u32p, _u32p)
_random_word = _sig("gqo_random_word", C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64)
_random_words = _sig("gqo_random_words", None, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int64, C.c_int, _u32p)
_global_norm = _sig("gqo_global_norm", C.c_int, C.POINTER(_f32p), C.c_int, C.c_int64, C.c_int, _f64p, _f32p)
_code = _sig("gqo_code", C.c_int32, C.c_int, C.c_float, C.c_float, C.c_int, C.c_uint32)
_quantize_with_words = _sig("gqo_quantize_with_words", None, _f32p, _u32p, C.c_int64, C.c_float,
                            C.c_int, C.c_int, _i32p)
_quantize = _sig("gqo_quantize", None, _f32p, C.c_int64, C.c_float, C.c_int, C.c_int,
                 C.c_uint64, C.c_uint32, C.c_uint64, C.c_int, _i32p)
_code_value = _sig("gqo_code_value", C.c_int64, C.c_int, C.c_int32)
_aggregate = _sig("gqo_aggregate", None, C.POINTER(_i32p), C.c_int, C.c_int64, C.c_int, _i64p)
_max_aggregate = _sig("gqo_max_aggregate", C.c_int64, C.c_int, C.c_int, C.c_int)
_check_width = _sig("gqo_check_width", C.c_int, C.c_int, C.c_int, C.c_int, C.c_int)
_fits_width = _sig("gqo_fits_width", C.c_int, _i64p, C.c_int64, C.c_int)
_dequantize = _sig("gqo_dequantize", None, _i64p, C.c_int64, C.c_double, C.c_int, C.c_int, C.c_int, _f64p)
_levels_bytes = _sig("gqo_levels_bytes", C.c_int64, C.c_int64, C.c_int)
_signplane_words = _sig("gqo_signplane_words", C.c_int64, C.c_int64)
_pack = _sig("gqo_pack", C.c_int, _i32p, C.c_int64, C.c_int, _u8p, _u32p)
_unpack = _sig("gqo_unpack", None, _u8p, _u32p, C.c_int64, C.c_int, _i32p)
_quantize_aggregate = _sig("gqo_quantize_aggregate", C.c_int, C.POINTER(_f32p), C.c_int, C.c_int64,
                           C.c_float, C.c_int, C.c_int, C.c_uint64, C.c_uint64, C.c_int, _i64p)


_alg2_k = _sig("gqo_alg2_k", C.c_int, C.c_uint32, C.c_int)
_alg2_draw = _sig("gqo_alg2_draw", C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int)
_alg2_field_bits = _sig("gqo_alg2_field_bits", C.c_int, C.c_int)
_exp_reduce_pair = _sig("gqo_exp_reduce_pair", None, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                        C.POINTER(C.c_int), C.POINTER(C.c_int))
_random_word_of = _sig("gqo_random_word_of", C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64)
_exp_tree_reduce = _sig("gqo_exp_tree_reduce", None, C.POINTER(_i32p), C.c_int, C.c_int64, C.c_int, C.c_uint64,
                        C.c_uint64, _i32p)
_exp_reduce_dequantize = _sig("gqo_exp_reduce_dequantize", None, _i32p, C.c_int64, C.c_double, C.c_int, _f64p)


_avg_pair = _sig("gqo_avg_pair", C.c_int32, C.c_int32, C.c_int32, C.c_int)
_avg_tree_reduce = _sig("gqo_avg_tree_reduce", None, C.POINTER(_i32p), C.c_int, C.c_int64, C.c_uint64, C.c_uint64, _i32p)
_avg_reduce_dequantize = _sig("gqo_avg_reduce_dequantize", None, _i32p, C.c_int64, C.c_double, C.c_int, C.c_int, _f64p)


_compact = _sig("gqo_compact", C.c_int64, _i32p, C.c_int64, C.c_int64, _u32p, _i32p)
_sparse_nnz_bound = _sig("gqo_sparse_nnz_bound", C.c_double, C.c_int, C.c_int, C.c_int, C.c_int64)
_sparse_aggregate = _sig("gqo_sparse_aggregate", None, C.POINTER(_u32p), C.POINTER(_i32p), _i64p, C.c_int, C.c_int64,
                         C.c_int, _i64p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _rows(xs, dtype, ctype):
    """List of K equally long 1-D arrays -> (kept-alive arrays, C array of row pointers, K, d)."""
    rows = [_arr(x, dtype).reshape(-1) for x in xs]
    d = rows[0].shape[0] if rows else 0
    for r in rows:
        if r.shape[0] != d:
            raise ValueError("workers must have equal length")
    ptrs = (C.POINTER(ctype) * len(rows))(*[_ptr(r, ctype) for r in rows])
    return rows, ptrs, len(rows), d


def philox4x32(ctr, key, rounds=10):
    """Philox4x32-`rounds` block function (Salmon et al., SC'11)."""
    c = _arr(ctr, np.uint32); k = _arr(key, np.uint32); o = np.zeros(4, np.uint32)
    _philox(int(rounds), _ptr(c, C.c_uint32), _ptr(k, C.c_uint32), _ptr(o, C.c_uint32))
    return o


def random_words(seed, worker, index_base, d, rng_bits=32):
    """The word that rounds each coordinate index_base .. index_base+d-1 of one worker: 32 random bits, or
    with rng_bits = 16 the coordinate's 16 random bits in the top half and zeros below."""
    r = np.zeros(int(d), np.uint32)
    _random_words(int(seed), int(worker), int(index_base), int(d), int(rng_bits), _ptr(r, C.c_uint32))
    return r


def global_norm(xs, kind):
    """Algorithm 1's norm step.  Returns (norm in binary64, norm rounded to binary32, flag bits)."""
    rows, ptrs, K, d = _rows(xs, np.float32, C.c_float)
    ne = C.c_double(0.0); nf = C.c_float(0.0)
    flags = _global_norm(ptrs, K, d, int(kind), C.byref(ne), C.byref(nf))
    return ne.value, np.float32(nf.value), flags


def code(scheme, x, norm, s, r):
    """Signed level integer of one coordinate for a given random word (Eq. (2))."""
    return int(_code(int(scheme), float(np.float32(x)), float(np.float32(norm)), int(s), int(r)))


def quantize_with_words(x, r, norm, scheme, s):
    """Eq. (2) for an array of coordinates with the random words given as an input."""
    x = _arr(x, np.float32).reshape(-1); r = _arr(r, np.uint32).reshape(-1)
    if x.shape != r.shape:
        raise ValueError("x and r must have equal length")
    q = np.zeros(x.shape[0], np.int32)
    _quantize_with_words(_ptr(x, C.c_float), _ptr(r, C.c_uint32), x.shape[0], float(np.float32(norm)),
                         int(scheme), int(s), _ptr(q, C.c_int32))
    return q


def quantize(x, norm, scheme, s, seed, worker, index_base=0, rng_bits=32):
    """Algorithm 1's quantisation loop for one worker: signed level integers, one int32 per coordinate."""
    x = _arr(x, np.float32).reshape(-1)
    q = np.zeros(x.shape[0], np.int32)
    _quantize(_ptr(x, C.c_float), x.shape[0], float(np.float32(norm)), int(scheme), int(s),
              int(seed), int(worker), int(index_base), int(rng_bits), _ptr(q, C.c_int32))
    return q


def code_value(scheme, q):
    """Integer that a signed code adds to the sum: q (linear) or sign*2^(|q|-1) (exponential)."""
    return int(_code_value(int(scheme), int(q)))


def aggregate(qs, scheme):
    """Algorithm 1's aggregation step: the integer sum over workers, in int64."""
    rows, ptrs, K, d = _rows(qs, np.int32, C.c_int32)
    A = np.zeros(d, np.int64)
    _aggregate(ptrs, K, d, int(scheme), _ptr(A, C.c_int64))
    return A


def max_aggregate(scheme, s, K):
    return int(_max_aggregate(int(scheme), int(s), int(K)))


def check_width(scheme, s, K, bits):
    """Section 4.2 headroom rule: does a signed `bits`-bit integer always hold the sum?"""
    return bool(_check_width(int(scheme), int(s), int(K), int(bits)))


def fits_width(A, bits):
    A = _arr(A, np.int64).reshape(-1)
    return bool(_fits_width(_ptr(A, C.c_int64), A.shape[0], int(bits)))


def dequantize(A, norm, scheme, s, K):
    """Eq. (1): norm * (1/n) * sum, in binary64."""
    A = _arr(A, np.int64).reshape(-1)
    out = np.zeros(A.shape[0], np.float64)
    _dequantize(_ptr(A, C.c_int64), A.shape[0], float(norm), int(scheme), int(s), int(K), _ptr(out, C.c_double))
    return out


def pack(q, fmt):
    """Signed codes -> (level bytes, sign words or None).  Raises if a code does not fit."""
    q = _arr(q, np.int32).reshape(-1)
    d = q.shape[0]
    lv = np.zeros(int(_levels_bytes(d, int(fmt))), np.uint8)
    sp = np.zeros(int(_signplane_words(d)), np.uint32)
    rc = _pack(_ptr(q, C.c_int32), d, int(fmt), _ptr(lv, C.c_uint8), _ptr(sp, C.c_uint32))
    if rc != 0:
        raise OverflowError("code does not fit pack format %d" % fmt)
    return lv, (sp if fmt in (PACK_U8_SIGNPLANE, PACK_U4_SIGNPLANE) else None)


def unpack(levels, signplane, d, fmt):
    lv = _arr(levels, np.uint8).reshape(-1)
    sp = _arr(signplane if signplane is not None else np.zeros(int(_signplane_words(d)), np.uint32), np.uint32)
    q = np.zeros(int(d), np.int32)
    _unpack(_ptr(lv, C.c_uint8), _ptr(sp, C.c_uint32), int(d), int(fmt), _ptr(q, C.c_int32))
    return q


def quantize_aggregate(xs, norm, scheme, s, seed, index_base=0, rng_bits=32):
    """Quantize every worker (worker word = position in xs) and sum: the unfused composition."""
    rows, ptrs, K, d = _rows(xs, np.float32, C.c_float)
    A = np.zeros(d, np.int64)
    rc = _quantize_aggregate(ptrs, K, d, float(np.float32(norm)), int(scheme), int(s), int(seed),
                             int(index_base), int(rng_bits), _ptr(A, C.c_int64))
    if rc != 0:
        raise MemoryError("oracle could not allocate the code vectors")
    return A


def alg2_k(r, s):
    """Algorithm 2, first statement: k = -floor(log2(max(p, 2^-m))), m = s + 1, for p = r / 2^s (r an s-bit integer)."""
    return int(_alg2_k(int(r), int(s)))


def alg2_draw(seed, node, g, s):
    """The s random bits of tree node `node` at coordinate g (stream 1 of the Philox counter)."""
    return int(_alg2_draw(int(seed), int(node), int(g), int(s)))


def alg2_field_bits(s):
    """Width W of the field a node's s random bits are the top of: 8, 16 or 32."""
    return int(_alg2_field_bits(int(s)))


def exp_reduce_pair(sign1, e1, sign2, e2, k):
    """Algorithm 2, the reduction of one pair, on (sign, e) pairs standing for sign * 2^-e (e = 0: zero)."""
    sr, er = C.c_int(0), C.c_int(0)
    _exp_reduce_pair(int(sign1), int(e1), int(sign2), int(e2), int(k), C.byref(sr), C.byref(er))
    return sr.value, er.value


def random_word_of(seed, word2, word3, g):
    """Philox4x32-10 word of coordinate g for counter words (lo32(g/4), hi32(g/4), word2, word3)."""
    return int(_random_word_of(int(seed), int(word2), int(word3), int(g)))


def exp_tree_reduce(qs, s, seed, index_base=0):
    """Algorithm 2 applied in tree order to K workers' exponential-grid codes: sign*e of the root."""
    rows, ptrs, K, d = _rows(qs, np.int32, C.c_int32)
    out = np.zeros(d, np.int32)
    _exp_tree_reduce(ptrs, K, d, int(s), int(seed), int(index_base), _ptr(out, C.c_int32))
    return out


def exp_reduce_dequantize(se, norm, K):
    """The mean that a reduced (sign, e) stands for: sign * 2^-e * 2n' * norm / K, in binary64."""
    se = _arr(se, np.int32).reshape(-1)
    out = np.zeros(se.shape[0], np.float64)
    _exp_reduce_dequantize(_ptr(se, C.c_int32), se.shape[0], float(norm), int(K), _ptr(out, C.c_double))
    return out


def avg_pair(a, b, coin):
    """Implementation section, one reduce step with averaging: round((a+b)/2), an odd sum going up iff coin."""
    return int(_avg_pair(int(a), int(b), int(coin)))


def avg_tree_reduce(qs, seed, index_base=0):
    """In-step averaging of K workers' linear codes in tree order: the root's code."""
    rows, ptrs, K, d = _rows(qs, np.int32, C.c_int32)
    out = np.zeros(d, np.int32)
    _avg_tree_reduce(ptrs, K, d, int(seed), int(index_base), _ptr(out, C.c_int32))
    return out


def avg_reduce_dequantize(code, norm, s, K):
    """The mean over K workers that an averaged code stands for, in binary64."""
    code = _arr(code, np.int32).reshape(-1)
    out = np.zeros(code.shape[0], np.float64)
    _avg_reduce_dequantize(_ptr(code, C.c_int32), code.shape[0], float(norm), int(s), int(K), _ptr(out, C.c_double))
    return out


def compact(q, capacity=None):
    """Algorithm 1's sparse branch, sender side: (count, indices, codes) of the non-zero codes, by increasing index.
    At most `capacity` pairs are returned; count is always the true number."""
    q = _arr(q, np.int32).reshape(-1)
    cap = q.shape[0] if capacity is None else int(capacity)
    idx = np.zeros(max(cap, 1), np.uint32); val = np.zeros(max(cap, 1), np.int32)
    n = int(_compact(_ptr(q, C.c_int32), q.shape[0], cap, _ptr(idx, C.c_uint32), _ptr(val, C.c_int32)))
    m = min(n, cap)
    return n, idx[:m].copy(), val[:m].copy()


def sparse_nnz_bound(scheme, s, K, d):
    """Theorem 1's sparsity statement as Eq. (2) implies it: E[non-zero codes over all K workers] <= top^2 + top*sqrt(K d)
    under the (2,2) norm, top = s or 2^(s-1); capped at K d; -1 for invalid arguments."""
    return float(_sparse_nnz_bound(int(scheme), int(s), int(K), int(d)))


def sparse_aggregate(indices, codes, d, scheme):
    """Algorithm 1's sparse branch, receiver side: the dense integer sum formed from K lists."""
    K = len(indices)
    ii = [_arr(a, np.uint32).reshape(-1) for a in indices]
    cc = [_arr(a, np.int32).reshape(-1) for a in codes]
    cnt = np.array([a.shape[0] for a in ii], np.int64)
    ip = (C.POINTER(C.c_uint32) * K)(*[_ptr(a, C.c_uint32) for a in ii])
    cp = (C.POINTER(C.c_int32) * K)(*[_ptr(a, C.c_int32) for a in cc])
    A = np.zeros(int(d), np.int64)
    _sparse_aggregate(ip, cp, _ptr(cnt, C.c_int64), K, int(d), int(scheme), _ptr(A, C.c_int64))
    return A
