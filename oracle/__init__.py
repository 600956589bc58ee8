"""ctypes front end of the CPU oracle (``bwta_oracle.c``).

Test infrastructure only: tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this; the product package never does, and this
module never imports the product package.  All arguments are numpy arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bwta_oracle.c")
_LIB = os.path.join(_HERE, "libbwta_oracle.so")

SCALE_NONE, SCALE_SCALAR, SCALE_VECTOR = 0, 1, 2


def build(force=False, out=None, extra_flags=()):
    """Compile the oracle with gcc (plain -O2, OpenMP for the row loops).  `out` / `extra_flags`:
    a second build elsewhere, e.g. an instrumented one for the sanitizer test."""
    if out is not None:
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]
                              + list(extra_flags) + ["-o", out, _SRC, "-lm"])
        return out
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # BWTA_ORACLE_LIB: load this build of the same source instead (the sanitizer test's)
        L = ctypes.CDLL(os.environ.get("BWTA_ORACLE_LIB") or build())
        c = ctypes
        P = c.c_void_p
        L.bwta_oracle_num_threads.restype = c.c_int
        L.bwta_oracle_set_num_threads.argtypes = [c.c_int]
        L.bwta_oracle_half_to_double.restype = c.c_double
        L.bwta_oracle_half_to_double.argtypes = [c.c_uint16]
        L.bwta_oracle_double_to_half.restype = c.c_uint16
        L.bwta_oracle_double_to_half.argtypes = [c.c_double]
        L.bwta_oracle_ternary_value.restype = c.c_int
        L.bwta_oracle_ternary_value.argtypes = [c.c_double, c.c_double]
        L.bwta_oracle_sign_value.restype = c.c_int
        L.bwta_oracle_sign_value.argtypes = [c.c_double]
        L.bwta_oracle_bool_value.restype = c.c_int
        L.bwta_oracle_bool_value.argtypes = [c.c_double, c.c_double]
        L.bwta_oracle_row_words.restype = c.c_int64
        L.bwta_oracle_row_words.argtypes = [c.c_int]
        L.bwta_oracle_ternarize.argtypes = [P, c.c_int64, P, c.c_int, c.c_int, c.c_int, P]
        L.bwta_oracle_sign_weights.argtypes = [P, c.c_int64, c.c_int, c.c_int, P]
        L.bwta_oracle_pack_act.argtypes = [P, c.c_int, c.c_int, P, P, P]
        L.bwta_oracle_pack_weights.argtypes = [P, c.c_int, c.c_int, P]
        L.bwta_oracle_unpack_act.argtypes = [P, P, c.c_int, c.c_int, P]
        L.bwta_oracle_unpack_weights.argtypes = [P, c.c_int, c.c_int, P]
        L.bwta_oracle_gemm_unpacked.argtypes = [P, P, c.c_int, c.c_int, c.c_int, P]
        L.bwta_oracle_gemm_packed.argtypes = [c.c_int, P, P, P, c.c_int, c.c_int, c.c_int, P]
        L.bwta_oracle_epilogue.argtypes = [P, P, c.c_int, P, c.c_int, c.c_int, c.c_int, P, c.c_int64]
        L.bwta_oracle_boolize.argtypes = [P, c.c_int64, P, c.c_int, c.c_int, c.c_int, P]
        L.bwta_oracle_matmul_tt_packed.argtypes = [c.c_int, P, P, P, P, c.c_int, c.c_int, c.c_int, P]
        L.bwta_oracle_epilogue_alpha.argtypes = [P, P, c.c_int, P, c.c_int, c.c_float, c.c_int, c.c_int, P, c.c_int64]
        L.bwta_oracle_prepare_weights.argtypes = [P, c.c_int64, c.c_int, c.c_int, P, P]
        L.bwta_oracle_act_scale.argtypes = [P, c.c_int64, c.c_int, c.c_int, P]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _half_bits(a):
    """View an fp16 (or already uint16) array as contiguous uint16 bit patterns."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _scale_mode(s, rows):
    if s is None:
        return SCALE_NONE
    n = int(np.asarray(s).size)
    if n == 1:
        return SCALE_SCALAR
    assert n == rows, (n, rows)
    return SCALE_VECTOR


def num_threads():
    return int(lib().bwta_oracle_num_threads())


def set_num_threads(n):
    lib().bwta_oracle_set_num_threads(int(n))


def half_to_double(bits):
    return float(lib().bwta_oracle_half_to_double(int(bits)))


def double_to_half(x):
    return int(lib().bwta_oracle_double_to_half(float(x)))


def ternary_value(a, s):
    return int(lib().bwta_oracle_ternary_value(float(a), float(s)))


def sign_value(w):
    return int(lib().bwta_oracle_sign_value(float(w)))


def bool_value(a, s):
    return int(lib().bwta_oracle_bool_value(float(a), float(s)))


def row_words(K):
    return int(lib().bwta_oracle_row_words(int(K)))


def ternarize(A, s_a=None):
    """fp16 [M, K] (+ scale None / [1] / [M]) -> int8 [M, K] in {-1, 0, +1}."""
    Ab = _half_bits(A)
    M, K = Ab.shape
    sb = _half_bits(s_a)
    t = np.empty((M, K), np.int8)
    lib().bwta_oracle_ternarize(_p(Ab), K, _p(sb), _scale_mode(sb, M), M, K, _p(t))
    return t


def sign_weights(W):
    """fp16 [N, K] -> int8 [N, K] in {-1, +1}."""
    Wb = _half_bits(W)
    N, K = Wb.shape
    w = np.empty((N, K), np.int8)
    lib().bwta_oracle_sign_weights(_p(Wb), K, N, K, _p(w))
    return w


def pack_act(t):
    """int8 ternary [M, K] -> (mask u32 [M, rw], sign u32 [M, rw], nnz i32 [M])."""
    t = np.ascontiguousarray(t, np.int8)
    M, K = t.shape
    rw = row_words(K)
    mask = np.empty((M, rw), np.uint32)
    sign = np.empty((M, rw), np.uint32)
    nnz = np.empty((M,), np.int32)
    lib().bwta_oracle_pack_act(_p(t), M, K, _p(mask), _p(sign), _p(nnz))
    return mask, sign, nnz


def pack_weights(w):
    """int8 +-1 [N, K] -> wsign u32 [N, rw]."""
    w = np.ascontiguousarray(w, np.int8)
    N, K = w.shape
    ws = np.empty((N, row_words(K)), np.uint32)
    lib().bwta_oracle_pack_weights(_p(w), N, K, _p(ws))
    return ws


def unpack_act(mask, sign, K):
    mask = np.ascontiguousarray(mask, np.uint32)
    sign = np.ascontiguousarray(sign, np.uint32)
    M = mask.shape[0]
    assert mask.shape[1] == row_words(K) and sign.shape == mask.shape
    t = np.empty((M, K), np.int8)
    lib().bwta_oracle_unpack_act(_p(mask), _p(sign), M, K, _p(t))
    return t


def unpack_weights(wsign, K):
    wsign = np.ascontiguousarray(wsign, np.uint32)
    N = wsign.shape[0]
    assert wsign.shape[1] == row_words(K)
    w = np.empty((N, K), np.int8)
    lib().bwta_oracle_unpack_weights(_p(wsign), N, K, _p(w))
    return w


def gemm_unpacked(t, w):
    """acc[m, n] = sum_k t[m, k] * w[n, k] (int32), the definition."""
    t = np.ascontiguousarray(t, np.int8)
    w = np.ascontiguousarray(w, np.int8)
    M, K = t.shape
    N, K2 = w.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    lib().bwta_oracle_gemm_unpacked(_p(t), _p(w), M, N, K, _p(acc))
    return acc


def gemm_packed(form, mask, sign, wsign, K):
    """The same product from bit planes; form 0 mask/sign, 1 xor-difference, 2 four-AND."""
    mask = np.ascontiguousarray(mask, np.uint32)
    sign = np.ascontiguousarray(sign, np.uint32)
    wsign = np.ascontiguousarray(wsign, np.uint32)
    M, N = mask.shape[0], wsign.shape[0]
    rw = row_words(K)
    assert mask.shape[1] == rw and sign.shape == mask.shape and wsign.shape[1] == rw
    acc = np.empty((M, N), np.int32)
    lib().bwta_oracle_gemm_packed(int(form), _p(mask), _p(sign), _p(wsign), M, N, K, _p(acc))
    return acc


def epilogue(acc, s_a=None, s_w=None):
    """fp16( s_w[n] * s_a[m] * acc[m, n] ) rounded once; returns a float16 array [M, N]."""
    acc = np.ascontiguousarray(acc, np.int32)
    M, N = acc.shape
    sa, sw = _half_bits(s_a), _half_bits(s_w)
    out = np.empty((M, N), np.uint16)
    lib().bwta_oracle_epilogue(_p(acc), _p(sa), _scale_mode(sa, M), _p(sw), _scale_mode(sw, N),
                               M, N, _p(out), N)
    return out.view(np.float16)


def boolize(A, s_a=None):
    """fp16 [M, K] (+ scale None / [1] / [M]) -> int8 [M, K] in {0, 1} by the bool function."""
    Ab = _half_bits(A)
    M, K = Ab.shape
    sb = _half_bits(s_a)
    b = np.empty((M, K), np.int8)
    lib().bwta_oracle_boolize(_p(Ab), K, _p(sb), _scale_mode(sb, M), M, K, _p(b))
    return b


def matmul_tt_packed(form, maskA, signA, maskB, signB, K):
    """a . b^T from (mask, sign) planes of both operands (sign None = boolean operand);
    form 0 four-AND (Cases 3 / 2), form 1 popc(u) - 2 popc(u & (sA ^ sB))."""
    maskA = np.ascontiguousarray(maskA, np.uint32)
    maskB = np.ascontiguousarray(maskB, np.uint32)
    signA = None if signA is None else np.ascontiguousarray(signA, np.uint32)
    signB = None if signB is None else np.ascontiguousarray(signB, np.uint32)
    M, N = maskA.shape[0], maskB.shape[0]
    assert maskA.shape[1] == row_words(K) == maskB.shape[1]
    acc = np.empty((M, N), np.int32)
    lib().bwta_oracle_matmul_tt_packed(int(form), _p(maskA), None if signA is None else _p(signA), _p(maskB),
                                       None if signB is None else _p(signB), M, N, K, _p(acc))
    return acc


def epilogue_alpha(acc, s_a=None, s_b=None, alpha=1.0):
    """fp16( acc * fp32(alpha * (s_a[m] * s_b[n])) ); returns a float16 array [M, N]."""
    acc = np.ascontiguousarray(acc, np.int32)
    M, N = acc.shape
    sa, sb = _half_bits(s_a), _half_bits(s_b)
    out = np.empty((M, N), np.uint16)
    lib().bwta_oracle_epilogue_alpha(_p(acc), _p(sa), _scale_mode(sa, M), _p(sb), _scale_mode(sb, N),
                                     float(np.float32(alpha)), M, N, _p(out), N)
    return out.view(np.float16)


def prepare_weights(W):
    """fp16 [N, K] -> (w int8 [N, K] = sign(W - row mean), s_w float16 [N] = row mean of |W - row mean|)."""
    Wb = _half_bits(W)
    N, K = Wb.shape
    w = np.empty((N, K), np.int8)
    s = np.empty(N, np.uint16)
    lib().bwta_oracle_prepare_weights(_p(Wb), K, N, K, _p(w), _p(s))
    return w, s.view(np.float16)


def act_scale(A):
    """fp16 [M, K] -> float16 [M]: 2 * mean_k |A[m, k]|, exact sum, one rounding."""
    Ab = _half_bits(A)
    M, K = Ab.shape
    s = np.empty(M, np.uint16)
    lib().bwta_oracle_act_scale(_p(Ab), K, M, K, _p(s))
    return s.view(np.float16)


def linear(A, s_a, w, s_w):
    """Whole layer: fp16 A [M, K], s_a, int8 +-1 weights [N, K], s_w -> (t, acc, out fp16)."""
    t = ternarize(A, s_a)
    acc = gemm_unpacked(t, w)
    return t, acc, epilogue(acc, s_a, s_w)
