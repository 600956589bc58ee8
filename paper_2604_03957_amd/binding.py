"""Thin ctypes binding of ``csrc/libbwta.so`` (the C ABI declared in ``include/bwta.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.  Tensors are
torch CUDA tensors used as device buffers; the current torch stream is passed through.
Importing this module without the compiled library raises -- there is no fallback.
"""
import ctypes
import os

# torch ships its own HIP runtime; load it first so that libbwta.so binds to the same runtime
# (same SONAME) instead of bringing a second one into the process.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
# BWTA_LIB: load this build of the same sources instead (the sanitizer test's host-instrumented one)
LIB_PATH = os.environ.get("BWTA_LIB") or os.path.join(_HERE, "csrc", "libbwta.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TOO_LARGE = -1, -2, -3, -4, -5, -6, -7
DTYPE_FP16, DTYPE_INT8 = 0, 1
SCALE_NONE, SCALE_SCALAR, SCALE_VECTOR = 0, 1, 2
PATH_AUTO, PATH_POPC, PATH_MFMA, PATH_FP4 = 0, 1, 2, 3
PREPARED_PLANES, PREPARED_FP4 = 1, 2
KERNEL_GEMV_POPC, KERNEL_GEMV_FP4, KERNEL_GEMM_FP4, KERNEL_GEMM_MFMA_I8, KERNEL_GEMM_POPC = 1, 2, 3, 4, 5

EXPORTS = ["bwta_plane_row_words", "bwta_workspace_bytes", "bwta_quantize_pack_act",
           "bwta_pack_weights", "bwta_gemm", "bwta_linear", "bwta_linear_static", "bwta_static_scratch_bytes",
           "bwta_static_scratch_init", "bwta_strerror", "bwta_last_hip_error",
           "bwta_build_id", "bwta_set_path", "bwta_get_path", "bwta_auto_path", "bwta_linear_launches", "bwta_version", "bwta_set_tile",
           "bwta_prepared_bytes", "bwta_prepared_format", "bwta_planned_kernel", "bwta_prepare_act", "bwta_gemm_prepared", "bwta_gemm_grouped",
           "bwta_quantize_pack_bool", "bwta_matmul_tt", "bwta_prepare_weights", "bwta_act_scale",
           "bwta_prepare_act_autoscale", "bwta_matmul_bool_prepared"]

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2604_03957_amd/build.py); there is no CPU fallback" % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)
_c = ctypes
_P = _c.c_void_p
_lib.bwta_plane_row_words.restype = _c.c_int64
_lib.bwta_plane_row_words.argtypes = [_c.c_int]
_lib.bwta_workspace_bytes.restype = _c.c_size_t
_lib.bwta_workspace_bytes.argtypes = [_c.c_int, _c.c_int, _c.c_int]
_lib.bwta_quantize_pack_act.restype = _c.c_int
_lib.bwta_quantize_pack_act.argtypes = [_P, _c.c_int, _c.c_int64, _P, _c.c_int, _c.c_int, _c.c_int,
                                        _P, _P, _P, _P]
_lib.bwta_pack_weights.restype = _c.c_int
_lib.bwta_pack_weights.argtypes = [_P, _c.c_int, _c.c_int64, _c.c_int, _c.c_int, _P, _P]
_lib.bwta_gemm.restype = _c.c_int
_lib.bwta_gemm.argtypes = [_P, _P, _P, _c.c_int, _c.c_int, _c.c_int, _P, _c.c_int, _P, _c.c_int,
                           _P, _P, _c.c_int64, _P, _c.c_size_t, _P]
_lib.bwta_linear.restype = _c.c_int
_lib.bwta_linear.argtypes = [_P, _c.c_int64, _P, _c.c_int, _P, _P, _c.c_int, _c.c_int, _c.c_int,
                             _c.c_int, _P, _c.c_int64, _P, _c.c_size_t, _P]
_lib.bwta_linear_static.restype = _c.c_int
_lib.bwta_linear_static.argtypes = [_P, _c.c_int64, _P, _c.c_int, _P, _P, _c.c_int, _c.c_int, _c.c_int,
                                    _c.c_int, _P, _c.c_int64, _P]
_lib.bwta_static_scratch_bytes.restype = _c.c_size_t
_lib.bwta_static_scratch_init.restype = _c.c_int
_lib.bwta_prepared_bytes.restype = _c.c_size_t
_lib.bwta_prepared_bytes.argtypes = [_c.c_int, _c.c_int]
_lib.bwta_prepare_act.restype = _c.c_int
_lib.bwta_planned_kernel.restype = _c.c_int
_lib.bwta_planned_kernel.argtypes = [_c.c_int, _c.c_int, _c.c_int, _c.c_int]
_lib.bwta_prepared_format.restype = _c.c_int
_lib.bwta_prepared_format.argtypes = [_c.c_int, _c.c_int]
_lib.bwta_prepare_act.argtypes = [_P, _c.c_int64, _P, _c.c_int, _c.c_int, _c.c_int, _P, _c.c_size_t,
                                  _c.POINTER(_c.c_int), _P]
_lib.bwta_gemm_prepared.restype = _c.c_int
_lib.bwta_gemm_prepared.argtypes = [_P, _c.c_size_t, _c.c_int, _P, _c.c_int, _c.c_int, _c.c_int, _P, _c.c_int, _P,
                                    _c.c_int, _P, _P, _c.c_int64, _P]


class GemmProblem(_c.Structure):
    _fields_ = [("mask", _P), ("sign", _P), ("wsign", _P), ("s_a", _P), ("s_w", _P), ("acc", _P), ("out", _P)]


_lib.bwta_gemm_grouped.restype = _c.c_int
_lib.bwta_gemm_grouped.argtypes = [_c.POINTER(GemmProblem), _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                   _c.c_int64, _P, _c.c_size_t, _P]
_lib.bwta_quantize_pack_bool.restype = _c.c_int
_lib.bwta_quantize_pack_bool.argtypes = [_P, _c.c_int64, _P, _c.c_int, _c.c_int, _c.c_int, _P, _P]
_lib.bwta_matmul_tt.restype = _c.c_int
_lib.bwta_matmul_tt.argtypes = [_P, _P, _c.c_int64, _P, _P, _c.c_int64, _c.c_int, _c.c_int, _c.c_int, _c.c_int,
                                _P, _c.c_int, _P, _c.c_int, _c.c_float, _P, _P, _c.c_int64, _c.c_int64, _P]
_lib.bwta_prepare_weights.restype = _c.c_int
_lib.bwta_prepare_weights.argtypes = [_P, _c.c_int64, _c.c_int, _c.c_int, _P, _P, _P]
_lib.bwta_act_scale.restype = _c.c_int
_lib.bwta_act_scale.argtypes = [_P, _c.c_int64, _c.c_int, _c.c_int, _P, _P]
_lib.bwta_prepare_act_autoscale.restype = _c.c_int
_lib.bwta_matmul_bool_prepared.restype = _c.c_int
_lib.bwta_matmul_bool_prepared.argtypes = [_P, _c.c_int64, _P, _c.c_size_t, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _c.c_int, _P, _c.c_int,
                                           _P, _c.c_int, _c.c_float, _P, _c.c_int64, _c.c_int64, _P]
_lib.bwta_prepare_act_autoscale.argtypes = [_P, _c.c_int64, _c.c_int, _c.c_int, _P, _P, _c.c_size_t,
                                            _c.POINTER(_c.c_int), _P]
_lib.bwta_strerror.restype = _c.c_char_p
_lib.bwta_strerror.argtypes = [_c.c_int]
_lib.bwta_last_hip_error.restype = _c.c_int
_lib.bwta_set_path.restype = _c.c_int
_lib.bwta_set_path.argtypes = [_c.c_int]
_lib.bwta_get_path.restype = _c.c_int
_lib.bwta_auto_path.restype = _c.c_int
_lib.bwta_auto_path.argtypes = [_c.c_int, _c.c_int, _c.c_int]
_lib.bwta_linear_launches.restype = _c.c_int
_lib.bwta_linear_launches.argtypes = [_c.c_int, _c.c_int, _c.c_int]
_lib.bwta_version.restype = _c.c_int
_lib.bwta_build_id.restype = _c.c_char_p
_lib.bwta_set_tile.restype = _c.c_int
_lib.bwta_set_tile.argtypes = [_c.c_int]


class BwtaError(RuntimeError):
    def __init__(self, code):
        self.code = code
        msg = _lib.bwta_strerror(code).decode()
        if code == ERR_HIP:
            msg += " [hipError %d]" % _lib.bwta_last_hip_error()
        super().__init__("bwta error %d: %s" % (code, msg))


def raw():
    """The ctypes library handle, for tests that probe error codes directly."""
    return _lib


def _check(code):
    if code != OK:
        raise BwtaError(code)


def _ptr(x):
    """Device pointer of a torch tensor, a raw integer address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


# The raw handle of torch's current stream: the two C entry points below cost ~0.3 us together,
# torch.cuda.current_stream().cuda_stream ~3 us (it builds a Python Stream object per call), which
# is as much as the kernel launch itself.
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_cur_device = getattr(torch._C, "_cuda_getDevice", None)


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    if _raw_stream is not None and _cur_device is not None:
        return _raw_stream(_cur_device())
    return torch.cuda.current_stream().cuda_stream


def _mode(s, mode):
    if mode is not None:
        return mode
    if s is None:
        return SCALE_NONE
    return SCALE_SCALAR if s.numel() == 1 else SCALE_VECTOR


def plane_row_words(K):
    return int(_lib.bwta_plane_row_words(K))


def workspace_bytes(M, N, K):
    return int(_lib.bwta_workspace_bytes(M, N, K))


def strerror(code):
    return _lib.bwta_strerror(code).decode()


def set_path(path):
    _check(_lib.bwta_set_path(path))


def get_path():
    return int(_lib.bwta_get_path())


def auto_path(M, N, K):
    return int(_lib.bwta_auto_path(M, N, K))


def linear_launches(M, N, K):
    return int(_lib.bwta_linear_launches(M, N, K))


def set_tile(tile):
    _check(_lib.bwta_set_tile(int(tile)))


def version():
    return int(_lib.bwta_version())


def build_id():
    return _lib.bwta_build_id().decode()


def bwta_quantize_pack_act(A, s_a, mask, sign, nnz=None, *, M, K, lda=None, a_dtype=DTYPE_FP16,
                           scale_mode=None, stream=None):
    lda = K if lda is None else lda
    _check(_lib.bwta_quantize_pack_act(_ptr(A), a_dtype, lda, _ptr(s_a), _mode(s_a, scale_mode), M, K,
                                       _ptr(mask), _ptr(sign), _ptr(nnz), _stream(stream)))


def bwta_pack_weights(W, wsign, *, N, K, ldw=None, w_dtype=DTYPE_INT8, stream=None):
    ldw = K if ldw is None else ldw
    _check(_lib.bwta_pack_weights(_ptr(W), w_dtype, ldw, N, K, _ptr(wsign), _stream(stream)))


def bwta_gemm(mask, sign, wsign, s_a, s_w, acc, out, workspace, *, M, N, K, ldo=None,
              a_scale_mode=None, w_scale_mode=None, workspace_bytes=None, stream=None):
    ldo = N if ldo is None else ldo
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()
    _check(_lib.bwta_gemm(_ptr(mask), _ptr(sign), _ptr(wsign), M, N, K, _ptr(s_a), _mode(s_a, a_scale_mode),
                          _ptr(s_w), _mode(s_w, w_scale_mode), _ptr(acc), _ptr(out), ldo,
                          _ptr(workspace), workspace_bytes, _stream(stream)))


def bwta_linear(A, s_a, wsign, s_w, out, workspace, *, M, N, K, lda=None, ldo=None, a_scale_mode=None,
                w_scale_mode=None, workspace_bytes=None, stream=None):
    lda = K if lda is None else lda
    ldo = N if ldo is None else ldo
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None or isinstance(workspace, int) else workspace.numel() * workspace.element_size()
    _check(_lib.bwta_linear(_ptr(A), lda, _ptr(s_a), _mode(s_a, a_scale_mode), _ptr(wsign), _ptr(s_w),
                            _mode(s_w, w_scale_mode), M, N, K, _ptr(out), ldo, _ptr(workspace),
                            workspace_bytes, _stream(stream)))


def static_scratch_bytes():
    return int(_lib.bwta_static_scratch_bytes())


def static_scratch_init():
    _check(_lib.bwta_static_scratch_init())


def bwta_linear_static(A, s_a, wsign, s_w, out, *, M, N, K, lda=None, ldo=None, a_scale_mode=None,
                       w_scale_mode=None, stream=None):
    lda = K if lda is None else lda
    ldo = N if ldo is None else ldo
    _check(_lib.bwta_linear_static(_ptr(A), lda, _ptr(s_a), _mode(s_a, a_scale_mode), _ptr(wsign), _ptr(s_w),
                                   _mode(s_w, w_scale_mode), M, N, K, _ptr(out), ldo, _stream(stream)))


def bwta_quantize_pack_bool(A, s_a, mask, *, M, K, lda=None, scale_mode=None, stream=None):
    lda = K if lda is None else lda
    _check(_lib.bwta_quantize_pack_bool(_ptr(A), lda, _ptr(s_a), _mode(s_a, scale_mode), M, K, _ptr(mask),
                                        _stream(stream)))


def bwta_matmul_tt(maskA, signA, maskB, signB, s_a, s_b, acc, out, *, batch, M, N, K, alpha=1.0, strideA=None,
                   strideB=None, ldo=None, stride_out=None, a_scale_mode=None, b_scale_mode=None, stream=None):
    rw = plane_row_words(K)
    strideA = M * rw if strideA is None else strideA
    strideB = N * rw if strideB is None else strideB
    ldo = N if ldo is None else ldo
    stride_out = M * ldo if stride_out is None else stride_out
    _check(_lib.bwta_matmul_tt(_ptr(maskA), _ptr(signA), strideA, _ptr(maskB), _ptr(signB), strideB, batch, M, N, K,
                               _ptr(s_a), _mode(s_a, a_scale_mode), _ptr(s_b), _mode(s_b, b_scale_mode), float(alpha),
                               _ptr(acc), _ptr(out), ldo, stride_out, _stream(stream)))


def bwta_prepare_weights(W, wsign, s_w, *, N, K, ldw=None, stream=None):
    ldw = K if ldw is None else ldw
    _check(_lib.bwta_prepare_weights(_ptr(W), ldw, N, K, _ptr(wsign), _ptr(s_w), _stream(stream)))


def bwta_act_scale(A, s, *, M, K, lda=None, stream=None):
    lda = K if lda is None else lda
    _check(_lib.bwta_act_scale(_ptr(A), lda, M, K, _ptr(s), _stream(stream)))


def _nbytes(buf, given):
    if given is not None:
        return given
    return 0 if buf is None or isinstance(buf, int) else buf.numel() * buf.element_size()


def prepared_bytes(M, K):
    return int(_lib.bwta_prepared_bytes(M, K))


def planned_kernel(operand, M, N, K):
    return int(_lib.bwta_planned_kernel(operand, M, N, K))


def prepared_format(M, K):
    return int(_lib.bwta_prepared_format(M, K))


def bwta_prepare_act(A, s_a, prepared, *, M, K, lda=None, a_scale_mode=None, prepared_bytes=None, stream=None):
    """Returns the format id of what was written; hand it to the call that consumes `prepared`."""
    lda = K if lda is None else lda
    fmt = _c.c_int(0)
    _check(_lib.bwta_prepare_act(_ptr(A), lda, _ptr(s_a), _mode(s_a, a_scale_mode), M, K, _ptr(prepared),
                                 _nbytes(prepared, prepared_bytes), _c.byref(fmt), _stream(stream)))
    return fmt.value


def bwta_prepare_act_autoscale(A, s_a, prepared, *, M, K, lda=None, prepared_bytes=None, stream=None):
    """Returns the format id of what was written, as bwta_prepare_act."""
    lda = K if lda is None else lda
    fmt = _c.c_int(0)
    _check(_lib.bwta_prepare_act_autoscale(_ptr(A), lda, M, K, _ptr(s_a), _ptr(prepared),
                                           _nbytes(prepared, prepared_bytes), _c.byref(fmt), _stream(stream)))
    return fmt.value


def bwta_matmul_bool_prepared(maskA, preparedB, s_a, s_b, out, *, fmt, batch, M, N, K, alpha=1.0, strideA=None, ldo=None,
                              stride_out=None, a_scale_mode=None, b_scale_mode=None, prepared_bytes=None, stream=None):
    rw = plane_row_words(K)
    strideA = M * rw if strideA is None else strideA
    ldo = N if ldo is None else ldo
    stride_out = M * ldo if stride_out is None else stride_out
    _check(_lib.bwta_matmul_bool_prepared(_ptr(maskA), strideA, _ptr(preparedB), _nbytes(preparedB, prepared_bytes),
                                          fmt, batch, M, N, K, _ptr(s_a), _mode(s_a, a_scale_mode), _ptr(s_b),
                                          _mode(s_b, b_scale_mode), float(alpha), _ptr(out), ldo, stride_out,
                                          _stream(stream)))


def bwta_gemm_prepared(prepared, wsign, s_a, s_w, acc, out, *, fmt, M, N, K, ldo=None, a_scale_mode=None,
                       w_scale_mode=None, prepared_bytes=None, stream=None):
    ldo = N if ldo is None else ldo
    _check(_lib.bwta_gemm_prepared(_ptr(prepared), _nbytes(prepared, prepared_bytes), fmt, _ptr(wsign), M, N, K,
                                   _ptr(s_a), _mode(s_a, a_scale_mode), _ptr(s_w), _mode(s_w, w_scale_mode),
                                   _ptr(acc), _ptr(out), ldo, _stream(stream)))


def make_problems(problems):
    """problems: list of (mask, sign, wsign, s_a, s_w, acc, out) tensors/addresses -> ctypes array
    (build once, reuse across calls)."""
    arr = (GemmProblem * len(problems))()
    for i, p in enumerate(problems):
        for name, v in zip(("mask", "sign", "wsign", "s_a", "s_w", "acc", "out"), p):
            setattr(arr[i], name, _ptr(v))
    return arr


def bwta_gemm_grouped(problem_array, workspace, *, M, N, K, a_scale_mode=SCALE_VECTOR, w_scale_mode=SCALE_VECTOR,
                      ldo=None, workspace_bytes=None, stream=None):
    ldo = N if ldo is None else ldo
    _check(_lib.bwta_gemm_grouped(problem_array, len(problem_array), M, N, K, a_scale_mode, w_scale_mode, ldo,
                                  _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream)))
