"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
the header declares, and rejects bad arguments before anything could be enqueued."""
import os
import re

import pytest

from paper_2604_03957_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # a well-aligned, never dereferenced "device" address


def declared_functions():
    names = set()
    for header in ("bwta.h", "bwta_tuning.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(bwta_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(B.raw(), n), n


def test_row_words_and_workspace():
    assert [B.plane_row_words(k) for k in (0, 1, 128, 129, 768, 4096, 11008)] == [0, 4, 4, 8, 24, 128, 344]
    assert B.workspace_bytes(0, 5, 5) == 0
    ws = B.workspace_bytes(4096, 3072, 768)
    assert ws % 256 == 0 and ws >= 2 * 4096 * 24 * 4 + 4096 * 768 // 2
    assert B.version() >= 1
    assert B.strerror(B.ERR_ALIGN) and B.strerror(0) == "ok"


def test_path_selection():
    assert B.get_path() == B.PATH_AUTO
    B.set_path(B.PATH_POPC)
    assert B.get_path() == B.PATH_POPC
    B.set_path(B.PATH_AUTO)
    with pytest.raises(B.BwtaError) as e:
        B.set_path(7)
    assert e.value.code == B.ERR_UNSUPPORTED
    assert B.auto_path(1, 11008, 4096) == B.PATH_POPC and B.auto_path(16, 11008, 4096) == B.PATH_FP4
    assert B.auto_path(2048, 4096, 4096) in (B.PATH_MFMA, B.PATH_FP4)
    # launches of bwta_linear: one kernel for short K on prefill shapes, two otherwise; the hook turns it off
    assert B.linear_launches(4096, 3072, 768) == 1 and B.linear_launches(4096, 768, 3072) == 2
    assert B.linear_launches(1, 768, 768) == 2 and B.linear_launches(16384, 11008, 1024) == 2
    assert B.linear_launches(16, 768, 768) == 1
    assert B.linear_launches(0, 8, 8) == 0 and B.linear_launches(8, 8, -1) == 0
    B.set_tile(900)
    try:
        assert B.linear_launches(4096, 3072, 768) == 2
    finally:
        B.set_tile(0)
    assert B.linear_launches(4096, 3072, 768) == 1


def _code(fn, *a, **k):
    with pytest.raises(B.BwtaError) as e:
        fn(*a, **k)
    return e.value.code


def test_quantize_pack_rejects_bad_arguments():
    q = B.bwta_quantize_pack_act
    kw = dict(M=4, K=256, stream=0, scale_mode=B.SCALE_VECTOR)
    assert _code(q, None, FAKE, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(q, FAKE, None, FAKE, FAKE, **kw) == B.ERR_NULL          # scale needed in VECTOR mode
    assert _code(q, FAKE, FAKE, FAKE + 4, FAKE, **kw) == B.ERR_ALIGN       # planes are 16-byte aligned
    assert _code(q, FAKE, FAKE, FAKE, FAKE, **dict(kw, lda=255)) == B.ERR_SHAPE
    assert _code(q, FAKE, FAKE, FAKE, FAKE, **dict(kw, M=-1)) == B.ERR_SHAPE
    assert _code(q, FAKE, FAKE, FAKE, FAKE, **dict(kw, K=0)) == B.ERR_SHAPE
    assert _code(q, FAKE, FAKE, FAKE, FAKE, **dict(kw, a_dtype=9)) == B.ERR_UNSUPPORTED
    assert _code(q, FAKE, FAKE, FAKE, FAKE, **dict(kw, scale_mode=5)) == B.ERR_UNSUPPORTED
    q(FAKE, FAKE, FAKE, FAKE, **dict(kw, M=0))                            # empty input is a no-op


def test_pack_weights_rejects_bad_arguments():
    p = B.bwta_pack_weights
    assert _code(p, None, FAKE, N=4, K=128, stream=0) == B.ERR_NULL
    assert _code(p, FAKE, FAKE + 8, N=4, K=128, stream=0) == B.ERR_ALIGN
    assert _code(p, FAKE, FAKE, N=4, K=128, ldw=64, stream=0) == B.ERR_SHAPE
    assert _code(p, FAKE, FAKE, N=4, K=128, w_dtype=3, stream=0) == B.ERR_UNSUPPORTED
    p(FAKE, FAKE, N=0, K=128, stream=0)


def test_gemm_and_linear_reject_bad_arguments():
    g = B.bwta_gemm
    ws = B.workspace_bytes(8, 8, 128)
    kw = dict(M=8, N=8, K=128, stream=0, workspace_bytes=ws, a_scale_mode=B.SCALE_VECTOR,
              w_scale_mode=B.SCALE_VECTOR)
    assert _code(g, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **kw) == B.ERR_NULL   # a NULL mask alone is legal (binary activations)
    assert _code(g, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, **kw) == B.ERR_NULL   # no output at all
    assert _code(g, FAKE, FAKE, FAKE + 4, FAKE, FAKE, FAKE, FAKE, FAKE, **kw) == B.ERR_ALIGN
    assert _code(g, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, ldo=7)) == B.ERR_SHAPE
    assert _code(g, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, **kw) == B.ERR_WORKSPACE
    assert _code(g, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, workspace_bytes=ws - 1)) == B.ERR_WORKSPACE
    assert _code(g, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 16, **kw) == B.ERR_ALIGN
    assert _code(g, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, **kw) == B.ERR_NULL    # s_a missing
    g(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, N=0))
    lin = B.bwta_linear
    assert _code(lin, FAKE, FAKE, FAKE, FAKE, None, FAKE, **kw) == B.ERR_NULL
    assert _code(lin, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, lda=100)) == B.ERR_SHAPE
    assert _code(lin, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, workspace_bytes=0)) == B.ERR_WORKSPACE
    lin(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, **dict(kw, M=0))


def test_prepare_and_gemm_prepared_reject_bad_arguments():
    pb = B.prepared_bytes(8, 128)
    assert pb % 256 == 0 and pb > 0 and B.prepared_bytes(0, 128) == 0
    kw = dict(M=8, K=128, stream=0, a_scale_mode=B.SCALE_VECTOR, prepared_bytes=pb)
    assert _code(B.bwta_prepare_act, None, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(B.bwta_prepare_act, FAKE, FAKE, FAKE, **dict(kw, prepared_bytes=pb - 1)) == B.ERR_WORKSPACE
    assert _code(B.bwta_prepare_act, FAKE, FAKE, FAKE + 32, **kw) == B.ERR_ALIGN
    assert _code(B.bwta_prepare_act, FAKE, FAKE, FAKE, **dict(kw, lda=64)) == B.ERR_SHAPE
    kw = dict(M=8, N=8, K=128, stream=0, a_scale_mode=B.SCALE_VECTOR, w_scale_mode=B.SCALE_VECTOR, prepared_bytes=pb,
              fmt=B.PREPARED_PLANES)
    g = B.bwta_gemm_prepared
    assert _code(g, None, FAKE, FAKE, FAKE, None, FAKE, **kw) == B.ERR_WORKSPACE
    assert _code(g, FAKE, None, FAKE, FAKE, None, FAKE, **kw) == B.ERR_NULL
    assert _code(g, FAKE, FAKE, FAKE, FAKE, None, None, **kw) == B.ERR_NULL
    assert _code(g, FAKE, FAKE, FAKE, FAKE, None, FAKE, **dict(kw, ldo=4)) == B.ERR_SHAPE
    # the operand's format travels with it: an id that names neither layout is refused before any launch
    for bad in (0, 3, -1, 77):
        assert _code(g, FAKE, FAKE, FAKE, FAKE, None, FAKE, **dict(kw, fmt=bad)) == B.ERR_UNSUPPORTED


def test_prepared_format_and_planned_kernel():
    """What bwta_prepare_act writes is decided once and reported; the consumer's kernel follows from
    that id and the shape, never from a second look at the path setting.  In particular prepared
    planes never resolve to the tiled FP4 kernel, which would need scratch the call does not have:
    that includes a decode-sized token count against a packed matrix too large for the decode
    kernel's 32-bit offsets (the shape that used to fall through to it)."""
    assert B.prepared_format(2048, 4096) == B.PREPARED_FP4 and B.prepared_format(16, 4096) == B.PREPARED_PLANES
    assert B.prepared_format(128, 11008) == B.PREPARED_PLANES and B.prepared_format(129, 11008) == B.PREPARED_FP4
    assert B.planned_kernel(B.PREPARED_FP4, 2048, 4096, 4096) == B.KERNEL_GEMM_FP4
    assert B.planned_kernel(B.PREPARED_PLANES, 16, 11008, 4096) == B.KERNEL_GEMV_FP4
    assert B.planned_kernel(0, 2048, 4096, 4096) == B.KERNEL_GEMM_FP4
    assert B.planned_kernel(0, 1, 4096, 4096) == B.KERNEL_GEMV_POPC
    huge_n = (1 << 32) // (344 * 4) + 1                       # (N + 4096) * row bytes no longer fits 32 bits
    for M in (2, 16, 128):
        assert B.planned_kernel(0, M, huge_n, 11008) == B.KERNEL_GEMM_FP4          # with a workspace: tiled kernel
        k = B.planned_kernel(B.PREPARED_PLANES, M, huge_n, 11008)
        assert k in (B.KERNEL_GEMM_MFMA_I8, B.KERNEL_GEMM_POPC, B.KERNEL_GEMV_POPC), k
    # prepared planes under every path setting, over a grid of shapes: never the kernel that needs scratch
    try:
        for path in (B.PATH_AUTO, B.PATH_POPC, B.PATH_MFMA, B.PATH_FP4):
            B.set_path(path)
            for M in (1, 2, 16, 128, 129, 2048):
                for N in (1, 128, 4096, huge_n):
                    for K in (32, 1024, 4096, 11008, 30000):
                        assert B.planned_kernel(B.PREPARED_PLANES, M, N, K) not in (0, B.KERNEL_GEMM_FP4)
                        assert B.planned_kernel(B.PREPARED_FP4, M, N, K) == B.KERNEL_GEMM_FP4
    finally:
        B.set_path(B.PATH_AUTO)
    assert B.planned_kernel(5, 8, 8, 8) == 0 and B.planned_kernel(0, 0, 8, 8) == 0


def test_attention_entry_points_reject_bad_arguments():
    qb = B.bwta_quantize_pack_bool
    kw = dict(M=4, K=256, stream=0, scale_mode=B.SCALE_SCALAR)
    assert _code(qb, None, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(qb, FAKE, None, FAKE, **kw) == B.ERR_NULL
    assert _code(qb, FAKE, FAKE, FAKE + 8, **kw) == B.ERR_ALIGN
    assert _code(qb, FAKE, FAKE, FAKE, **dict(kw, lda=100)) == B.ERR_SHAPE
    qb(FAKE, FAKE, FAKE, **dict(kw, M=0))                                   # empty: nothing enqueued
    mm = B.bwta_matmul_tt
    kw = dict(batch=2, M=8, N=8, K=128, stream=0, a_scale_mode=B.SCALE_NONE, b_scale_mode=B.SCALE_NONE)
    assert _code(mm, None, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(mm, FAKE, None, FAKE, None, None, None, None, None, **kw) == B.ERR_NULL      # no output at all
    assert _code(mm, FAKE, FAKE + 4, FAKE, FAKE, None, None, FAKE, FAKE, **kw) == B.ERR_ALIGN
    assert _code(mm, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, strideA=8)) == B.ERR_SHAPE
    assert _code(mm, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, strideA=8 * 4 + 2)) == B.ERR_ALIGN
    assert _code(mm, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, ldo=4)) == B.ERR_SHAPE
    assert _code(mm, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, alpha=float("inf"))) == B.ERR_UNSUPPORTED
    assert _code(mm, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, batch=-1)) == B.ERR_SHAPE
    mm(FAKE, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, **dict(kw, batch=0))  # empty batch: nothing enqueued


def test_weight_preparation_entry_points_reject_bad_arguments():
    pw = B.bwta_prepare_weights
    kw = dict(N=4, K=256, stream=0)
    assert _code(pw, None, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(pw, FAKE, FAKE, None, **kw) == B.ERR_NULL
    assert _code(pw, FAKE, FAKE + 4, FAKE, **kw) == B.ERR_ALIGN
    assert _code(pw, FAKE, FAKE, FAKE, **dict(kw, ldw=255)) == B.ERR_SHAPE
    assert _code(pw, FAKE, FAKE, FAKE, **dict(kw, K=32769)) == B.ERR_UNSUPPORTED
    pw(FAKE, FAKE, FAKE, **dict(kw, N=0))
    sc = B.bwta_act_scale
    kw = dict(M=4, K=256, stream=0)
    assert _code(sc, None, FAKE, **kw) == B.ERR_NULL
    assert _code(sc, FAKE, FAKE + 1, **kw) == B.ERR_ALIGN
    assert _code(sc, FAKE, FAKE, **dict(kw, lda=8)) == B.ERR_SHAPE
    assert _code(sc, FAKE, FAKE, **dict(kw, K=40000)) == B.ERR_UNSUPPORTED
    sc(FAKE, FAKE, **dict(kw, M=0))
    au = B.bwta_prepare_act_autoscale
    kw = dict(M=4, K=256, stream=0, prepared_bytes=B.prepared_bytes(4, 256))
    assert _code(au, None, FAKE, FAKE, **kw) == B.ERR_NULL
    assert _code(au, FAKE, None, FAKE, **kw) == B.ERR_NULL
    assert _code(au, FAKE, FAKE + 1, FAKE, **kw) == B.ERR_ALIGN
    assert _code(au, FAKE, FAKE, FAKE + 16, **kw) == B.ERR_ALIGN
    assert _code(au, FAKE, FAKE, FAKE, **dict(kw, lda=8)) == B.ERR_SHAPE
    assert _code(au, FAKE, FAKE, FAKE, **dict(kw, prepared_bytes=16)) == B.ERR_WORKSPACE
    assert _code(au, FAKE, FAKE, None, **kw) == B.ERR_WORKSPACE
    assert _code(au, FAKE, FAKE, FAKE, **dict(kw, K=40000, prepared_bytes=1 << 30)) == B.ERR_UNSUPPORTED
    au(FAKE, FAKE, FAKE, **dict(kw, M=0))


def test_prepared_attention_product_rejects_bad_arguments():
    f = B.bwta_matmul_bool_prepared
    kw = dict(batch=2, M=64, N=128, K=256, stream=0, prepared_bytes=B.prepared_bytes(256, 256), fmt=B.PREPARED_FP4)
    assert _code(f, None, FAKE, None, None, FAKE, **kw) == B.ERR_NULL
    assert _code(f, FAKE, FAKE, None, None, None, **kw) == B.ERR_NULL
    assert _code(f, FAKE, None, None, None, FAKE, **kw) == B.ERR_WORKSPACE
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, prepared_bytes=64)) == B.ERR_WORKSPACE
    assert _code(f, FAKE, FAKE + 16, None, None, FAKE, **kw) == B.ERR_ALIGN
    assert _code(f, FAKE + 4, FAKE, None, None, FAKE, **kw) == B.ERR_ALIGN
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, strideA=64 * 8 + 2)) == B.ERR_ALIGN
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, N=96)) == B.ERR_UNSUPPORTED      # not a multiple of 128
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, fmt=B.PREPARED_PLANES)) == B.ERR_UNSUPPORTED  # needs fragments
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, fmt=0)) == B.ERR_UNSUPPORTED
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, alpha=float("nan"))) == B.ERR_UNSUPPORTED
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, ldo=64)) == B.ERR_SHAPE
    assert _code(f, FAKE, FAKE, None, None, FAKE, **dict(kw, strideA=8)) == B.ERR_SHAPE
    f(FAKE, FAKE, None, None, FAKE, **dict(kw, batch=0))


def test_static_scratch_entry_point_refuses_oversized_shapes_on_the_host():
    assert B.static_scratch_bytes() == 32 << 20
    lin = B.bwta_linear_static
    kw = dict(stream=0, a_scale_mode=B.SCALE_VECTOR, w_scale_mode=B.SCALE_VECTOR)
    assert B.workspace_bytes(8192, 768, 11008) > B.static_scratch_bytes()
    assert _code(lin, FAKE, FAKE, FAKE, FAKE, FAKE, M=8192, N=768, K=11008, **kw) == B.ERR_TOO_LARGE
    assert _code(lin, None, None, None, None, None, M=8192, N=768, K=11008, **kw) == B.ERR_TOO_LARGE  # size first
    assert B.strerror(B.ERR_TOO_LARGE) != "unknown error code"
    lin(FAKE, FAKE, FAKE, FAKE, FAKE, M=0, N=768, K=11008, **kw)   # empty: a no-op, no device needed
