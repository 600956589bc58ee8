"""GPU parity of the attention MatMuls (BWTA_QK: ternary x ternary, BWTA_Att: bool x ternary) and of
the boolean packer against the oracle, through the C ABI.  Planes and int32 accumulators must be
bit-identical; fp16 outputs within 1e-3 relative (and, as built, bit-identical)."""
import math

import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, host_u32, max_rel_err, same_half
from paper_2604_03957_amd import binding as B
import synth

pytestmark = pytest.mark.gpu
RTOL = 1e-3
DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


def gpu_pack_bool(A, s_a, lda=None, K=None):
    M = A.shape[0]
    K = A.shape[1] if K is None else K
    mask = torch.full((M, B.plane_row_words(K)), -1, dtype=torch.int32, device=DEV)
    B.bwta_quantize_pack_bool(dev(A), dev(s_a), mask, M=M, K=K, lda=A.shape[1] if lda is None else lda)
    torch.cuda.synchronize()
    return host_u32(mask)


@pytest.mark.parametrize("M,K,lda", [(5, 40, None), (64, 768, None), (33, 300, 304), (257, 1001, 1003), (2, 11008, None)])
def test_bool_pack_matches_oracle(M, K, lda):
    _say("bool pack", M, K, lda)
    x = np.abs(synth.gaussian(40 + M, 1, M * (lda or K))).astype(np.float16).reshape(M, -1)   # non-negative, like probabilities
    x[0, :4] = [0.0, np.float16(0.5), np.float16(0.4998), np.nan]
    s = synth.scales(40 + M, 2, M)
    s[-1] = np.float16(1.0)
    x[-1, :3] = [0.5, np.float16(0.49976), np.inf]                # exact tie at 0.5 s -> 1, just below -> 0
    want, _, _ = oracle.pack_act(oracle.boolize(np.ascontiguousarray(x[:, :K]), s))
    assert np.array_equal(gpu_pack_bool(x, s, lda=lda, K=K), want)


@pytest.mark.parametrize("M,K,lda", [(2100, 4096, None), (2300, 3720, 3728)])
def test_bool_pack_large_aligned_rows(M, K, lda):
    """Sizes at which the boolean packer takes its four-groups-per-thread kernel."""
    _say("bool pack large", M, K, lda)
    x = np.abs(synth.gaussian(60 + M, 1, M * (lda or K))).astype(np.float16).reshape(M, -1)
    s = synth.scales(60 + M, 2, M)
    s[3], s[M - 2] = np.nan, -1.0
    want, _, _ = oracle.pack_act(oracle.boolize(np.ascontiguousarray(x[:, :K]), s))
    assert np.array_equal(gpu_pack_bool(x, s, lda=lda, K=K), want)
    one = np.array([0.3], np.float16)
    want, _, _ = oracle.pack_act(oracle.boolize(np.ascontiguousarray(x[:, :K]), one))
    assert np.array_equal(gpu_pack_bool(x, one, lda=lda, K=K), want)


def test_bool_pack_every_half_pattern_and_bad_scales():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(64, 1024)
    A = bits.view(np.float16)
    for s in (1.0, 0.37, 2.0 ** -24, 65504.0, -1.0, 0.0, float("nan"), float("inf")):
        sc = np.array([s], np.float16)
        want, _, _ = oracle.pack_act(oracle.boolize(A, sc))
        assert np.array_equal(gpu_pack_bool(A, sc), want), s


@pytest.fixture(params=["matrix_cores", "popcount"])
def family(request):
    """Both kernels behind bwta_matmul_tt: the FP4 matrix-core one (default) and the wave64 popcount one."""
    if request.param == "popcount":
        B.set_path(B.PATH_POPC)
    yield request.param
    B.set_path(B.PATH_AUTO)


def _operands(seed, batch, M, N, K, a_bool, p0a=0.45, p0b=0.5):
    a = synth.ternary(seed, 1, (batch, M, K), p0a)
    if a_bool:
        a = (a != 0).astype(np.int8)
    b = synth.ternary(seed, 2, (batch, N, K), p0b)
    return a, b


def _run(a, b, s_a, s_b, alpha, a_bool, *, pad_a=0, pad_b=0, ldo=None, pad_out=0, dirty=False, b_bool=False):
    batch, M, K = a.shape
    N = b.shape[1]
    rw = B.plane_row_words(K)
    planes = [oracle.pack_act(a[i])[:2] + oracle.pack_act(b[i])[:2] for i in range(batch)]

    def stack(idx, rows, pad):
        buf = np.zeros((batch, rows * rw + pad), np.uint32)
        for i in range(batch):
            buf[i, :rows * rw] = planes[i][idx].reshape(-1)
        return buf
    ma, sa, mb, sb = stack(0, M, pad_a), stack(1, M, pad_a), stack(2, N, pad_b), stack(3, N, pad_b)
    if dirty:                                                      # sign bits under a zero mask must be ignored
        sa = sa | (~ma & np.uint32(0x5A5A5A5A))
        sb = sb | (~mb & np.uint32(0xA5A5A5A5))
    ldo = N if ldo is None else ldo
    stride_out = M * ldo + pad_out
    acc = torch.full((batch, M, N), 12345, dtype=torch.int32, device=DEV)
    out = torch.full((batch * stride_out,), float("nan"), dtype=torch.float16, device=DEV)
    B.bwta_matmul_tt(dev(ma), None if a_bool else dev(sa), dev(mb), None if b_bool else dev(sb), dev(s_a), dev(s_b), acc, out,
                     batch=batch, M=M, N=N, K=K, alpha=alpha, strideA=M * rw + pad_a, strideB=N * rw + pad_b,
                     ldo=ldo, stride_out=stride_out)
    torch.cuda.synchronize()
    acc, out = acc.cpu().numpy(), out.cpu().numpy()
    exact = True
    for i in range(batch):
        want_acc = oracle.gemm_unpacked(a[i], b[i])
        assert np.array_equal(acc[i], want_acc), "int32 accumulators differ in batch %d" % i
        sai = s_a if s_a is None or s_a.size == 1 else s_a.reshape(batch, M)[i]
        sbi = s_b if s_b is None or s_b.size == 1 else s_b.reshape(batch, N)[i]
        want = oracle.epilogue_alpha(want_acc, sai, sbi, alpha)
        got = np.stack([out[i * stride_out + m * ldo: i * stride_out + m * ldo + N] for m in range(M)])
        assert max_rel_err(got, want) <= RTOL
        exact = exact and same_half(got, want)
        if ldo > N:                                                # columns past N were not touched
            gap = np.stack([out[i * stride_out + m * ldo + N: i * stride_out + (m + 1) * ldo] for m in range(M - 1)])
            assert np.isnan(gap).all()
    return exact


QK_SHAPES = [(1, 64, 64, 128), (3, 70, 130, 128), (2, 1, 5, 33), (2, 257, 65, 64), (1, 130, 200, 1000), (1, 129, 260, 1300)]


@pytest.mark.parametrize("batch,M,N,K", QK_SHAPES)
def test_qk_product_matches_oracle(batch, M, N, K, family):
    """BWTA_QK: ternary(Q) x ternary(K)^T with layerwise scales and 1/sqrt(D)."""
    _say("qk", batch, M, N, K)
    q, k = _operands(600 + M, batch, M, N, K, a_bool=False)
    s_q, s_k = synth.scales(600, 1, 1), synth.scales(600, 2, 1)
    assert _run(q, k, s_q, s_k, 1.0 / math.sqrt(K), False, dirty=True)


@pytest.mark.parametrize("batch,M,N,K", [(1, 64, 64, 64), (3, 70, 64, 200), (2, 1, 5, 33), (2, 200, 128, 1000)])
def test_att_v_product_matches_oracle(batch, M, N, K, family):
    """BWTA_Att: bool(Att) x ternary(V); V arrives transposed (packed along the sequence)."""
    _say("att", batch, M, N, K)
    att, vt = _operands(700 + M, batch, M, N, K, a_bool=True, p0a=0.8)
    assert _run(att, vt, synth.scales(700, 1, 1), synth.scales(700, 2, 1), 1.0, True, dirty=True)


def test_two_boolean_operands(family):
    """No sign plane on either side: the product counts the positions where both bits are set."""
    a, b = _operands(750, 2, 70, 130, 300, a_bool=True)
    b = (b != 0).astype(np.int8)
    assert _run(a, b, synth.scales(750, 1, 1), None, 0.5, True, b_bool=True)


def test_products_seeded_random_shapes(family):
    """Twelve products with shapes, sparsities and operand kinds drawn from a seeded generator:
    ragged tiles in both directions, K tails inside and across the 256-k slabs."""
    rng = np.random.default_rng(20260404)
    for case in range(12):
        batch, M, N = int(rng.integers(1, 4)), int(rng.integers(1, 300)), int(rng.integers(1, 300))
        K = int(rng.integers(1, 1500))
        a_bool, b_bool = bool(rng.integers(0, 2)), bool(rng.integers(0, 4) == 0)
        _say("tt random", case, batch, M, N, K, a_bool, b_bool)
        a, b = _operands(5000 + case, batch, M, N, K, a_bool, p0a=float(rng.uniform(0.2, 0.9)))
        if b_bool:
            b = (b != 0).astype(np.int8)
        s_a = synth.scales(5000 + case, 3, batch * M) if case % 2 else synth.scales(5000 + case, 3, 1)
        s_b = synth.scales(5000 + case, 4, batch * N) if case % 3 == 0 else None
        assert _run(a, b, s_a, s_b, float(rng.uniform(0.05, 2.0)), a_bool, b_bool=b_bool, dirty=not (a_bool or b_bool))


def test_vector_scales_strides_and_no_scale(family):
    q, k = _operands(800, 2, 37, 50, 160, a_bool=False)
    s_q, s_k = synth.scales(800, 1, 2 * 37), synth.scales(800, 2, 2 * 50)
    assert _run(q, k, s_q, s_k, 0.125, False, pad_a=8, pad_b=12, ldo=56, pad_out=24)
    assert _run(q, k, None, None, 1.0, False)
    assert _run(q, k, None, s_k, 3.0, False)


def test_attention_head_shapes_full_size(family):
    """The paper's attention shapes for a 7B-class block: 2048 tokens, head dimension 128."""
    S, D, heads = 2048, 128, 2
    _say("full-size heads", S, D, heads)
    q, k = _operands(900, heads, S, S, D, a_bool=False)
    assert _run(q, k, synth.scales(900, 1, 1), synth.scales(900, 2, 1), 1.0 / math.sqrt(D), False)
    att, vt = _operands(901, heads, S, D, S, a_bool=True, p0a=0.9)
    assert _run(att, vt, synth.scales(901, 1, 1), synth.scales(901, 2, 1), 1.0, True)


def test_empty_inputs_are_noops():
    z = torch.zeros(16, dtype=torch.int32, device=DEV)
    B.bwta_matmul_tt(z, z, z, z, None, None, z, None, batch=0, M=4, N=4, K=32)
    B.bwta_matmul_tt(z, z, z, z, None, None, z, None, batch=1, M=0, N=4, K=32)
    B.bwta_quantize_pack_bool(z, None, z, M=0, K=32)
    torch.cuda.synchronize()


@pytest.mark.parametrize("batch,M,N,K,vec", [(2, 200, 128, 300, False), (3, 257, 256, 1000, True), (1, 64, 256, 128, False),
                                             (2, 130, 128, 2048, True), (8, 300, 128, 200, True), (16, 33, 256, 64, False)])
def test_att_v_with_v_prepared_once(batch, M, N, K, vec):
    """BWTA_Att through bwta_matmul_bool_prepared: the boolean plane against V^T prepared like an
    activation (bwta_prepare_act).  Ragged attention rows, K tails, vector and scalar scales, a scale
    prefix, padded strides; nothing is written between rows or batch entries.  Batch counts that are
    and are not multiples of 8 (the two workgroup-to-head mappings)."""
    _say("att prepared", batch, M, N, K, vec)
    att, vt = _operands(900 + M, batch, M, N, K, a_bool=True, p0a=0.8)
    rw = B.plane_row_words(K)
    pad_a, ldo, pad_out = 8, N + 8, 24
    ma = np.zeros((batch, M * rw + pad_a), np.uint32)
    for i in range(batch):
        ma[i, :M * rw] = oracle.pack_act(att[i])[0].reshape(-1)
    s_a = synth.scales(900, 1, batch * M) if vec else synth.scales(900, 1, 1)
    s_b = synth.scales(900, 2, batch * N) if vec else None
    alpha = 0.37
    v16 = np.ascontiguousarray(vt.reshape(batch * N, K).astype(np.float16))     # +-1 and 0: ternarised as they are
    prep = torch.empty(B.prepared_bytes(batch * N, K), dtype=torch.uint8, device=DEV)
    stride_out = M * ldo + pad_out
    out = torch.full((batch * stride_out,), float("nan"), dtype=torch.float16, device=DEV)
    fmt = B.bwta_prepare_act(dev(v16), None, prep, M=batch * N, K=K)
    B.bwta_matmul_bool_prepared(dev(ma), prep, dev(s_a), dev(s_b), out, fmt=fmt, batch=batch, M=M, N=N, K=K, alpha=alpha,
                                strideA=M * rw + pad_a, ldo=ldo, stride_out=stride_out)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    for i in range(batch):
        want_acc = oracle.gemm_unpacked(att[i], vt[i])
        sai = s_a if s_a.size == 1 else s_a.reshape(batch, M)[i]
        sbi = None if s_b is None else s_b.reshape(batch, N)[i]
        want = oracle.epilogue_alpha(want_acc, sai, sbi, alpha)
        got = np.stack([out[i * stride_out + m * ldo: i * stride_out + m * ldo + N] for m in range(M)])
        assert max_rel_err(got, want) <= RTOL
        assert same_half(got, want)
        gap = np.stack([out[i * stride_out + m * ldo + N: i * stride_out + (m + 1) * ldo] for m in range(M - 1)])
        assert np.isnan(gap).all()
        assert np.isnan(out[i * stride_out + M * ldo - (ldo - N): (i + 1) * stride_out]).all()
