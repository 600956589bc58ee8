"""GPU parity of weight preparation (mean-centring, sign, channel scale) and of the activation
scale's starting value against the oracle, through the C ABI.  Planes are bit-identical (every
decision is an exact integer comparison on both sides); the fp16 scales are compared to 1e-3
relative, the bar for floating point, and are in fact bit-identical on these inputs."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, gpu_gemm, host_u32, max_rel_err, same_half
from paper_2604_03957_amd import binding as B
import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


def gpu_prepare(W, K=None):
    N = W.shape[0]
    K = W.shape[1] if K is None else K
    ws = torch.full((N, B.plane_row_words(K)), -1, dtype=torch.int32, device=DEV)
    sw = torch.full((N,), float("nan"), dtype=torch.float16, device=DEV)
    B.bwta_prepare_weights(dev(W), ws, sw, N=N, K=K, ldw=W.shape[1])
    torch.cuda.synchronize()
    return host_u32(ws), sw.cpu().numpy()


@pytest.mark.parametrize("N,K,ldw", [(5, 40, 40), (768, 768, 768), (17, 1001, 1003), (3, 11008, 11008), (2, 32768, 32768)])
def test_prepare_weights_matches_oracle(N, K, ldw):
    _say("prepare weights", N, K, ldw)
    W = (synth.gaussian(50 + N, 1, N * ldw) * 0.03 + 0.002).astype(np.float16).reshape(N, ldw)
    W[0, :min(K, 6)] = np.array([6e-8, -6e-8, 65504.0, -65504.0, 0.0, -0.0], np.float16)[:min(K, 6)]
    Wk = np.ascontiguousarray(W[:, :K])
    w, s = oracle.prepare_weights(Wk)
    planes, sw = gpu_prepare(W, K)
    assert np.array_equal(planes, oracle.pack_weights(w))
    assert max_rel_err(sw.reshape(1, -1), s.reshape(1, -1)) <= 1e-3
    assert same_half(sw, s)


def test_prepare_weights_special_rows():
    K = 300
    W = (synth.laplace(60, 1, 6 * K) * 0.02).astype(np.float16).reshape(6, K)
    W[0] = np.float16(0.125)                                   # all equal to the mean: every sign +1, scale 0
    W[1, :4] = [np.inf, -np.inf, np.nan, 1.0]                  # non-finite entries stay out of mean and scale
    W[2] = 0.0
    W[3, ::2] = np.float16(1.0); W[3, 1::2] = np.float16(-1.0) # mean exactly 0: ties nowhere, scale exactly 1
    W[4] = np.float16(2.0 ** -24)                              # smallest subnormal everywhere
    w, s = oracle.prepare_weights(W)
    planes, sw = gpu_prepare(W)
    assert np.array_equal(planes, oracle.pack_weights(w))
    assert same_half(sw, s)
    assert sw[0] == 0 and sw[3] == 1 and not planes[0].any()


@pytest.mark.parametrize("M,K,lda", [(5, 40, 40), (64, 768, 768), (33, 300, 304), (7, 11008, 11008), (3, 32768, 32768)])
def test_act_scale_matches_oracle(M, K, lda):
    _say("act scale", M, K, lda)
    A = np.ascontiguousarray(synth.gaussian_outlier_activations(70 + M, 1, M, lda))
    A[0, :min(K, 4)] = np.array([np.nan, np.inf, 65504.0, 6e-8], np.float16)[:min(K, 4)]
    want = oracle.act_scale(np.ascontiguousarray(A[:, :K]))
    s = torch.full((M,), float("nan"), dtype=torch.float16, device=DEV)
    B.bwta_act_scale(dev(A), s, M=M, K=K, lda=lda)
    torch.cuda.synchronize()
    got = s.cpu().numpy()
    assert max_rel_err(got.reshape(1, -1), want.reshape(1, -1)) <= 1e-3
    assert same_half(got, want)


def test_prepared_weights_feed_the_linear_layer():
    """fp16 checkpoint -> prepare -> BWTA linear equals the oracle's chain on the same inputs."""
    M, N, K = 70, 130, 1000
    W = (synth.gaussian(80, 1, N * K) * 0.02 + 0.001).astype(np.float16).reshape(N, K)
    t = synth.ternary(80, 2, (M, K), 0.5)
    s_a = synth.scales(80, 3, M)
    w, s_w = oracle.prepare_weights(W)
    want_acc = oracle.gemm_unpacked(t, w)
    want = oracle.epilogue(want_acc, s_a, s_w)
    ws = torch.empty((N, B.plane_row_words(K)), dtype=torch.int32, device=DEV)
    sw = torch.empty((N,), dtype=torch.float16, device=DEV)
    B.bwta_prepare_weights(dev(W), ws, sw, N=N, K=K)
    mask, sign, _ = oracle.pack_act(t)
    acc, out = gpu_gemm(mask, sign, ws, s_a, sw.cpu().numpy(), M, N, K)
    assert np.array_equal(acc, want_acc) and same_half(out, want)


@pytest.mark.parametrize("path", [B.PATH_AUTO, B.PATH_POPC, B.PATH_FP4])
@pytest.mark.parametrize("M,N,K,lda", [(5, 40, 40, 40), (64, 70, 768, 768), (33, 50, 300, 304), (130, 96, 1001, 1003),
                                       (257, 130, 4096, 4096), (300, 64, 11008, 11008), (200, 33, 520, 528)])
def test_scale_and_ternarise_in_one_pass(M, N, K, lda, path):
    """bwta_prepare_act_autoscale: the token scales it writes are the oracle's act_scale (to the
    floating-point bar, and bit for bit on these inputs), and the operand it prepares, fed to
    bwta_gemm_prepared with those scales, gives the oracle's linear layer exactly.  Both operand
    forms (bit planes below 129 tokens and on the popcount path, matrix-core fragments above),
    ragged and strided rows, NaN / Inf entries, an all-zero token (scale 0: the token is zero)."""
    _say("scale + ternarise", M, N, K, lda, "path", path)
    A = np.ascontiguousarray(synth.gaussian_outlier_activations(90 + M, 1, M, lda))
    A[0, :min(K, 4)] = np.array([np.nan, np.inf, 65504.0, 6e-8], np.float16)[:min(K, 4)]
    A[2, :] = 0
    Ak = np.ascontiguousarray(A[:, :K])
    s_want = oracle.act_scale(Ak)
    assert s_want[2] == 0
    w = synth.binary_pm1(91, M + N, (N, K))
    s_w = synth.scales(91, 3, N)
    _, _, want = oracle.linear(Ak, s_want, w, s_w)
    B.set_path(path)
    try:
        s = torch.full((M,), float("nan"), dtype=torch.float16, device=DEV)
        prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device=DEV)
        out = torch.full((M, N), 7.0, dtype=torch.float16, device=DEV)
        ws = torch.empty((N, B.plane_row_words(K)), dtype=torch.int32, device=DEV)
        B.bwta_pack_weights(dev(w), ws, N=N, K=K)
        fmt = B.bwta_prepare_act_autoscale(dev(A), s, prep, M=M, K=K, lda=lda)
        B.bwta_gemm_prepared(prep, ws, s, dev(s_w), None, out, fmt=fmt, M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    got_s = s.cpu().numpy()
    assert max_rel_err(got_s.reshape(1, -1), s_want.reshape(1, -1)) <= 1e-3
    assert same_half(got_s, s_want)
    assert same_half(out.cpu().numpy(), want)
