"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (path
AUTO), every output element compared with the oracle: no sampling.  Every output buffer starts
from a sentinel no correct result can equal, so a tile the kernels never wrote fails the test."""
import numpy as np
import pytest
import torch

import inputs
import oracle
import synth
from gpu_util import dev, gpu_pack_weights, host_u32, same_half, workspace
from paper_2604_03957_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ACC_SENTINEL = 0x7FFFFFF0      # |acc| <= K always
NAN = float("nan")             # no product of finite scales and an integer is NaN


def _sentinel_out(M, N):
    return torch.full((M, N), NAN, dtype=torch.float16, device=DEV)


def _sentinel_acc(M, N):
    return torch.full((M, N), ACC_SENTINEL, dtype=torch.int32, device=DEV)


def _sentinel_planes(M, rw):
    # all ones: pad bits must come back zero, and sign is a subset of mask in every written word
    return (torch.full((M, rw), -1, dtype=torch.int32, device=DEV), torch.full((M, rw), -1, dtype=torch.int32, device=DEV))


@pytest.mark.parametrize("which", ["up", "down"])
def test_config2_ffn_every_element(which):
    """Encoder FFN layers, whole path from fp16: planes (bwta_quantize_pack_act), int32 accumulators
    (bwta_gemm) and fp16 outputs (bwta_gemm, and bwta_linear as benchmarked), all 4096 tokens."""
    c = inputs.config2(which)
    M, N, K = c["M"], c["N"], c["K"]
    print("config2", which, M, N, K, flush=True)
    t, acc_want, out_want = oracle.linear(c["A"], c["s_a"], c["w"], c["s_w"])
    mask_want, sign_want, nnz_want = oracle.pack_act(t)
    rw = B.plane_row_words(K)
    A, s_a, s_w = dev(c["A"]), dev(c["s_a"]), dev(c["s_w"])
    wsign = gpu_pack_weights(c["w"])
    assert np.array_equal(host_u32(wsign), oracle.pack_weights(c["w"]))
    mask, sign = _sentinel_planes(M, rw)
    nnz = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    B.bwta_quantize_pack_act(A, s_a, mask, sign, nnz, M=M, K=K)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(mask), mask_want)
    assert np.array_equal(host_u32(sign), sign_want)
    assert np.array_equal(nnz.cpu().numpy(), nnz_want)
    ws = workspace(M, N, K)
    acc, out_g, out_l = _sentinel_acc(M, N), _sentinel_out(M, N), _sentinel_out(M, N)
    B.bwta_gemm(mask, sign, wsign, s_a, s_w, acc, None, ws, M=M, N=N, K=K)
    B.bwta_gemm(mask, sign, wsign, s_a, s_w, None, out_g, ws, M=M, N=N, K=K)
    B.bwta_linear(A, s_a, wsign, s_w, out_l, ws, M=M, N=N, K=K)        # as benchmarked
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_want)
    assert same_half(out_g.cpu().numpy(), out_want) and not np.isnan(out_want).any()
    assert same_half(out_l.cpu().numpy(), out_want)


@pytest.mark.parametrize("which", ["qkvo", "upgate", "down"])
def test_config3_prefill_every_element(which):
    """7B prefill shapes from ternary input: planes, int32 accumulators and fp16 outputs of bwta_gemm
    (the call the benchmark's headline times), all 2048 tokens."""
    c = synth.config3(which)
    M, N, K = c["M"], c["N"], c["K"]
    print("config3", which, M, N, K, flush=True)
    rw = B.plane_row_words(K)
    mask, sign = _sentinel_planes(M, rw)
    B.bwta_quantize_pack_act(dev(c["t"]), None, mask, sign, None, M=M, K=K, a_dtype=B.DTYPE_INT8)
    wsign = gpu_pack_weights(c["w"])
    out, acc = _sentinel_out(M, N), _sentinel_acc(M, N)
    ws = workspace(M, N, K)
    s_a, s_w = dev(c["s_a"]), dev(c["s_w"])
    B.bwta_gemm(mask, sign, wsign, s_a, s_w, None, out, ws, M=M, N=N, K=K)     # as benchmarked
    B.bwta_gemm(mask, sign, wsign, s_a, s_w, acc, None, ws, M=M, N=N, K=K)     # int32 accumulators
    torch.cuda.synchronize()
    mask_want, sign_want, _ = oracle.pack_act(c["t"])
    assert np.array_equal(host_u32(mask), mask_want) and np.array_equal(host_u32(sign), sign_want)
    want_acc = oracle.gemm_unpacked(c["t"], c["w"])
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    del acc
    want_out = oracle.epilogue(want_acc, c["s_a"], c["s_w"])
    assert same_half(out.cpu().numpy(), want_out) and not np.isnan(want_out).any()


@pytest.mark.parametrize("which", ["upgate", "down"])
@pytest.mark.parametrize("M", [1, 4, 16])
def test_config4_decode_every_element(which, M):
    c = synth.config4(which, M)
    N, K = c["N"], c["K"]
    print("config4", which, M, N, K, flush=True)
    rw = B.plane_row_words(K)
    mask, sign = _sentinel_planes(M, rw)
    B.bwta_quantize_pack_act(dev(c["t"]), None, mask, sign, None, M=M, K=K, a_dtype=B.DTYPE_INT8)
    wsign = gpu_pack_weights(c["w"])
    out, acc = _sentinel_out(M, N), _sentinel_acc(M, N)
    B.bwta_gemm(mask, sign, wsign, dev(c["s_a"]), dev(c["s_w"]), acc, out, workspace(M, N, K), M=M, N=N, K=K)
    torch.cuda.synchronize()
    want_acc = oracle.gemm_unpacked(c["t"], c["w"])
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    assert same_half(out.cpu().numpy(), oracle.epilogue(want_acc, c["s_a"], c["s_w"]))


def test_config4_decode_grouped_as_benchmarked():
    """The decode benchmark's launch: several distinct weight matrices of one shape in one grouped
    call; every output of every matrix against the oracle."""
    c = synth.config4("down", 16)
    M, N, K = c["M"], c["N"], c["K"]
    rw = B.plane_row_words(K)
    mask, sign = _sentinel_planes(M, rw)
    B.bwta_quantize_pack_act(dev(c["t"]), None, mask, sign, None, M=M, K=K, a_dtype=B.DTYPE_INT8)
    wsign = gpu_pack_weights(c["w"])
    nmat = 5
    mats = [torch.roll(wsign, shifts=i, dims=0).contiguous() for i in range(nmat)]
    outs = [_sentinel_out(M, N) for _ in range(nmat)]
    s_a, s_w = dev(c["s_a"]), dev(c["s_w"])
    ws = torch.empty(max(B.workspace_bytes(M, N, K), 256) * nmat, dtype=torch.uint8, device=DEV)
    probs = B.make_problems([(mask, sign, w, s_a, s_w, None, o) for w, o in zip(mats, outs)])
    B.bwta_gemm_grouped(probs, ws, M=M, N=N, K=K)
    torch.cuda.synchronize()
    for i in range(nmat):
        want = oracle.epilogue(oracle.gemm_unpacked(c["t"], np.roll(c["w"], i, axis=0)), c["s_a"], c["s_w"])
        assert same_half(outs[i].cpu().numpy(), want), i


def _check_block_linears(blk, cfg):
    """Every BWTA step of the decoder block against the oracle, on the block's own intermediates:
    the four per-token scale vectors (the s_A^0 statistic) and the seven linear layers (ternary
    function with those scales, then the BWTA linear equation), every element, bit for bit."""
    host = lambda t: t.detach().cpu().numpy()
    feeds = [("h", blk.s_h, [("wq", blk.q), ("wk", blk.k), ("wv", blk.v)]),
             ("att", blk.s_att, [("wo", blk.o)]),
             ("h2", blk.s_h2, [("wgate", blk.g), ("wup", blk.u)]),
             ("act", blk.s_act, [("wdown", blk.d)])]
    for name, s_gpu, outs in feeds:
        a = host(getattr(blk, name))
        assert np.isfinite(a).all(), name
        s_want = oracle.act_scale(a)
        assert np.array_equal(host(s_gpu).view(np.uint16), s_want.view(np.uint16)), name
        t = oracle.ternarize(a, s_want)
        for wname, out in outs:
            want = oracle.epilogue(oracle.gemm_unpacked(t, cfg[wname]), s_want, cfg["s_" + wname])
            got = host(out)
            assert not np.isnan(want).any() and same_half(got, want), (name, wname)
            print("block linear", wname, got.shape, "ok", flush=True)


def test_config5_block_every_linear_every_element():
    """The fused decoder block at its full size (2048 tokens, hidden 4096, FFN 11008): run the block
    as the benchmark does, then check all 7 linears and all 4 scale computations on the tensors the
    block really produced."""
    import bench
    cfg = synth.config5()
    blk = bench.Block(cfg, torch, B)
    for t in (blk.q, blk.k, blk.v, blk.o, blk.g, blk.u, blk.d):
        t.fill_(NAN)
    y = blk.forward()
    torch.cuda.synchronize()
    assert y.shape == (2048, 4096) and bool(torch.isfinite(y).all())
    _check_block_linears(blk, cfg)
    # the residual stream the harness assembles around the layers (plain tensor ops)
    x1 = blk.x + blk.o
    assert torch.equal(y, x1 + blk.d)
    # the timing-only pass (BWTA kernels alone on the stored intermediates) writes the same bits
    before = [t.clone() for t in (blk.q, blk.k, blk.v, blk.o, blk.g, blk.u, blk.d)]
    for t in (blk.q, blk.k, blk.v, blk.o, blk.g, blk.u, blk.d):
        t.fill_(NAN)
    blk.forward(bwta_only=True)
    torch.cuda.synchronize()
    for a, b in zip(before, (blk.q, blk.k, blk.v, blk.o, blk.g, blk.u, blk.d)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_config5_block_ragged_sequence():
    """The same block on a sequence that fills neither a 128-token tile nor a 32-token strip."""
    import bench
    cfg = synth.config5(seq=333)
    blk = bench.Block(cfg, torch, B)
    y = blk.forward()
    torch.cuda.synchronize()
    assert y.shape == (333, 4096) and bool(torch.isfinite(y).all())
    _check_block_linears(blk, cfg)


def _check_block_attention(blk):
    """The block's two attention MatMuls against the oracle on the block's own tensors, every head and
    every element: the per-row scales (the s_A^0 statistic), BWTA_QK = ternary(Q) (x) ternary(K)^T with
    the 1/sqrt(d) prefix (arithmetic Case 3), and BWTA_Att = bool(softmax) (x) ternary(V) (Case 2)."""
    host = lambda t: t.detach().cpu().numpy()
    S, heads, hd = blk.S, blk.heads, blk.H // blk.heads
    qh, kh, vt = host(blk.qh), host(blk.kh), host(blk.vt)
    s_q, s_k, s_v = oracle.act_scale(qh), oracle.act_scale(kh), oracle.act_scale(vt)
    for got, want, name in ((blk.s_q, s_q, "s_q"), (blk.s_k, s_k, "s_k"), (blk.s_v, s_v, "s_v")):
        assert np.array_equal(host(got).view(np.uint16), want.view(np.uint16)), name
    tq, tk, tv = oracle.ternarize(qh, s_q), oracle.ternarize(kh, s_k), oracle.ternarize(vt, s_v)
    alpha = 1.0 / hd ** 0.5
    scores = host(blk.scores)
    for h in range(heads):
        r = slice(h * S, (h + 1) * S)
        want = oracle.epilogue_alpha(oracle.gemm_unpacked(tq[r], tk[r]), s_q[r], s_k[r], alpha)
        assert not np.isnan(want).any() and same_half(scores[h], want), ("scores", h)
    print("block attention scores ok", scores.shape, flush=True)
    del scores
    probs = host(blk.probs).reshape(heads * S, S)
    assert np.isfinite(probs).all()
    s_p = oracle.act_scale(probs)
    assert np.array_equal(host(blk.s_p).view(np.uint16), s_p.view(np.uint16))
    ctx = host(blk.ctx)
    ones = 0
    for h in range(heads):
        r = slice(h * S, (h + 1) * S)
        b = oracle.boolize(probs[r], s_p[r])
        ones += int(b.sum())
        d = slice(h * hd, (h + 1) * hd)
        want = oracle.epilogue_alpha(oracle.gemm_unpacked(b, tv[d]), s_p[r], s_v[d], 1.0)
        assert not np.isnan(want).any() and same_half(ctx[h], want), ("context", h)
    assert 0 < ones < heads * S * S // 2                       # the boolean attention is neither empty nor dense
    print("block attention context ok", ctx.shape, "ones per row %.1f" % (ones / (heads * S)), flush=True)


@pytest.mark.parametrize("seq", [2048, 333])
def test_config5_block_with_bwta_attention(seq):
    """The block with the paper's attention MatMuls instead of fp16 attention: both attention products
    and all 7 linears (whose inputs now come out of that attention) against the oracle, full size and a
    ragged sequence."""
    import bench
    cfg = synth.config5(seq=seq)
    blk = bench.Block(cfg, torch, B)
    y = blk.forward(attention="bwta")
    torch.cuda.synchronize()
    assert y.shape == (seq, 4096) and bool(torch.isfinite(y).all())
    _check_block_attention(blk)
    _check_block_linears(blk, cfg)
