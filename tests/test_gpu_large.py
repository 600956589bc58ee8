"""GPU parity where an operand or the output has more than 2^31 elements, so that any 32-bit
index arithmetic left in a kernel shows up.  The tall operand repeats a block of PERIOD seeded
rows (PERIOD is prime, so a row fetched 2^31 or 2^32 elements early is a different row of the
block); the oracle computes the block and every row of the device result is compared with the
block's row it repeats, on the device."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, dev, gpu_pack_weights, workspace
from paper_2604_03957_amd import binding as B
import synth

pytestmark = pytest.mark.gpu

PERIOD = 4099


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.float16 else t


def _same_rows(got, want_block, idx, chunk=1 << 16):
    """got[m] == want_block[idx[m]] for every m, bit for bit, in chunks of rows."""
    got, want_block = _bits(got), _bits(want_block)
    for r0 in range(0, got.shape[0], chunk):
        r1 = min(r0 + chunk, got.shape[0])
        if not torch.equal(got[r0:r1], want_block[idx[r0:r1]]):
            return False
    return True


def test_ternarise_more_than_2g_input_elements():
    M, K, N = 1_052_000, 2048, 128
    assert M * K > 2**31
    print("tall input", M, K, flush=True)
    base = synth.gaussian_outlier_activations(21, 0, PERIOD, K)
    s_base = oracle.act_scale(base)
    w = synth.binary_pm1(21, 1, (N, K))
    s_w = synth.scales(21, 2, N)
    t = oracle.ternarize(base, s_base)
    mask_b, sign_b, nnz_b = oracle.pack_act(t)
    _, _, out_b = oracle.linear(base, s_base, w, s_w)

    idx = torch.arange(M, device=DEV) % PERIOD
    A = dev(base)[idx]
    s_a = dev(s_base)[idx]
    rw = B.plane_row_words(K)
    mask = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
    sign = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
    nnz = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    B.bwta_quantize_pack_act(A, s_a, mask, sign, nnz, M=M, K=K)
    torch.cuda.synchronize()
    assert _same_rows(mask, dev(mask_b), idx)
    assert _same_rows(sign, dev(sign_b), idx)
    assert torch.equal(nnz, dev(nnz_b)[idx])
    del mask, sign, nnz

    # the same input through the fragment form and the tiled kernel
    prepared = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device=DEV)
    wsign = gpu_pack_weights(w)
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    fmt = B.bwta_prepare_act(A, s_a, prepared, M=M, K=K)
    B.bwta_gemm_prepared(prepared, wsign, s_a, dev(s_w), None, out, fmt=fmt, M=M, N=N, K=K)
    torch.cuda.synchronize()
    assert _same_rows(out, dev(out_b), idx)

    # and with the token scales computed in the same pass
    s_got = torch.zeros(M, dtype=torch.float16, device=DEV)
    out.fill_(float("nan"))
    fmt = B.bwta_prepare_act_autoscale(A, s_got, prepared, M=M, K=K)
    B.bwta_gemm_prepared(prepared, wsign, s_got, dev(s_w), None, out, fmt=fmt, M=M, N=N, K=K)
    torch.cuda.synchronize()
    assert torch.equal(_bits(s_got), _bits(dev(oracle.act_scale(base)))[idx])
    assert np.array_equal(oracle.act_scale(base).view(np.uint16), s_base.view(np.uint16))  # same scales as above
    assert _same_rows(out, dev(out_b), idx)


@pytest.mark.parametrize("entry", ["gemm", "gemm_acc", "linear"])
def test_more_than_2g_output_elements(entry):
    M, K, N = 585_000, 128, 3712
    assert M * N > 2**31
    print("tall output", entry, M, N, K, flush=True)
    base = synth.gaussian_outlier_activations(22, 0, PERIOD, K)
    s_base = oracle.act_scale(base)
    w = synth.binary_pm1(22, 1, (N, K))
    s_w = synth.scales(22, 2, N)
    _, acc_b, out_b = oracle.linear(base, s_base, w, s_w)

    idx = torch.arange(M, device=DEV) % PERIOD
    A = dev(base)[idx]
    s_a = dev(s_base)[idx]
    wsign = gpu_pack_weights(w)
    ws = workspace(M, N, K)
    if entry == "linear":  # one launch: ternarisation and product in the same kernel
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        B.bwta_linear(A, s_a, wsign, dev(s_w), out, ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
        assert _same_rows(out, dev(out_b), idx)
        return
    rw = B.plane_row_words(K)
    mask = torch.empty((M, rw), dtype=torch.int32, device=DEV)
    sign = torch.empty_like(mask)
    B.bwta_quantize_pack_act(A, s_a, mask, sign, None, M=M, K=K)
    if entry == "gemm":
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        B.bwta_gemm(mask, sign, wsign, s_a, dev(s_w), None, out, ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
        assert _same_rows(out, dev(out_b), idx)
    else:
        acc = torch.full((M, N), 123456, dtype=torch.int32, device=DEV)
        B.bwta_gemm(mask, sign, wsign, None, None, acc, None, ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
        assert _same_rows(acc, dev(acc_b), idx)


def test_score_product_more_than_2g_output_elements():
    """BWTA_QK over 136 heads of 4096 x 4096 scores; head b repeats seeded head b % 3."""
    batch, M, N, K, distinct = 136, 4096, 4096, 128, 3
    assert batch * M * N > 2**31
    print("scores", batch, M, N, K, flush=True)
    s_q, s_k, alpha = synth.scales(23, 1, 1), synth.scales(23, 2, 1), 1.0 / np.sqrt(K)
    planes, want_acc, want_out = [], [], []
    for h in range(distinct):
        q = synth.ternary(23, 10 + h, (M, K), 0.5)
        k = synth.ternary(23, 20 + h, (N, K), 0.5)
        mq, sq, _ = oracle.pack_act(q)
        mk, sk, _ = oracle.pack_act(k)
        planes.append((mq, sq, mk, sk))
        acc = oracle.gemm_unpacked(q, k)
        want_acc.append(acc)
        want_out.append(oracle.epilogue_alpha(acc, s_q, s_k, alpha))
    hidx = torch.arange(batch, device=DEV) % distinct
    mqs, sqs, mks, sks = (dev(np.stack([p[i] for p in planes]))[hidx].contiguous() for i in range(4))
    acc = torch.full((batch, M, N), 12345, dtype=torch.int32, device=DEV)
    out = torch.full((batch, M, N), float("nan"), dtype=torch.float16, device=DEV)
    B.bwta_matmul_tt(mqs, sqs, mks, sks, dev(s_q), dev(s_k), acc, out, batch=batch, M=M, N=N, K=K, alpha=alpha)
    torch.cuda.synchronize()
    want_acc, want_out = dev(np.stack(want_acc)), _bits(dev(np.stack(want_out)))
    for b in range(batch):
        assert torch.equal(acc[b], want_acc[b % distinct]), "accumulators of head %d" % b
        assert torch.equal(_bits(out[b]), want_out[b % distinct]), "scores of head %d" % b
