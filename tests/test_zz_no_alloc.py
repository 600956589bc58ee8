"""The entry point that allocates nothing (bwta_linear_static: scratch inside the library's own
device image) against bwta_linear with a caller workspace, through the C ABI: identical bits, on
calls in a row that share the scratch, the later ones on smaller inputs.  Both are also checked
against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import dev, gpu_pack_weights, same_half, workspace
from paper_2604_03957_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, M, N, K):
    A = synth.laplace_activations(seed, 1, M, K)
    s_a = oracle.act_scale(A)
    w = synth.binary_pm1(seed, 2, (N, K))
    s_w = synth.scales(seed, 3, N)
    return A, s_a, w, s_w


def test_static_scratch_linear_matches_workspace_linear_on_calls_in_a_row():
    assert B.static_scratch_bytes() == 32 << 20
    B.static_scratch_init()
    # two-kernel shapes (K > 1024: ternarise into the scratch, then the product reads it), the second
    # and third smaller than the first; then a decode-sized one (bit planes in the scratch) and a
    # one-launch one (short K: the scratch is not touched)
    shapes = [(700, 900, 3000), (150, 300, 1500), (2048, 512, 11008), (16, 1000, 4096), (300, 256, 768)]
    for i, (M, N, K) in enumerate(shapes):
        print("static scratch", M, N, K, flush=True)
        assert B.workspace_bytes(M, N, K) <= B.static_scratch_bytes()
        A, s_a, w, s_w = _case(80 + i, M, N, K)
        dA, dsa, dsw, wsign = dev(A), dev(s_a), dev(s_w), gpu_pack_weights(w)
        got = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        ref = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        B.bwta_linear_static(dA, dsa, wsign, dsw, got, M=M, N=N, K=K)
        B.bwta_linear(dA, dsa, wsign, dsw, ref, workspace(M, N, K), M=M, N=N, K=K)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), (M, N, K)
        _, _, want = oracle.linear(A, s_a, w, s_w)
        assert same_half(got.cpu().numpy(), want), (M, N, K)


def test_static_scratch_linear_rejects_what_does_not_fit():
    M, N, K = 8192, 768, 11008
    assert B.workspace_bytes(M, N, K) > B.static_scratch_bytes()
    A = torch.zeros((8, 8), dtype=torch.float16, device=DEV)  # never read: the call is refused on the host
    with pytest.raises(B.BwtaError) as e:
        B.bwta_linear_static(A, None, A, None, A, M=M, N=N, K=K)
    assert e.value.code == B.ERR_TOO_LARGE
    B.bwta_linear_static(A, None, A, None, A, M=0, N=N, K=K)      # empty: nothing enqueued
