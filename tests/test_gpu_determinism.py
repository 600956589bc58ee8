"""Run-to-run determinism on the GPU: every entry point called twice on the same inputs (fresh
output buffers each time, other work in between) must write identical bits.  The contraction is
integer arithmetic in any order, so nothing may depend on launch timing; a difference here means
a race or an uninitialised read."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, gpu_pack_weights
from paper_2604_03957_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(t):
    t = t.contiguous()
    return t.view(torch.int16) if t.dtype == torch.float16 else t


def _twice(run):
    """run() -> list of output tensors; called twice with a large unrelated launch in between."""
    a = run()
    torch.cuda.synchronize()
    junk = torch.randn(1 << 22, device=DEV).sin_()  # different cache and scheduler state
    b = run()
    torch.cuda.synchronize()
    del junk
    assert len(a) == len(b)
    for i, (x, y) in enumerate(zip(a, b)):
        assert torch.equal(_bits(x), _bits(y)), i


@pytest.mark.parametrize("M,K", [(300, 1000), (2048, 4096), (5, 11008)])
def test_packers_twice(M, K):
    print("determinism packers", M, K, flush=True)
    A = dev(synth.laplace_activations(70, M, M, K))
    s = dev(synth.scales(70, 2, M))
    W = dev(synth.binary_pm1(70, 3, (M, K)))
    rw = B.plane_row_words(K)

    def run():
        mask = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
        sign = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
        nnz = torch.full((M,), -1, dtype=torch.int32, device=DEV)
        bmask = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
        wsign = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
        sc = torch.full((M,), 7.0, dtype=torch.float16, device=DEV)
        wsign2 = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
        sw = torch.full((M,), 7.0, dtype=torch.float16, device=DEV)
        B.bwta_quantize_pack_act(A, s, mask, sign, nnz, M=M, K=K)
        B.bwta_quantize_pack_bool(A, s, bmask, M=M, K=K)
        B.bwta_pack_weights(W, wsign, N=M, K=K)
        B.bwta_act_scale(A, sc, M=M, K=K)
        B.bwta_prepare_weights(A, wsign2, sw, N=M, K=K)
        return [mask, sign, nnz, bmask, wsign, sc, wsign2, sw]

    _twice(run)


@pytest.mark.parametrize("path", [B.PATH_AUTO, B.PATH_POPC, B.PATH_MFMA, B.PATH_FP4])
@pytest.mark.parametrize("M,N,K", [(1, 1000, 4096), (16, 300, 11008), (100, 520, 768), (700, 900, 3000)])
def test_products_twice(M, N, K, path):
    print("determinism products", M, N, K, path, flush=True)
    A = dev(synth.laplace_activations(71, M, M, K))
    s_a = dev(synth.scales(71, 2, M))
    s_w = dev(synth.scales(71, 3, N))
    wsign = gpu_pack_weights(synth.binary_pm1(71, 4, (N, K)))
    rw = B.plane_row_words(K)
    mask = torch.empty((M, rw), dtype=torch.int32, device=DEV)
    sign = torch.empty_like(mask)
    B.bwta_quantize_pack_act(A, s_a, mask, sign, None, M=M, K=K)

    def run():
        ws = torch.zeros(B.workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
        prep = torch.zeros(B.prepared_bytes(M, K), dtype=torch.uint8, device=DEV)
        acc = torch.full((M, N), -9, dtype=torch.int32, device=DEV)
        o1, o2, o3, o4 = (torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV) for _ in range(4))
        s2 = torch.full((M,), 7.0, dtype=torch.float16, device=DEV)
        B.bwta_gemm(mask, sign, wsign, s_a, s_w, acc, o1, ws, M=M, N=N, K=K)
        B.bwta_linear(A, s_a, wsign, s_w, o2, ws, M=M, N=N, K=K)
        fmt = B.bwta_prepare_act(A, s_a, prep, M=M, K=K)
        B.bwta_gemm_prepared(prep, wsign, s_a, s_w, None, o3, fmt=fmt, M=M, N=N, K=K)
        fmt = B.bwta_prepare_act_autoscale(A, s2, prep, M=M, K=K)
        B.bwta_gemm_prepared(prep, wsign, s2, s_w, None, o4, fmt=fmt, M=M, N=N, K=K)
        outs = [torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV) for _ in range(3)]
        probs = B.make_problems([(mask, sign, wsign, s_a, s_w, None, o) for o in outs])
        wsg = torch.zeros(3 * max(B.workspace_bytes(M, N, K), 256), dtype=torch.uint8, device=DEV)
        B.bwta_gemm_grouped(probs, wsg, M=M, N=N, K=K)
        return [acc, o1, o2, o3, o4, s2] + outs

    B.set_path(path)
    try:
        _twice(run)
    finally:
        B.set_path(B.PATH_AUTO)


@pytest.mark.parametrize("path", [B.PATH_AUTO, B.PATH_POPC])
def test_attention_products_twice(path):
    H, S, D = 3, 300, 128
    print("determinism attention", H, S, D, path, flush=True)
    q = dev(synth.laplace_activations(72, 1, H * S, D))
    k = dev(synth.laplace_activations(72, 2, H * S, D))
    vt = dev(synth.laplace_activations(72, 3, H * D, S))
    att = dev((np.abs(synth.gaussian(72, 4, H * S * S)) * 0.3).astype(np.float16).reshape(H * S, S))
    one = torch.ones(1, dtype=torch.float16, device=DEV)
    rw_d, rw_s = B.plane_row_words(D), B.plane_row_words(S)
    planes = lambda rows, rw: (torch.empty((rows, rw), dtype=torch.int32, device=DEV),
                               torch.empty((rows, rw), dtype=torch.int32, device=DEV))
    qm, qs = planes(H * S, rw_d)
    km, ks = planes(H * S, rw_d)
    vm, vs = planes(H * D, rw_s)
    am, _ = planes(H * S, rw_s)
    B.bwta_quantize_pack_act(q, one, qm, qs, None, M=H * S, K=D)
    B.bwta_quantize_pack_act(k, one, km, ks, None, M=H * S, K=D)
    B.bwta_quantize_pack_act(vt, one, vm, vs, None, M=H * D, K=S)
    B.bwta_quantize_pack_bool(att, one, am, M=H * S, K=S)

    def run():
        scores = torch.full((H, S, S), float("nan"), dtype=torch.float16, device=DEV)
        ctx = torch.full((H, S, D), float("nan"), dtype=torch.float16, device=DEV)
        ctx2 = torch.full((H, S, D), float("nan"), dtype=torch.float16, device=DEV)
        acc = torch.full((H, S, D), -9, dtype=torch.int32, device=DEV)
        prep = torch.zeros(B.prepared_bytes(H * D, S), dtype=torch.uint8, device=DEV)
        B.bwta_matmul_tt(qm, qs, km, ks, one, one, None, scores, batch=H, M=S, N=S, K=D, alpha=D ** -0.5)
        B.bwta_matmul_tt(am, None, vm, vs, one, one, acc, ctx, batch=H, M=S, N=D, K=S)
        outs = [scores, ctx, acc]
        if path == B.PATH_AUTO:
            fmt = B.bwta_prepare_act(vt, one, prep, M=H * D, K=S)
            B.bwta_matmul_bool_prepared(am, prep, one, one, ctx2, fmt=fmt, batch=H, M=S, N=D, K=S)
            outs.append(ctx2)
        return outs

    B.set_path(path)
    try:
        _twice(run)
    finally:
        B.set_path(B.PATH_AUTO)


@pytest.mark.parametrize("variant", [243, 223, 323])
@pytest.mark.parametrize("M,N,K", [(700, 900, 3000), (2048, 4096, 4096), (130, 520, 512)])
def test_lds_staged_kernel_twice(M, N, K, variant):
    """The LDS-staged tiled kernel, whose wavefronts enter the epilogue without a workgroup barrier:
    int32 accumulators and fp16 outputs of two runs must be the same bits."""
    print("determinism lds-staged", M, N, K, variant, flush=True)
    t = dev(synth.ternary(73, 1, (M, K), 0.5))
    s_a = dev(synth.scales(73, 2, M))
    s_w = dev(synth.scales(73, 3, N))
    wsign = gpu_pack_weights(synth.binary_pm1(73, 4, (N, K)))
    rw = B.plane_row_words(K)
    mask = torch.empty((M, rw), dtype=torch.int32, device=DEV)
    sign = torch.empty_like(mask)
    B.bwta_quantize_pack_act(t, None, mask, sign, None, M=M, K=K, a_dtype=B.DTYPE_INT8)

    def run():
        ws = torch.zeros(B.workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
        acc = torch.full((M, N), -9, dtype=torch.int32, device=DEV)
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        B.bwta_gemm(mask, sign, wsign, s_a, s_w, acc, None, ws, M=M, N=N, K=K)
        B.bwta_gemm(mask, sign, wsign, s_a, s_w, None, out, ws, M=M, N=N, K=K)
        return [acc, out]

    B.set_path(B.PATH_FP4)
    B.set_tile(variant)
    try:
        _twice(run)
    finally:
        B.set_tile(0)
        B.set_path(B.PATH_AUTO)
