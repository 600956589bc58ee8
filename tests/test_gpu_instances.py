"""GPU parity over the kernel instances behind the dispatchers: every template instance the library
can launch for the decode kernels and the row-wise preparation kernels is chosen by K, by the token
count, by how much work a launch holds, or by a tuning hook; these tests walk those axes so that no
instance goes out untested (checked with a kernel trace of the test suite against the library's
symbol list)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev, gpu_pack_weights, same_half
from paper_2604_03957_amd import binding as B
import synth

pytestmark = pytest.mark.gpu

# K = 128 * chunks - 8: the chunk counts at which the popcount decode kernel changes its lanes per
# row or chunks per lane, and one below each (rows that are not whole 128-byte lines)
POPC_K = [128 * c - 8 * r for c in (8, 16, 32, 64, 96, 128) for r in (0, 16)]


_blocks = {}


def _weights(N, K, i):
    """Seeded +-1 weights [N, K]: a block of 64 generated rows (kept per K), repeated down the rows
    with a generated sign per row, so that tall matrices cost little to make."""
    if K not in _blocks:
        _blocks[K] = synth.binary_pm1(77, K % 1000, (64, K))
    flips = synth.binary_pm1(78 + i, N % 1000, (N,))
    return np.ascontiguousarray(_blocks[K][(np.arange(N) + 7 * i) % 64] * flips[:, None]).astype(np.int8)


def _grouped(M, N, K, count, path, seed, distinct=2):
    """count problems in one grouped call: `distinct` weight matrices and activations, cycled."""
    acts, weights = [], []
    for i in range(distinct):
        t = synth.ternary(seed, 10 + i, (M, K), 0.5)
        s_a = synth.scales(seed, 20 + i, M)
        mask, sign, _ = oracle.pack_act(t)
        acts.append((t, s_a, dev(mask), dev(sign), dev(s_a)))
        w = _weights(N, K, i)
        s_w = synth.scales(seed, 40 + i, N)
        weights.append((w, s_w, gpu_pack_weights(w), dev(s_w)))
    want = {}
    for a in range(distinct):
        for b in range(distinct):
            acc = oracle.gemm_unpacked(acts[a][0], weights[b][0])
            want[(a, b)] = (acc, oracle.epilogue(acc, acts[a][1], weights[b][1]))
    probs, outs = [], []
    for i in range(count):
        a, b = i % distinct, (i // distinct) % distinct
        acc = torch.full((M, N), -9, dtype=torch.int32, device="cuda:0")
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
        outs.append((a, b, acc, out))
        probs.append((acts[a][2], acts[a][3], weights[b][2], acts[a][4], weights[b][3], acc, out))
    ws = torch.empty(max(B.workspace_bytes(M, N, K), 256) * count, dtype=torch.uint8, device="cuda:0")
    B.set_path(path)
    try:
        B.bwta_gemm_grouped(B.make_problems(probs), ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    for a, b, acc, out in outs:
        if not (np.array_equal(acc.cpu().numpy(), want[(a, b)][0]) and same_half(out.cpu().numpy(), want[(a, b)][1])):
            return False
    return True


@pytest.mark.parametrize("K", POPC_K)
@pytest.mark.parametrize("M", [1, 2, 3, 7])
def test_popcount_decode_instances_by_shape(M, K):
    """Token tile (1, 2, 4, 8) x lanes per row and chunks per lane (by K) x streamed or cached
    weight loads (whole 128-byte rows or not), each as a single small matrix (one pass per
    wavefront) and as a grouped launch with enough work for several passes per wavefront."""
    print("popcount decode", M, K, flush=True)
    assert _grouped(M, 100, K, 1, B.PATH_POPC, 5000 + M)
    N = 1024 if K <= 1024 else 512 if K <= 2048 else 256
    assert _grouped(M, N, K, 64, B.PATH_POPC, 5100 + M)


@pytest.mark.parametrize("lanes,chunks", [(8, 4), (16, 2), (32, 1), (16, 6), (32, 3), (8, 11), (16, 4), (32, 2), (32, 4)])
def test_popcount_decode_forced_row_splits(lanes, chunks):
    """The row splits the tuning hook can force, at the largest K each holds and one with ragged
    rows, for every token tile that fits the registers."""
    B.set_tile(1000 + 16 * lanes + chunks)
    try:
        for M in (1, 2, 4, 8):
            if (1 if M == 1 else 2 if M == 2 else 4 if M <= 4 else 8) * chunks > 16:
                continue
            for K in (128 * lanes * chunks, 128 * lanes * chunks - 200):
                print("popcount decode forced", lanes, chunks, M, K, flush=True)
                assert _grouped(M, 90, K, 1, B.PATH_POPC, 5200 + M)
                assert _grouped(M, 1024 if lanes == 8 else 512, K, 64, B.PATH_POPC, 5300 + M)
    finally:
        B.set_tile(0)


@pytest.mark.parametrize("rpw,pf", [(1, 1), (1, 2), (1, 3), (1, 4), (2, 1), (2, 2), (2, 3), (2, 4), (3, 1), (3, 2), (3, 3),
                                    (4, 1), (4, 2)])
def test_matrix_core_decode_instances(rpw, pf):
    """Chunks per wavefront x ring depth x wavefronts per workgroup (4, 8 or 16 by K) x streamed or
    cached weight loads of the matrix-core decode kernel."""
    B.set_tile(2000 + 1024 * pf + 64 * rpw + 2 * pf)
    try:
        for kw in (3, 4, 7, 8, 12, 16):          # wavefronts per workgroup -> instances of 4, 8, 16
            for K in (512 * rpw * kw, 512 * rpw * kw - 264):
                if K > 24576 or -(-B.plane_row_words(K) // 16) > 16 * rpw:
                    continue
                print("decode fp4", rpw, pf, kw, K, flush=True)
                assert _grouped(5, 70, K, 3, B.PATH_FP4, 5400 + rpw)
    finally:
        B.set_tile(0)


@pytest.mark.parametrize("K", [1000, 2048, 3000, 4096, 6000, 8192, 11008, 16384, 20000, 32768])
def test_row_kernels_every_group_count(K):
    """bwta_act_scale, bwta_prepare_act_autoscale (planes on a decode-sized M, fragments on a
    prefill-sized one) and bwta_prepare_weights pick their 128-bit groups per thread and threads per
    row by K."""
    print("row kernels", K, flush=True)
    for M in (5, 160):
        A = synth.gaussian_outlier_activations(5500 + M, 1, M, K)
        want_s = oracle.act_scale(A)
        s = torch.zeros(M, dtype=torch.float16, device="cuda:0")
        B.bwta_act_scale(dev(A), s, M=M, K=K)
        torch.cuda.synchronize()
        assert np.array_equal(s.cpu().numpy().view(np.uint16), want_s.view(np.uint16))
        N = 48
        w = synth.binary_pm1(5600, 2, (N, K))
        s_w = synth.scales(5600, 3, N)
        _, _, want = oracle.linear(A, want_s, w, s_w)
        prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device="cuda:0")
        s2 = torch.zeros(M, dtype=torch.float16, device="cuda:0")
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
        fmt = B.bwta_prepare_act_autoscale(dev(A), s2, prep, M=M, K=K)
        B.bwta_gemm_prepared(prep, gpu_pack_weights(w), s2, dev(s_w), None, out, fmt=fmt, M=M, N=N, K=K)
        torch.cuda.synchronize()
        assert np.array_equal(s2.cpu().numpy().view(np.uint16), want_s.view(np.uint16))
        assert same_half(out.cpu().numpy(), want)
    Wf = synth.gaussian_outlier_activations(5700, 4, 40, K)      # any fp16 matrix serves as full-precision weights
    w_want, sw_want = oracle.prepare_weights(Wf)
    wsign = torch.full((40, B.plane_row_words(K)), -1, dtype=torch.int32, device="cuda:0")
    s_w = torch.zeros(40, dtype=torch.float16, device="cuda:0")
    B.bwta_prepare_weights(dev(Wf), wsign, s_w, N=40, K=K)
    torch.cuda.synchronize()
    assert np.array_equal(wsign.cpu().numpy().view(np.uint32), oracle.pack_weights(w_want))
    assert np.array_equal(s_w.cpu().numpy().view(np.uint16), sw_want.view(np.uint16))


@pytest.mark.parametrize("M,N,K", [(2048, 4096, 520), (4096, 6144, 200)])
def test_int8_matrix_core_kernel_large_tiles(M, N, K):
    """The int8 MFMA comparison kernel picks 128x256 and 256x256 workgroup tiles once a launch
    holds enough of them; both on full outputs, int32 and fp16."""
    print("int8 mfma large tiles", M, N, K, flush=True)
    t = synth.ternary(5800, 1, (M, K), 0.5)
    w = _weights(N, K, 0)
    s_a, s_w = synth.scales(5800, 2, M), synth.scales(5800, 3, N)
    mask, sign, _ = oracle.pack_act(t)
    want_acc = oracle.gemm_unpacked(t, w)
    want = oracle.epilogue(want_acc, s_a, s_w)
    acc = torch.full((M, N), -9, dtype=torch.int32, device="cuda:0")
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    ws = torch.empty(max(B.workspace_bytes(M, N, K), 256), dtype=torch.uint8, device="cuda:0")
    B.set_path(B.PATH_MFMA)
    try:
        B.bwta_gemm(dev(mask), dev(sign), gpu_pack_weights(w), dev(s_a), dev(s_w), acc, out, ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    assert np.array_equal(acc.cpu().numpy(), want_acc)
    assert same_half(out.cpu().numpy(), want)
