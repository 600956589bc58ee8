"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element.

Bars: packed planes, nnz and int32 accumulators bit-exact; fp16 outputs within 1e-3
relative (the kernels are built to round exactly once, so in practice they are bit-equal
and the tests report that too).
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import (dev, gpu_gemm, gpu_linear, gpu_pack_weights, gpu_quantize_pack, host_u32,
                      max_rel_err, same_half)
from paper_2604_03957_amd import binding as B
import inputs
import synth

pytestmark = pytest.mark.gpu
RTOL = 1e-3
PATHS = [B.PATH_POPC, B.PATH_MFMA, B.PATH_FP4]


def _say(*a):
    print(*a, flush=True)


# ---- ternarise + pack ---------------------------------------------------------------------

def _activation_case(seed, M, K, lda=None):
    lda = K if lda is None else lda
    A = (synth.gaussian(seed, 1, M * lda).reshape(M, lda) * 1.3).astype(np.float16)
    s = synth.scales(seed, 2, M, 0.3, 2.5)
    # plant exact ties and special values
    for m in range(min(M, 6)):
        h = np.float16(0.5 * float(s[m]))
        vals = [h, -h, np.nextafter(h, np.float16(0)), np.nextafter(-h, np.float16(-np.inf)),
                np.float16(np.nan), np.float16(np.inf), np.float16(-np.inf), np.float16(-0.0)]
        for i, v in enumerate(vals):
            if i < K:
                A[m, (7 * m + 5 * i) % K] = v
    return A, s


@pytest.mark.parametrize("M,K,lda", [(5, 40, None), (64, 768, None), (33, 300, 304), (257, 1001, 1003),
                                     (3, 4096, None), (2, 11008, None), (1, 1, None), (130, 129, 136)])
def test_quantize_pack_fp16_matches_oracle(M, K, lda):
    _say("quantize fp16", M, K, lda)
    A, s = _activation_case(100 + M, M, K, lda)
    t = oracle.ternarize(np.ascontiguousarray(A[:, :K]), s)
    want = oracle.pack_act(t)
    got = gpu_quantize_pack(A, s, K=K)
    for w, g, name in zip(want, got, ("mask", "sign", "nnz")):
        assert np.array_equal(w, g), name


@pytest.mark.parametrize("M,K,lda", [(2100, 4096, None), (2300, 3720, 3728), (70000, 128, None)])
def test_quantize_pack_fp16_large_aligned_rows(M, K, lda):
    """Sizes at which aligned fp16 rows take the four-groups-per-thread kernel: whole rows, rows with
    padding groups past K, rows narrower than a wavefront's span; a few invalid scales among them."""
    _say("quantize fp16 large", M, K, lda)
    A, s = _activation_case(300 + K, M, K, lda)
    s[5], s[17], s[M - 1] = 0.0, np.nan, np.inf
    want = oracle.pack_act(oracle.ternarize(np.ascontiguousarray(A[:, :K]), s))
    got = gpu_quantize_pack(A, s, K=K)
    for w, g, name in zip(want, got, ("mask", "sign", "nnz")):
        assert np.array_equal(w, g), name
    sc = np.array([0.75], np.float16)                                  # one scale for the whole tensor
    want = oracle.pack_act(oracle.ternarize(np.ascontiguousarray(A[:, :K]), sc))
    got = gpu_quantize_pack(A, sc, K=K)
    assert all(np.array_equal(w, g) for w, g in zip(want, got))


def test_quantize_pack_scale_modes_and_bad_scales():
    M, K = 9, 200
    A, _ = _activation_case(7, M, K)
    one = oracle.pack_act(oracle.ternarize(A, None))
    got = gpu_quantize_pack(A, None)
    assert all(np.array_equal(w, g) for w, g in zip(one, got))
    sc = np.array([0.75], np.float16)
    want = oracle.pack_act(oracle.ternarize(A, sc))
    got = gpu_quantize_pack(A, sc)
    assert all(np.array_equal(w, g) for w, g in zip(want, got))
    bad = np.array([1.0, 0.0, -1.0, np.inf, np.nan, 2.0 ** -24, 6e-5, 65504.0, 1.5], np.float16)
    want = oracle.pack_act(oracle.ternarize(A, bad))
    got = gpu_quantize_pack(A, bad)
    assert all(np.array_equal(w, g) for w, g in zip(want, got))
    assert not got[0][1:5].any()          # rows with an invalid scale are all zero


def test_quantize_pack_every_half_pattern():
    A = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16).reshape(16, 4096)
    for sv in (1.0, 0.37, 2.0 ** -14, 2.0 ** -24, 900.0):
        s = np.full(16, sv, np.float16)
        want = oracle.pack_act(oracle.ternarize(A, s))
        got = gpu_quantize_pack(A, s)
        assert all(np.array_equal(w, g) for w, g in zip(want, got)), sv


def test_fragment_routes_every_half_pattern():
    """All 65 536 fp16 bit patterns, each under every one of 14 scales, through the two kernels that
    ternarise straight into matrix-core fragments (bwta_prepare_act on the tiled path, and the
    one-launch linear).  The scales include the smallest subnormal, odd and even subnormals, the
    values around 2^-14 and 2^-13 (where half the scale stops being a binary16 value) and the largest
    finite one.  The fragments are opaque, so the check is on what they produce against 64 random
    weight rows: one wrong decision changes every accumulator of its token by 1 or 2."""
    M, K, N = 256, 256, 64
    A = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16).reshape(M, K)
    svals = np.array([0x3c00, 0x3800, 0x3e00, 0x0001, 0x0002, 0x0003, 0x03ff, 0x0400, 0x0401, 0x07ff, 0x0800,
                      0x0801, 0x7bff, 0x2e65], np.uint16).view(np.float16)
    w = synth.binary_pm1(35, 1, (N, K))
    ones = np.ones(N, np.float16)
    wsign = gpu_pack_weights(w)
    wsign2 = gpu_pack_weights(np.concatenate([w, w], axis=0))  # the one-launch kernel wants at least 128 channels
    prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(B.workspace_bytes(M, 128, K), dtype=torch.uint8, device="cuda:0")
    B.set_path(B.PATH_FP4)
    try:
        for rot in range(len(svals)):
            s = svals[(np.arange(M) + rot) % len(svals)]
            _, want_acc, want_out = oracle.linear(A, s, w, ones)
            acc = torch.full((M, N), 123456, dtype=torch.int32, device="cuda:0")
            B.set_tile(0)
            fmt = B.bwta_prepare_act(dev(A), dev(s), prep, M=M, K=K)
            B.bwta_gemm_prepared(prep, wsign, dev(s), dev(ones), acc, None, fmt=fmt, M=M, N=N, K=K)
            torch.cuda.synchronize()
            assert np.array_equal(acc.cpu().numpy(), want_acc), rot
            out = torch.full((M, 128), 7.0, dtype=torch.float16, device="cuda:0")
            B.set_tile(901)
            B.bwta_linear(dev(A), dev(s), wsign2, dev(np.ones(128, np.float16)), out, ws, M=M, N=128, K=K)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert same_half(np.ascontiguousarray(got[:, :N]), want_out), rot
            assert same_half(np.ascontiguousarray(got[:, N:]), want_out), rot
    finally:
        B.set_tile(0)
        B.set_path(B.PATH_AUTO)


@pytest.mark.parametrize("M,K,lda", [(64, 768, None), (7, 333, 335), (2, 11008, None)])
def test_quantize_pack_int8_matches_oracle(M, K, lda):
    lda = K if lda is None else lda
    t = synth.ternary(5, M, (M, lda), 0.4)
    want = oracle.pack_act(np.ascontiguousarray(t[:, :K]))
    got = gpu_quantize_pack(t, None, K=K)
    assert all(np.array_equal(w, g) for w, g in zip(want, got))


def test_quantize_pack_unaligned_base_pointer():
    M, K = 6, 264
    A, s = _activation_case(3, M, K + 8)
    flat = dev(A.reshape(-1))
    view = flat[1:]                                   # 2-byte aligned only
    ref = A.reshape(-1)[1:1 + (M - 1) * (K + 8) + K]
    rows = np.stack([ref[m * (K + 8): m * (K + 8) + K] for m in range(M)])
    want = oracle.pack_act(oracle.ternarize(rows, s))
    rw = B.plane_row_words(K)
    mask = torch.zeros((M, rw), dtype=torch.int32, device="cuda:0")
    sign = torch.zeros_like(mask)
    B.bwta_quantize_pack_act(view, dev(s), mask, sign, None, M=M, K=K, lda=K + 8)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(mask), want[0]) and np.array_equal(host_u32(sign), want[1])


@pytest.mark.parametrize("N,K", [(5, 40), (768, 768), (17, 1001), (3, 11008)])
def test_pack_weights_matches_oracle(N, K):
    w = synth.binary_pm1(11, N, (N, K))
    want = oracle.pack_weights(w)
    assert np.array_equal(host_u32(gpu_pack_weights(w)), want)
    Wf = (synth.gaussian(12, N, N * K).reshape(N, K)).astype(np.float16)
    Wf[0, :4] = np.array([0.0, -0.0, np.nan, -1e-7], np.float16)
    want = oracle.pack_weights(oracle.sign_weights(Wf))
    assert np.array_equal(host_u32(gpu_pack_weights(Wf)), want)


# ---- product + epilogue ---------------------------------------------------------------------

def _gemm_case(seed, M, N, K, p0=0.45):
    t = synth.ternary(seed, 1, (M, K), p0)
    w = synth.binary_pm1(seed, 2, (N, K))
    return t, w, synth.scales(seed, 3, M), synth.scales(seed, 4, N)


def _check_gemm(t, w, s_a, s_w, path, dirty_sign=False):
    M, K = t.shape
    N = w.shape[0]
    mask, sign, _ = oracle.pack_act(t)
    ws = oracle.pack_weights(w)
    want_acc = oracle.gemm_unpacked(t, w)
    want_out = oracle.epilogue(want_acc, s_a, s_w)
    if dirty_sign:
        sign = sign | (~mask & np.uint32(0x5A5A5A5A))
    acc, out = gpu_gemm(mask, sign, ws, s_a, s_w, M, N, K, path=path)
    assert np.array_equal(acc, want_acc), "int32 accumulators differ"
    err = max_rel_err(out, want_out)
    assert err <= RTOL, err
    return same_half(out, want_out)


GEMM_SHAPES = [(64, 768, 768), (1, 64, 128), (3, 5, 33), (16, 100, 4096), (130, 200, 1000),
               (300, 260, 2048), (257, 513, 1408), (70, 129, 11008), (4, 300, 11008)]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_matches_oracle(M, N, K, path):
    _say("gemm", M, N, K, "path", path)
    t, w, s_a, s_w = _gemm_case(1000 + M + N, M, N, K)
    exact = _check_gemm(t, w, s_a, s_w, path)
    assert exact, "fp16 outputs are within tolerance but not bit-equal"


DECODE_SHAPES = [(1, 7, 33), (2, 130, 128), (3, 257, 1000), (1, 1001, 4096), (4, 999, 4096), (8, 300, 4096),
                 (5, 258, 8192), (1, 515, 11008), (4, 130, 11008), (8, 67, 11008), (2, 70, 16384),
                 (3, 40, 16512), (9, 100, 4096), (13, 77, 1408), (16, 257, 11008), (16, 90, 768),
                 (16, 40, 17000), (7, 33, 30000), (12, 16, 512), (15, 17, 513), (17, 100, 4096), (33, 70, 11008),
                 (64, 130, 1000), (48, 17, 128), (65, 200, 4096), (100, 70, 11008), (128, 129, 1000)]


@pytest.mark.parametrize("M,N,K", DECODE_SHAPES)
def test_decode_shaped_gemm_matches_oracle(M, N, K):
    _say("decode gemm", M, N, K)
    t, w, s_a, s_w = _gemm_case(2000 + M + N, M, N, K, p0=0.5)
    assert _check_gemm(t, w, s_a, s_w, B.PATH_AUTO)
    assert _check_gemm(t, w, s_a, s_w, B.PATH_POPC, dirty_sign=True)
    assert _check_gemm(t, w, s_a, s_w, B.PATH_FP4, dirty_sign=True)


@pytest.mark.parametrize("rpw,tiles,pf", [(1, 2, 2), (1, 8, 2), (1, 8, 4), (1, 6, 3), (2, 2, 2), (2, 4, 2), (2, 8, 2),
                                          (2, 8, 4), (2, 16, 4), (2, 6, 3), (2, 4, 4), (3, 2, 2), (3, 4, 2), (3, 8, 2),
                                          (3, 6, 3), (3, 9, 3), (4, 2, 2), (4, 4, 2), (4, 8, 2),
                                          (1, 1, 1), (2, 1, 1), (2, 3, 1), (3, 1, 1), (4, 1, 1)])
def test_matrix_core_decode_every_work_split(rpw, tiles, pf):
    """Chunks per wavefront x channel tiles per workgroup x ring depth of the matrix-core decode
    kernel, on shapes with ragged N, a K tail inside a chunk, and more tiles than one workgroup takes."""
    _say("decode fp4 split", rpw, tiles, pf)
    B.set_tile(2000 + 1024 * pf + 64 * rpw + tiles)
    try:
        for M, N, K in [(16, 100, 4096), (11, 70, 11008), (1, 33, 200), (5, 1000, 1000), (40, 50, 600)]:
            if -(-B.plane_row_words(K) // 16) > 16 * rpw:
                continue
            t, w, s_a, s_w = _gemm_case(2500 + M + rpw, M, N, K, p0=0.5)
            assert _check_gemm(t, w, s_a, s_w, B.PATH_FP4)
    finally:
        B.set_tile(0)


def test_decode_seeded_random_shapes():
    """Twenty decode-sized problems with shapes drawn from a seeded generator (token counts across
    the token-group boundaries, ragged channel counts, K tails anywhere inside a 512-k chunk), on
    both decode kernel families and the dispatcher's choice."""
    rng = np.random.default_rng(20260403)
    for case in range(20):
        M = int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 31, 33, 48, 63, 64, 65, 96, 127, 128]))
        N = int(rng.integers(1, 700))
        K = int(rng.integers(1, 9000))
        _say("decode random", case, M, N, K)
        t, w, s_a, s_w = _gemm_case(4000 + case, M, N, K, p0=float(rng.uniform(0.1, 0.9)))
        assert _check_gemm(t, w, s_a, s_w, B.PATH_AUTO, dirty_sign=True)
        assert _check_gemm(t, w, s_a, s_w, B.PATH_FP4)
        if M <= 16:
            assert _check_gemm(t, w, s_a, s_w, B.PATH_POPC)


@pytest.mark.parametrize("tile", [0, 22, 23, 21, 12, 11, 13, 222])
def test_tiled_matrix_core_kernel_every_tile_variant(tile):
    """The tiled FP4 kernel's workgroup tiles (128x128 at two and three wavefronts per SIMD, 128x64,
    64x128, 64x64, 128x96, split-K) and the dispatcher's own choice (0: 64x64 tiles for these few-tile
    shapes), fp16 output only (the int32 output always takes the 128x128 variant), ragged in M, N and K."""
    _say("fp4 tile variant", tile)
    B.set_tile(tile)
    try:
        for M, N, K in [(300, 260, 2048), (129, 70, 1100), (200, 513, 4096 + 64)]:
            t, w, s_a, s_w = _gemm_case(3000 + M, M, N, K)
            mask, sign, _ = oracle.pack_act(t)
            want = oracle.epilogue(oracle.gemm_unpacked(t, w), s_a, s_w)
            _, out = gpu_gemm(mask, sign, oracle.pack_weights(w), s_a, s_w, M, N, K, path=B.PATH_FP4, want_acc=False)
            assert same_half(out, want)
    finally:
        B.set_tile(0)


@pytest.mark.parametrize("path", PATHS)
def test_gemm_config1_tiny(path):
    c = synth.config1()
    assert _check_gemm(c["t"], c["w"], c["s_a"], c["s_w"], path)


@pytest.mark.parametrize("path", PATHS)
def test_gemm_degenerate_inputs(path):
    M, N, K = 40, 70, 600
    t, w, s_a, s_w = _gemm_case(77, M, N, K)
    _check_gemm(np.zeros_like(t), w, s_a, s_w, path)              # all-zero activation -> all-zero output
    _check_gemm(np.ones_like(t), np.ones_like(w), s_a, s_w, path)   # every product +1 -> K
    _check_gemm(-np.ones_like(t), np.ones_like(w), s_a, s_w, path)  # -> -K
    _check_gemm(t, w, s_a, s_w, path, dirty_sign=True)            # sign bits under a zero mask are ignored
    big = s_a.copy(); big[:] = np.float16(60000.0)                # overflow to +-Inf in the epilogue
    _check_gemm(t, w, big, s_w, path)
    tiny = s_w.copy(); tiny[:] = np.float16(2.0 ** -24)           # subnormal fp16 results
    assert _check_gemm(t, w, np.full(M, 2.0 ** -10, np.float16), tiny, path)
    neg = s_a.copy(); neg[::2] *= -1                              # negative scales, signed zeros
    sparse = t.copy(); sparse[:, 3:] = 0
    assert _check_gemm(sparse, w, neg, s_w, path)
    assert _check_gemm(t, w, neg, -s_w, path)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("M,N,K", [(20, 36, 256), (200, 130, 600)])  # decode kernels / tiled kernels
def test_gemm_output_selection_and_scale_modes(path, M, N, K):
    t, w, s_a, s_w = _gemm_case(5, M, N, K)
    mask, sign, _ = oracle.pack_act(t)
    ws = oracle.pack_weights(w)
    want_acc = oracle.gemm_unpacked(t, w)
    acc, out = gpu_gemm(mask, sign, ws, None, None, M, N, K, path=path)
    assert np.array_equal(acc, want_acc) and same_half(out, oracle.epilogue(want_acc, None, None))
    acc, _ = gpu_gemm(mask, sign, ws, s_a, s_w, M, N, K, path=path, want_out=False)
    assert np.array_equal(acc, want_acc)
    _, out = gpu_gemm(mask, sign, ws, s_a[:1], s_w[:1], M, N, K, path=path, want_acc=False)
    assert same_half(out, oracle.epilogue(want_acc, s_a[:1], s_w[:1]))


def test_empty_problem_is_a_noop():
    ws = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    z = torch.empty(0, dtype=torch.int32, device="cuda:0")
    B.bwta_gemm(z, z, z, None, None, z, None, ws, M=0, N=8, K=128)
    B.bwta_quantize_pack_act(z, None, z, z, None, M=0, K=128)
    torch.cuda.synchronize()


# ---- the whole layer ----------------------------------------------------------------------

@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("which", ["up", "down"])
def test_linear_ffn_reduced_m(which, path):
    c = inputs.config2(which, M=200)
    _say("linear", c["name"], "path", path)
    _, _, want = oracle.linear(c["A"], c["s_a"], c["w"], c["s_w"])
    wsign = gpu_pack_weights(c["w"])
    out = gpu_linear(c["A"], c["s_a"], wsign, c["s_w"], c["N"], path=path)
    assert max_rel_err(out, want) <= RTOL
    assert same_half(out, want)


@pytest.mark.parametrize("path", PATHS)
def test_linear_laplace_block_input(path):
    x = synth.laplace_activations(4, 1, 96, 4096)
    s = oracle.act_scale(x)
    w = synth.binary_pm1(4, 10, (160, 4096))
    s_w = synth.scales(4, 11, 160)
    _, _, want = oracle.linear(x, s, w, s_w)
    out = gpu_linear(x, s, gpu_pack_weights(w), s_w, 160, path=path)
    assert same_half(out, want)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("M,N,K", [(1, 9, 40), (37, 130, 1001), (130, 70, 129), (257, 300, 2500), (33, 64, 11008)])
def test_linear_ragged_shapes_and_special_values(M, N, K, path):
    _say("linear ragged", M, N, K, "path", path)
    A, s = _activation_case(300 + M, M, K)          # ties, NaN, Inf, -0.0 planted
    if M > 4:
        s[3] = np.float16(0.0)                      # an invalid scale zeroes the token
    w = synth.binary_pm1(31, M + N, (N, K))
    s_w = synth.scales(31, 5, N)
    _, _, want = oracle.linear(A, s, w, s_w)
    out = gpu_linear(A, s, gpu_pack_weights(w), s_w, N, path=path)
    assert same_half(out, want)


@pytest.mark.parametrize("hook", [0, 901, 902, 903, 906, 912])
@pytest.mark.parametrize("M,N,K", [(256, 128, 128), (300, 260, 768), (1000, 3072, 768), (289, 1000, 1000), (700, 513, 1024), (257, 130, 136),
                                   (129, 130, 136), (200, 513, 768), (2, 130, 136), (16, 513, 768), (100, 3072, 1000)])
def test_linear_one_launch_short_k(M, N, K, hook):
    """bwta_linear as a single kernel (K <= 1024): every chunk count, channel splits forced to
    1, 2, 3, 6 and 12 as well as the launcher's own choice (which makes every group width appear; 0 = the
    dispatcher decides whether to use the kernel at all),
    ragged M and N, special values, an invalid token scale."""
    _say("one-launch linear", M, N, K, "hook", hook)
    A, s = _activation_case(500 + M, M, K)
    s[min(5, M - 1)] = np.float16(0.0)
    w = synth.binary_pm1(33, M + N, (N, K))
    s_w = synth.scales(33, 7, N)
    _, _, want = oracle.linear(A, s, w, s_w)
    B.set_tile(hook)
    try:
        out = gpu_linear(A, s, gpu_pack_weights(w), s_w, N, path=B.PATH_FP4)
    finally:
        B.set_tile(0)
    assert same_half(out, want)


@pytest.mark.parametrize("K", [200, 504, 760, 1000])
@pytest.mark.parametrize("N", [250, 440, 512, 1000])
def test_linear_one_launch_every_kernel_instance(N, K):
    """With two channel splits forced, N = 250 / 440 / 512 / 1000 leaves a workgroup 4 / 7 / 8 / 16
    channel blocks: workgroups of 4 or 8 wavefronts with groups of one or two blocks; K = 200 ..
    1000 gives one to four chunks of 256 k.  Together every instance of the kernel runs, on ragged
    M, N and K."""
    M = 300
    _say("one-launch linear, instance sweep", M, N, K)
    A, s = _activation_case(900 + N + K, M, K)
    w = synth.binary_pm1(36, N + K, (N, K))
    s_w = synth.scales(36, 8, N)
    _, _, want = oracle.linear(A, s, w, s_w)
    B.set_tile(902)
    try:
        assert B.linear_launches(M, N, K) == 1
        out = gpu_linear(A, s, gpu_pack_weights(w), s_w, N, path=B.PATH_FP4)
    finally:
        B.set_tile(0)
    assert same_half(out, want)


def test_linear_one_launch_seeded_random_shapes():
    """40 seeded random shapes (M 256..1500, N 128..2500, K 8..1024 in steps of 8) through the
    dispatcher's own choice of launch form, split count and kernel instance."""
    rng = np.random.default_rng(20260404)
    for case in range(40):
        M, N, K = int(rng.integers(256, 1501)), int(rng.integers(128, 2501)), 8 * int(rng.integers(1, 129))
        _say("one-launch linear, random shape", case, M, N, K)
        A, s = _activation_case(2000 + case, M, K)
        w = synth.binary_pm1(37, case, (N, K))
        s_w = synth.scales(37, 100 + case, N)
        _, _, want = oracle.linear(A, s, w, s_w)
        assert B.linear_launches(M, N, K) == 1
        out = gpu_linear(A, s, gpu_pack_weights(w), s_w, N)
        assert same_half(out, want), (case, M, N, K)


def test_every_entry_and_family_seeded_random_shapes():
    """60 seeded random problems (prefill-sized with any K, short K, decode-sized) with planted
    ties, infinities, NaN, -0 and now and then an invalid token scale: bwta_linear as dispatched,
    and bwta_gemm on the dispatcher's choice and on each kernel family, int32 and fp16."""
    rng = np.random.default_rng(20260405)
    for case in range(60):
        kind = case % 3
        if kind == 0:
            M, N, K = int(rng.integers(129, 1200)), int(rng.integers(1, 1500)), int(rng.integers(1, 3000))
        elif kind == 1:
            M, N, K = int(rng.integers(256, 3000)), int(rng.integers(128, 3000)), 8 * int(rng.integers(1, 129))
        else:
            M, N, K = int(rng.integers(1, 129)), int(rng.integers(1, 2000)), int(rng.integers(1, 12000))
        _say("random problem", case, M, N, K)
        A = (synth.gaussian(9000 + case, 1, M * K) * float(rng.uniform(0.01, 30))).astype(np.float16).reshape(M, K)
        s = oracle.act_scale(A)
        if M * K > 8:
            flat = A.reshape(-1)
            idx = rng.integers(0, flat.size, 6)
            flat[idx[0]] = np.float16(0.5) * s[idx[0] // K]
            flat[idx[1]] = -(np.float16(0.5) * s[idx[1] // K])
            flat[idx[2]], flat[idx[3]], flat[idx[4]], flat[idx[5]] = np.inf, -np.inf, np.nan, -0.0
        if case % 4 == 0:
            s[int(rng.integers(0, M))] = np.float16([0.0, -1.0, np.inf, np.nan][(case // 4) % 4])
        w = synth.binary_pm1(9100 + case, 2, (N, K))
        s_w = synth.scales(9200 + case, 3, N)
        t, acc_want, want = oracle.linear(A, s, w, s_w)
        wsign = gpu_pack_weights(w)
        assert same_half(gpu_linear(A, s, wsign, s_w, N), want), (case, M, N, K)
        mask, sign, _ = oracle.pack_act(t)
        for path in [B.PATH_AUTO] + PATHS:
            acc, out = gpu_gemm(mask, sign, wsign, s, s_w, M, N, K, path=path)
            assert np.array_equal(acc, acc_want) and same_half(out, want), (case, M, N, K, path)


def test_linear_one_launch_scale_modes_and_strides():
    """The one-launch kernel with layerwise (scalar) scales, with no scales at all, and with strided
    input and output (nothing written past N)."""
    M, N, K, lda = 300, 260, 512, 520
    A, _ = _activation_case(601, M, lda)
    w = synth.binary_pm1(34, 1, (N, K))
    Ak = np.ascontiguousarray(A[:, :K])
    one_a, one_w = np.array([0.75], np.float16), np.array([1.25], np.float16)
    ws = torch.empty(B.workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda:0")
    wsign = gpu_pack_weights(w)
    B.set_tile(901)
    B.set_path(B.PATH_FP4)
    try:
        for (s_a, s_w), ldo in (((one_a, one_w), 272), ((None, None), 263)):  # 263: rows not 16-byte aligned
            fa = np.full(M, 1.0 if s_a is None else s_a[0], np.float16)
            fw = np.full(N, 1.0 if s_w is None else s_w[0], np.float16)
            _, _, want = oracle.linear(Ak, fa, w, fw)
            out = torch.full((M, ldo), 7.0, dtype=torch.float16, device="cuda:0")
            B.bwta_linear(dev(A), None if s_a is None else dev(s_a), wsign, None if s_w is None else dev(s_w), out, ws,
                          M=M, N=N, K=K, lda=lda, ldo=ldo)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert same_half(np.ascontiguousarray(got[:, :N]), want)
            assert np.all(got[:, N:] == 7.0)
    finally:
        B.set_path(B.PATH_AUTO)
        B.set_tile(0)


def test_linear_strided_input_and_output():
    M, N, K, lda, ldo = 50, 72, 520, 528, 80
    A, s = _activation_case(9, M, lda)
    w = synth.binary_pm1(32, 1, (N, K))
    s_w = synth.scales(32, 2, N)
    _, _, want = oracle.linear(np.ascontiguousarray(A[:, :K]), s, w, s_w)
    out = torch.full((M, ldo), 7.0, dtype=torch.float16, device="cuda:0")
    ws = torch.empty(B.workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda:0")
    for path in PATHS:
        B.set_path(path)
        out.fill_(7.0)
        B.bwta_linear(dev(A), dev(s), gpu_pack_weights(w), dev(s_w), out, ws, M=M, N=N, K=K, lda=lda, ldo=ldo)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert same_half(np.ascontiguousarray(got[:, :N]), want), path
        assert np.all(got[:, N:] == 7.0)            # nothing written past N
    B.set_path(B.PATH_AUTO)


@pytest.mark.parametrize("path", PATHS)
def test_prepare_once_feed_several_weight_matrices(path):
    M, K = 70, 1300
    A, s = _activation_case(55, M, K)
    prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device="cuda:0")
    B.set_path(path)
    try:
        fmt = B.bwta_prepare_act(dev(A), dev(s), prep, M=M, K=K)
        for i, N in enumerate((40, 129)):
            w = synth.binary_pm1(60 + i, 1, (N, K))
            s_w = synth.scales(60 + i, 2, N)
            t, acc_want, want = oracle.linear(A, s, w, s_w)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda:0")
            acc = torch.empty((M, N), dtype=torch.int32, device="cuda:0")
            B.bwta_gemm_prepared(prep, gpu_pack_weights(w), dev(s), dev(s_w), acc, out, fmt=fmt, M=M, N=N, K=K)
            torch.cuda.synchronize()
            assert np.array_equal(acc.cpu().numpy(), acc_want)
            assert same_half(out.cpu().numpy(), want)
    finally:
        B.set_path(B.PATH_AUTO)


@pytest.mark.parametrize("path", [B.PATH_AUTO, B.PATH_POPC, B.PATH_FP4])
@pytest.mark.parametrize("M,N,K,count", [(1, 300, 4096, 3), (4, 130, 11008, 2), (8, 70, 1000, 35), (16, 64, 512, 2), (37, 50, 640, 3)])
def test_gemm_grouped_matches_oracle(M, N, K, count, path):
    _say("grouped", M, N, K, count, path)
    t, _, s_a, _ = _gemm_case(3000 + M, M, N, K, p0=0.5)
    mask, sign, _ = oracle.pack_act(t)
    dm, dsg, dsa = dev(mask), dev(sign), dev(s_a)
    keep, probs, want = [], [], []
    for i in range(count):
        w = synth.binary_pm1(3100 + i, M, (N, K))
        s_w = synth.scales(3200 + i, M, N)
        acc_want = oracle.gemm_unpacked(t, w)
        want.append((acc_want, oracle.epilogue(acc_want, s_a, s_w)))
        dw, dsw = gpu_pack_weights(w), dev(s_w)
        acc = torch.full((M, N), -9, dtype=torch.int32, device="cuda:0")
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
        keep.append((dw, dsw, acc, out))
        probs.append((dm, dsg, dw, dsa, dsw, acc, out))
    ws = torch.empty(max(B.workspace_bytes(M, N, K), 256) * count, dtype=torch.uint8, device="cuda:0")
    B.set_path(path)
    try:
        B.bwta_gemm_grouped(B.make_problems(probs), ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    for (dw, dsw, acc, out), (acc_want, out_want) in zip(keep, want):
        assert np.array_equal(acc.cpu().numpy(), acc_want)
        assert same_half(out.cpu().numpy(), out_want)


@pytest.mark.parametrize("path", [B.PATH_AUTO, B.PATH_POPC, B.PATH_FP4])
@pytest.mark.parametrize("M", [1, 5, 12, 40])
def test_gemm_grouped_mixed_null_scales(M, path):
    """Problems of one grouped call may leave either scale out (NULL reads as 1) independently of
    their neighbours, the first problem included."""
    N, K = 150, 700
    _say("grouped mixed scales", M, N, K, path)
    t, _, s_a, _ = _gemm_case(3300 + M, M, N, K, p0=0.5)
    mask, sign, _ = oracle.pack_act(t)
    dm, dsg, dsa = dev(mask), dev(sign), dev(s_a)
    have = [(False, False), (True, True), (False, True), (True, False), (True, True)]  # (s_a, s_w) present?
    keep, probs, want = [], [], []
    for i, (ha, hw) in enumerate(have):
        w = synth.binary_pm1(3400 + i, M, (N, K))
        s_w = synth.scales(3500 + i, M, N)
        acc_want = oracle.gemm_unpacked(t, w)
        want.append(oracle.epilogue(acc_want, s_a if ha else None, s_w if hw else None))
        dw, dsw = gpu_pack_weights(w), dev(s_w)
        out = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
        keep.append((dw, dsw, out))
        probs.append((dm, dsg, dw, dsa if ha else None, dsw if hw else None, None, out))
    ws = torch.empty(max(B.workspace_bytes(M, N, K), 256) * len(have), dtype=torch.uint8, device="cuda:0")
    B.set_path(path)
    try:
        B.bwta_gemm_grouped(B.make_problems(probs), ws, M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    for i, ((dw, dsw, out), out_want) in enumerate(zip(keep, want)):
        assert same_half(out.cpu().numpy(), out_want), (i, have[i])


@pytest.mark.parametrize("path", [B.PATH_AUTO] + PATHS)
@pytest.mark.parametrize("M,N,K", [(64, 96, 768), (3, 130, 1000), (130, 70, 129), (16, 257, 4096), (300, 200, 1000)])
def test_binary_activations_w1a1(M, N, K, path):
    """mask == NULL: binary (+-1) activations, the W1A1 "Binary Linear" special case
    acc = K - 2 popc(x ^ w); the activation signs are packed with the sign packer."""
    _say("w1a1", M, N, K, path)
    x = synth.binary_pm1(4000 + M, 1, (M, K))
    w = synth.binary_pm1(4000 + M, 2, (N, K))
    s_a, s_w = synth.scales(4000, 3, M), synth.scales(4000, 4, N)
    want_acc = oracle.gemm_unpacked(x, w)
    xs, wsn = oracle.pack_weights(x), oracle.pack_weights(w)
    xor_popc = np.array([[bin(int.from_bytes((xs[m] ^ wsn[n]).tobytes(), "little")).count("1") for n in range(N)] for m in range(min(M, 4))])
    assert np.array_equal(want_acc[:min(M, 4)], K - 2 * xor_popc)           # the textbook XNOR-popcount form
    acc, out = gpu_gemm(None, xs, wsn, s_a, s_w, M, N, K, path=path)
    assert np.array_equal(acc, want_acc)
    assert same_half(out, oracle.epilogue(want_acc, s_a, s_w))


@pytest.mark.parametrize("variant", [223, 243, 323])
@pytest.mark.parametrize("M,N,K", [(129, 256, 256), (300, 200, 1000), (257, 513, 2100), (1000, 700, 4096), (130, 90, 11008),
                                   (1000, 704, 4096), (256, 288, 256), (136, 64, 11008), (2048, 1024, 768),
                                   (4096, 4608, 384)])
def test_lds_staged_tiled_kernel_variants(M, N, K, variant):
    """The tiled FP4 kernel whose operands reach LDS by direct global->LDS loads, every tile / ring
    variant forced through the tuning hook: int32 accumulators and fp16 outputs, from planes
    (bwta_gemm) and from fp16 activations (bwta_linear's two-kernel form)."""
    _say("lds-staged", M, N, K, variant)
    t, w, s_a, s_w = _gemm_case(5000 + M + variant, M, N, K, p0=0.5)
    mask, sign, _ = oracle.pack_act(t)
    wsign = oracle.pack_weights(w)
    want_acc = oracle.gemm_unpacked(t, w)
    want_out = oracle.epilogue(want_acc, s_a, s_w)
    B.set_tile(variant)
    try:
        acc, out = gpu_gemm(mask, sign, wsign, s_a, s_w, M, N, K, path=B.PATH_FP4, want_acc=True, want_out=False)
        assert np.array_equal(acc, want_acc)
        _, out = gpu_gemm(mask, sign, wsign, s_a, s_w, M, N, K, path=B.PATH_FP4, want_acc=False, want_out=True)
        assert same_half(out, want_out)
        # from fp16 activations: +-1 / 0 under a unit scale ternarise to themselves
        B.set_tile(variant)
        A16 = t.astype(np.float16)
        dA = dev(A16)
        prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device="cuda:0")
        B.set_path(B.PATH_FP4)
        if B.prepared_format(M, K) == B.PREPARED_FP4:
            fmt = B.bwta_prepare_act(dA, None, prep, M=M, K=K)
            o2 = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
            B.bwta_gemm_prepared(prep, dev(wsign), dev(s_a), dev(s_w), None, o2, fmt=fmt, M=M, N=N, K=K)
            torch.cuda.synchronize()
            assert same_half(o2.cpu().numpy(), want_out)
    finally:
        B.set_path(B.PATH_AUTO)
        B.set_tile(0)


def test_lds_staged_seeded_random_shapes():
    """30 seeded random problems on the LDS-staged tiled kernel (every tile variant in turn, forced
    through the tuning hook): ragged token and channel counts, any K from two slabs up, planted
    ties / infinities / NaN, from fp16 through bwta_linear's two-kernel form and from planes,
    int32 and fp16."""
    rng = np.random.default_rng(20261128)
    variants = [243, 223, 323]
    for case in range(30):
        M, N, K = int(rng.integers(129, 900)), int(rng.integers(1, 1300)), int(rng.integers(129, 7000))  # tiled-kernel token counts
        variant = variants[case % 3]
        _say("random lds-staged problem", case, M, N, K, variant)
        A = (synth.gaussian(9500 + case, 1, M * K) * float(rng.uniform(0.01, 30))).astype(np.float16).reshape(M, K)
        s = oracle.act_scale(A)
        flat = A.reshape(-1)
        idx = rng.integers(0, flat.size, 6)
        flat[idx[0]] = np.float16(0.5) * s[idx[0] // K]
        flat[idx[1]] = -(np.float16(0.5) * s[idx[1] // K])
        flat[idx[2]], flat[idx[3]], flat[idx[4]], flat[idx[5]] = np.inf, -np.inf, np.nan, -0.0
        w = synth.binary_pm1(9600 + case, 2, (N, K))
        s_w = synth.scales(9700 + case, 3, N)
        t, acc_want, want = oracle.linear(A, s, w, s_w)
        wsign = gpu_pack_weights(w)
        mask, sign, _ = oracle.pack_act(t)
        B.set_tile(variant)
        try:
            acc, out = gpu_gemm(mask, sign, wsign, s, s_w, M, N, K, path=B.PATH_FP4)
            assert np.array_equal(acc, acc_want) and same_half(out, want), (case, M, N, K, variant)
            B.set_tile(variant)
            if K > 1024:  # longer than the one-launch linear takes: ternarise to fragments, then this kernel
                assert same_half(gpu_linear(A, s, wsign, s_w, N, path=B.PATH_FP4), want), (case, M, N, K, variant)
        finally:
            B.set_tile(0)
