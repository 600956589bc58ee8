"""Pins for the CPU oracle: each part is checked against something other than itself --
IEEE-754 as numpy implements it, exact rational arithmetic, closed forms, brute
force, algebraic invariants and special cases that reduce to textbook routines.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import inputs
import synth

ALL_HALF = np.arange(65536, dtype=np.uint32).astype(np.uint16)


# ---- fp16 codec -------------------------------------------------------------------------

def test_half_decode_matches_ieee_for_every_pattern():
    want = ALL_HALF.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in ALL_HALF])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_paper_hex_constants():
    """The bitpack constants the kernel section prints (tests/golden/bitpack_constants.txt): two
    binary16 values per 32-bit register; the decoder must read +0.5, -0.5 and a bare sign bit, and
    the ternary rule must put exactly these thresholds (times the scale) on the +1 / -1 side."""
    rows = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bitpack_constants.txt")):
        if line.strip() and not line.startswith("#"):
            name, reg, half, value = line.split()[:4]
            rows[name] = (int(reg, 16), int(half, 16), float(value))
    assert set(rows) == {"sign_mask", "plus_half", "minus_half"}
    for reg, half, value in rows.values():
        assert reg == (half << 16 | half)                       # the same pattern in both halves
        got = oracle.half_to_double(half)
        assert got == value and math.copysign(1, got) == math.copysign(1, value)
    plus, minus = np.array([rows["plus_half"][1]], np.uint16).view(np.float16), np.array([rows["minus_half"][1]], np.uint16).view(np.float16)
    one = np.array([1.0], np.float16)
    assert oracle.ternarize(plus.reshape(1, 1), one)[0, 0] == 1     # a / s = +0.5 -> +1 (the printed ">= 0.5")
    assert oracle.ternarize(minus.reshape(1, 1), one)[0, 0] == 0    # a / s = -0.5 -> 0  (the printed "-0.5 <= a / s")
    below = np.nextafter(minus, np.float16(-np.inf))
    assert oracle.ternarize(below.reshape(1, 1), one)[0, 0] == -1
    w = np.array([[1.0, -1.0, -0.0, 0.0]], np.float16)               # sign bit set -> bit 1, except -0.0 (w >= 0 -> +1)
    assert list(oracle.sign_weights(w)[0]) == [1, -1, 1, 1]


def test_half_encode_round_to_nearest_even():
    rng = np.random.default_rng(5)
    vals = [0.0, -0.0, 1.0, 65504.0, 65519.99, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0000001, 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25,
            float("inf"), float("-inf")]
    # every tie between neighbouring fp16 values, and points just around it
    finite = ALL_HALF[(ALL_HALF & 0x7C00) != 0x7C00].view(np.float16).astype(np.float64)
    pos = np.sort(finite[finite >= 0])
    mid = (pos[:-1] + pos[1:]) / 2
    vals += list(mid[::7]) + list(np.nextafter(mid[::11], 0)) + list(np.nextafter(mid[::13], 1e9))
    vals += list(rng.standard_normal(4000) * 10.0 ** rng.integers(-8, 5, 4000))
    vals = np.array(vals, np.float64)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(v) for v in vals], np.uint16)
    assert np.array_equal(got, want)
    assert oracle.double_to_half(float("nan")) & 0x7C00 == 0x7C00
    # every fp16 value survives a round trip
    back = np.array([oracle.double_to_half(v) for v in finite], np.uint16)
    assert np.array_equal(back.view(np.float16).astype(np.float64), finite)


# ---- ternary / sign / bool definitions ----------------------------------------------------

def test_ternary_ties_follow_the_printed_equation():
    for s in (1.0, 0.5, 1.5, 2.0 ** -14, 3.0):
        assert oracle.ternary_value(0.5 * s, s) == 1          # a/s = 0.5 belongs to the +1 case
        assert oracle.ternary_value(-0.5 * s, s) == 0         # -0.5 <= a/s belongs to the 0 case
        assert oracle.ternary_value(np.nextafter(0.5 * s, 0), s) == 0
        assert oracle.ternary_value(np.nextafter(-0.5 * s, -9), s) == -1
    assert oracle.ternary_value(float("inf"), 1.0) == 1
    assert oracle.ternary_value(float("-inf"), 1.0) == -1
    assert oracle.ternary_value(float("nan"), 1.0) == 0
    assert oracle.ternary_value(-0.0, 1.0) == 0
    for bad in (0.0, -1.0, float("inf"), float("nan")):       # scale must be a finite positive
        assert oracle.ternary_value(3.0, bad) == 0


def test_ternarize_every_half_pattern_against_round_of_clip():
    # The paper regards ternary as round(clip(a/s, -1, 1)); with a power-of-two scale the
    # division is exact, and numpy's rint (half to even) agrees everywhere except the two
    # ties, where the printed case analysis sends +0.5 to +1 (rint: 0).
    a = ALL_HALF.view(np.float16).reshape(1, -1)
    af = a.astype(np.float64)
    for s in (1.0, 0.5, 4.0, 2.0 ** -10, 2.0 ** -14, 2.0 ** -24, 1024.0):
        got = oracle.ternarize(a, np.array([s], np.float16))[0].astype(np.int64)
        with np.errstate(invalid="ignore"):
            q = af[0] / s
            want = np.rint(np.clip(q, -1, 1))
        want = np.where(np.isnan(q), 0, want).astype(np.int64)
        want[q == 0.5] = 1
        assert np.array_equal(got, want), s


def test_ternarize_against_exact_rational_division():
    # Literal a/s with exact rationals, scales that are not powers of two.
    rng = np.random.default_rng(11)
    s_bits = rng.integers(0x0001, 0x7C00, 300).astype(np.uint16)
    for sb in s_bits:
        s = float(np.array([sb], np.uint16).view(np.float16)[0])
        half = np.float16(0.5 * s)
        cand = np.array([half, -half, np.nextafter(half, np.float16(0)), np.nextafter(half, np.float16(np.inf)),
                         np.nextafter(-half, np.float16(-np.inf)), np.float16(s), np.float16(-s)], np.float16)
        cand = np.concatenate([cand, rng.integers(0, 65536, 8).astype(np.uint16).view(np.float16)])
        cand = cand[np.isfinite(cand)]
        got = oracle.ternarize(cand.reshape(1, -1), np.array([sb], np.uint16))[0]
        for a, g in zip(cand, got):
            q = Fraction(float(a)) / Fraction(s)
            want = 1 if q >= Fraction(1, 2) else (0 if q >= Fraction(-1, 2) else -1)
            assert g == want, (float(a), s)


def test_ternarize_scale_modes_and_strides():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((5, 40)).astype(np.float16)
    s = np.array([0.5, 1.0, 1.5, 2.0, 0.25], np.float16)
    per_row = oracle.ternarize(A, s)
    for m in range(5):
        assert np.array_equal(per_row[m], oracle.ternarize(A[m:m + 1], s[m:m + 1])[0])
    assert np.array_equal(oracle.ternarize(A, None), oracle.ternarize(A, np.ones(1, np.float16)))


def test_zero_fraction_closed_forms():
    # scale = 2 E|x| puts the zero band at |x| < E|x|: Gaussian -> erf(sqrt(2/pi)/sqrt(2)),
    # Laplace(0,1) -> 1 - exp(-1).  (The paper quotes ~57 % zeros for Gaussian-like inputs.)
    n = 400000
    g = synth.gaussian(7, 1, n)
    s = np.array([2 * math.sqrt(2 / math.pi)], np.float16)
    z = np.mean(oracle.ternarize(g.astype(np.float16).reshape(1, -1), s) == 0)
    assert abs(z - math.erf(math.sqrt(2 / math.pi) / math.sqrt(2))) < 4e-3
    lp = synth.laplace(7, 2, n)
    z = np.mean(oracle.ternarize(lp.astype(np.float16).reshape(1, -1), np.array([2.0], np.float16)) == 0)
    assert abs(z - (1 - math.exp(-1))) < 4e-3


def test_sign_and_bool_definitions():
    assert oracle.sign_value(0.0) == 1 and oracle.sign_value(-0.0) == 1      # w >= 0 -> +1
    assert oracle.sign_value(-1e-8) == -1 and oracle.sign_value(float("nan")) == -1
    W = np.array([[0.0, -0.0, 1.0, -1.0, 6e-8, -6e-8]], np.float16)
    assert oracle.sign_weights(W).tolist() == [[1, 1, 1, -1, 1, -1]]
    assert oracle.bool_value(0.5, 1.0) == 1 and oracle.bool_value(0.4999, 1.0) == 0
    assert oracle.bool_value(-3.0, 1.0) == 0


# ---- packing ------------------------------------------------------------------------------

def test_pack_hand_example_bit_order_and_polarity():
    # element k -> word k/32, bit k%32, LSB first; negative -> sign bit 1
    t = np.zeros((1, 40), np.int8)
    t[0, [0, 2, 33]] = [1, -1, -1]
    mask, sign, nnz = oracle.pack_act(t)
    assert mask.shape == (1, 4)                       # 40 bits padded to 128
    assert mask[0].tolist() == [0b101, 0b10, 0, 0]
    assert sign[0].tolist() == [0b100, 0b10, 0, 0]
    assert nnz.tolist() == [3]
    w = np.ones((1, 40), np.int8)
    w[0, [1, 39]] = -1
    assert oracle.pack_weights(w)[0].tolist() == [0b10, 1 << 7, 0, 0]


@pytest.mark.parametrize("K", [1, 31, 32, 33, 127, 128, 129, 300])
def test_pack_round_trip_and_plane_invariants(K):
    t = synth.ternary(9, K, (7, K), 0.45)
    w = synth.binary_pm1(9, 1000 + K, (5, K))
    mask, sign, nnz = oracle.pack_act(t)
    ws = oracle.pack_weights(w)
    assert mask.shape[1] == 4 * ((K + 127) // 128) == oracle.row_words(K)
    assert np.array_equal(oracle.unpack_act(mask, sign, K), t)
    assert np.array_equal(oracle.unpack_weights(ws, K), w)
    assert not np.any(sign & ~mask)                                   # sign is a subset of mask
    popc = np.array([[bin(int(x)).count("1") for x in row] for row in mask]).sum(1)
    assert np.array_equal(popc, nnz) and np.array_equal(nnz, np.count_nonzero(t, axis=1))
    bits = np.unpackbits(mask.view(np.uint8), axis=1, bitorder="little")
    assert not bits[:, K:].any()                                      # pad bits are zero
    assert not np.unpackbits(ws.view(np.uint8), axis=1, bitorder="little")[:, K:].any()
    # numpy's own little-endian bit packer is the textbook routine for this layout
    want = np.packbits((t != 0).astype(np.uint8), axis=1, bitorder="little")
    assert np.array_equal(mask.view(np.uint8)[:, :want.shape[1]], want)
    want = np.packbits((w < 0).astype(np.uint8), axis=1, bitorder="little")
    assert np.array_equal(ws.view(np.uint8)[:, :want.shape[1]], want)


# ---- integer product ----------------------------------------------------------------------

def _all_forms(t, w):
    K = t.shape[1]
    mask, sign, _ = oracle.pack_act(t)
    ws = oracle.pack_weights(w)
    return [oracle.gemm_unpacked(t, w)] + [oracle.gemm_packed(f, mask, sign, ws, K) for f in (0, 1, 2)]


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5])
def test_brute_force_every_operand_pair_tiny_k(K):
    t = np.array(list(itertools.product((-1, 0, 1), repeat=K)), np.int8)       # 3^K rows
    w = np.array(list(itertools.product((-1, 1), repeat=K)), np.int8)          # 2^K rows
    want = t.astype(np.int64) @ w.astype(np.int64).T
    for got in _all_forms(t, w):
        assert np.array_equal(got, want)


@pytest.mark.parametrize("K", [1, 31, 32, 33, 127, 128, 129, 768])
def test_four_forms_equal_numpy_matmul(K):
    t = synth.ternary(21, K, (9, K), 0.4)
    w = synth.binary_pm1(21, 500 + K, (11, K))
    want = t.astype(np.int64) @ w.astype(np.int64).T
    for got in _all_forms(t, w):
        assert got.dtype == np.int32 and np.array_equal(got, want)


def test_product_invariants():
    K = 200
    t = synth.ternary(33, 1, (6, K), 0.5)
    w = synth.binary_pm1(33, 2, (8, K))
    acc = oracle.gemm_unpacked(t, w)
    nnz = np.count_nonzero(t, axis=1)
    assert np.array_equal(oracle.gemm_unpacked(-t, w), -acc)
    assert np.array_equal(oracle.gemm_unpacked(t, -w), -acc)
    assert np.all(np.abs(acc) <= nnz[:, None])
    assert np.all((acc - nnz[:, None]) % 2 == 0)
    assert not oracle.gemm_unpacked(np.zeros_like(t), w).any()        # all-zero activation
    ones_t, ones_w = np.ones((2, K), np.int8), np.ones((3, K), np.int8)
    assert np.all(oracle.gemm_unpacked(ones_t, ones_w) == K)
    # sign bits under a zero mask must not matter in any packed form
    mask, sign, _ = oracle.pack_act(t)
    ws = oracle.pack_weights(w)
    dirty = sign | (~mask & np.uint32(0xA5A5A5A5))
    assert np.array_equal(oracle.gemm_packed(0, mask, dirty, ws, K), acc)
    # a masked-out lane contributes nothing whatever the weight is
    t2 = t.copy(); t2[:, 17] = 0
    w2 = w.copy(); w2[:, 17] *= -1
    assert np.array_equal(oracle.gemm_unpacked(t2, w), oracle.gemm_unpacked(t2, w2))


def test_full_mask_reduces_to_xnor_popcount():
    # With no zeros the layer is the classic binary linear: K - 2 popc(x ^ w).
    K = 333
    x = synth.binary_pm1(44, 1, (5, K))
    w = synth.binary_pm1(44, 2, (7, K))
    xs, wsb = oracle.pack_weights(x), oracle.pack_weights(w)
    xor = xs[:, None, :] ^ wsb[None, :, :]
    popc = np.unpackbits(xor.view(np.uint8), axis=2).sum(2).astype(np.int64)
    assert np.array_equal(oracle.gemm_unpacked(x, w), K - 2 * popc)


# ---- epilogue -----------------------------------------------------------------------------

def test_epilogue_unit_scales_are_exact_casts():
    acc = np.arange(-2048, 2049, dtype=np.int32).reshape(1, -1)
    out = oracle.epilogue(acc, None, None)
    assert np.array_equal(out.astype(np.int64), acc)
    assert np.array_equal(out, oracle.epilogue(acc, np.ones(1, np.float16), np.ones(acc.shape[1], np.float16)))


def test_epilogue_against_exact_rational_product():
    rng = np.random.default_rng(8)
    M, N = 12, 40
    acc = rng.integers(-11008, 11009, (M, N)).astype(np.int32)
    acc[0, :4] = [0, 1, -1, 11008]
    s_a = synth.scales(8, 1, M)
    s_w = synth.scales(8, 2, N)
    s_a[1] = np.float16(60000.0)       # overflow to +-Inf
    s_w[3] = np.float16(2.0 ** -24)    # smallest subnormal scale
    got = oracle.epilogue(acc, s_a, s_w)
    with np.errstate(over="ignore"):
        for m in range(M):
            for n in range(N):
                exact = Fraction(int(acc[m, n])) * Fraction(float(s_a[m])) * Fraction(float(s_w[n]))
                as_double = float(exact)
                assert Fraction(as_double) == exact          # the product fits a double exactly
                want = np.float64(as_double).astype(np.float16)
                assert got[m, n].view(np.uint16) == want.view(np.uint16), (m, n)
    assert np.isinf(got[1]).any()


def test_linear_is_the_composition():
    c = inputs.config2("up", M=8)
    t, acc, out = oracle.linear(c["A"], c["s_a"], c["w"], c["s_w"])
    assert np.array_equal(t, oracle.ternarize(c["A"], c["s_a"]))
    assert np.array_equal(acc, t.astype(np.int64) @ c["w"].astype(np.int64).T)
    ref = acc.astype(np.float64) * c["s_a"].astype(np.float64)[:, None] * c["s_w"].astype(np.float64)[None, :]
    assert np.allclose(out.astype(np.float64), ref, rtol=2.0 ** -11, atol=0)


# ---- attention MatMuls (BWTA_QK: ternary x ternary; BWTA_Att: bool x ternary) -----------------

def test_boolize_every_half_pattern_and_ties():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(1, -1)
    A = bits.view(np.float16)
    for s in (1.0, 0.5, 1.5, 2.0 ** -24, 65504.0):
        got = oracle.boolize(A, np.array([s], np.float16))[0]
        a = A[0].astype(np.float64)
        with np.errstate(invalid="ignore"):
            want = np.where(np.isnan(a), 0, (a >= 0.5 * float(np.float16(s))).astype(np.int8))
        assert np.array_equal(got, want), s
    # exactly 0.5 s -> 1 (the >= of the printed rule); just below -> 0; negative scale clears the row
    assert oracle.boolize(np.array([[0.75, 0.7495]], np.float16), np.array([1.5], np.float16)).tolist() == [[1, 0]]
    assert oracle.boolize(np.array([[5.0]], np.float16), np.array([-1.0], np.float16)).tolist() == [[0]]
    # bool(a) agrees with the positive part of ternary(a)
    x = synth.gaussian(5, 9, 4096).astype(np.float16).reshape(4, -1)
    s = np.array([0.7], np.float16)
    assert np.array_equal(oracle.boolize(x, s), (oracle.ternarize(x, s) == 1).astype(np.int8))


def _tt_forms(a, b, a_bool=False):
    K = a.shape[1]
    ma, sa, _ = oracle.pack_act(a)
    mb, sb, _ = oracle.pack_act(b)
    if a_bool:
        assert not sa.any()
        sa = None
    return [oracle.gemm_unpacked(a, b)] + [oracle.matmul_tt_packed(f, ma, sa, mb, sb, K) for f in (0, 1)]


@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_ternary_ternary_brute_force_every_operand_pair(K):
    t = np.array(list(itertools.product((-1, 0, 1), repeat=K)), np.int8)       # 3^K rows on both sides
    want = t.astype(np.int64) @ t.astype(np.int64).T
    for got in _tt_forms(t, t):
        assert np.array_equal(got, want)
    b = np.array(list(itertools.product((0, 1), repeat=K)), np.int8)           # 2^K boolean rows
    want = b.astype(np.int64) @ t.astype(np.int64).T
    for got in _tt_forms(b, t, a_bool=True):
        assert np.array_equal(got, want)


@pytest.mark.parametrize("K", [1, 31, 32, 33, 127, 128, 129, 2048])
def test_attention_products_equal_numpy_matmul(K):
    q = synth.ternary(31, K, (10, K), 0.4)
    k = synth.ternary(31, 700 + K, (13, K), 0.55)
    want = q.astype(np.int64) @ k.astype(np.int64).T
    for got in _tt_forms(q, k):
        assert got.dtype == np.int32 and np.array_equal(got, want)
    att = (synth.ternary(32, K, (10, K), 0.7) != 0).astype(np.int8)            # boolean, ~30 % ones
    want = att.astype(np.int64) @ k.astype(np.int64).T
    for got in _tt_forms(att, k, a_bool=True):
        assert np.array_equal(got, want)


def test_attention_product_invariants():
    K = 200
    q = synth.ternary(33, 1, (7, K), 0.4)
    k = synth.ternary(33, 2, (9, K), 0.4)
    ma, sa, _ = oracle.pack_act(q)
    mb, sb, _ = oracle.pack_act(k)
    base = oracle.matmul_tt_packed(1, ma, sa, mb, sb, K)
    assert np.array_equal(base.T, oracle.matmul_tt_packed(1, mb, sb, ma, sa, K))           # symmetry of the rule
    assert np.array_equal(oracle.gemm_unpacked(-q, k), -base)                               # sign flips
    dirty_a = sa | (~ma & np.uint32(0xA5A5A5A5))                                            # sign bits under a zero mask
    dirty_b = sb | (~mb & np.uint32(0x5A5A5A5A))
    for f in (0, 1):
        assert np.array_equal(oracle.matmul_tt_packed(f, ma, dirty_a, mb, dirty_b, K), base)
    # a binary (+-1) second operand reduces the rule to the BWTA linear product
    w = synth.binary_pm1(33, 3, (9, K))
    mw, sw, _ = oracle.pack_act(w)
    assert np.array_equal(oracle.matmul_tt_packed(1, ma, sa, mw, sw, K), oracle.gemm_packed(0, ma, sa, oracle.pack_weights(w), K))
    # |acc| <= number of positions where both are non-zero, and same parity
    both = (q != 0).astype(np.int64) @ (k != 0).astype(np.int64).T
    assert np.all(np.abs(base) <= both) and np.all((base - both) % 2 == 0)


def test_epilogue_alpha_against_exact_rational_arithmetic():
    rng = np.random.default_rng(9)
    M, N = 6, 30
    acc = rng.integers(-2048, 2049, (M, N)).astype(np.int32)
    s_a, s_b = synth.scales(9, 1, M), synth.scales(9, 2, N)
    alpha = np.float32(1.0 / math.sqrt(128.0))
    got = oracle.epilogue_alpha(acc, s_a, s_b, alpha)
    for m in range(M):
        for n in range(N):
            prod = Fraction(float(alpha)) * Fraction(float(s_a[m])) * Fraction(float(s_b[n]))
            s32 = np.float32(float(prod))            # the exact product (46 bits) fits a double; one rounding to fp32
            assert Fraction(float(prod)) == prod
            exact = Fraction(int(acc[m, n])) * Fraction(float(s32))
            assert Fraction(float(exact)) == exact
            want = np.float64(float(exact)).astype(np.float16)
            assert got[m, n].view(np.uint16) == want.view(np.uint16), (m, n)
    # alpha = 1 reduces to the linear layer's epilogue
    assert np.array_equal(oracle.epilogue_alpha(acc, s_a, s_b, 1.0).view(np.uint16), oracle.epilogue(acc, s_a, s_b).view(np.uint16))


# ---- weight preparation and the activation scale's starting value --------------------------

def _exact_prepare(row):
    vals = [Fraction(float(x)) for x in row]
    mu = sum(vals) / len(vals)
    w = [1 if v - mu >= 0 else -1 for v in vals]
    s = sum(abs(v - mu) for v in vals) / len(vals)
    return w, s


def _half_of_fraction(q):
    """Correctly rounded binary16 of a non-negative rational, by bisection over all finite halfs."""
    halfs = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16)            # ascending
    fr = [Fraction(float(h)) for h in (halfs[0], halfs[-1])]
    lo, hi = 0, len(halfs) - 1
    if q >= fr[1]:
        return halfs[-1]
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if Fraction(float(halfs[mid])) <= q:
            lo = mid
        else:
            hi = mid
    a, b = Fraction(float(halfs[lo])), Fraction(float(halfs[hi]))
    if q - a < b - q or (q - a == b - q and lo % 2 == 0):
        return halfs[lo]
    return halfs[hi]


def test_prepare_weights_against_exact_rational_arithmetic():
    W = (synth.gaussian(41, 1, 6 * 37) * 0.05 + 0.01).astype(np.float16).reshape(6, 37)
    W[0, :3] = [0.25, 0.25, 0.25]
    W[1] = np.float16(0.125)                         # every element equals the mean: all +1, scale 0
    W[2, :4] = [6e-8, -6e-8, 65504.0, -65504.0]      # subnormals and the largest finite values
    w, s = oracle.prepare_weights(W)
    for n in range(W.shape[0]):
        we, se = _exact_prepare(W[n])
        assert w[n].tolist() == we, n
        assert s[n].view(np.uint16) == _half_of_fraction(se).view(np.uint16), n
    assert w[1].tolist() == [1] * 37 and s[1] == 0


def test_prepare_weights_scale_is_the_least_squares_optimum():
    W = (synth.laplace(42, 1, 3 * 64) * 0.02).astype(np.float16).reshape(3, 64)
    w, s = oracle.prepare_weights(W)
    for n in range(3):
        vals = [Fraction(float(x)) for x in W[n]]
        mu = sum(vals) / len(vals)
        c = [v - mu for v in vals]
        err = lambda sc: sum((ci - sc * wi) ** 2 for ci, wi in zip(c, w[n].tolist()))
        s_opt = sum(abs(ci) for ci in c) / len(c)                # d/ds of the error vanishes here
        assert err(s_opt) <= err(s_opt * Fraction(1001, 1000)) and err(s_opt) <= err(s_opt * Fraction(999, 1000))
        assert abs(Fraction(float(s[n])) - s_opt) <= s_opt * Fraction(1, 2048)   # one rounding to binary16
        assert sum(w[n].tolist()) != 64                          # centred weights are not all of one sign


def test_prepare_weights_matches_float64_numpy_and_special_values():
    W = (synth.gaussian(43, 1, 40 * 768) * 0.03 + 0.004).astype(np.float16).reshape(40, 768)
    w, s = oracle.prepare_weights(W)
    W64 = W.astype(np.float64)
    c = W64 - W64.mean(axis=1, keepdims=True)
    assert np.array_equal(w, np.where(c >= 0, 1, -1))            # no element sits within rounding of its row mean
    ref = np.abs(c).mean(axis=1)
    assert np.all(np.abs(s.astype(np.float64) - ref) <= ref * 2.0 ** -11)
    V = np.array([[1.0, np.inf, -np.inf, np.nan, -1.0, 3.0]], np.float16)
    w, s = oracle.prepare_weights(V)                             # finite part: {1, -1, 3}, sum 3 over K = 6 -> mean 0.5
    assert w.tolist() == [[1, 1, -1, -1, -1, 1]]
    assert s[0] == np.float16((0.5 + 1.5 + 2.5) / 6)


def test_act_scale_is_twice_the_mean_absolute_value():
    A16 = synth.config2("up", M=16)["A"]
    got = oracle.act_scale(A16)
    ref = 2.0 * np.mean(np.abs(A16.astype(np.float64)), axis=1)               # float64: 1e-13 relative, then one rounding
    assert np.all(np.abs(got.astype(np.float64) - ref) <= ref * 2.0 ** -11)
    # random rows against exact rational arithmetic, rounded once to binary16 by bisection on the grid
    rows = (synth.laplace(44, 1, 5 * 37) * np.repeat([1e-3, 0.3, 1.0, 40.0, 3000.0], 37)).astype(np.float16).reshape(5, 37)
    want = [_half_of_fraction(2 * sum(abs(Fraction(float(x))) for x in r) / len(r)) for r in rows]
    assert [x.view(np.uint16) for x in oracle.act_scale(rows)] == [x.view(np.uint16) for x in want]
    A = np.array([[1.0, -2.0, 0.5, 0.0], [6e-8, 6e-8, 0.0, 0.0], [65504.0] * 4], np.float16)
    with np.errstate(over="ignore"):
        want = [np.float16(1.75), _half_of_fraction(Fraction(float(np.float16(6e-8))) * 2 * 2 / 4), np.float16(np.inf)]
    assert [x.view(np.uint16) for x in oracle.act_scale(A)] == [x.view(np.uint16) for x in want]
