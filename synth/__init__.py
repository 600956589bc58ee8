"""Seeded synthetic inputs shaped like the paper's transformer workloads.

This module (outside the product package and outside the oracle) only *draws numbers*: a counter-based generator (SplitMix64 finaliser
over seed, tensor id and element index) turned into uniform, Gaussian, Laplace,
ternary and +-1 tensors.  It holds none of the method's arithmetic (no
ternarisation, packing, product or epilogue) and imports neither the oracle nor
the HIP binding, so both sides of a parity test can be fed from it.

numpy only; every value is a pure function of (seed, tensor_id, index), so any
slice of any tensor can be regenerated anywhere.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def raw_u64(seed, tensor_id, start, count):
    """64 random bits for element indices start .. start+count-1 of one tensor."""
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * _GOLDEN + np.uint64(tensor_id) + np.uint64(0x632BE59BD9B4E019))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(key + (idx + np.uint64(1)) * _GOLDEN)


def _chunks(n):
    for s in range(0, n, _CHUNK):
        yield s, min(_CHUNK, n - s)


def uniform01(seed, tensor_id, n, stream=0):
    """float64 in (0, 1), 53 bits, never exactly 0 or 1."""
    out = np.empty(n, np.float64)
    for s, c in _chunks(n):
        r = raw_u64(seed, tensor_id * 16 + stream, s, c)
        out[s:s + c] = ((r >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    return out


def ternary(seed, tensor_id, shape, p_zero):
    """int8 in {-1, 0, +1}: P(0) = p_zero, the two signs equally likely."""
    n = int(np.prod(shape))
    u = uniform01(seed, tensor_id, n)
    t = np.zeros(n, np.int8)
    half = (1.0 - p_zero) / 2.0
    t[u < half] = -1
    t[u >= 1.0 - half] = 1
    return t.reshape(shape)


def binary_pm1(seed, tensor_id, shape):
    """int8 in {-1, +1}, equally likely."""
    n = int(np.prod(shape))
    out = np.empty(n, np.int8)
    for s, c in _chunks(n):
        r = raw_u64(seed, tensor_id * 16, s, c)
        out[s:s + c] = np.where((r >> np.uint64(63)) == 1, -1, 1).astype(np.int8)
    return out.reshape(shape)


def scales(seed, tensor_id, n, lo=0.5, hi=1.5):
    """fp16 scales ~ U(lo, hi)."""
    return (lo + (hi - lo) * uniform01(seed, tensor_id, n)).astype(np.float16)


def gaussian(seed, tensor_id, n):
    """float64 N(0, 1) by Box-Muller on two independent streams."""
    u1 = uniform01(seed, tensor_id, n, stream=1)
    u2 = uniform01(seed, tensor_id, n, stream=2)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def laplace(seed, tensor_id, n):
    """float64 Laplace(0, 1) by inverse CDF."""
    u = uniform01(seed, tensor_id, n, stream=3) - 0.5
    return -np.sign(u) * np.log1p(-2.0 * np.abs(u))


def gaussian_outlier_activations(seed, tensor_id, M, K, outlier_frac=0.02, outlier_gain=20.0):
    """fp16 [M, K] ~ N(0,1); a fixed random `outlier_frac` of the K channels is scaled
    by `outlier_gain` (the heavy-channel structure of transformer activations)."""
    a = gaussian(seed, tensor_id, M * K).reshape(M, K)
    chan = uniform01(seed, tensor_id, K, stream=4) < outlier_frac
    a[:, chan] *= outlier_gain
    return a.astype(np.float16)


def laplace_activations(seed, tensor_id, M, K):
    return laplace(seed, tensor_id, M * K).reshape(M, K).astype(np.float16)


# ---- the five benchmark configurations -------------------------------------------------

def config1():
    """Tiny GEMM: ternary [64, 768] with P(0)=0.4, +-1 weights [768, 768], seed 0."""
    seed = 0
    return dict(name="c1_tiny", M=64, N=768, K=768,
                t=ternary(seed, 1, (64, 768), 0.4), w=binary_pm1(seed, 2, (768, 768)),
                s_a=scales(seed, 3, 64), s_w=scales(seed, 4, 768))


FFN_SHAPES = {"up": (768, 3072), "down": (3072, 768)}            # K -> N
PREFILL_SHAPES = {"qkvo": (4096, 4096), "upgate": (4096, 11008), "down": (11008, 4096)}
DECODE_SHAPES = {"upgate": (4096, 11008), "down": (11008, 4096)}


def config2(which, M=4096):
    """Encoder FFN: fp16 activations with outlier channels, full path.  The per-token activation
    scale is an input of the layer too (at inference a trained parameter; the synthetic stand-in
    is the value training starts it from), but deriving it from A is the method's arithmetic, so
    it is not computed here: each side's harness derives `s_a` from A with its own
    implementation of that statistic (the oracle's in tests, the library's in the benchmark)."""
    seed = 1
    K, N = FFN_SHAPES[which]
    tid = 10 if which == "up" else 20
    A = gaussian_outlier_activations(seed, tid + 1, M, K)
    return dict(name="c2_ffn_" + which, M=M, N=N, K=K, A=A,
                w=binary_pm1(seed, tid + 2, (N, K)), s_w=scales(seed, tid + 3, N))


def config3(which, M=2048):
    """7B-decoder prefill linears from ternary activations with P(0)=0.5."""
    seed = 2
    K, N = PREFILL_SHAPES[which]
    tid = {"qkvo": 10, "upgate": 20, "down": 30}[which]
    return dict(name="c3_prefill_" + which, M=M, N=N, K=K,
                t=ternary(seed, tid + 1, (M, K), 0.5), w=binary_pm1(seed, tid + 2, (N, K)),
                s_a=scales(seed, tid + 3, M), s_w=scales(seed, tid + 4, N))


def config4(which, M):
    """7B-decoder decode linears, M in {1, 4, 16} tokens."""
    seed = 3
    K, N = DECODE_SHAPES[which]
    tid = (10 if which == "upgate" else 20) + 100 * M
    return dict(name="c4_decode_%s_m%d" % (which, M), M=M, N=N, K=K,
                t=ternary(seed, tid + 1, (M, K), 0.5), w=binary_pm1(seed, tid + 2, (N, K)),
                s_a=scales(seed, tid + 3, M), s_w=scales(seed, tid + 4, N))


BLOCK_LINEARS = [("wq", 4096, 4096), ("wk", 4096, 4096), ("wv", 4096, 4096), ("wo", 4096, 4096),
                 ("wgate", 4096, 11008), ("wup", 4096, 11008), ("wdown", 11008, 4096)]


def config5(seq=2048, hidden=4096, ffn=11008):
    """One decoder block: Laplace hidden states and the seven +-1 weight matrices.  Channel scales
    are U(0.5, 1.5) / sqrt(K), the size mean|W| has in a trained layer of fan-in K, so that the
    block's fp16 intermediates stay in range."""
    seed = 4
    out = dict(name="c5_block", seq=seq, hidden=hidden, ffn=ffn, heads=32,
               x=laplace_activations(seed, 1, seq, hidden))
    dims = {"wq": (hidden, hidden), "wk": (hidden, hidden), "wv": (hidden, hidden),
            "wo": (hidden, hidden), "wgate": (hidden, ffn), "wup": (hidden, ffn),
            "wdown": (ffn, hidden)}
    for i, (nm, _, _) in enumerate(BLOCK_LINEARS):
        K, N = dims[nm]
        out[nm] = binary_pm1(seed, 10 + 2 * i, (N, K))
        out["s_" + nm] = scales(seed, 11 + 2 * i, N, lo=0.5 / np.sqrt(K), hi=1.5 / np.sqrt(K))
    return out
