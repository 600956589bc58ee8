"""Helpers shared by the GPU parity tests: move numpy inputs to the device, run the HIP path
through the C ABI binding, bring results back as numpy."""
import numpy as np
import torch

from paper_2604_03957_amd import binding as B

DEV = "cuda:0"


def dev(a):
    """numpy -> device tensor (uint32 planes travel as int32 bit patterns)."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def workspace(M, N, K):
    n = max(B.workspace_bytes(M, N, K), 256)
    return torch.empty(n, dtype=torch.uint8, device=DEV)


def gpu_quantize_pack(A, s_a, dtype=None, lda=None, want_nnz=True, K=None):
    """A: numpy fp16/int8 [M, lda]; returns (mask, sign, nnz) as numpy."""
    M = A.shape[0]
    K = A.shape[1] if K is None else K
    dtype = (B.DTYPE_FP16 if A.dtype == np.float16 else B.DTYPE_INT8) if dtype is None else dtype
    rw = B.plane_row_words(K)
    dA, ds = dev(A), dev(s_a)
    mask = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
    sign = torch.full((M, rw), -1, dtype=torch.int32, device=DEV)
    nnz = torch.full((M,), -7, dtype=torch.int32, device=DEV) if want_nnz else None
    B.bwta_quantize_pack_act(dA, ds, mask, sign, nnz, M=M, K=K, lda=A.shape[1] if lda is None else lda,
                             a_dtype=dtype)
    torch.cuda.synchronize()
    return host_u32(mask), host_u32(sign), (nnz.cpu().numpy() if want_nnz else None)


def gpu_pack_weights(W, K=None):
    N = W.shape[0]
    K = W.shape[1] if K is None else K
    dtype = B.DTYPE_FP16 if W.dtype == np.float16 else B.DTYPE_INT8
    ws = torch.full((N, B.plane_row_words(K)), -1, dtype=torch.int32, device=DEV)
    B.bwta_pack_weights(dev(W), ws, N=N, K=K, ldw=W.shape[1], w_dtype=dtype)
    torch.cuda.synchronize()
    return ws


def gpu_gemm(mask, sign, wsign, s_a, s_w, M, N, K, path=B.PATH_AUTO, want_acc=True, want_out=True):
    """Planes may be numpy or device tensors.  Returns (acc int32 numpy, out fp16 numpy)."""
    dm = mask if torch.is_tensor(mask) or mask is None else dev(mask)
    dsg = sign if torch.is_tensor(sign) else dev(sign)
    dw = wsign if torch.is_tensor(wsign) else dev(wsign)
    acc = torch.full((M, N), 123456, dtype=torch.int32, device=DEV) if want_acc else None
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV) if want_out else None
    B.set_path(path)
    try:
        B.bwta_gemm(dm, dsg, dw, dev(s_a), dev(s_w), acc, out, workspace(M, N, K), M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    return (acc.cpu().numpy() if want_acc else None), (out.cpu().numpy() if want_out else None)


def gpu_linear(A, s_a, wsign_dev, s_w, N, path=B.PATH_AUTO):
    M, K = A.shape
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    B.set_path(path)
    try:
        B.bwta_linear(dev(A), dev(s_a), wsign_dev, dev(s_w), out, workspace(M, N, K), M=M, N=N, K=K)
        torch.cuda.synchronize()
    finally:
        B.set_path(B.PATH_AUTO)
    return out.cpu().numpy()


def same_half(a, b):
    """Bit-equality of two fp16 arrays, NaNs compared as equal."""
    a16, b16 = a.view(np.uint16), b.view(np.uint16)
    both_nan = np.isnan(a) & np.isnan(b)
    return bool(np.all((a16 == b16) | both_nan))


def max_rel_err(got, want):
    g, w = got.astype(np.float64), want.astype(np.float64)
    fin = np.isfinite(w)
    if not np.array_equal(np.isfinite(g), fin):
        return np.inf
    if not np.array_equal(g[~fin & ~np.isnan(w)], w[~fin & ~np.isnan(w)]):
        return np.inf
    denom = np.maximum(np.abs(w[fin]), 1e-30)
    err = np.abs(g[fin] - w[fin]) / denom
    err[(w[fin] == 0) & (g[fin] == 0)] = 0
    return float(err.max()) if err.size else 0.0
