"""fp64 reference results, one operator at a time -- TEST INFRASTRUCTURE ONLY.

What a superkernel must produce for each packed operator is the plain result
of that operator (Sections 1 and 5.3; Figure 6 caption: the GEMM that backs a
convolution).  `gemm` / `conv2d_nhwc` / `conv2d_nchw` call the plain C loops in sk_oracle.c;
`gemm_py` / `conv2d_nhwc_py` / `conv2d_nchw_py` are the same definitions as pure-Python loops for
tiny cases; `gemm_at` / `conv2d_at` evaluate single output elements so that
full-size runs can be checked on a sample.

Conventions (the paper fixes none of them; these are this build's reading):
  * GEMM  C[m,n] = sum_k A[m,k] * B[n,k]; the weight operand is stored
    K-contiguous as [N,K]; alpha = 1, beta = 0.
  * Convolution is cross-correlation over NHWC activations and [Cout,R,S,Cin]
    filters, one stride for both directions, dilation 1, one group, zero padding, no bias.
  * The GEMM that backs a convolution has rows m = (b*Ho + ho)*Wo + wo,
    columns n = co and reduction index k = (r*S + s)*Cin + c.
  * The channel-major form (X [Nb,Cin,H,W], W [Cout,Cin,R,S], Y [Nb,Cout,Ho,Wo]) is the same
    operator on the other storage order; its reduction index is k = (c*R + r)*S + s.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build()
        lib = ctypes.CDLL(path)
        lib.sk_oracle_gemm.restype = None
        lib.sk_oracle_gemm.argtypes = [ctypes.c_int] * 3 + [
            ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p, ctypes.c_long,
            ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p]
        lib.sk_oracle_conv2d_nhwc.restype = None
        lib.sk_oracle_conv2d_nhwc.argtypes = [ctypes.c_int] * 10 + [ctypes.c_void_p] * 4
        lib.sk_oracle_conv2d_nchw.restype = None
        lib.sk_oracle_conv2d_nchw.argtypes = [ctypes.c_int] * 10 + [ctypes.c_void_p] * 4
        _lib = lib
    return _lib


def set_threads(n: int) -> None:
    """Number of host threads the C loops may use (OpenMP over output rows)."""
    os.environ["OMP_NUM_THREADS"] = str(int(n))
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(int(n))
    except OSError:
        pass


def _f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def gemm(A, B, want_mag: bool = False):
    """A [M,K], B [N,K] (values already rounded to the storage type) -> C fp64 [M,N]."""
    A = _f32(A)
    B = _f32(B)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_mag else None
    _load().sk_oracle_gemm(M, N, K, A.ctypes.data, K, B.ctypes.data, K, C.ctypes.data, N,
                           S.ctypes.data if want_mag else None)
    return (C, S) if want_mag else C


def conv2d_nhwc(X, W, pad_h: int, pad_w: int, want_mag: bool = False, stride: int = 1):
    """X [Nb,H,W,Cin], W [Cout,R,S,Cin] -> Y fp64 [Nb,Ho,Wo,Cout]; filter positions `stride` apart."""
    X = _f32(X)
    W = _f32(W)
    Nb, H, Wd, Cin = X.shape
    Cout, R, S, Cin2 = W.shape
    assert Cin == Cin2
    assert stride >= 1 and H + 2 * pad_h >= R and Wd + 2 * pad_w >= S
    Ho = (H + 2 * pad_h - R) // stride + 1
    Wo = (Wd + 2 * pad_w - S) // stride + 1
    Y = np.empty((Nb, Ho, Wo, Cout), dtype=np.float64)
    Sm = np.empty_like(Y) if want_mag else None
    _load().sk_oracle_conv2d_nhwc(Nb, H, Wd, Cin, Cout, R, S, pad_h, pad_w, stride,
                                  X.ctypes.data, W.ctypes.data, Y.ctypes.data,
                                  Sm.ctypes.data if want_mag else None)
    return (Y, Sm) if want_mag else Y


def conv2d_nchw(X, W, pad_h: int, pad_w: int, want_mag: bool = False, stride: int = 1):
    """X [Nb,Cin,H,W], W [Cout,Cin,R,S] -> Y fp64 [Nb,Cout,Ho,Wo]."""
    X = _f32(X)
    W = _f32(W)
    Nb, Cin, H, Wd = X.shape
    Cout, Cin2, R, S = W.shape
    assert Cin == Cin2
    assert stride >= 1 and H + 2 * pad_h >= R and Wd + 2 * pad_w >= S
    Ho = (H + 2 * pad_h - R) // stride + 1
    Wo = (Wd + 2 * pad_w - S) // stride + 1
    Y = np.empty((Nb, Cout, Ho, Wo), dtype=np.float64)
    Sm = np.empty_like(Y) if want_mag else None
    _load().sk_oracle_conv2d_nchw(Nb, H, Wd, Cin, Cout, R, S, pad_h, pad_w, stride,
                                  X.ctypes.data, W.ctypes.data, Y.ctypes.data,
                                  Sm.ctypes.data if want_mag else None)
    return (Y, Sm) if want_mag else Y


# ---- the same definitions as pure-Python loops (tiny inputs only) ------------

def gemm_py(A, B):
    M, K = len(A), len(A[0])
    N = len(B)
    C = [[0.0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            s = 0.0
            for k in range(K):
                s += float(A[m][k]) * float(B[n][k])
            C[m][n] = s
    return np.array(C, dtype=np.float64)


def conv2d_nhwc_py(X, W, pad_h, pad_w, stride=1):
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Nb, H, Wd, Cin = X.shape
    Cout, R, S, _ = W.shape
    Ho = (H + 2 * pad_h - R) // stride + 1
    Wo = (Wd + 2 * pad_w - S) // stride + 1
    Y = np.zeros((Nb, Ho, Wo, Cout), dtype=np.float64)
    for b in range(Nb):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    s = 0.0
                    for r in range(R):
                        for t in range(S):
                            h = ho * stride - pad_h + r
                            w = wo * stride - pad_w + t
                            if 0 <= h < H and 0 <= w < Wd:
                                for c in range(Cin):
                                    s += X[b, h, w, c] * W[co, r, t, c]
                    Y[b, ho, wo, co] = s
    return Y


def conv2d_nchw_py(X, W, pad_h, pad_w, stride=1):
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Nb, Cin, H, Wd = X.shape
    Cout, _, R, S = W.shape
    Ho = (H + 2 * pad_h - R) // stride + 1
    Wo = (Wd + 2 * pad_w - S) // stride + 1
    Y = np.zeros((Nb, Cout, Ho, Wo), dtype=np.float64)
    for b in range(Nb):
        for co in range(Cout):
            for ho in range(Ho):
                for wo in range(Wo):
                    s = 0.0
                    for c in range(Cin):
                        for r in range(R):
                            for t in range(S):
                                h = ho * stride - pad_h + r
                                w = wo * stride - pad_w + t
                                if 0 <= h < H and 0 <= w < Wd:
                                    s += X[b, c, h, w] * W[co, c, r, t]
                    Y[b, co, ho, wo] = s
    return Y


# ---- single output elements (sampled checks at full size) -------------------

def gemm_at(A_row, B_row):
    """One output element from row m of A and row n of the [N,K] weight."""
    a = np.asarray(A_row, dtype=np.float64)
    b = np.asarray(B_row, dtype=np.float64)
    s = 0.0
    mag = 0.0
    for k in range(a.shape[0]):
        s += a[k] * b[k]
        mag += abs(a[k]) * abs(b[k])
    return s, mag


def conv2d_at(X, W_co, b, ho, wo, pad_h, pad_w, stride=1):
    """One output element Y[b,ho,wo,co] from the full X and filter W[co] ([R,S,Cin])."""
    X = np.asarray(X)
    W_co = np.asarray(W_co)
    _, H, Wd, Cin = X.shape
    R, S, _ = W_co.shape
    s = 0.0
    mag = 0.0
    for r in range(R):
        h = ho * stride - pad_h + r
        if h < 0 or h >= H:
            continue
        for t in range(S):
            w = wo * stride - pad_w + t
            if w < 0 or w >= Wd:
                continue
            x = X[b, h, w, :].astype(np.float64)
            f = W_co[r, t, :].astype(np.float64)
            for c in range(Cin):
                s += x[c] * f[c]
                mag += abs(x[c]) * abs(f[c])
    return s, mag


def patch_matrix(X, R, S, pad_h, pad_w, stride=1):
    """Explicit patch (im2col) matrix [Nb*Ho*Wo, R*S*Cin] with k = (r*S+s)*Cin + c.

    Only used to pin the direct convolution against patch-matrix x GEMM.
    """
    X = np.asarray(X)
    Nb, H, Wd, Cin = X.shape
    Ho = (H + 2 * pad_h - R) // stride + 1
    Wo = (Wd + 2 * pad_w - S) // stride + 1
    P = np.zeros((Nb * Ho * Wo, R * S * Cin), dtype=X.dtype)
    for b in range(Nb):
        for ho in range(Ho):
            for wo in range(Wo):
                m = (b * Ho + ho) * Wo + wo
                for r in range(R):
                    for t in range(S):
                        h = ho * stride - pad_h + r
                        w = wo * stride - pad_w + t
                        if 0 <= h < H and 0 <= w < Wd:
                            k0 = (r * S + t) * Cin
                            P[m, k0:k0 + Cin] = X[b, h, w, :]
    return P
