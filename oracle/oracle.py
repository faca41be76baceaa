"""ctypes front end of the CPU oracle -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It loads `libsolar_oracle.so`, built from `solar_oracle.c` with plain gcc,
and converts numpy arrays to the double-precision host buffers the C code expects.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "solar_oracle.c")
_LIB = os.path.join(_HERE, "libsolar_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no BLAS, no threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        _lib.solar_oracle_gram.argtypes = [dp, ip, ci, ci, ci, dp]
        _lib.solar_oracle_svd_factorize.argtypes = [dp, ip, ci, ci, ci, ci, dp, dp, dp, dp, ip]
        _lib.solar_oracle_svd_attention.argtypes = [dp, dp, ip, dp, dp, ci, ci, ci, ci, ci,
                                                    ctypes.c_double, ci, dp]
        _lib.solar_oracle_dense_attention.argtypes = [dp, dp, ip, ci, ci, ci, ci,
                                                      ctypes.c_double, dp]
        for f in (_lib.solar_oracle_gram, _lib.solar_oracle_svd_factorize,
                  _lib.solar_oracle_svd_attention, _lib.solar_oracle_dense_attention):
            f.restype = ci
    return _lib


def _d(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _len(lengths) -> Optional[np.ndarray]:
    return None if lengths is None else np.ascontiguousarray(lengths, dtype=np.int32)


def gram(X, lengths=None) -> np.ndarray:
    X = _f64(X)
    B, N, d = X.shape
    L = _len(lengths)
    G = np.empty((B, d, d), dtype=np.float64)
    rc = _load().solar_oracle_gram(_d(X), _i(L), B, N, d, _d(G))
    if rc != 0:
        raise RuntimeError(f"solar_oracle_gram failed: {rc}")
    return G


def svd_factorize(X, r: int, lengths=None, want_u: bool = False, want_full: bool = False):
    """Returns dict(S [B,r], V [B,d,r], U [B,N,r] or None, S_full [B,d] or None, info [B])."""
    X = _f64(X)
    B, N, d = X.shape
    L = _len(lengths)
    S = np.empty((B, r), dtype=np.float64)
    V = np.empty((B, d, r), dtype=np.float64)
    U = np.zeros((B, N, r), dtype=np.float64) if want_u else None
    SF = np.zeros((B, d), dtype=np.float64) if want_full else None
    info = np.zeros((B,), dtype=np.int32)
    rc = _load().solar_oracle_svd_factorize(_d(X), _i(L), B, N, d, r, _d(S), _d(V), _d(U),
                                            _d(SF), _i(info))
    if rc < 0:
        raise RuntimeError(f"solar_oracle_svd_factorize failed: {rc}")
    return dict(S=S, V=V, U=U, S_full=SF, info=info, status=rc)


def svd_attention(Q, X, S, V, scale: float, mode: int, lengths=None) -> np.ndarray:
    Q = _f64(Q)
    S = _f64(S)
    V = _f64(V)
    B, M, d = Q.shape
    r = S.shape[1]
    if X is not None:
        X = _f64(X)
        N = X.shape[1]
    else:
        N = 1
    L = _len(lengths)
    O = np.empty((B, M, d), dtype=np.float64)
    rc = _load().solar_oracle_svd_attention(_d(Q), _d(X), _i(L), _d(S), _d(V), B, N, d, r, M,
                                            float(scale), int(mode), _d(O))
    if rc != 0:
        raise RuntimeError(f"solar_oracle_svd_attention failed: {rc}")
    return O


def dense_attention(Q, X, scale: float, lengths=None) -> np.ndarray:
    Q = _f64(Q)
    X = _f64(X)
    B, M, d = Q.shape
    N = X.shape[1]
    L = _len(lengths)
    O = np.empty((B, M, d), dtype=np.float64)
    rc = _load().solar_oracle_dense_attention(_d(Q), _d(X), _i(L), B, N, d, M, float(scale), _d(O))
    if rc != 0:
        raise RuntimeError(f"solar_oracle_dense_attention failed: {rc}")
    return O


def rsvd_alg1(X, Omega, n_iter: int, lengths=None):
    """Algorithm 1 ("Randomized SVD with Power Iteration") as printed, in double precision.

    Per user: Omega (d x r, passed in: the Gaussian draw is an input so that the GPU path can
    use the same one), n_iter times Omega <- H^T (H Omega) with no re-orthonormalisation,
    Q = orthonormal basis of H Omega by a Householder QR (library routine), the SVD of the small
    matrix Q^T H (the oracle's own Jacobi SVD), s = its singular values, R = its right
    singular vectors (sign rule of the oracle: largest-magnitude entry positive).
    Returns dict(S [B,r], V [B,d,r]).
    """
    X = _f64(X)
    Omega = _f64(Omega)
    B, N, d = X.shape
    r = Omega.shape[2]
    L = _len(lengths)
    S = np.empty((B, r), dtype=np.float64)
    V = np.empty((B, d, r), dtype=np.float64)
    for b in range(B):
        n = N if L is None else int(L[b])
        H = X[b, :n]
        Om = Omega[b].copy()
        for _ in range(n_iter):
            Om = H.T @ (H @ Om)
        Qm, _ = np.linalg.qr(H @ Om, mode="reduced")
        Bm = Qm.T @ H                               # r x d
        f = svd_factorize(Bm[None], r)              # singular values and right vectors of Q^T H
        S[b] = f["S"][0]
        V[b] = f["V"][0]
    return dict(S=S, V=V)


def linear_attention(Q, X, scale: float, lengths=None) -> np.ndarray:
    """Attn_lin = Query (Key^T Value) of the Preliminaries with Key = Value = X (W = I):
    O_b = scale * Q_b (X_b^T X_b) over the valid rows, evaluated in that order."""
    Q = _f64(Q)
    X = _f64(X)
    L = _len(lengths)
    B, N, _ = X.shape
    O = np.empty_like(Q)
    for b in range(B):
        n = N if L is None else int(L[b])
        H = X[b, :n]
        O[b] = scale * (Q[b] @ (H.T @ H))
    return O


def apply_weights(In, W) -> np.ndarray:
    """Rows times a shared d x d matrix: the projections Query = C W_Q etc. of the Preliminaries."""
    return _f64(In) @ _f64(W)


def svd_backward(X, r: int, S_bar, V_bar, lengths=None, gap_rel: float = 0.0) -> np.ndarray:
    """Gradient of a loss through the truncated SVD with respect to X ("Backward Pass Through
    SVD", the form with U-bar = 0): dL/dX = U [diag(S_bar) + 2 S sym(F o (V^T V_bar))] V^T with
    sym(A) = (A + A^T)/2 and F_ij = 1/(s_j^2 - s_i^2) off the diagonal, 0 on it -- the orientation
    of F that central finite differences confirm (the printed F_ij = 1/(s_i^2 - s_j^2) is its
    transpose).  Pairs with |s_i^2 - s_j^2| <= gap_rel * s_1^2 get F_ij = 0.  U, S, V come from the
    oracle's own Jacobi SVD.  Rows past the valid length get zero gradient."""
    X = _f64(X)
    S_bar = _f64(S_bar)
    V_bar = _f64(V_bar)
    B, N, d = X.shape
    L = _len(lengths)
    f = svd_factorize(X, r, lengths, want_u=True)
    dX = np.zeros_like(X)
    for b in range(B):
        n = N if L is None else int(L[b])
        U, S, V = f["U"][b, :n], f["S"][b], f["V"][b]
        A = V.T @ V_bar[b]
        s2 = S * S
        diff = s2[None, :] - s2[:, None]                 # [i, j] = s_j^2 - s_i^2
        F = np.zeros((r, r))
        ok = np.abs(diff) > gap_rel * s2[0]
        np.fill_diagonal(ok, False)
        F[ok] = 1.0 / diff[ok]
        Bm = F * A
        K = np.diag(S_bar[b]) + 2.0 * np.diag(S) @ (0.5 * (Bm + Bm.T))
        dX[b, :n] = U @ K @ V.T
    return dX
