"""ctypes binding of libsolar.so: same names as the C entry points of
include/solar.h, argument marshalling only.  torch supplies device memory and the
stream; every step of the computation runs in the library's HIP kernels.  There
is no fallback: if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsolar.so")

SOLAR_OK = 0
SOLAR_ERR_NOT_CONVERGED = 5
SOLAR_ERR_SCRATCH_LIMIT = 6
SOLAR_DEBUG_EIG_MAX_ITER = 0
SOLAR_DEBUG_FORCE_GUARDED_PASS = 1
SOLAR_STATIC_SCRATCH_BYTES = 48 * 1024 * 1024
SOLAR_F32 = 0
SOLAR_BF16 = 1
SOLAR_ATTN_SEQ_SOFTMAX = 0
SOLAR_ATTN_EIGEN_SOFTMAX = 1
SOLAR_ATTN_LINEAR = 2

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2603_02561_amd.build` "
        "(hipcc, gfx950). There is no CPU fallback.")

_lib = ctypes.CDLL(LIB_PATH)
_vp, _ci, _cf, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
_lib.solar_status_string.argtypes = [_ci]
_lib.solar_status_string.restype = ctypes.c_char_p
_lib.solar_workspace_bytes.argtypes = [_ci, _ci, _ci, _ci, _ci, _ci]
_lib.solar_workspace_bytes.restype = _sz
_lib.solar_gram.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp, _sz, _vp]
_lib.solar_gram.restype = _ci
_lib.solar_svd_factorize.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _vp, _vp, _vp,
                                     _sz, _vp]
_lib.solar_svd_factorize.restype = _ci
_lib.solar_svd_factorize_static.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _vp, _vp, _vp]
_lib.solar_svd_factorize_static.restype = _ci
_lib.solar_svd_attention.argtypes = [_vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _cf, _ci,
                                     _ci, _vp, _vp, _sz, _vp]
_lib.solar_svd_attention.restype = _ci
_lib.solar_svd_attention_from_x.argtypes = [_vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _cf, _ci, _vp, _vp,
                                            _sz, _vp]
_lib.solar_svd_attention_from_x.restype = _ci
_lib.solar_dense_attention_ref.argtypes = [_vp, _vp, _vp, _ci, _ci, _ci, _ci, _cf, _ci, _vp, _vp,
                                           _sz, _vp]
_lib.solar_dense_attention_ref.restype = _ci
_lib.solar_rsvd_workspace_bytes.argtypes = [_ci, _ci, _ci, _ci]
_lib.solar_rsvd_workspace_bytes.restype = _sz
_lib.solar_svd_factorize_rsvd.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _ci, _vp, _vp, _vp,
                                          _vp, _vp, _sz, _vp]
_lib.solar_svd_factorize_rsvd.restype = _ci
_lib.solar_linear_attention.argtypes = [_vp, _vp, _vp, _ci, _ci, _ci, _ci, _cf, _ci, _vp, _vp, _sz, _vp]
_lib.solar_linear_attention.restype = _ci
_lib.solar_apply_weights.argtypes = [_vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp]
_lib.solar_apply_weights.restype = _ci
_lib.solar_svd_backward.argtypes = [_vp, _vp, _vp, _vp, _vp, _ci, _ci, _ci, _ci, _cf, _vp, _vp, _sz, _vp]
_lib.solar_svd_backward.restype = _ci
_lib.solar_info_status.argtypes = [_vp, _ci]
_lib.solar_info_status.restype = _ci
_lib.solar_debug_option.argtypes = [_ci, _ci]
_lib.solar_debug_option.restype = _ci
_lib.solar_phase_timing_begin.argtypes = []
_lib.solar_phase_timing_begin.restype = None
_lib.solar_phase_timing_end.argtypes = [ctypes.POINTER(ctypes.c_float)]
_lib.solar_phase_timing_end.restype = _ci


class SolarError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"solar status {code}: {solar_status_string(code)}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SOLAR_F32
    if t.dtype == torch.bfloat16:
        return SOLAR_BF16
    raise TypeError(f"X and Q must be float32 or bfloat16, got {t.dtype}")


def _check(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous CUDA tensors")


def solar_status_string(code: int) -> str:
    return _lib.solar_status_string(int(code)).decode()


def solar_workspace_bytes(B: int, N: int, d: int, r: int, M: int, dtype_code: int) -> int:
    return int(_lib.solar_workspace_bytes(B, N, d, r, M, dtype_code))


def solar_info_status(info) -> int:
    """Status over a factorization's per-user info (waits for the device and copies it to the host)."""
    host = info.detach().to("cpu", torch.int32).contiguous()
    return int(_lib.solar_info_status(ctypes.c_void_p(host.data_ptr()), host.numel()))


def solar_debug_option(key: int, value: int) -> int:
    return int(_lib.solar_debug_option(int(key), int(value)))


def solar_phase_timing_begin() -> None:
    _lib.solar_phase_timing_begin()


def solar_phase_timing_end():
    """Returns (calls, [gram_ms, eig_ms, project_ms]) summed over the timed calls."""
    buf = (ctypes.c_float * 3)()
    n = _lib.solar_phase_timing_end(buf)
    return int(n), [float(buf[i]) for i in range(3)]


def solar_gram(X, lengths, G, workspace, raise_on_error: bool = True) -> int:
    _check(X, lengths, G, workspace)
    B, N, d = X.shape
    rc = _lib.solar_gram(_ptr(X), _ptr(lengths), B, N, d, _dtype_code(X), _ptr(G), _ptr(workspace),
                         workspace.numel() * workspace.element_size(), _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_svd_factorize(X, lengths, r: int, S, V, P, info, workspace,
                        raise_on_error: bool = True) -> int:
    _check(X, lengths, S, V, P, info, workspace)
    B, N, d = X.shape
    rc = _lib.solar_svd_factorize(_ptr(X), _ptr(lengths), B, N, d, int(r), _dtype_code(X), _ptr(S),
                                  _ptr(V), _ptr(P), _ptr(info), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_svd_factorize_static(X, lengths, r: int, S, V, P, info, raise_on_error: bool = True) -> int:
    """solar_svd_factorize with the library's built-in scratch array instead of a workspace."""
    _check(X, lengths, S, V, P, info)
    B, N, d = X.shape
    rc = _lib.solar_svd_factorize_static(_ptr(X), _ptr(lengths), B, N, d, int(r), _dtype_code(X), _ptr(S),
                                         _ptr(V), _ptr(P), _ptr(info), _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_rsvd_workspace_bytes(B: int, N: int, d: int, r: int) -> int:
    return int(_lib.solar_rsvd_workspace_bytes(B, N, d, r))


def solar_svd_factorize_rsvd(X, lengths, r: int, Omega, n_iter: int, S, V, P, info, workspace,
                             raise_on_error: bool = True) -> int:
    _check(X, lengths, Omega, S, V, P, info, workspace)
    B, N, d = X.shape
    rc = _lib.solar_svd_factorize_rsvd(_ptr(X), _ptr(lengths), B, N, d, int(r), _dtype_code(X),
                                       _ptr(Omega), int(n_iter), _ptr(S), _ptr(V), _ptr(P), _ptr(info),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_svd_attention(Q, S, V, P, lengths, N: int, scale: float, mode: int, O, workspace=None,
                        raise_on_error: bool = True) -> int:
    _check(Q, S, V, P, lengths, O, workspace)
    B, M, d = Q.shape
    r = V.shape[2]
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = _lib.solar_svd_attention(_ptr(Q), _ptr(S), _ptr(V), _ptr(P), _ptr(lengths), B, int(N), d,
                                  r, M, float(scale), int(mode), _dtype_code(Q), _ptr(O),
                                  _ptr(workspace), wsb, _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_svd_attention_from_x(Q, X, S, V, lengths, scale: float, O, raise_on_error: bool = True) -> int:
    _check(Q, X, S, V, lengths, O)
    B, M, d = Q.shape
    N = X.shape[1]
    r = V.shape[2]
    rc = _lib.solar_svd_attention_from_x(_ptr(Q), _ptr(X), _ptr(S), _ptr(V), _ptr(lengths), B, N, d, r, M,
                                         float(scale), _dtype_code(Q), _ptr(O), None, 0, _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_dense_attention_ref(Q, X, lengths, scale: float, O, workspace=None,
                              raise_on_error: bool = True) -> int:
    _check(Q, X, lengths, O, workspace)
    B, M, d = Q.shape
    N = X.shape[1]
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = _lib.solar_dense_attention_ref(_ptr(Q), _ptr(X), _ptr(lengths), B, N, d, M, float(scale),
                                        _dtype_code(Q), _ptr(O), _ptr(workspace), wsb, _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_svd_backward(S, V, P, S_bar, V_bar, gap_rel: float, dX, workspace,
                       raise_on_error: bool = True) -> int:
    _check(S, V, P, S_bar, V_bar, dX, workspace)
    B, N, r = P.shape
    d = V.shape[1]
    rc = _lib.solar_svd_backward(_ptr(S), _ptr(V), _ptr(P), _ptr(S_bar), _ptr(V_bar), B, N, d, r,
                                 float(gap_rel), _ptr(dX), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_linear_attention(Q, X, lengths, scale: float, O, workspace, raise_on_error: bool = True) -> int:
    _check(Q, X, lengths, O, workspace)
    B, M, d = Q.shape
    N = X.shape[1]
    rc = _lib.solar_linear_attention(_ptr(Q), _ptr(X), _ptr(lengths), B, N, d, M, float(scale),
                                     _dtype_code(Q), _ptr(O), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


def solar_apply_weights(In, W, Out, raise_on_error: bool = True) -> int:
    _check(In, W, Out)
    d = In.shape[-1]
    rows = In.numel() // d
    rc = _lib.solar_apply_weights(_ptr(In), _ptr(W), rows, d, _dtype_code(In), _dtype_code(Out), _ptr(Out),
                                  _stream())
    if rc != SOLAR_OK and raise_on_error:
        raise SolarError(rc)
    return rc


# ---------------------------------------------------------------------------------------
# Convenience for tests and the benchmark: device buffers for one workload.

class DeviceBatch:
    """Device-resident inputs, outputs and workspace of one batch (allocation only)."""

    def __init__(self, X_host, Q_host, lengths_host, r: int, bf16: bool, device="cuda:0"):
        dev = torch.device(device)
        X = torch.from_numpy(X_host)
        Q = torch.from_numpy(Q_host)
        if bf16:
            # the host values are already bf16-representable, so this conversion is exact
            X = X.to(torch.bfloat16)
            Q = Q.to(torch.bfloat16)
        self.X = X.to(dev).contiguous()
        self.Q = Q.to(dev).contiguous()
        self.lengths = None if lengths_host is None else torch.from_numpy(lengths_host).to(dev)
        B, N, d = X_host.shape
        M = Q_host.shape[1]
        self.B, self.N, self.d, self.r, self.M = B, N, d, r, M
        self.S = torch.empty((B, r), dtype=torch.float32, device=dev)
        self.V = torch.empty((B, d, r), dtype=torch.float32, device=dev)
        self.P = torch.empty((B, N, r), dtype=torch.float32, device=dev)
        self.O = torch.empty((B, M, d), dtype=torch.float32, device=dev)
        self.info = torch.zeros((B,), dtype=torch.int32, device=dev)
        nbytes = solar_workspace_bytes(B, N, d, r, M, SOLAR_BF16 if bf16 else SOLAR_F32)
        self.workspace = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=dev)

    def factorize(self):
        return solar_svd_factorize(self.X, self.lengths, self.r, self.S, self.V, self.P, self.info,
                                   self.workspace)

    def factorize_rsvd(self, Omega, n_iter: int):
        """Algorithm 1 as printed (passes over X); Omega is a [B,d,r] float device tensor."""
        if getattr(self, "rsvd_workspace", None) is None:
            nbytes = solar_rsvd_workspace_bytes(self.B, self.N, self.d, self.r)
            self.rsvd_workspace = torch.empty((max(nbytes, 256),), dtype=torch.uint8,
                                              device=self.X.device)
        return solar_svd_factorize_rsvd(self.X, self.lengths, self.r, Omega, n_iter, self.S, self.V,
                                        self.P, self.info, self.rsvd_workspace)

    def attention(self, scale: float, mode: int = SOLAR_ATTN_SEQ_SOFTMAX, O=None):
        return solar_svd_attention(self.Q, self.S, self.V, self.P, self.lengths, self.N, scale,
                                   mode, self.O if O is None else O, self.workspace)

    def backward(self, S_bar, V_bar, gap_rel: float = 0.0, dX=None):
        """Gradient through the factorization held in S, V, P; S_bar [B,r] and V_bar [B,d,r] are
        float device tensors.  Returns dX [B,N,d] float."""
        if dX is None:
            dX = torch.empty((self.B, self.N, self.d), dtype=torch.float32, device=self.X.device)
        solar_svd_backward(self.S, self.V, self.P, S_bar, V_bar, gap_rel, dX, self.workspace)
        return dX

    def attention_from_x(self, scale: float, O=None):
        """Mode 0 with P = X V formed inside the attention kernel (bf16 inputs, r a multiple of 4)."""
        return solar_svd_attention_from_x(self.Q, self.X, self.S, self.V, self.lengths, scale,
                                          self.O if O is None else O)

    def factorize_no_p(self):
        return solar_svd_factorize(self.X, self.lengths, self.r, self.S, self.V, None, self.info,
                                   self.workspace)

    def linear(self, scale: float, O=None):
        return solar_linear_attention(self.Q, self.X, self.lengths, scale, self.O if O is None else O,
                                      self.workspace)

    def dense(self, scale: float, O=None):
        return solar_dense_attention_ref(self.Q, self.X, self.lengths, scale,
                                         self.O if O is None else O, self.workspace)
