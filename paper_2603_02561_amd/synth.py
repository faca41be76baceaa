"""Seeded synthetic workloads for SVD-Attention (numpy only, no method arithmetic).

The paper's workloads are production behaviour sequences of roughly ten thousand
items attended by a few thousand candidates, whose embedding matrices are close to
rank ~30 (evaluation-settings table and the low-rank figure of the introduction).
None of that data is public, so every input here is a seeded random matrix with the
same shapes and the same (approximately) low-rank structure.

This module is shared by the tests, the benchmark and the CPU oracle harness.  It
only *builds inputs*: Gaussian draws, products of Gaussian factors, prescribed
singular spectra and bf16 rounding.  Nothing in it computes a factorization of an
input or an attention output.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence

import numpy as np

SEED0 = 20260302

F32 = 0
BF16 = 1


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x_rounded: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x_rounded, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclasses.dataclass
class Workload:
    """One batch of users.  X and Q hold the values both sides consume (float32;
    already rounded to bf16-representable values when dtype == BF16)."""

    name: str
    B: int
    N: int
    d: int
    r: int
    M: int
    dtype: int
    X: np.ndarray          # [B, N, d] float32
    Q: np.ndarray          # [B, M, d] float32
    lengths: np.ndarray    # [B] int32
    sharp_scale: float     # 3 / rms(X): makes the softmax peaked
    recipe: str

    @property
    def X_bits(self) -> np.ndarray:
        return bf16_bits(self.X)

    @property
    def Q_bits(self) -> np.ndarray:
        return bf16_bits(self.Q)


def _orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q


def user_matrix(rng: np.random.Generator, n: int, d: int, r: int, kind: str,
                decay: float = 1.0, noise: float = 0.0) -> np.ndarray:
    """One user's n x d sequence matrix (float64).

    kind == "gauss_lowrank": X = A @ Bm with A (n x r), Bm (r x d) i.i.d. Gaussian
        with standard deviation 1/sqrt(r); X has rank exactly r and entry std
        1/sqrt(r).
    kind == "spectrum": X = U0 diag(sigma) V0^T + E with orthonormal U0, V0,
        sigma_k = c * k**-decay scaled so that the signal has RMS 1/sqrt(r), and
        E i.i.d. N(0, noise) (noise = standard deviation).
    """
    if kind == "gauss_lowrank":
        # Both factors i.i.d. N(0, 1/sqrt(r)) read as standard deviation 1/sqrt(r).
        s = 1.0 / np.sqrt(r)
        a = rng.standard_normal((n, r)) * s
        bm = rng.standard_normal((r, d)) * s
        return a @ bm
    if kind == "spectrum":
        u0 = _orthonormal(rng, n, r)
        v0 = _orthonormal(rng, d, r)
        k = np.arange(1, r + 1, dtype=np.float64)
        sig = k ** (-decay)
        sig *= np.sqrt(n * d / r / np.sum(sig * sig))
        x = (u0 * sig) @ v0.T
        if noise > 0.0:
            x = x + rng.standard_normal((n, d)) * noise
        return x
    raise ValueError(kind)


def make_workload(name: str, B: int, N: int, d: int, r: int, M: int, dtype: int,
                  kind: str, decay: float = 1.0, noise: float = 0.0,
                  var_len: Optional[Sequence[int]] = None, seed: int = SEED0,
                  users: Optional[Sequence[int]] = None) -> Workload:
    """Build a batch.  `users` selects a subset of user indices (their per-user
    seeds are unchanged, so a subset reproduces the same matrices as the full batch).
    var_len = (lo, hi): per-user valid length uniform in [lo, hi]; rows past the
    valid length are filled with finite garbage (not zeros) so that masking is
    exercised."""
    idx = list(range(B)) if users is None else list(users)
    nb = len(idx)
    X = np.empty((nb, N, d), dtype=np.float32)
    Q = np.empty((nb, M, d), dtype=np.float32)
    lengths = np.empty((nb,), dtype=np.int32)
    for o, b in enumerate(idx):
        rng = np.random.default_rng(seed + b)
        if var_len is not None:
            n_b = int(rng.integers(var_len[0], var_len[1] + 1))
        else:
            n_b = N
        lengths[o] = n_b
        X[o, :n_b] = user_matrix(rng, n_b, d, r, kind, decay, noise).astype(np.float32)
        if n_b < N:
            X[o, n_b:] = (rng.standard_normal((N - n_b, d)) * 3.0 + 1.0).astype(np.float32)
        Q[o] = (rng.standard_normal((M, d)) / np.sqrt(d)).astype(np.float32)
    if dtype == BF16:
        X = round_to_bf16(X)
        Q = round_to_bf16(Q)
    ms = 0.0
    cnt = 0
    for o in range(nb):
        v = X[o, : lengths[o]].astype(np.float64)
        ms += float(np.sum(v * v))
        cnt += v.size
    rms = np.sqrt(ms / max(cnt, 1))
    recipe = (f"{kind}, decay={decay}, noise_std={noise}, var_len={var_len}, "
              f"seed={seed}+user, dtype={'bf16' if dtype == BF16 else 'f32'}")
    return Workload(name, nb, N, d, r, M, dtype, X, Q, lengths, float(3.0 / rms), recipe)


# The five workloads the build is measured and tested on.  Index 0 is the small
# case the CPU oracle finishes in seconds; index 2 is the one the headline metric
# is quoted on.
CONFIGS = {
    "C1": dict(B=1, N=1024, d=64, r=8, M=64, dtype=F32, kind="gauss_lowrank"),
    "C2": dict(B=32, N=4096, d=128, r=16, M=512, dtype=F32, kind="gauss_lowrank"),
    "C3": dict(B=64, N=10000, d=128, r=32, M=1000, dtype=BF16, kind="spectrum",
               decay=1.0, noise=0.01),
    "C4": dict(B=16, N=16384, d=256, r=32, M=4096, dtype=BF16, kind="gauss_lowrank"),
    "C5": dict(B=128, N=10000, d=128, r=64, M=2000, dtype=BF16, kind="spectrum",
               decay=0.5, noise=0.05, var_len=(2000, 10000)),
}


def make_config(name: str, users: Optional[Sequence[int]] = None,
                B: Optional[int] = None) -> Workload:
    """Workload `name` in CONFIGS.  `users` picks a subset of its users; `B`
    overrides the batch size (users 0..B-1)."""
    cfg = dict(CONFIGS[name])
    if B is not None:
        cfg["B"] = B
    seed = SEED0 + 1000 * (int(name[1:]))
    return make_workload(name, seed=seed, users=users, **cfg)


def make_omega(B: int, d: int, r: int, seed: int = SEED0 + 77) -> np.ndarray:
    """Standard normal start blocks Omega [B, d, r] (float32) for the randomized SVD of
    Algorithm 1, one independent stream per user."""
    out = np.empty((B, d, r), dtype=np.float32)
    for b in range(B):
        out[b] = np.random.default_rng(seed + b).standard_normal((d, r)).astype(np.float32)
    return out


def make_cotangents(B: int, d: int, r: int, seed: int = SEED0 + 99):
    """Upstream gradients for the backward pass through the factorization: S_bar [B, r] and
    V_bar [B, d, r], float32, standard normal, one independent stream per user."""
    S_bar = np.empty((B, r), dtype=np.float32)
    V_bar = np.empty((B, d, r), dtype=np.float32)
    for b in range(B):
        g = np.random.default_rng(seed + b)
        S_bar[b] = g.standard_normal(r).astype(np.float32)
        V_bar[b] = g.standard_normal((d, r)).astype(np.float32)
    return S_bar, V_bar
