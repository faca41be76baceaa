"""GPU parity at the edges of the contract, against the CPU oracle through the C ABI:

* falling scores -- a row of the first 32-row block scores 12 to 20 log2 units above a tail of
  more than ten thousand rows, so every tail weight of the fp16 attention kernel's first pass
  lies in the subnormal range of its 16-bit weights while the tail as a whole carries a
  visible share of the softmax mass (the mirror image of the rising-scores cases);
* rank(X) < r -- not an error: the trailing singular values are 0 and every mode still
  matches the oracle;
* slowly converging spectra -- a plateau of unwanted singular values just below s_r, which makes
  the eigen-iteration add its filtered power steps;
* the resolution limit of the float Gram route -- prescribed spectra with s_r / s_1 from 1e-1
  down to 1e-3: components above the documented limit come back, with the accuracy the header
  states; components below it come back as S = 0 with a zero column of V (visible to the
  caller), and what remains is still the exact factorization of the resolved part.

Tolerances: 1e-4 (float inputs) and 2e-2 (bf16 inputs), errors relative to the largest oracle
output per user, unless a case states its own bound.
"""
import numpy as np
import pytest

from paper_2603_02561_amd import synth

pytestmark = pytest.mark.gpu

LOG2E = 1.4426950408889634


@pytest.fixture(scope="module")
def lib():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU")
    from paper_2603_02561_amd import binding
    return binding


@pytest.fixture(scope="module")
def oracle():
    from oracle import oracle as o
    return o


def rel_err(got, want):
    return max(np.abs(got[b] - want[b]).max() / np.abs(want[b]).max() for b in range(want.shape[0]))


@pytest.mark.parametrize("N,r,M", [(16384, 32, 96), (12000, 64, 80), (10240, 32, 64), (40000, 32, 48),
                                   (100000, 32, 40)])
def test_scores_falling_from_the_first_block(lib, oracle, N, r, M):
    import torch
    d, B = 128, 2
    print(f"[case] falling scores N={N} d={d} r={r} M={M}", flush=True)
    w = synth.make_workload("t", B, N, d, r, M, synth.BF16, "gauss_lowrank", seed=9100 + r)
    X = w.X.copy()
    X[:, :32, :] *= 8.0                     # a power of two: the values stay bf16
    # tail scores of about one log2 unit of spread: scale * log2(e) * std(q . x) = 1
    sd = float(np.std(np.einsum("bmd,bnd->bmn", w.Q[:, :8].astype(np.float64), X[:, 64:2064].astype(np.float64))))
    scale = 1.0 / (LOG2E * sd)
    f = oracle.svd_factorize(X, r, w.lengths)
    n_in_range = 0
    for b in range(B):
        Xr = (X[b].astype(np.float64) @ f["V"][b]) @ f["V"][b].T
        sc = scale * LOG2E * (w.Q[b].astype(np.float64) @ Xr.T)
        head = sc[:, :32].max(axis=1)
        drop = head[:, None] - sc[:, 32:]
        frac = np.mean((drop > 12.0) & (drop < 20.0), axis=1)          # share of the tail 12..20 below the head
        tail_mass = np.exp2(sc[:, 32:] - head[:, None]).sum(axis=1)    # relative to the head row's weight
        ok = (frac > 0.5) & (tail_mass > 0.02)
        n_in_range += int(ok.sum())
        print(f"  user {b}: candidates with most of the tail 12-20 log2 units below the head and a tail mass "
              f"above 2 %: {int(ok.sum())} of {M} (median tail mass {np.median(tail_mass):.3f})", flush=True)
    assert n_in_range >= M // 2            # precondition on the input, not on the library
    db = lib.DeviceBatch(X, w.Q, w.lengths, r, True)
    db.factorize()
    torch.cuda.synchronize()
    assert np.all(db.info.cpu().numpy() == 0)
    want = oracle.svd_attention(w.Q, X, f["S"], f["V"], scale, 0, w.lengths)
    db.attention(scale, 0)
    torch.cuda.synchronize()
    err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
    db.attention_from_x(scale)
    torch.cuda.synchronize()
    err_fx = rel_err(db.O.cpu().numpy().astype(np.float64), want)
    lib.solar_debug_option(lib.SOLAR_DEBUG_FORCE_GUARDED_PASS, 1)
    try:
        db.attention(scale, 0)
        torch.cuda.synchronize()
    finally:
        lib.solar_debug_option(lib.SOLAR_DEBUG_FORCE_GUARDED_PASS, 0)
    err_g = rel_err(db.O.cpu().numpy().astype(np.float64), want)
    print(f"  err stored-P {err:.3e}  fused projection {err_fx:.3e}  guarded pass {err_g:.3e}", flush=True)
    assert err < 2e-2 and err_fx < 2e-2 and err_g < 2e-2


@pytest.mark.parametrize("dtype,d,r,rank,N,M", [(synth.F32, 64, 8, 5, 600, 50), (synth.F32, 128, 32, 20, 900, 70),
                                                (synth.F32, 256, 16, 9, 500, 40)])
def test_rank_below_r_is_not_an_error(lib, oracle, dtype, d, r, rank, N, M):
    """X of exact rank `rank` < r with well separated singular values (so that mode 1, which
    depends on the individual vectors, is pinned too)."""
    import torch
    B = 2
    print(f"[case] rank {rank} < r = {r}, d={d}", flush=True)
    X = np.empty((B, N, d), dtype=np.float32)
    Q = np.empty((B, M, d), dtype=np.float32)
    for b in range(B):
        g = np.random.default_rng(5150 + 17 * b + d)
        U0, _ = np.linalg.qr(g.standard_normal((N, rank)))
        V0, _ = np.linalg.qr(g.standard_normal((d, rank)))
        sig = 40.0 * 0.8 ** np.arange(rank)
        X[b] = ((U0 * sig) @ V0.T).astype(np.float32)
        Q[b] = (g.standard_normal((M, d)) / np.sqrt(d)).astype(np.float32)
    f = oracle.svd_factorize(X, r)
    assert np.all(f["S"][:, rank:] < 1e-5 * f["S"][:, :1])          # the oracle sees the rank as well
    db = lib.DeviceBatch(X, Q, None, r, False)
    db.factorize()
    torch.cuda.synchronize()
    assert np.all(db.info.cpu().numpy() == 0)
    S = db.S.cpu().numpy().astype(np.float64)
    V = db.V.cpu().numpy().astype(np.float64)
    assert np.all(S[:, rank:] == 0.0) and np.all(V[:, :, rank:] == 0.0)
    for b in range(B):
        assert np.abs(S[b, :rank] - f["S"][b, :rank]).max() < 1e-4 * f["S"][b, 0]
        pg = V[b, :, :rank] @ V[b, :, :rank].T
        po = f["V"][b, :, :rank] @ f["V"][b, :, :rank].T
        assert np.abs(pg - po).max() < 1e-4
    rms = float(np.sqrt(np.mean(X.astype(np.float64) ** 2)))
    for mode, scale in ((0, 1.0), (0, 3.0 / rms), (2, 1.0), (1, 0.02)):
        want = oracle.svd_attention(Q, X, f["S"], f["V"], scale, mode)
        db.attention(scale, mode)
        torch.cuda.synchronize()
        err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
        print(f"  mode {mode} scale {scale:.3g}: {err:.3e}", flush=True)
        assert err < 1e-4
    # exact rank <= r: mode 0 is dense softmax attention
    dense = oracle.dense_attention(Q, X, 3.0 / rms)
    db.attention(3.0 / rms, 0)
    torch.cuda.synchronize()
    assert rel_err(db.O.cpu().numpy().astype(np.float64), dense) < 1e-4


def _prescribed(N, d, sig, seed):
    g = np.random.default_rng(seed)
    U0, _ = np.linalg.qr(g.standard_normal((N, len(sig))))
    V0, _ = np.linalg.qr(g.standard_normal((d, len(sig))))
    return ((U0 * sig) @ V0.T).astype(np.float32), V0


# s_r / s_1, and what the header promises there: (components returned, bound on |S - S_oracle| / s_1,
# bound on the projector of the returned columns, bound on mode 0 relative to the oracle)
# (measured: S 1e-7 throughout; projector 3e-7, 2e-6, 2e-5, 7e-5 at 1e-1, 3e-2, 1e-2, 5e-3; mode 0 <= 4e-6)
RESOLUTION = [
    (1e-1, 8, 2e-6, 5e-6, 1e-4),
    (3e-2, 8, 2e-6, 3e-5, 1e-4),
    (1e-2, 8, 2e-6, 2e-4, 1e-4),
    (5e-3, 8, 2e-6, 1e-3, 1e-4),
    (4e-3, 8, 2e-6, 2e-3, 1e-4),
    (2e-3, 7, 2e-6, 5e-6, None),
    (1e-3, 7, 2e-6, 5e-6, None),
]


@pytest.mark.parametrize("ratio,kept,s_tol,p_tol,o_tol", RESOLUTION, ids=[f"{c[0]:g}" for c in RESOLUTION])
def test_resolution_of_small_components(lib, oracle, ratio, kept, s_tol, p_tol, o_tol):
    """Float inputs of exact rank r = 8 whose first seven singular values fall geometrically from
    1 to 0.2 and whose last one is ratio * s_1: on the resolved side of the documented limit
    (3.2e-3 of s_1) all eight come back, the direction of the smallest with an accuracy that
    degrades as 2^-24 / ratio^2 while S and the attention output stay inside the 1e-4 contract;
    below the limit the eighth component comes back as S = 0 with a zero column of V, and the
    seven resolved ones stay accurate."""
    import torch
    N, d, r, M, B = 1500, 64, 8, 60, 2
    print(f"[case] resolution s_r/s_1 = {ratio:g}", flush=True)
    sig = np.concatenate([30.0 * np.geomspace(1.0, 0.2, r - 1), [30.0 * ratio]])
    X = np.stack([_prescribed(N, d, sig, 880 + b)[0] for b in range(B)])
    g = np.random.default_rng(881)
    Q = (g.standard_normal((B, M, d)) / np.sqrt(d)).astype(np.float32)
    f = oracle.svd_factorize(X, r)
    db = lib.DeviceBatch(X, Q, None, r, False)
    db.factorize()
    torch.cuda.synchronize()
    assert np.all(db.info.cpu().numpy() == 0)
    S = db.S.cpu().numpy().astype(np.float64)
    V = db.V.cpu().numpy().astype(np.float64)
    for b in range(B):
        n_pos = int((S[b] > 0).sum())
        s_err = np.abs(S[b, :kept] - f["S"][b, :kept]).max() / f["S"][b, 0]
        pg = V[b, :, :kept] @ V[b, :, :kept].T
        po = f["V"][b, :, :kept] @ f["V"][b, :, :kept].T
        p_err = np.abs(pg - po).max()
        print(f"  user {b}: {n_pos} components returned, S err {s_err:.2e}, projector err {p_err:.2e}, "
              f"S_r gpu {S[b, r - 1]:.5g} oracle {f['S'][b, r - 1]:.5g}", flush=True)
        assert n_pos == kept
        assert np.all(S[b, kept:] == 0.0) and np.all(V[b, :, kept:] == 0.0)
        assert s_err < s_tol and p_err < p_tol
    rms = float(np.sqrt(np.mean(X.astype(np.float64) ** 2)))
    if o_tol is None:
        # the dropped component is gone from the output as well: mode 0 equals the oracle's
        # mode 0 on the rank-7 factorization
        f7 = oracle.svd_factorize(X, kept)
        for scale in (1.0, 3.0 / rms):
            want = oracle.svd_attention(Q, X, f7["S"], f7["V"], scale, 0)
            db.attention(scale, 0)
            torch.cuda.synchronize()
            err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
            print(f"  mode 0 scale {scale:.3g} against the rank-{kept} oracle: {err:.3e}", flush=True)
            assert err < 1e-4
    else:
        for scale in (1.0, 3.0 / rms):
            want = oracle.svd_attention(Q, X, f["S"], f["V"], scale, 0)
            db.attention(scale, 0)
            torch.cuda.synchronize()
            err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
            print(f"  mode 0 scale {scale:.3g}: {err:.3e}", flush=True)
            assert err < o_tol


# (lambda_(r+1) / lambda_r of the Gram matrix, bound on the projector error, bound on mode 0)
# (measured: S 1.3e-7; eigen-residual 9e-7; projector 1.5e-5; mode 0 1.7e-5 at most)
SLOW_SPECTRA = [(0.35, 3e-5, 1e-4), (0.6, 5e-5, 1e-4), (0.75, 1e-4, 1e-4)]


@pytest.mark.parametrize("rho,p_tol,o_tol", SLOW_SPECTRA, ids=[f"{c[0]:g}" for c in SLOW_SPECTRA])
@pytest.mark.parametrize("d,r", [(128, 16), (64, 8)])
def test_slowly_converging_spectra(lib, oracle, d, r, rho, p_tol, o_tol):
    """Full-rank float inputs whose singular values fall geometrically from 1 to 0.3 over the r
    wanted components and then sit on a plateau at sqrt(rho) * s_r: the block iteration converges
    like rho per power step, slowly enough that the eigen-iteration adds filtered power steps
    (rate estimate above 0.3).  Every user must converge (info 0), the singular values must agree
    with the oracle to 2e-6 of the largest, each returned pair must be an eigenpair of X^T X to
    2e-5 of the largest eigenvalue (formed here in double precision), and the projector and mode 0
    must agree with the oracle."""
    import torch
    N, M, B = 1200, 40, 3
    print(f"[case] slow spectrum d={d} r={r} rho={rho:g}", flush=True)
    sig = 30.0 * np.concatenate([np.geomspace(1.0, 0.3, r), np.full(d - r, 0.3 * np.sqrt(rho))])
    X = np.stack([_prescribed(N, d, sig, 660 + b)[0] for b in range(B)])
    g = np.random.default_rng(661)
    Q = (g.standard_normal((B, M, d)) / np.sqrt(d)).astype(np.float32)
    f = oracle.svd_factorize(X, r)
    db = lib.DeviceBatch(X, Q, None, r, False)
    db.factorize()
    torch.cuda.synchronize()
    info = db.info.cpu().numpy()
    assert np.all(info == 0), info
    S = db.S.cpu().numpy().astype(np.float64)
    V = db.V.cpu().numpy().astype(np.float64)
    for b in range(B):
        G = X[b].astype(np.float64).T @ X[b].astype(np.float64)
        s_err = np.abs(S[b] - f["S"][b]).max() / f["S"][b, 0]
        res = np.abs(G @ V[b] - V[b] * S[b] ** 2).max() / S[b, 0] ** 2
        orth = np.abs(V[b].T @ V[b] - np.eye(r)).max()
        p_err = np.abs(V[b] @ V[b].T - f["V"][b] @ f["V"][b].T).max()
        print(f"  user {b}: S err {s_err:.2e} eigen-residual {res:.2e} VtV-I {orth:.2e} projector err {p_err:.2e}",
              flush=True)
        assert s_err < 2e-6 and res < 2e-5 and orth < 2e-5 and p_err < p_tol
    rms = float(np.sqrt(np.mean(X.astype(np.float64) ** 2)))
    for scale in (1.0, 3.0 / rms):
        want = oracle.svd_attention(Q, X, f["S"], f["V"], scale, 0)
        db.attention(scale, 0)
        torch.cuda.synchronize()
        err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
        print(f"  mode 0 scale {scale:.3g}: {err:.3e}", flush=True)
        assert err < o_tol
