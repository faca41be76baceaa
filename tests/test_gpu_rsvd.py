"""GPU parity of the factorization by Algorithm 1 (passes over X, QR through the Cholesky factor
of Y^T Y, small SVD by one-sided Jacobi) against the double-precision oracle of the printed
algorithm on the same Gaussian start blocks.

The oracle runs the power steps exactly as printed, with no re-orthonormalisation, which double
precision can afford.  The library replaces the block by an orthonormal basis of its range after
every power step: every output of the algorithm depends on the block only through its range, so
the two compute the same thing, and the library's float arithmetic survives the power steps
(without that step cond(H Omega) grows by (sigma_1/sigma_r)^2 per power step and the float
Cholesky factor of Y^T Y breaks down after the first one on the headline workload).

Tolerances.  No power step: singular values to 1e-3 of the largest (the bf16 inputs' exact-rank
case loses the most: its smallest singular values sit 1e-3 below the largest and Y = H Omega
inherits the conditioning of the raw Gaussian block), projectors V V^T to 1e-4.  One or two power
steps: 1e-5 for both (measured at most 3e-6), and no user may be flagged.
"""
import numpy as np
import pytest

from paper_2603_02561_amd import synth

pytestmark = pytest.mark.gpu

TOL_ATTN = {synth.F32: 1e-4, synth.BF16: 2e-2}


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


def workloads():
    out = []
    out.append(("f32_d128_r16", synth.make_workload("t", 3, 777, 128, 16, 150, synth.F32, "gauss_lowrank", seed=102)))
    out.append(("bf16_d128_r32_noise", synth.make_workload("t", 3, 1100, 128, 32, 200, synth.BF16, "spectrum",
                                                           1.0, 0.01, seed=103)))
    out.append(("bf16_d128_r64_varlen", synth.make_workload("t", 4, 900, 128, 64, 130, synth.BF16, "spectrum",
                                                            0.5, 0.02, var_len=(300, 900), seed=104)))
    out.append(("bf16_d64_r16", synth.make_workload("t", 2, 400, 64, 16, 33, synth.BF16, "gauss_lowrank", seed=106)))
    out.append(("f32_d64_r48_varlen", synth.make_workload("t", 2, 600, 64, 48, 40, synth.F32, "spectrum",
                                                          0.3, 0.05, var_len=(200, 600), seed=109)))
    return out


WORKLOADS = workloads()
IDS = [n for n, _ in WORKLOADS]


@pytest.mark.parametrize("name,w", WORKLOADS, ids=IDS)
def test_rsvd_factorize(lib, oracle, name, w):
    import torch
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, w.dtype == synth.BF16)
    Om = synth.make_omega(w.B, w.d, w.r)
    Omd = torch.from_numpy(Om).cuda()
    for q in (0, 1, 2):
        print(f"[case] rsvd {name} n_iter={q}", flush=True)
        db.factorize_rsvd(Omd, q)
        torch.cuda.synchronize()
        S = db.S.cpu().numpy().astype(np.float64)
        V = db.V.cpu().numpy().astype(np.float64)
        P = db.P.cpu().numpy().astype(np.float64)
        info = db.info.cpu().numpy()
        f = oracle.rsvd_alg1(w.X, Om, q, w.lengths)
        tol_s, tol_p = [(1e-3, 1e-4), (1e-5, 1e-5), (1e-5, 1e-5)][q]
        for b in range(w.B):
            assert info[b] == 0, f"user {b} flagged {info[b]} with {q} power steps"
            s_err = np.abs(S[b] - f["S"][b]).max() / f["S"][b][0]
            proj_err = np.abs(V[b] @ V[b].T - f["V"][b] @ f["V"][b].T).max()
            orth = np.abs(V[b].T @ V[b] - np.eye(w.r)).max()
            n = int(w.lengths[b])
            p_want = w.X[b, :n].astype(np.float64) @ V[b]
            p_err = np.abs(P[b, :n] - p_want).max() / np.abs(p_want).max()
            print(f"  user {b}: S {s_err:.2e} proj {proj_err:.2e} VtV-I {orth:.2e} P {p_err:.2e}", flush=True)
            assert s_err < tol_s and proj_err < tol_p and orth < 2e-5 and p_err < 1e-5
            assert np.all(P[b, n:] == 0)
            assert np.all(np.diff(S[b]) <= 0)


def test_rsvd_headline_size_with_power_steps(lib, oracle):
    """The headline workload (B=64, N=10000, d=128, r=32, bf16, spectrum 1/k + noise), where
    sigma_1/sigma_32 = 32: no user may be flagged after one or two power steps, V^T V = I for
    every user (P^T P = diag(S^2) is not a property of the randomized algorithm: its V are the
    singular vectors of Q^T H, not of H), and four users agree with the oracle of the printed
    algorithm."""
    import torch
    w = synth.make_config("C3")
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, True)
    Om = synth.make_omega(w.B, w.d, w.r)
    Omd = torch.from_numpy(Om).cuda()
    users = [0, 21, 42, 63]
    for q in (1, 2):
        print(f"[case] rsvd C3 n_iter={q}", flush=True)
        db.factorize_rsvd(Omd, q)
        torch.cuda.synchronize()
        info = db.info.cpu().numpy()
        assert np.all(info == 0), info
        V = db.V.double()
        eye = torch.eye(w.r, dtype=torch.float64, device=V.device)
        vtv = (V.transpose(1, 2) @ V - eye).abs().amax().item()
        print(f"  all users: |VtV-I| {vtv:.2e}", flush=True)
        assert vtv < 2e-5
        f = oracle.rsvd_alg1(w.X[users], Om[users], q, w.lengths[users])
        Sg = db.S.cpu().numpy().astype(np.float64)
        Vg = db.V.cpu().numpy().astype(np.float64)
        for i, u in enumerate(users):
            s_err = np.abs(Sg[u] - f["S"][i]).max() / f["S"][i][0]
            proj_err = np.abs(Vg[u] @ Vg[u].T - f["V"][i] @ f["V"][i].T).max()
            print(f"  user {u}: S {s_err:.2e} proj {proj_err:.2e}", flush=True)
            assert s_err < 1e-5 and proj_err < 1e-4


@pytest.mark.parametrize("n_iter", [0, 1])
@pytest.mark.parametrize("name,w", WORKLOADS[:2], ids=IDS[:2])
def test_rsvd_then_attention(lib, oracle, name, w, n_iter):
    """mode 0 on the factors of Algorithm 1 against the oracle's attention on the oracle's
    factors of the same algorithm."""
    import torch
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, w.dtype == synth.BF16)
    Om = synth.make_omega(w.B, w.d, w.r)
    db.factorize_rsvd(torch.from_numpy(Om).cuda(), n_iter)
    f = oracle.rsvd_alg1(w.X, Om, n_iter, w.lengths)
    for scale in (1.0, w.sharp_scale):
        db.attention(scale, 0)
        torch.cuda.synchronize()
        want = oracle.svd_attention(w.Q, w.X, f["S"], f["V"], scale, 0, w.lengths)
        got = db.O.cpu().numpy().astype(np.float64)
        err = max(np.abs(got[b] - want[b]).max() / np.abs(want[b]).max() for b in range(w.B))
        print(f"[case] rsvd attention {name} scale={scale:.3g} err {err:.3e}", flush=True)
        assert err < TOL_ATTN[w.dtype]


def test_rsvd_argument_errors(lib):
    import torch
    w = WORKLOADS[0][1]
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, False)
    Om = torch.from_numpy(synth.make_omega(w.B, w.d, w.r)).cuda()
    ws = torch.empty((lib.solar_rsvd_workspace_bytes(w.B, w.N, w.d, w.r),), dtype=torch.uint8, device="cuda")
    rc = lib.solar_svd_factorize_rsvd(db.X, db.lengths, w.r, Om, -1, db.S, db.V, db.P, db.info, ws,
                                      raise_on_error=False)
    assert rc == 1
    rc = lib.solar_svd_factorize_rsvd(db.X, db.lengths, w.r, Om, 0, db.S, db.V, db.P, db.info, ws[:1024],
                                      raise_on_error=False)
    assert rc == 3
    assert lib.solar_rsvd_workspace_bytes(2, 100, 256, 16) == 0   # d = 256 is not supported on this route
