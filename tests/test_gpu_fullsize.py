"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole batch runs on the GPU.  The oracle (seconds per user at these sizes) checks every
user and candidate of the small workload and, of the large ones, eight users (the shortest
and the longest among them) on sampled candidates; every user and candidate is additionally
checked through what holds at any size: convergence flags, V^T V = I, P^T P = diag(S^2)
(which is U^T U = I), descending S, and equality with the GPU's dense softmax attention --
on X itself where X has rank r exactly, on the rank-r projection P V^T otherwise -- which
itself is oracle-checked on the sampled users.
"""
import numpy as np
import pytest

from paper_2603_02561_amd import synth

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

N_QUERIES = 48   # candidates per sampled user that the oracle evaluates


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


def rel(got, want):
    return float(np.abs(np.asarray(got, np.float64) - want).max() / np.abs(want).max())


# name, oracle-checked users (None = eight of them: the shortest, the longest and six spread over
# the batch; "all" = every user), tolerance, exact rank?
CASES = [
    ("C1", "all", 1e-4, True),
    ("C2", [0, 31], 1e-4, True),
    ("C3", None, 2e-2, False),
    ("C4", [5], 2e-2, True),
    ("C5", None, 2e-2, False),
]


def eight_users(lengths):
    B = len(lengths)
    picks = {int(np.argmin(lengths)), int(np.argmax(lengths))}
    for u in np.linspace(0, B - 1, 8).astype(int):
        if len(picks) < 8:
            picks.add(int(u))
    u = 1
    while len(picks) < min(8, B):
        picks.add(u)
        u += 1
    return sorted(picks)


@pytest.mark.parametrize("name,users,tol,exact", CASES, ids=[c[0] for c in CASES])
def test_full_size(lib, oracle, name, users, tol, exact):
    import torch
    from concurrent.futures import ThreadPoolExecutor
    print(f"[case] full size {name}: generating", flush=True)
    w = synth.make_config(name)
    bf16 = w.dtype == synth.BF16
    if users is None:
        users = eight_users(w.lengths)
    all_candidates = users == "all"
    if all_candidates:
        users = list(range(w.B))
    print(f"  B={w.B} N={w.N} d={w.d} r={w.r} M={w.M} users={users} "
          f"lengths={[int(w.lengths[u]) for u in users]}", flush=True)
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, bf16)
    db.factorize()
    torch.cuda.synchronize()
    info = db.info.cpu().numpy()
    print(f"  info nonzero: {int((info != 0).sum())}", flush=True)
    assert np.all(info == 0)

    # properties for every user, evaluated on the device in float64
    V = db.V.double()
    P = db.P.double()
    S = db.S.double()
    eye = torch.eye(w.r, dtype=torch.float64, device=V.device)
    vtv = (V.transpose(1, 2) @ V - eye).abs().amax().item()
    ptp = P.transpose(1, 2) @ P
    utu = ((ptp - torch.diag_embed(S * S)).abs().amax(dim=(1, 2)) / (S[:, 0] ** 2)).max().item()
    desc = bool((S[:, 1:] <= S[:, :-1]).all().item())
    print(f"  all users: |VtV-I| {vtv:.2e}  |PtP-diag(S^2)|/S1^2 {utu:.2e}  descending {desc}", flush=True)
    assert vtv < 2e-5 and utu < 1e-4 and desc
    del V, P, ptp

    O0 = {}
    for scale in (1.0, w.sharp_scale):
        db.attention(scale, 0)
        torch.cuda.synchronize()
        O0[scale] = db.O.clone()
    Od = torch.empty_like(db.O)
    if exact:
        # lossless reading: equals dense softmax attention for every user
        for scale in (1.0, w.sharp_scale):
            db.dense(scale, Od)
            torch.cuda.synchronize()
            num = (O0[scale] - Od).abs().amax(dim=(1, 2))
            den = Od.abs().amax(dim=(1, 2))
            err = (num / den).max().item()
            print(f"  svd vs gpu dense, all users, scale={scale:.3g}: {err:.3e}", flush=True)
            assert err < tol
    else:
        # rank > r: mode 0 is dense softmax attention on the rank-r projection X_r = P V^T.  X_r is
        # formed here from the library's own P and V (which the properties above and the oracle
        # below check) and handed, as float, to the dense reference kernel (itself oracle-checked
        # on the sampled users below): every candidate of every user is compared.
        Xr = torch.bmm(db.P, db.V.transpose(1, 2)).contiguous()          # [B, N, d] float
        Qf = db.Q.float().contiguous()
        for scale in (1.0, w.sharp_scale):
            lib.solar_dense_attention_ref(Qf, Xr, db.lengths, scale, Od)
            torch.cuda.synchronize()
            num = (O0[scale] - Od).abs().amax(dim=(1, 2))
            den = Od.abs().amax(dim=(1, 2))
            err = (num / den).max().item()
            print(f"  svd vs gpu dense on X_r = P V^T, all users, scale={scale:.3g}: {err:.3e}", flush=True)
            assert err < tol
        del Xr, Qf

    # oracle on sampled users / sampled candidates (one user per thread: the C oracle releases the GIL)
    qsel = np.arange(w.M) if all_candidates else np.linspace(0, w.M - 1, N_QUERIES).astype(int)
    db.attention(1.0, 2)
    torch.cuda.synchronize()
    O2 = db.O.clone()
    db.dense(1.0)
    torch.cuda.synchronize()
    Odense = db.O.clone()
    S_gpu = db.S.cpu().numpy()
    V_gpu = db.V.cpu().numpy().astype(np.float64)

    def check(u):
        Xu = w.X[u:u + 1]
        Lu = w.lengths[u:u + 1]
        Qu = w.Q[u:u + 1][:, qsel]
        f = oracle.svd_factorize(Xu, w.r, Lu)
        out = {"u": u, "S": float(np.abs(S_gpu[u] - f["S"][0]).max() / f["S"][0][0]),
               "proj": float(np.abs(V_gpu[u] @ V_gpu[u].T - f["V"][0] @ f["V"][0].T).max())}
        for scale in (1.0, w.sharp_scale):
            want = oracle.svd_attention(Qu, Xu, f["S"], f["V"], scale, 0, Lu)[0]
            out[f"mode0@{scale:.3g}"] = rel(O0[scale][u].cpu().numpy()[qsel], want)
        want2 = oracle.svd_attention(Qu, None, f["S"], f["V"], 1.0, 2)[0]
        out["mode2"] = rel(O2[u].cpu().numpy()[qsel], want2)
        wantd = oracle.dense_attention(Qu, Xu, 1.0, Lu)[0]
        out["dense"] = rel(Odense[u].cpu().numpy()[qsel], wantd)
        if exact:
            out["mode0_vs_dense"] = rel(O0[1.0][u].cpu().numpy()[qsel], wantd)
        return out

    print(f"  oracle: {len(users)} users, {len(qsel)} candidates each", flush=True)
    with ThreadPoolExecutor(max_workers=8) as pool:
        results = list(pool.map(check, users))
    for res in results:
        print("  user " + " ".join(f"{k}={v:.2e}" if k != "u" else str(v) for k, v in res.items()), flush=True)
        assert res["S"] < (1e-4 if not bf16 else 1e-3) and res["proj"] < 1e-2
        for k, v in res.items():
            if k.startswith("mode0") or k == "mode2":
                assert v < tol, (res["u"], k, v)
        assert res["dense"] < 1e-4
