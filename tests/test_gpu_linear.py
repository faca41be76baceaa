"""GPU parity of linear attention (Query (Key^T Value) with Key = Value = X) and of the folded
projections against the oracle.  Tolerances: products accumulate in float over <= N terms twice;
1e-4 for float inputs; 1e-3 for bf16 inputs (the inputs are exact, the only 16-bit rounding is the
optional bf16 output of the folding step, 2^-9 relative, tested at 5e-3)."""
import numpy as np
import pytest

from paper_2603_02561_amd import synth

pytestmark = pytest.mark.gpu


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


CASES = [
    ("f32_d64", synth.make_workload("t", 2, 333, 64, 8, 70, synth.F32, "gauss_lowrank", seed=201)),
    ("bf16_d128_varlen", synth.make_workload("t", 3, 900, 128, 32, 130, synth.BF16, "spectrum", 0.5, 0.02,
                                             var_len=(300, 900), seed=202)),
    ("f32_d256", synth.make_workload("t", 2, 300, 256, 16, 41, synth.F32, "gauss_lowrank", seed=203)),
]


def rel_err(got, want):
    return max(np.abs(got[b] - want[b]).max() / np.abs(want[b]).max() for b in range(want.shape[0]))


@pytest.mark.parametrize("name,w", CASES, ids=[c[0] for c in CASES])
def test_linear_attention(lib, oracle, name, w):
    import torch
    print(f"[case] linear attention {name}", flush=True)
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, w.dtype == synth.BF16)
    db.linear(0.37)
    torch.cuda.synchronize()
    want = oracle.linear_attention(w.Q, w.X, 0.37, w.lengths)
    err = rel_err(db.O.cpu().numpy().astype(np.float64), want)
    print(f"  err {err:.3e}", flush=True)
    assert err < (1e-4 if w.dtype == synth.F32 else 1e-3)


@pytest.mark.parametrize("name,w", CASES, ids=[c[0] for c in CASES])
def test_folded_projections(lib, oracle, name, w):
    """C (W_Q W_K^T) -> SVD-attention (mode 0) -> W_V on the GPU against the oracle doing the same
    steps in double on the same folded candidates."""
    import torch
    print(f"[case] folded projections {name}", flush=True)
    g = np.random.default_rng(7)
    d = w.d
    Wf = (np.eye(d) + 0.1 * g.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32)
    Wv = (np.eye(d) + 0.1 * g.standard_normal((d, d)) / np.sqrt(d)).astype(np.float32)
    bf16 = w.dtype == synth.BF16
    db = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, bf16)
    Wf_d, Wv_d = torch.from_numpy(Wf).cuda(), torch.from_numpy(Wv).cuda()
    Qf = torch.empty_like(db.Q)
    lib.solar_apply_weights(db.Q, Wf_d, Qf)
    torch.cuda.synchronize()
    want_qf = oracle.apply_weights(w.Q, Wf)
    got_qf = Qf.float().cpu().numpy().astype(np.float64)
    e1 = rel_err(got_qf, want_qf)
    print(f"  folded candidates err {e1:.3e}", flush=True)
    assert e1 < (1e-5 if not bf16 else 5e-3)
    # the operator on the folded candidates (the GPU's own, rounded if bf16), then W_V
    db.Q = Qf
    db.factorize()
    db.attention(1.0, 0)
    Of = torch.empty_like(db.O)
    lib.solar_apply_weights(db.O, Wv_d, Of)
    torch.cuda.synchronize()
    f = oracle.svd_factorize(w.X, w.r, w.lengths)
    want = oracle.apply_weights(oracle.svd_attention(got_qf, w.X, f["S"], f["V"], 1.0, 0, w.lengths), Wv)
    e2 = rel_err(Of.cpu().numpy().astype(np.float64), want)
    print(f"  output err {e2:.3e}", flush=True)
    assert e2 < (1e-4 if not bf16 else 2e-2)
