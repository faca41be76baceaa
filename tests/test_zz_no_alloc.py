"""The allocation-free factorization, solar_svd_factorize_static, against solar_svd_factorize
(caller's workspace) through the C ABI: two calls in a row on the library's built-in scratch
array, the second on a smaller problem, so that whatever the first call left in the array would
show if the second read it.  Both entry points run the same kernels in the same order with
fixed-order reductions, so the outputs must agree bit for bit (which is inside every tolerance
of the parity tests); the existing entry point is itself checked against the oracle elsewhere.
"""
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


def _both_ways(lib, w, tag):
    import torch
    bf16 = w.dtype == synth.BF16
    ref = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, bf16)
    got = lib.DeviceBatch(w.X, w.Q, w.lengths, w.r, bf16)
    for t in (got.S, got.V, got.P):
        t.fill_(float("nan"))
    got.info.fill_(-77)
    print(f"[case] factorize_static {tag} B={w.B} N={w.N} d={w.d} r={w.r} bf16={bf16}", flush=True)
    ref.factorize()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = lib.solar_svd_factorize_static(got.X, got.lengths, w.r, got.S, got.V, got.P, got.info)
    after = torch.cuda.memory_allocated()
    torch.cuda.synchronize()
    assert rc == lib.SOLAR_OK
    assert after == before
    assert ref.info.cpu().tolist() == [0] * w.B, ref.info
    assert torch.equal(got.info, ref.info)
    assert torch.equal(got.S, ref.S), (got.S - ref.S).abs().max()
    assert torch.equal(got.V, ref.V), (got.V - ref.V).abs().max()
    assert torch.equal(got.P, ref.P), (got.P - ref.P).abs().max()
    # and the factors are sane in absolute terms: V^T V = I, P^T P = diag(S^2)
    V = got.V.double()
    P = got.P.double()
    S = got.S.double()
    eye = torch.eye(w.r, dtype=torch.float64, device=V.device)
    assert (V.transpose(1, 2) @ V - eye).abs().max().item() < 2e-5
    ptp = P.transpose(1, 2) @ P
    assert ((ptp - torch.diag_embed(S * S)).abs().amax(dim=(1, 2)) / (S[:, 0] ** 2)).max().item() < 1e-4
    return got


def test_two_calls_in_a_row_second_smaller(lib):
    big = synth.make_workload("t", 6, 2100, 128, 32, 16, synth.BF16, "spectrum", 1.0, 0.01,
                              var_len=(700, 2100), seed=7701)
    small = synth.make_workload("t", 3, 700, 64, 8, 16, synth.F32, "gauss_lowrank", seed=7702)
    _both_ways(lib, big, "first, larger")
    _both_ways(lib, small, "second, smaller")
    # d = 256 goes through G in the scratch array (the eigen-iteration reads it from there)
    wide = synth.make_workload("t", 2, 900, 256, 16, 16, synth.BF16, "gauss_lowrank", seed=7703)
    _both_ways(lib, wide, "third, d = 256")


def test_sizes_beyond_the_array_are_rejected(lib):
    import torch
    B, N, d, r = 64, 100000, 256, 32
    assert lib.solar_workspace_bytes(B, N, d, r, 0, lib.SOLAR_BF16) > lib.SOLAR_STATIC_SCRATCH_BYTES
    # nothing is dereferenced or launched: one-element tensors stand in for the arrays
    one = torch.zeros((1,), dtype=torch.float32, device="cuda")
    import ctypes
    rc = lib._lib.solar_svd_factorize_static(ctypes.c_void_p(one.data_ptr()), None, B, N, d, r, lib.SOLAR_BF16,
                                             ctypes.c_void_p(one.data_ptr()), ctypes.c_void_p(one.data_ptr()),
                                             None, None, None)
    assert rc == lib.SOLAR_ERR_SCRATCH_LIMIT
    assert "scratch" in lib.solar_status_string(rc)
