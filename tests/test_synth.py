"""Seeded input generators: determinism, bf16 rounding, stated structure."""
import numpy as np

from paper_2603_02561_amd import synth


def test_bf16_rounding_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -3.1415927, 1e-30, 0.0], dtype=np.float32)
    r = synth.round_to_bf16(x)
    assert np.array_equal(synth.round_to_bf16(r), r)
    assert r[0] == 1.0
    assert r[1] == np.float32(1.0)           # tie, rounds to even mantissa
    assert r[2] == np.float32(1.0078125)     # above the tie
    assert r[3] == 1.0                       # below the tie
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    bits = synth.bf16_bits(r)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, r)


def test_subset_of_users_reproduces_full_batch():
    full = synth.make_workload("t", 4, 64, 16, 4, 8, synth.BF16, "spectrum", 1.0, 0.01, seed=7)
    sub = synth.make_workload("t", 4, 64, 16, 4, 8, synth.BF16, "spectrum", 1.0, 0.01, seed=7,
                              users=[2, 3])
    assert np.array_equal(full.X[2:], sub.X)
    assert np.array_equal(full.Q[2:], sub.Q)


def test_structure_of_the_recipes():
    w = synth.make_workload("t", 2, 256, 32, 4, 8, synth.F32, "gauss_lowrank", seed=11)
    s = np.linalg.svd(w.X[0].astype(np.float64), compute_uv=False)
    assert s[4] < 1e-5 * s[0]                # exactly rank r up to float32 rounding
    assert abs(w.X.std() * 2.0 - 1.0) < 0.2  # entry std 1/sqrt(r)
    w = synth.make_workload("t", 1, 512, 32, 8, 8, synth.F32, "spectrum", 1.0, 0.0, seed=12)
    s = np.linalg.svd(w.X[0].astype(np.float64), compute_uv=False)
    assert np.allclose(s[:8] * np.arange(1, 9), s[0], rtol=1e-4)   # sigma_k = c / k
    w = synth.make_workload("t", 6, 300, 16, 4, 8, synth.F32, "spectrum", 0.5, 0.05,
                            var_len=(100, 300), seed=13)
    assert np.all((w.lengths >= 100) & (w.lengths <= 300))
    short = int(np.argmin(w.lengths))
    if w.lengths[short] < 300:
        assert np.all(np.isfinite(w.X[short])) and np.abs(w.X[short, w.lengths[short]:]).mean() > 0.5
