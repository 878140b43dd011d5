"""The seeded input generator: counter-based (slices reproduce), normal moments, exact bf16 rounding."""
import numpy as np

import spmoe_inputs as si


def test_slices_reproduce_and_streams_differ():
    a = si.normal_f32(0, 5, 10001)
    assert np.array_equal(si.normal_f32(0, 5, 1000, offset=777), a[777:1777])
    assert np.array_equal(si.normal_f32(0, 5, 3, offset=9998), a[9998:])
    assert not np.array_equal(si.normal_f32(0, 6, 100), a[:100])
    assert not np.array_equal(si.normal_f32(1, 5, 100), a[:100])


def test_moments_and_independence():
    a = si.normal_f32(3, 9, 2_000_000).astype(np.float64)
    assert abs(a.mean()) < 3e-3 and abs(a.std() - 1) < 3e-3
    assert abs((a ** 3).mean()) < 1e-2 and abs((a ** 4).mean() - 3) < 3e-2
    assert abs(np.corrcoef(a[::2], a[1::2])[0, 1]) < 3e-3          # the two Box-Muller outputs of a pair
    w = si.normal_f32(3, 10, 200_000, std=0.02)
    assert abs(w.std() - 0.02) < 2e-4


def test_bf16_is_nearest_even_rounding_of_the_fp32_stream():
    f = si.normal_f32(4, 2, 50_000, std=0.02)
    b = si.normal_bf16(4, 2, 50_000, std=0.02)
    assert np.array_equal(b, si.round_bf16(f))
    up = si.bf16_to_f32(b)
    # nearest: error at most half a bf16 ulp (8 significant bits)
    assert np.all(np.abs(up - f) <= np.abs(f) * 2.0 ** -8)
    # ties-to-even on constructed halfway cases: 1 + 2^-8 -> 1.0 (even), 1 + 3*2^-8 -> 1 + 2^-6
    halfway = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)
    assert np.array_equal(si.bf16_to_f32(si.round_bf16(halfway)), np.array([1.0, 1.0 + 2.0 ** -6], np.float32))


def test_layout_shapes():
    g, u, dn = si.expert_weights(0, 1, 2, 64, 96, "bf16")
    assert g.shape == (96, 64) and u.shape == (96, 64) and dn.shape == (64, 96) and g.dtype == np.uint16
    assert si.gate_weights(0, 0, 8, 64, "f32").shape == (8, 64)
    assert si.hidden(0, 5, 64).shape == (5, 64)


def test_correlated_tokens_share_a_sequence_component():
    x0 = si.hidden_correlated(5, 32, 4096, 0.0, 4)
    assert np.array_equal(x0, si.hidden(5, 32, 4096))
    x = si.hidden_correlated(5, 32, 4096, 0.8, 4).astype(np.float64)
    assert abs(x.std() - 1.0) < 2e-2
    c = np.corrcoef(x)
    same = np.mean([c[i, j] for i in range(32) for j in range(32) if i != j and i // 8 == j // 8])
    other = np.mean([c[i, j] for i in range(32) for j in range(32) if i // 8 != j // 8])
    assert abs(same - 0.64) < 0.03 and abs(other) < 0.03          # rho^2 inside a sequence, 0 across
