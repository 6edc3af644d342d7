"""The seeded input generator: determinism, distributions, sub-batch consistency, bf16 rounding."""
import numpy as np

from paper_2211_16270_amd import synth


def test_workload_shapes_and_lengths():
    for name, wl in synth.WORKLOADS.items():
        T, U, lab = synth.draw_lengths_labels(wl)
        assert T.shape == (wl.B,) and U.shape == (wl.B,) and lab.shape == (wl.B, wl.U_max)
        assert T.min() >= 1 and T.max() <= wl.T_max and U.min() >= 0 and U.max() <= wl.U_max
        assert lab.min() >= 1 and lab.max() <= wl.V - 1
    T, U, _ = synth.draw_lengths_labels(synth.WORKLOADS["C2"])
    assert T.min() >= 150 and U.min() >= 20
    T, U, lab = synth.draw_lengths_labels(synth.WORKLOADS["C5"])
    assert T.min() >= 50 and np.all(U == np.floor(0.3 * T + 0.5))
    assert (lab == 1).mean() > 0.05          # Zipf head


def test_sub_batch_matches_full_batch_and_is_deterministic():
    full = synth.make_batch("C1")
    again = synth.make_batch("C1")
    np.testing.assert_array_equal(full.enc, again.enc)
    sub = synth.make_batch("C1", sample_ids=[1])
    np.testing.assert_array_equal(sub.enc[0], full.enc[1])
    np.testing.assert_array_equal(sub.pred[0], full.pred[1])
    np.testing.assert_array_equal(sub.labels[0], full.labels[1])
    np.testing.assert_array_equal(sub.W_out, full.W_out)
    assert full.rows == 240


def test_bf16_rounding_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.001953125, 1.005859375, -3.14159, 1e-30, 65504.0], dtype=np.float32)
    r = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-9 is nearer to 1 + 2^-7
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 and r[3] == np.float32(1.0078125)
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(r)), r)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    b = synth.make_batch("C2", sample_ids=[0, 5], pad="zero")
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(b.enc)), b.enc)
    assert abs(float(b.W_out.std()) - 512 ** -0.5) < 2e-3
