"""The seeded input generators: exact counts, reproducibility, stated distributions."""
import numpy as np

import synth
from synth import inputs as si


def test_uniform_mask_exact_count_and_reproducible():
    M = synth.uniform_mask(1, 2, 48, 96, 0.05)
    assert M.dtype == np.uint8 and M.shape == (48, 96)
    assert int(M.sum()) == si.active_count(48 * 96, 0.05) == 230
    np.testing.assert_array_equal(M, synth.uniform_mask(1, 2, 48, 96, 0.05))
    assert (M != synth.uniform_mask(2, 2, 48, 96, 0.05)).any()
    assert synth.uniform_mask(1, 2, 4, 4, 1.0).all() and not synth.uniform_mask(1, 2, 4, 4, 0.0).any()


def test_config1_active_count():
    assert si.active_count(768 * 3072, 0.05) == 117965


def test_powerlaw_mask_row_lengths():
    O, I = 768, 768
    M = synth.powerlaw_mask(3, 5, O, I, 0.02)
    lens = M.sum(axis=1)
    assert int(lens.sum()) == si.active_count(O * I, 0.02)
    np.testing.assert_array_equal(lens, si.powerlaw_row_lengths(3, 5, O, I, 0.02))
    assert lens.max() >= 20 * np.median(lens)          # heavy tail: a few long rows
    assert np.median(lens) <= 8                          # most rows hold a handful


def test_bf16_rounding_is_nearest_even_and_exact_to_widen():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.3895314e38], dtype=np.float32)
    b = synth.to_bf16_bits(x)
    y = synth.bf16_bits_to_f32(b)
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.0 + 2 ** -7 and y[3] == 1.0 + 2 ** -6
    assert abs(y[4] + 0.3) <= 0.3 * 2 ** -8
    np.testing.assert_array_equal(synth.to_bf16_bits(y), b)     # idempotent


def test_layer_and_activations():
    W, M = synth.make_layer(0, 1, 32, 48, 0.1)
    assert W.shape == (48, 32) and W.dtype == np.float32 and not W[M == 0].any()
    assert abs(W[M != 0].std() - 0.02) < 0.01
    X, dY = synth.make_activations(0, 1, 64, 32, 48)
    assert X.shape == (64, 32) and dY.shape == (64, 48) and abs(X.std() - 1) < 0.1
    Xf, dYf, xb, yb = synth.make_activations(0, 1, 64, 32, 48, "bf16")
    assert xb.dtype == np.uint16 and np.abs(Xf - X).max() <= np.abs(X).max() * 2 ** -8
