"""Pins of the oracle's activation normalisation (Sec. 3.1) to facts that do not come from the oracle."""
import math

import numpy as np

from oracle import clt_oracle as O


def _batches(seed, L=3, d=16, sizes=(5, 9, 2)):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((L, b, d)) * (1.0 + np.arange(L))[:, None, None] for b in sizes]


def test_constant_rows_have_the_textbook_norm():
    # every token of layer l is v_l * ones(d): ||.||_2 = |v_l| sqrt(d)
    L, B, d = 4, 7, 25
    v = np.array([0.5, -2.0, 3.0, 1e-3])
    a = np.ones((L, B, d)) * v[:, None, None]
    np.testing.assert_allclose(O.normalisation_factor([a]), np.abs(v) * math.sqrt(d), rtol=1e-14)


def test_three_four_five():
    a = np.zeros((1, 2, 8))
    a[0, 0, 1], a[0, 0, 6] = 3.0, -4.0       # norm 5
    a[0, 1, 0], a[0, 1, 3] = 5.0, 12.0       # norm 13
    np.testing.assert_allclose(O.normalisation_factor([a]), [9.0], rtol=1e-15)


def test_brute_force_over_unequal_batches_weights_tokens_not_batches():
    bs = _batches(0)
    L = bs[0].shape[0]
    want = np.zeros(L)
    n = 0
    for a in bs:
        for b in range(a.shape[1]):
            n += 1
            for l in range(L):
                want[l] += math.sqrt(sum(float(t) ** 2 for t in a[l, b]))
    want /= n
    np.testing.assert_allclose(O.normalisation_factor(bs), want, rtol=1e-13)
    # the same tokens in one batch give the same factor
    np.testing.assert_allclose(O.normalisation_factor([np.concatenate(bs, axis=1)]), want, rtol=1e-13)
    # and a mean of per-batch means would not
    per_batch = np.mean([O.normalisation_factor([a]) for a in bs], axis=0)
    assert np.abs(per_batch / want - 1).max() > 1e-3


def test_normalised_estimation_set_has_unit_mean_norm_per_layer():
    bs = _batches(1)
    c = O.normalisation_factor(bs)
    after = [O.normalise_activations(a, c) for a in bs]
    np.testing.assert_allclose(O.normalisation_factor(after), np.ones_like(c), rtol=1e-13)
    # the factor is per layer: layers of very different scale all end up at one
    assert c.max() / c.min() > 2.0


def test_factor_is_absolutely_homogeneous():
    bs = _batches(2)
    c = O.normalisation_factor(bs)
    np.testing.assert_allclose(O.normalisation_factor([-3.5 * a for a in bs]), 3.5 * c, rtol=1e-13)


def test_dividing_the_input_equals_dividing_the_encoder_weights():
    # pre(x / c; W) = pre(x; W / c): pins "divide", per layer, against eq. (1)
    rng = np.random.default_rng(3)
    L, B, d, F = 3, 6, 8, 16
    x = rng.standard_normal((L, B, d))
    W = rng.standard_normal((L, d, F))
    b = rng.standard_normal((L, F))
    c = np.array([0.5, 2.0, 7.0])
    lhs = O.encoder_preact(O.normalise_activations(x, c), W, b)
    rhs = O.encoder_preact(x, W / c[:, None, None], b)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    for l in range(L):
        np.testing.assert_allclose(O.normalise_activations(x, c)[l] * c[l], x[l], rtol=1e-15)


def test_all_zero_layer_is_left_alone():
    a = np.zeros((2, 3, 4))
    a[1] = 2.0
    c = O.normalisation_factor([a])
    assert c[0] == 1.0 and abs(c[1] - 4.0) < 1e-15
    assert np.all(O.normalise_activations(a, c)[0] == 0.0)


def test_folding_into_the_row_scale_is_the_same_division():
    # int8 cache (Sec. 3.1): x = q * s, so x / c = q * (s / c)
    rng = np.random.default_rng(4)
    q = rng.integers(-127, 128, size=(2, 5, 8))
    s = rng.uniform(0.01, 0.1, size=(2, 5))
    c = O.normalisation_factor([O.dequantize_rows(q, s)])
    np.testing.assert_allclose(O.dequantize_rows(q, s / c[:, None]),
                               O.normalise_activations(O.dequantize_rows(q, s), c), rtol=1e-14)
