"""Pins for the oracle of the SREM convolution (no GPU needed): the paper's identity initialisation, a library
routine for the plain case, a hand-worked corner, and what transposing / flipping the sequence does to the taps."""
import numpy as np
import pytest
import torch

from oracle import srem_oracle as so


def test_identity_initialisation_is_the_identity():
    # kernel centre one, rest zero (Sec. 3.3): the module starts as a no-op, in every orientation
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 6 * 5, 7))
    for orient in range(4):
        np.testing.assert_array_equal(so.srem_dwconv(x, so.identity_weights(7), None, 6, 5, orient), x)


def test_against_library_depthwise_convolution():
    rng = np.random.default_rng(1)
    B, gh, gw, D = 2, 5, 7, 6
    x = rng.standard_normal((B, gh * gw, D))
    w = rng.standard_normal((D, 3, 3))
    b = rng.standard_normal(D)
    img = torch.from_numpy(x.reshape(B, gh, gw, D)).permute(0, 3, 1, 2)
    ref = torch.nn.functional.conv2d(img, torch.from_numpy(w).reshape(D, 1, 3, 3), torch.from_numpy(b), padding=1,
                                     groups=D).permute(0, 2, 3, 1).reshape(B, gh * gw, D).numpy()
    np.testing.assert_allclose(so.srem_dwconv(x, w, b, gh, gw, 0), ref, rtol=1e-12, atol=1e-12)


def test_corner_token_by_hand():
    # 2 x 2 matrix, one channel, x = [[1, 2], [3, 4]], w = [[1..9]]: the top-left output sees
    # x[0,0] w[1,1] + x[0,1] w[1,2] + x[1,0] w[2,1] + x[1,1] w[2,2] = 5 + 12 + 24 + 36 = 77
    x = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 4, 1)
    w = np.arange(1.0, 10.0).reshape(1, 3, 3)
    y = so.srem_dwconv(x, w, np.array([0.5]), 2, 2, 0)
    assert y[0, 0, 0] == 77.5
    # bottom-right: x[1,1] w[1,1] + x[1,0] w[1,0] + x[0,1] w[0,1] + x[0,0] w[0,0] = 20 + 12 + 4 + 1 = 37
    assert y[0, 3, 0] == 37.5


def test_orientations_permute_the_taps():
    """Convolving the reversed / transposed token matrix equals convolving the canonical one with the kernel
    rotated by 180 degrees / transposed (and both for the column-major reversed order)."""
    rng = np.random.default_rng(2)
    B, gh, gw, D = 1, 4, 6, 3
    x = rng.standard_normal((B, gh * gw, D))
    w = rng.standard_normal((D, 3, 3))
    b = rng.standard_normal(D)
    base = lambda ww: so.srem_dwconv(x, ww, b, gh, gw, 0)
    np.testing.assert_allclose(so.srem_dwconv(x, w, b, gh, gw, 1), base(w[:, ::-1, ::-1]), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(so.srem_dwconv(x, w, b, gh, gw, 2), base(w.transpose(0, 2, 1)), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(so.srem_dwconv(x, w, b, gh, gw, 3), base(w.transpose(0, 2, 1)[:, ::-1, ::-1]),
                               rtol=1e-13, atol=1e-13)
    # and the orientations really differ for an asymmetric kernel
    assert np.abs(so.srem_dwconv(x, w, b, gh, gw, 2) - base(w)).max() > 1e-3


def test_single_row_and_single_column_matrices():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 5, 2))
    w = rng.standard_normal((2, 3, 3))
    # a 1 x 5 matrix only ever meets the middle row of the kernel
    y = so.srem_dwconv(x, w, None, 1, 5, 0)
    ref = np.zeros_like(x)
    for c in range(5):
        for dx in (-1, 0, 1):
            if 0 <= c + dx < 5:
                ref[0, c] += x[0, c + dx] * w[:, 1, dx + 1]
    np.testing.assert_allclose(y, ref, rtol=1e-14, atol=1e-14)
    with pytest.raises(ValueError):
        so.srem_dwconv(x, w, None, 2, 2, 0)
