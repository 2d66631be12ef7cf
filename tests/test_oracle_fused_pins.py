"""Pins for the oracle of the gate prologue and the output epilogue (no GPU needed).

Expected values come from closed forms and from a two-token example evaluated by hand; citations name the
equations of the DiG paper (Sec. 3.1) that define each step.
"""
import math

import numpy as np
import pytest

from oracle import gla_oracle, gla_oracle_fused as fo

LN3 = math.log(3.0)


def test_log_sigmoid_closed_forms():
    # sigmoid(0) = 1/2, sigmoid(ln 3) = 3/4, sigmoid(-ln 3) = 1/4
    z = np.array([0.0, LN3, -LN3])
    np.testing.assert_allclose(fo.log_sigmoid(z), [math.log(0.5), math.log(0.75), math.log(0.25)], rtol=1e-15)


def test_log_sigmoid_identities_and_tails():
    rng = np.random.default_rng(0)
    z = rng.standard_normal(1000) * 6
    ls, lsn = fo.log_sigmoid(z), fo.log_sigmoid(-z)
    np.testing.assert_allclose(ls - lsn, z, atol=1e-13)                 # log s(z) - log s(-z) = z
    np.testing.assert_allclose(np.exp(ls) + np.exp(lsn), 1.0, atol=1e-15)  # s(z) + s(-z) = 1
    assert fo.log_sigmoid(-800.0) == -800.0                            # no overflow on the far left
    assert abs(fo.log_sigmoid(40.0) + math.exp(-40.0)) < 1e-30         # log(1 - e^-40 + ...) on the right
    assert np.all(fo.log_sigmoid(z) < 0)


def test_alpha_is_the_tau_th_root_of_sigmoid():
    # Eq. (gate_gla): alpha = sigmoid(z)^(1/tau)
    z = np.array([-3.0, -0.5, 0.0, 1.25, 4.0])
    for tau in (1.0, 2.0, 16.0):
        alpha = np.exp(fo.log_alpha_from_z(z, tau))
        np.testing.assert_allclose(alpha ** tau, 1.0 / (1.0 + np.exp(-z)), rtol=1e-13)
    # temperature 16 keeps the gate close to one: sigmoid(0)^(1/16) = 2^(-1/16)
    assert abs(math.exp(fo.log_alpha_from_z(0.0, 16.0)) - 2.0 ** (-1.0 / 16.0)) < 1e-15


def test_swish_closed_forms():
    # Eq. (attn_gla) row 4: Swish(x) = x sigmoid(x)
    np.testing.assert_allclose(fo.swish(np.array([0.0, LN3, -LN3])), [0.0, 0.75 * LN3, -0.25 * LN3], rtol=1e-15)
    x = np.linspace(-20, 20, 401)
    np.testing.assert_allclose(fo.swish(x) - fo.swish(-x), x, atol=1e-13)   # x s(x) + x s(-x) = x
    assert fo.swish(-1.278464542761074) == pytest.approx(-0.2784645427610738, abs=1e-12)   # the minimum of Swish


def test_layer_norm_hand_example():
    # o = (1, 2, 3, 4): mean 5/2, biased variance 5/4
    o = np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 1, 4)
    s = math.sqrt(1.25)
    np.testing.assert_allclose(fo.layer_norm_heads(o, eps=0.0).ravel(), [-1.5 / s, -0.5 / s, 0.5 / s, 1.5 / s],
                               rtol=1e-15)
    w = np.array([[2.0, 1.0, 0.5, -1.0]])
    b = np.array([[0.0, 1.0, 2.0, 3.0]])
    np.testing.assert_allclose(fo.layer_norm_heads(o, w, b, eps=0.0).ravel(),
                               [-3.0 / s, 1 - 0.5 / s, 2 + 0.25 / s, 3 - 1.5 / s], rtol=1e-15)
    # eps sits inside the square root
    np.testing.assert_allclose(fo.layer_norm_heads(o, eps=0.75).ravel(), np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(2.0),
                               rtol=1e-15)


def test_layer_norm_invariants():
    rng = np.random.default_rng(1)
    B, H, T, dv = 2, 3, 5, 24
    o = rng.standard_normal((B, H, T, dv)) * 3 + 1
    y = fo.layer_norm_heads(o, eps=0.0)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-14)
    np.testing.assert_allclose((y ** 2).mean(-1), 1.0, rtol=1e-13)
    # shift and positive scale of a token's row leave LN unchanged (eps = 0)
    np.testing.assert_allclose(fo.layer_norm_heads(2.5 * o + 7.0, eps=0.0), y, atol=1e-12)
    # statistics are per (batch, head, token): changing one head's row does not touch another head
    o2 = o.copy()
    o2[:, 1] += rng.standard_normal((B, T, dv))
    y2 = fo.layer_norm_heads(o2, eps=0.0)
    np.testing.assert_array_equal(y2[:, 0], y[:, 0])
    np.testing.assert_array_equal(y2[:, 2], y[:, 2])
    # per-head affine rows
    w = rng.standard_normal((H, dv))
    b = rng.standard_normal((H, dv))
    ya = fo.layer_norm_heads(o, w, b, eps=0.0)
    for h in range(H):
        np.testing.assert_allclose(ya[:, h], y[:, h] * w[h] + b[h], rtol=1e-14, atol=1e-14)
    # a constant row has zero variance: with eps > 0 the result is the bias
    c = np.full((1, H, 1, dv), 4.0)
    np.testing.assert_allclose(fo.layer_norm_heads(c, w, b, eps=1e-5), np.broadcast_to(b.reshape(1, H, 1, dv), c.shape),
                               atol=1e-12)


def test_fused_two_token_example_by_hand():
    """T = 2, d_k = 1, d_v = 2, tau = 2, z_2 = ln 3 so that alpha_2 = sqrt(3)/2.

    S_1 = k_1 v_1 = (2, 0), O_1 = q_1 S_1 = (2, 0); S_2 = alpha_2 S_1 + k_2 v_2 = (sqrt 3, 4), O_2 = 2 S_2.
    LN over two entries (eps = 0) is (+1, -1) or (-1, +1); weight (2, 3), bias (1/2, -1/2).
    r_1 = (ln 3, 0), r_2 = (-ln 3, ln 3): Swish = (3/4 ln 3, 0) and (-1/4 ln 3, 3/4 ln 3).
    """
    q = np.array([1.0, 2.0]).reshape(1, 1, 2, 1)
    k = np.array([1.0, 1.0]).reshape(1, 1, 2, 1)
    v = np.array([[2.0, 0.0], [0.0, 4.0]]).reshape(1, 1, 2, 2)
    z = np.array([-5.0, LN3]).reshape(1, 1, 2, 1)      # the first gate multiplies the zero state
    r = np.array([[LN3, 0.0], [-LN3, LN3]]).reshape(1, 1, 2, 2)
    w = np.array([[2.0, 3.0]])
    b = np.array([[0.5, -0.5]])
    o, fin = fo.gla_fused(q, k, v, z, 2.0, None, None, None, 0.0, 1, 2)
    np.testing.assert_allclose(o.reshape(2, 2), [[2.0, 0.0], [2 * math.sqrt(3.0), 8.0]], rtol=1e-15)
    np.testing.assert_allclose(fin.ravel(), [math.sqrt(3.0), 4.0], rtol=1e-15)
    y, fin2 = fo.gla_fused(q, k, v, z, 2.0, r, w, b, 0.0, 1, 2)
    np.testing.assert_allclose(y.reshape(2, 2), [[0.75 * LN3 * 2.5, 0.0], [0.375 * LN3, 1.875 * LN3]], rtol=1e-14,
                               atol=1e-15)
    np.testing.assert_array_equal(fin, fin2)


def test_fused_composition_and_scan_orders():
    rng = np.random.default_rng(2)
    B, H, gh, gw, dk, dv = 1, 2, 3, 4, 3, 5
    T = gh * gw
    q, k = rng.standard_normal((2, B, H, T, dk))
    v, r = rng.standard_normal((2, B, H, T, dv))
    z = rng.standard_normal((B, H, T, dk)) * 2
    w, b = rng.standard_normal((2, H, dv))
    for scan in range(4):
        y, fin = fo.gla_fused(q, k, v, z, 16.0, r, w, b, 1e-5, gh, gw, scan)
        # the epilogue is token-wise: it commutes with the permutation that the scan order applies
        perm = gla_oracle.scan_order(scan, gh, gw)
        yp, finp = fo.gla_fused(q[:, :, perm], k[:, :, perm], v[:, :, perm], z[:, :, perm], 16.0, r[:, :, perm],
                                w, b, 1e-5, 1, T, 0)
        np.testing.assert_allclose(y[:, :, perm], yp, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(fin, finp, rtol=1e-12, atol=1e-12)
    # all gates wide open (z -> +inf): plain causal linear attention, by brute force over token pairs
    o, _ = fo.gla_fused(q, k, v, np.full_like(z, 60.0), 16.0, None, None, None, 0.0, 1, T, 0)
    a = np.tril(np.einsum("bhic,bhjc->bhij", q, k))
    np.testing.assert_allclose(o, np.einsum("bhij,bhjn->bhin", a, v), rtol=1e-10, atol=1e-10)
