"""Pins of the two-sided-gate oracle (``oracle/gla_oracle_gates.py``) against what the paper and the mathematics fix.

Sec. 3.1: G_t = alpha_t^T beta_t (Eqs. (gate_gla), (gate_gla_2)) applied element-wise in Eq. (attn_gla) rows 1-3.
"""
import numpy as np
import pytest

from oracle import gla_oracle as orc
from oracle import gla_oracle_gates as og


def _rand(B, H, gh, gw, dk, dv, seed):
    rng = np.random.default_rng(seed)
    T = gh * gw
    q = rng.standard_normal((B, H, T, dk))
    k = rng.standard_normal((B, H, T, dk))
    v = rng.standard_normal((B, H, T, dv))
    la = -rng.uniform(0.01, 0.5, (B, H, T, dk))
    lb = -rng.uniform(0.01, 0.5, (B, H, T, dv))
    return q, k, v, la, lb


def test_unit_beta_is_the_key_side_recurrence():
    q, k, v, la, lb = _rand(2, 2, 4, 5, 3, 4, 1)
    for d in range(4):
        o1, f1 = og.gla_fwd_gates(q, k, v, la, np.zeros_like(lb), 4, 5, d)
        o0, f0 = orc.gla_fwd(q, k, v, la, 4, 5, d)
        np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(f1, f0, rtol=1e-12, atol=1e-12)


def test_unrolled_definition_brute_force():
    """o_t[n] = sum_{i<=t} sum_c q_t[c] k_i[c] v_i[n] prod_{i<s<=t} alpha_s[c] beta_s[n]: the recurrence unrolled by
    hand (token t's own gate never touches its own k_t^T v_t, and the gate at the first step decays only S_0 = 0)."""
    q, k, v, la, lb = _rand(1, 1, 1, 7, 3, 2, 2)
    out, fin = og.gla_fwd_gates(q, k, v, la, lb, 1, 7, 0)
    T, dk, dv = 7, 3, 2
    for t in range(T):
        for n in range(dv):
            acc = 0.0
            for i in range(t + 1):
                for c in range(dk):
                    w = 1.0
                    for s in range(i + 1, t + 1):
                        w *= np.exp(la[0, 0, s, c]) * np.exp(lb[0, 0, s, n])
                    acc += q[0, 0, t, c] * k[0, 0, i, c] * v[0, 0, i, n] * w
            assert abs(out[0, 0, t, n] - acc) < 1e-12
    # the final state from the same unrolling
    for c in range(dk):
        for n in range(dv):
            acc = 0.0
            for i in range(T):
                w = np.exp(la[0, 0, i + 1:, c].sum() + lb[0, 0, i + 1:, n].sum())
                acc += k[0, 0, i, c] * v[0, 0, i, n] * w
            assert abs(fin[0, 0, c, n] - acc) < 1e-12


def test_column_uniform_beta_folds_into_alpha():
    """If beta_t is the same number b_t for every value column, G_t = (b_t alpha_t)^T 1: the key-side recurrence with
    log_alpha + log b (checked against the C oracle of that recurrence)."""
    q, k, v, la, lb = _rand(1, 2, 3, 4, 4, 5, 3)
    lb_u = np.repeat(lb[..., :1], lb.shape[-1], axis=-1)
    o1, f1 = og.gla_fwd_gates(q, k, v, la, lb_u, 3, 4, 2)
    o0, f0 = orc.gla_fwd(q, k, v, la + lb[..., :1], 3, 4, 2)
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(f1, f0, rtol=1e-12, atol=1e-12)


def test_state_is_symmetric_under_swapping_the_two_sides():
    """S^T obeys the same recurrence with (k, alpha) and (v, beta) exchanged."""
    q, k, v, la, lb = _rand(1, 1, 2, 5, 3, 4, 4)
    _, f = og.gla_fwd_gates(q, k, v, la, lb, 2, 5, 1)
    q2 = np.zeros_like(v)
    _, ft = og.gla_fwd_gates(q2, v, k, lb, la, 2, 5, 1)
    np.testing.assert_allclose(ft, np.swapaxes(f, -1, -2), rtol=1e-12, atol=1e-12)


def test_scalar_geometric_series():
    """dk = dv = 1, q = k = v = 1, constant gates a and b: S_t = sum_{i=0}^{t} (a b)^i."""
    T, a, b = 9, 0.8, 0.9
    one = np.ones((1, 1, T, 1))
    out, fin = og.gla_fwd_gates(one, one, one, np.log(a) * one, np.log(b) * one, 1, T, 0)
    r = a * b
    expect = np.array([(1 - r ** (t + 1)) / (1 - r) for t in range(T)])
    np.testing.assert_allclose(out[0, 0, :, 0], expect, rtol=1e-13)
    assert abs(fin[0, 0, 0, 0] - expect[-1]) < 1e-13


def test_initial_state_decays_on_both_sides():
    q, k, v, la, lb = _rand(1, 1, 1, 3, 2, 2, 5)
    s0 = np.random.default_rng(6).standard_normal((1, 1, 2, 2))
    zero = np.zeros_like
    out, fin = og.gla_fwd_gates(q, zero(k), zero(v), la, lb, 1, 3, 0, initial_state=s0)
    w = np.exp(la[0, 0].sum(0)[:, None] + lb[0, 0].sum(0)[None, :])
    np.testing.assert_allclose(fin[0, 0], s0[0, 0] * w, rtol=1e-12)
    w1 = np.exp(la[0, 0, 0][:, None] + lb[0, 0, 0][None, :])
    np.testing.assert_allclose(out[0, 0, 0], q[0, 0, 0] @ (s0[0, 0] * w1), rtol=1e-12)


@pytest.mark.parametrize("d", [2, 3])
def test_column_scans_are_row_scans_of_the_transposed_grid(d):
    gh, gw = 3, 4
    q, k, v, la, lb = _rand(1, 1, gh, gw, 2, 3, 7)
    o, f = og.gla_fwd_gates(q, k, v, la, lb, gh, gw, d)

    def tr(x):   # tokens of the transposed grid in row-major order
        return np.ascontiguousarray(x.reshape(1, 1, gh, gw, -1).swapaxes(2, 3).reshape(1, 1, gh * gw, -1))
    ot, ft = og.gla_fwd_gates(tr(q), tr(k), tr(v), tr(la), tr(lb), gw, gh, d - 2)
    np.testing.assert_allclose(tr(o), ot, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(f, ft, rtol=1e-12, atol=1e-12)
