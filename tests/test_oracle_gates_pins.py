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


def test_fused_gates_two_tokens_by_hand():
    """dk = 1, dv = 2, two tokens, tau = 1, every step written out: gates sigmoid(z), state, output, LayerNorm over
    the two value columns (mean of two numbers, variance ((a-b)/2)^2), Swish gate."""
    from oracle import gla_oracle_fused as fo
    q = np.array([[[[2.0], [3.0]]]]); k = np.array([[[[1.0], [0.5]]]])
    v = np.array([[[[1.0, -1.0], [2.0, 4.0]]]])
    za = np.array([[[[0.3], [np.log(3.0)]]]])                 # alpha_2 = 3/4
    zb = np.array([[[[0.1, 0.2], [0.0, np.log(1.0 / 3.0)]]]])  # beta_2 = (1/2, 1/4)
    r = np.array([[[[1.0, 2.0], [0.5, -1.0]]]])
    y, fin = fo.gla_fused_gates(q, k, v, za, zb, 1.0, r, None, None, 0.0, 1, 2, 0)
    # token 1: S = k v = (1, -1), o = 2 S = (2, -2); token 2: S = 3/4 (1/2, 1/4) * (1, -1) + 0.5 (2, 4)
    s2 = np.array([0.75 * 0.5 * 1.0 + 1.0, 0.75 * 0.25 * -1.0 + 2.0])
    np.testing.assert_allclose(fin[0, 0, 0], s2, rtol=1e-14)
    o1, o2 = np.array([2.0, -2.0]), 3.0 * s2
    sw = lambda x: x / (1.0 + np.exp(-x))
    ln = lambda o: (o - o.mean()) / abs((o[0] - o[1]) / 2.0)      # eps = 0: a two-entry row normalises to (+-1)
    np.testing.assert_allclose(y[0, 0, 0], sw(r[0, 0, 0]) * ln(o1), rtol=1e-13)
    np.testing.assert_allclose(y[0, 0, 1], sw(r[0, 0, 1]) * ln(o2), rtol=1e-13)


def test_fused_gates_large_negative_z_beta_forgets_the_past():
    """beta -> 0 on every column wipes the previous state: each output is q_t (k_t^T v_t)."""
    from oracle import gla_oracle_fused as fo
    q, k, v, la, lb = _rand(1, 1, 2, 3, 3, 2, 9)
    z_a = np.zeros_like(la)
    z_b = np.full_like(lb, -800.0)
    o, _ = fo.gla_fused_gates(q, k, v, z_a, z_b, 1.0, None, None, None, 0.0, 2, 3, 0)
    expect = np.einsum("bhtc,bhtc->bht", q, k)[..., None] * v
    np.testing.assert_allclose(o, expect, rtol=1e-12, atol=1e-12)


# ---- reverse mode of the two-sided-gate recurrence ----

def _loss(q, k, v, la, lb, w, gh, gw, d):
    o, _ = og.gla_fwd_gates(q, k, v, la, lb, gh, gw, d)
    return float((o * w).sum())


@pytest.mark.parametrize("d", [0, 1, 2, 3])
def test_backward_matches_central_differences(d):
    """Every gradient entry against (L(x + h) - L(x - h)) / 2h for L = <out, w> (fp64, h = 1e-6)."""
    gh, gw = 2, 3
    q, k, v, la, lb = _rand(1, 2, gh, gw, 3, 2, 20 + d)
    w = np.random.default_rng(30 + d).standard_normal(v.shape)
    grads = og.gla_bwd_gates(q, k, v, la, lb, w, gh, gw, d)
    args = [q, k, v, la, lb]
    h = 1e-6
    for a_i, g in enumerate(grads):
        x = args[a_i]
        num = np.empty_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            keep = x[idx]
            x[idx] = keep + h
            lp = _loss(*args, w, gh, gw, d)
            x[idx] = keep - h
            lm = _loss(*args, w, gh, gw, d)
            x[idx] = keep
            num[idx] = (lp - lm) / (2 * h)
        np.testing.assert_allclose(g, num, rtol=2e-6, atol=2e-8)


def test_backward_with_unit_beta_is_the_key_side_backward():
    q, k, v, la, lb = _rand(2, 2, 4, 5, 3, 4, 41)
    w = np.random.default_rng(42).standard_normal(v.shape)
    for d in (0, 3):
        dq, dk, dvv, dla, dlb = og.gla_bwd_gates(q, k, v, la, np.zeros_like(lb), w, 4, 5, d)
        r = orc.gla_bwd(q, k, v, la, w, 4, 5, d)
        for got, ref in zip((dq, dk, dvv, dla), r):
            np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_gate_gradients_are_reverse_cumulative_sums():
    """d log alpha = reverse cumulative sum over the scan of (q * dq - k * dk); d log beta likewise of
    (o * dO - v * dv): the identities the GPU path evaluates, checked on the oracle's direct formulas."""
    gh, gw, d = 3, 4, 2
    q, k, v, la, lb = _rand(1, 2, gh, gw, 3, 4, 43)
    w = np.random.default_rng(44).standard_normal(v.shape)
    dq, dk, dvv, dla, dlb = og.gla_bwd_gates(q, k, v, la, lb, w, gh, gw, d)
    o, _ = og.gla_fwd_gates(q, k, v, la, lb, gh, gw, d)
    pi = orc.scan_order(d, gh, gw)
    ta = (q * dq - k * dk)[:, :, pi, :]
    tb = (o * w - v * dvv)[:, :, pi, :]
    ra = np.flip(np.cumsum(np.flip(ta, 2), 2), 2)
    rb = np.flip(np.cumsum(np.flip(tb, 2), 2), 2)
    np.testing.assert_allclose(dla[:, :, pi, :], ra, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dlb[:, :, pi, :], rb, rtol=1e-10, atol=1e-12)
