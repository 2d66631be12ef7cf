"""Pins of the backward oracle (oracle/gla_oracle_bwd.c) against things other than itself: a hand-worked scalar
example, central finite differences of the forward oracle, closed forms for one token and for absent decay
(brute-force causal linear attention), and the reverse-cumulative-sum identity of the gate gradient."""
import os

import numpy as np
import pytest

from oracle import gla_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_problem(rng, B, H, gh, gw, dk, dv, decay=0.3):
    T = gh * gw
    q, k = rng.standard_normal((2, B, H, T, dk))
    v, w = rng.standard_normal((2, B, H, T, dv))
    g = -np.abs(rng.standard_normal((B, H, T, dk))) * decay
    return q, k, v, g, w


def test_two_token_scalar_example_from_golden_file():
    vals = {}
    for line in open(os.path.join(HERE, "golden", "two_token_backward.txt")):
        if line.strip() and not line.startswith("#"):
            name, x = line.split()
            vals[name] = float(x)
    q = np.array([0.5, -1.5]).reshape(1, 1, 2, 1)
    k = np.array([2.0, 0.25]).reshape(1, 1, 2, 1)
    v = np.array([-1.0, 3.0]).reshape(1, 1, 2, 1)
    w = np.array([0.75, -2.0]).reshape(1, 1, 2, 1)
    g = np.array([-0.7, np.log(0.5)]).reshape(1, 1, 2, 1)
    dq, dk, dv, dg = orc.gla_bwd(q, k, v, g, w, 1, 2, orc.SCAN_ROW_FWD)
    got = {"dq0": dq[0, 0, 0, 0], "dq1": dq[0, 0, 1, 0], "dk0": dk[0, 0, 0, 0], "dk1": dk[0, 0, 1, 0],
           "dv0": dv[0, 0, 0, 0], "dv1": dv[0, 0, 1, 0], "dg0": dg[0, 0, 0, 0], "dg1": dg[0, 0, 1, 0]}
    for name, x in vals.items():
        assert got[name] == pytest.approx(x, abs=1e-13), name


@pytest.mark.parametrize("scan", [0, 1, 2, 3])
def test_central_differences_of_the_forward_oracle(scan):
    """dL/dx for L = sum(out * w), every input tensor, sampled entries; T = 170 crosses a checkpoint block."""
    rng = np.random.default_rng(100 + scan)
    B, H, gh, gw, dk, dv = 1, 2, 10, 17, 3, 2
    q, k, v, g, w = rand_problem(rng, B, H, gh, gw, dk, dv, decay=0.05)
    grads = orc.gla_bwd(q, k, v, g, w, gh, gw, scan)

    def loss(args):
        return float((orc.gla_fwd(args[0], args[1], args[2], args[3], gh, gw, scan)[0] * w).sum())

    h = 1e-6
    for which, grad in enumerate(grads):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in grad.shape)
            args = [q.copy(), k.copy(), v.copy(), g.copy()]
            args[which][idx] += h
            up = loss(args)
            args[which][idx] -= 2 * h
            fd = (up - loss(args)) / (2 * h)
            assert grad[idx] == pytest.approx(fd, rel=1e-6, abs=1e-7), (which, idx)


def test_single_token_closed_form():
    """T = 1: o = (q.k) v, so dq = (w.v) k, dk = (w.v) q, dv = (q.k) w and the gate has no effect."""
    rng = np.random.default_rng(5)
    q, k, v, g, w = rand_problem(rng, 2, 3, 1, 1, 4, 5)
    dq, dk, dv, dg = orc.gla_bwd(q, k, v, g, w, 1, 1, 0)
    wv = (w * v).sum(-1, keepdims=True)
    qk = (q * k).sum(-1, keepdims=True)
    np.testing.assert_allclose(dq, wv * k, atol=1e-13)
    np.testing.assert_allclose(dk, wv * q, atol=1e-13)
    np.testing.assert_allclose(dv, qk * w, atol=1e-13)
    np.testing.assert_allclose(dg, 0.0, atol=0)


def test_absent_decay_is_causal_linear_attention():
    """log_alpha = 0: o_t = sum_{i<=t} (q_t.k_i) v_i; its gradients by explicit double loops (Eq. (attn_simple))."""
    rng = np.random.default_rng(6)
    B, H, gh, gw, dk, dv = 1, 2, 3, 5, 3, 4
    T = gh * gw
    q, k, v, _, w = rand_problem(rng, B, H, gh, gw, dk, dv)
    g = np.zeros_like(q)
    for scan in range(4):
        pi = orc.scan_order(scan, gh, gw)
        dq, dk, dv_, _ = orc.gla_bwd(q, k, v, g, w, gh, gw, scan)
        rq, rk, rv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
        for b in range(B):
            for hh in range(H):
                for t in range(T):
                    for i in range(t + 1):
                        nt, ni = pi[t], pi[i]
                        wv = w[b, hh, nt] @ v[b, hh, ni]
                        qk = q[b, hh, nt] @ k[b, hh, ni]
                        rq[b, hh, nt] += wv * k[b, hh, ni]
                        rk[b, hh, ni] += wv * q[b, hh, nt]
                        rv[b, hh, ni] += qk * w[b, hh, nt]
        np.testing.assert_allclose(dq, rq, atol=1e-12)
        np.testing.assert_allclose(dk, rk, atol=1e-12)
        np.testing.assert_allclose(dv_, rv, atol=1e-12)


def test_gate_gradient_is_a_reverse_cumulative_sum():
    """In the unrolled form of Eq. (attn_gla), o_t = sum_{i<=t} sum_c q_t[c] k_i[c] exp(sum_{m=i+1..t} g_m[c]) v_i,
    the gate g_s[c] sits in exactly the terms with i < s <= t.  q_t[c] dL/dq_t[c] collects the terms of output
    step t, k_i[c] dL/dk_i[c] those of input step i; summed over steps >= s, the first gives the terms with
    t >= s and the second those with i >= s, and their difference is the terms with i < s <= t:
    dL/dg_s = sum_{s' >= s} (q * dq - k * dk).  The oracle computes the left side from its definition."""
    rng = np.random.default_rng(7)
    B, H, gh, gw, dk, dv = 2, 2, 6, 7, 4, 3
    q, k, v, g, w = rand_problem(rng, B, H, gh, gw, dk, dv, decay=0.2)
    for scan in range(4):
        pi = orc.scan_order(scan, gh, gw)
        dq, dk, _, dg = orc.gla_bwd(q, k, v, g, w, gh, gw, scan)
        term = (q * dq - k * dk)[:, :, pi]                       # in scan order
        suffix = np.flip(np.cumsum(np.flip(term, axis=2), axis=2), axis=2)
        np.testing.assert_allclose(dg[:, :, pi], suffix, atol=1e-11)


def test_linear_in_the_upstream_gradient_and_zero_for_zero():
    rng = np.random.default_rng(8)
    q, k, v, g, w = rand_problem(rng, 1, 2, 4, 5, 3, 3)
    w2 = rng.standard_normal(w.shape)
    a = orc.gla_bwd(q, k, v, g, w, 4, 5, 2)
    b = orc.gla_bwd(q, k, v, g, w2, 4, 5, 2)
    c = orc.gla_bwd(q, k, v, g, 2.0 * w - 3.0 * w2, 4, 5, 2)
    for x, y, z in zip(a, b, c):
        np.testing.assert_allclose(z, 2.0 * x - 3.0 * y, atol=1e-11)
    for x in orc.gla_bwd(q, k, v, g, np.zeros_like(w), 4, 5, 2):
        assert np.all(x == 0.0)


def test_first_scan_step_gate_has_zero_gradient_and_threads_agree():
    rng = np.random.default_rng(9)
    q, k, v, g, w = rand_problem(rng, 2, 2, 5, 4, 3, 2)
    for scan in range(4):
        first = orc.scan_order(scan, 5, 4)[0]
        one = orc.gla_bwd(q, k, v, g, w, 5, 4, scan, nthreads=1)
        many = orc.gla_bwd(q, k, v, g, w, 5, 4, scan)
        assert np.all(one[3][:, :, first] == 0.0)
        for x, y in zip(one, many):
            assert np.array_equal(x, y)
