"""CPU fp64 oracle for the GLA recurrence with the full gate matrix of DiG (key-side and value-side factors).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the ``cpu_baseline`` leg of the benchmark may
import this module; the product package never does, and this module never imports the product package.

Sec. 3.1 builds the gate of a token as an outer product, G_t = alpha_t^T beta_t, with alpha_t in (0,1)^{1 x dk}
(Eq. (gate_gla)) and beta_t in (0,1)^{1 x dv} (Eq. (gate_gla_2)), and applies it element-wise to the previous
state (Eq. (attn_gla), rows 1-3):

    S_t = (alpha_t^T beta_t) * S_{t-1} + k_t^T v_t ,     o_t = q_t S_t ,     S_0 = initial state (or 0),

run along a scan order of the token grid (Sec. 3.3 / Algorithm 1).  :func:`gla_fwd_gates` is that recurrence taken
token by token in numpy float64 (vectorised over batch and head only); the gates arrive as logarithms.
With ``log_beta = 0`` it is the recurrence of ``gla_oracle.gla_fwd``.
"""
from __future__ import annotations

import numpy as np

from .gla_oracle import scan_order


def gla_fwd_gates(q, k, v, log_alpha, log_beta, grid_h, grid_w, scan_dir=0, initial_state=None):
    """q, k, log_alpha: [B,H,T,dk]; v, log_beta: [B,H,T,dv].  Returns (out [B,H,T,dv], final_state [B,H,dk,dv])."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    lb = np.asarray(log_beta, dtype=np.float64)
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    if k.shape != q.shape or la.shape != q.shape or v.shape != (B, H, T, dv) or lb.shape != v.shape:
        raise ValueError("shape mismatch")
    if grid_h * grid_w != T:
        raise ValueError("grid does not match T")
    pi = scan_order(scan_dir, grid_h, grid_w)
    S = np.zeros((B, H, dk, dv)) if initial_state is None else np.array(initial_state, dtype=np.float64)
    out = np.empty((B, H, T, dv))
    for s in range(T):
        n = pi[s]
        G = np.exp(la[:, :, n, :, None] + lb[:, :, n, None, :])          # alpha_t^T beta_t
        S = G * S + k[:, :, n, :, None] * v[:, :, n, None, :]            # decayed state plus k_t^T v_t
        out[:, :, n, :] = np.einsum("bhc,bhcn->bhn", q[:, :, n, :], S)   # o_t = q_t S_t
    return out, S


def gla_bwd_gates(q, k, v, log_alpha, log_beta, d_out, grid_h, grid_w, scan_dir=0):
    """Reverse-mode derivative of :func:`gla_fwd_gates` (zero initial state) for a given d_out = dL/d out.

    The forward recurrence is replayed keeping every state S_s; the adjoint state G_s = dL/dS_s is then carried
    backwards over the scan: G_s = q_s^T dO_s + (alpha_{s+1}^T beta_{s+1}) * G_{s+1}, and at every step
        dq_s = S_s dO_s^T,  dk_s = G_s v_s^T,  dv_s = k_s G_s,
        d log alpha_s[c] = sum_n (G_s * A_s * S_{s-1})[c, n],   d log beta_s[n] = sum_c (G_s * A_s * S_{s-1})[c, n],
    with A_s = alpha_s^T beta_s (the derivative of exp(la + lb) w.r.t. either logarithm is A_s itself).
    Returns (dq, dk, dv, dlog_alpha, dlog_beta) in float64, shaped like q, k, v, log_alpha, log_beta.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_alpha, dtype=np.float64)
    lb = np.asarray(log_beta, dtype=np.float64)
    do = np.asarray(d_out, dtype=np.float64)
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    if T * B * H * dk * dv * 8 > (4 << 30):
        raise ValueError("too large for the state history kept by this oracle")
    pi = scan_order(scan_dir, grid_h, grid_w)
    hist = np.empty((T + 1, B, H, dk, dv))
    hist[0] = 0.0
    for s in range(T):
        n = pi[s]
        A = np.exp(la[:, :, n, :, None] + lb[:, :, n, None, :])
        hist[s + 1] = A * hist[s] + k[:, :, n, :, None] * v[:, :, n, None, :]
    dq, dkk, dvv = np.empty_like(q), np.empty_like(k), np.empty_like(v)
    dla, dlb = np.empty_like(la), np.empty_like(lb)
    G = np.zeros((B, H, dk, dv))
    for s in range(T - 1, -1, -1):
        n = pi[s]
        G = G + q[:, :, n, :, None] * do[:, :, n, None, :]           # dL/dS_s, all later uses included
        dq[:, :, n, :] = np.einsum("bhcn,bhn->bhc", hist[s + 1], do[:, :, n, :])
        dkk[:, :, n, :] = np.einsum("bhcn,bhn->bhc", G, v[:, :, n, :])
        dvv[:, :, n, :] = np.einsum("bhc,bhcn->bhn", k[:, :, n, :], G)
        A = np.exp(la[:, :, n, :, None] + lb[:, :, n, None, :])
        GAS = G * A * hist[s]
        dla[:, :, n, :] = GAS.sum(-1)
        dlb[:, :, n, :] = GAS.sum(-2)
        G = A * G                                                    # what reaches S_{s-1}
    return dq, dkk, dvv, dla, dlb
