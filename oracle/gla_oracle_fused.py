"""CPU fp64 oracle for the GLA mixer with its gate prologue and its output epilogue.

TEST INFRASTRUCTURE ONLY (same rules as ``gla_oracle.py``: used by the tests, the smoke check and the
benchmark's CPU leg; never imported by the product package, and never importing it).

The steps, in the paper's order and notation (Sec. 3.1):

* Eq. (gate_gla):        alpha_t = sigmoid(z_t)^(1/tau), z = X W_alpha + b_alpha given as input;
                         log alpha_t = logsigmoid(z_t) / tau
* Eq. (attn_gla) rows 1-3 with beta = 1:  the recurrence of ``gla_oracle.gla_fwd`` -> O_t
* Eq. (attn_gla) row 4:  R_t = Swish(r_t), r = X W_r + b_r given as input; Swish(x) = x * sigmoid(x)
* Eq. (attn_gla) row 5, before the output projection:  Y_t = R_t * LN(O_t)

LN normalises the d_v entries of one head's O_t (mean and biased variance over d_v, eps inside the square
root) and applies an affine map with per-head weight and bias rows ``[H, d_v]``.
"""
from __future__ import annotations

import numpy as np

from . import gla_oracle


def log_sigmoid(z):
    """log(sigmoid(z)) in fp64, written so that neither branch overflows."""
    z = np.asarray(z, dtype=np.float64)
    return -(np.maximum(-z, 0.0) + np.log1p(np.exp(-np.abs(z))))


def log_alpha_from_z(z, tau):
    """Eq. (gate_gla): log of alpha = sigmoid(z)^(1/tau)."""
    return log_sigmoid(z) / float(tau)


def swish(x):
    """Swish with unit slope parameter: x * sigmoid(x) (Eq. (attn_gla) row 4)."""
    x = np.asarray(x, dtype=np.float64)
    return x * np.exp(log_sigmoid(x))


def layer_norm_heads(o, weight=None, bias=None, eps=1e-5):
    """LN over the last axis of o [B,H,T,dv]; weight, bias: [H,dv] or None (1 and 0)."""
    o = np.asarray(o, dtype=np.float64)
    B, H, T, dv = o.shape
    mean = o.mean(axis=-1, keepdims=True)
    var = ((o - mean) ** 2).mean(axis=-1, keepdims=True)
    y = (o - mean) / np.sqrt(var + float(eps))
    if weight is not None:
        y = y * np.asarray(weight, dtype=np.float64).reshape(1, H, 1, dv)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, H, 1, dv)
    return y


def gla_fused(q, k, v, z, tau, r_pre, ln_weight, ln_bias, ln_eps, grid_h, grid_w,
              scan_dir=gla_oracle.SCAN_ROW_FWD, nthreads=0):
    """Gate prologue + recurrence + (if r_pre is given) Swish gate times LayerNorm.

    Returns (y [B,H,T,dv], final_state [B,H,dk,dv]) in float64; with ``r_pre is None`` y is the plain O.
    """
    log_alpha = log_alpha_from_z(z, tau)
    o, fin = gla_oracle.gla_fwd(q, k, v, log_alpha, grid_h, grid_w, scan_dir, nthreads=nthreads)
    if r_pre is None:
        return o, fin
    return swish(r_pre) * layer_norm_heads(o, ln_weight, ln_bias, ln_eps), fin


def gla_fused_gates(q, k, v, z_alpha, z_beta, tau, r_pre, ln_weight, ln_bias, ln_eps, grid_h, grid_w,
                    scan_dir=gla_oracle.SCAN_ROW_FWD):
    """The whole mixer of Sec. 3.1 up to the projection W_O: both gates from their pre-activations
    (Eq. (gate_gla): alpha = sigmoid(z_alpha)^(1/tau); Eq. (gate_gla_2): beta = sigmoid(z_beta)^(1/tau)), the recurrence
    with G_t = alpha_t^T beta_t (Eq. (attn_gla) rows 1-3) and, if ``r_pre`` is given, Swish(r) * LN(o) (rows 4-5).

    Returns (y [B,H,T,dv], final_state [B,H,dk,dv]) in float64.
    """
    from . import gla_oracle_gates
    o, fin = gla_oracle_gates.gla_fwd_gates(q, k, v, log_alpha_from_z(z_alpha, tau), log_alpha_from_z(z_beta, tau),
                                            grid_h, grid_w, scan_dir)
    if r_pre is None:
        return o, fin
    return swish(r_pre) * layer_norm_heads(o, ln_weight, ln_bias, ln_eps), fin
