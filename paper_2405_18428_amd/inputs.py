"""Seeded synthetic inputs for the GLA forward path (host side, numpy only).

This module is the one piece shared by the GPU tests / benchmark and the CPU
oracle's tests.  It holds none of the method's arithmetic: it only draws the
tensors that stand in for the activations of a DiG block (the q/k/v
projections and the pre-activation z of the gate alpha = sigmoid(z)^(1/tau),
Sec. 3.1, Eq. (qkv_gla) and Eq. (gate_gla)), with the head counts and head
dimensions of the DiG-S/2 and DiG-XL/2 sizes (Table "model variants": D = 384
and D = 1152) at 256 to 2048 px (T = (px/16)^2 tokens for patch size 2 on the
8x down-sampled latent, Sec. 3.2).

Recipe (fixed; every consumer gets bit-identical arrays for a given config):
  * generator numpy.random.Generator(PCG64(seed)), draw order q, k, v, z, each
    standard_normal(float32) of its full shape;
  * q is multiplied by dk**-0.5 in fp32 (the path itself applies no scale);
  * z = z_mean + z;  log_alpha = logsigmoid(z) / tau in fp32, computed as
    -(max(-z, 0) + log1p(exp(-|z|))) / tau, tau = 16;
  * for bf16 configs q, k, v are rounded fp32 -> bf16 round-to-nearest-even;
    the rounded values are what both sides consume, so input quantisation is
    not part of any error.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

TAU = 16.0

SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV = 0, 1, 2, 3
ALL_SCANS = (SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV)


@dataclass(frozen=True)
class GlaConfig:
    name: str
    B: int
    H: int
    grid_h: int
    grid_w: int
    dk: int
    dv: int
    dtype: str                      # "f32" or "bf16": element type of q, k, v
    scans: Tuple[int, ...] = (SCAN_ROW_FWD,)
    z_mean: float = 0.0
    seed: int = 0

    @property
    def T(self) -> int:
        return self.grid_h * self.grid_w


# The five workloads of the build contract, plus the long-memory variant of the
# headline shape (gates near 1) and the 1792 px shape the paper's Fig. 1 quotes.
CONFIGS: Dict[str, GlaConfig] = {c.name: c for c in [
    GlaConfig("tiny_f32", 1, 2, 16, 16, 32, 64, "f32", (SCAN_ROW_FWD,)),
    GlaConfig("dig_s2_256", 8, 6, 16, 16, 32, 64, "bf16", ALL_SCANS),
    GlaConfig("dig_xl2_512", 4, 16, 32, 32, 36, 72, "bf16", (SCAN_ROW_FWD, SCAN_COL_REV)),
    GlaConfig("dig_xl2_1024", 2, 16, 64, 64, 36, 72, "bf16", ALL_SCANS),
    GlaConfig("dig_xl2_2048", 1, 16, 128, 128, 36, 72, "bf16", (SCAN_ROW_FWD,)),
    GlaConfig("dig_xl2_2048_longmem", 1, 16, 128, 128, 36, 72, "bf16", (SCAN_ROW_FWD,), z_mean=3.0),
    GlaConfig("dig_s2_1792", 1, 6, 112, 112, 32, 64, "bf16", (SCAN_ROW_FWD,)),
    GlaConfig("dig_s2_1792_longmem", 1, 6, 112, 112, 32, 64, "bf16", (SCAN_ROW_FWD,), z_mean=3.0),
    GlaConfig("dig_xl2_1792", 1, 16, 112, 112, 36, 72, "bf16", (SCAN_ROW_FWD,)),
]}
CONFIG_ORDER = ["tiny_f32", "dig_s2_256", "dig_xl2_512", "dig_xl2_1024", "dig_xl2_2048"]


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even; NaN kept quiet."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + rounding) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def log_sigmoid_f32(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.float32)
    return -(np.maximum(-z, np.float32(0)) + np.log1p(np.exp(-np.abs(z)))).astype(np.float32)


def make_inputs(B, H, T, dk, dv, dtype="bf16", seed=0, z_mean=0.0, tau=TAU):
    """Returns a dict of host arrays.

    'q','k','v'      float32 arrays holding the values the path consumes
                     (already rounded to bf16 values when dtype == "bf16");
    'q_bits', ...    uint16 bf16 bit patterns (bf16 configs only);
    'log_alpha'      float32 [B,H,T,dk], <= 0.
    """
    if dtype not in ("f32", "bf16"):
        raise ValueError("dtype must be 'f32' or 'bf16'")
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    k = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    v = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    z = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    q = (q * np.float32(dk ** -0.5)).astype(np.float32)
    z = (z + np.float32(z_mean)).astype(np.float32)
    log_alpha = (log_sigmoid_f32(z) / np.float32(tau)).astype(np.float32)
    d = {"log_alpha": log_alpha, "dtype": dtype}
    if dtype == "bf16":
        for name, a in (("q", q), ("k", k), ("v", v)):
            bits = round_to_bf16_bits(a)
            d[name + "_bits"] = bits
            d[name] = bf16_bits_to_f32(bits)
    else:
        d.update(q=q, k=k, v=v)
    return d


def make_fused_inputs(B, H, T, dk, dv, dtype="bf16", seed=0, z_mean=0.0):
    """Inputs of the forward pass with gate prologue and output epilogue: q, k, v and the gate pre-activation z
    drawn exactly as in :func:`make_inputs` (same generator, same order), plus the output-gate pre-activation
    ``r`` (standard normal, shaped like v) and LayerNorm rows ``ln_w = 1 + 0.1 n``, ``ln_b = 0.1 n`` of shape
    [H, dv] from a second generator.  For "bf16" q, k, v, z, r hold bf16-representable values and the
    ``*_bits`` entries their bit patterns."""
    if dtype not in ("f32", "bf16"):
        raise ValueError("dtype must be 'f32' or 'bf16'")
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    k = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    v = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    z = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    q = (q * np.float32(dk ** -0.5)).astype(np.float32)
    z = (z + np.float32(z_mean)).astype(np.float32)
    rng2 = np.random.Generator(np.random.PCG64(seed + 2000))
    r = rng2.standard_normal((B, H, T, dv), dtype=np.float32)
    ln_w = (np.float32(1) + np.float32(0.1) * rng2.standard_normal((H, dv), dtype=np.float32)).astype(np.float32)
    ln_b = (np.float32(0.1) * rng2.standard_normal((H, dv), dtype=np.float32)).astype(np.float32)
    d = {"dtype": dtype, "ln_w": ln_w, "ln_b": ln_b}
    for name, a in (("q", q), ("k", k), ("v", v), ("z", z), ("r", r)):
        if dtype == "bf16":
            bits = round_to_bf16_bits(a)
            d[name + "_bits"] = bits
            d[name] = bf16_bits_to_f32(bits)
        else:
            d[name] = a
    return d


def make_gate_inputs(B, H, T, dk, dv, dtype="bf16", seed=0, z_mean=0.0, tau=TAU):
    """:func:`make_inputs` plus ``log_beta`` [B,H,T,dv] (fp32, <= 0) for the value-side gate: logsigmoid of a
    standard-normal pre-activation (+ z_mean) from a second generator, divided by tau like log_alpha."""
    d = make_inputs(B, H, T, dk, dv, dtype, seed, z_mean, tau)
    rng2 = np.random.Generator(np.random.PCG64(seed + 3000))
    zb = (rng2.standard_normal((B, H, T, dv), dtype=np.float32) + np.float32(z_mean)).astype(np.float32)
    d["log_beta"] = (log_sigmoid_f32(zb) / np.float32(tau)).astype(np.float32)
    return d


def make_fused_gate_inputs(B, H, T, dk, dv, dtype="bf16", seed=0, z_mean=0.0):
    """:func:`make_fused_inputs` plus ``zb`` [B,H,T,dv], the pre-activation of the value-side gate (standard normal
    + z_mean, third generator; bf16-representable with its ``zb_bits`` for "bf16")."""
    d = make_fused_inputs(B, H, T, dk, dv, dtype, seed, z_mean)
    rng3 = np.random.Generator(np.random.PCG64(seed + 4000))
    zb = (rng3.standard_normal((B, H, T, dv), dtype=np.float32) + np.float32(z_mean)).astype(np.float32)
    if dtype == "bf16":
        d["zb_bits"] = round_to_bf16_bits(zb)
        d["zb"] = bf16_bits_to_f32(d["zb_bits"])
    else:
        d["zb"] = zb
    return d


def make_config_inputs(cfg: GlaConfig):
    return make_inputs(cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv, cfg.dtype, cfg.seed, cfg.z_mean)
