"""Host-side input recipe: determinism, distributions, bf16 rounding."""
import numpy as np
import torch

from paper_2405_18428_amd import inputs as gi


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(100000).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40, -65504.0]  # ties and extremes
    bits = gi.round_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    np.testing.assert_array_equal(gi.bf16_bits_to_f32(bits), t.float().numpy())


def test_recipe_is_deterministic_and_shaped():
    cfg = gi.CONFIGS["dig_s2_256"]
    a = gi.make_config_inputs(cfg)
    b = gi.make_config_inputs(cfg)
    for name in ("q", "k", "v", "log_alpha", "q_bits"):
        np.testing.assert_array_equal(a[name], b[name])
    assert a["q"].shape == (8, 6, 256, 32) and a["v"].shape == (8, 6, 256, 64)
    assert a["log_alpha"].dtype == np.float32 and (a["log_alpha"] <= 0).all()
    # q carries the dk^-0.5 scale, k and v are unit normal
    assert abs(a["q"].std() * 32 ** 0.5 - 1) < 0.02
    assert abs(a["k"].std() - 1) < 0.02 and abs(a["v"].std() - 1) < 0.02


def test_log_alpha_is_logsigmoid_over_tau():
    z = np.linspace(-30, 30, 241).astype(np.float32)
    got = gi.log_sigmoid_f32(z) / np.float32(16)
    ref = torch.nn.functional.logsigmoid(torch.from_numpy(z).double()).numpy() / 16
    np.testing.assert_allclose(got, ref, rtol=2e-6, atol=1e-9)


def test_contract_configs_present():
    assert gi.CONFIG_ORDER == ["tiny_f32", "dig_s2_256", "dig_xl2_512", "dig_xl2_1024", "dig_xl2_2048"]
    c = gi.CONFIGS["dig_xl2_2048"]
    assert (c.B, c.H, c.T, c.dk, c.dv, c.dtype) == (1, 16, 16384, 36, 72, "bf16")


def test_gate_input_recipes_extend_the_plain_ones():
    """The two-sided-gate generators leave q, k, v and the key-side gate exactly as the plain recipes draw them and
    add the value-side tensors from generators of their own."""
    a = gi.make_inputs(1, 2, 40, 8, 16, "bf16", seed=5, z_mean=0.5)
    g = gi.make_gate_inputs(1, 2, 40, 8, 16, "bf16", seed=5, z_mean=0.5)
    for name in ("q", "k", "v", "log_alpha", "q_bits"):
        np.testing.assert_array_equal(a[name], g[name])
    lb = g["log_beta"]
    assert lb.shape == (1, 2, 40, 16) and lb.dtype == np.float32 and (lb <= 0).all() and (lb > -2).all()
    np.testing.assert_array_equal(lb, gi.make_gate_inputs(1, 2, 40, 8, 16, "bf16", seed=5, z_mean=0.5)["log_beta"])
    f = gi.make_fused_inputs(1, 2, 40, 8, 16, "bf16", seed=5)
    fg = gi.make_fused_gate_inputs(1, 2, 40, 8, 16, "bf16", seed=5)
    for name in ("q", "k", "v", "z", "r", "ln_w", "ln_b"):
        np.testing.assert_array_equal(f[name], fg[name])
    assert fg["zb"].shape == (1, 2, 40, 16)
    np.testing.assert_array_equal(gi.bf16_bits_to_f32(fg["zb_bits"]), fg["zb"])   # bf16-representable
