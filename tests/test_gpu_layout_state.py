"""GPU parity of gla_fwd_layout: the [B,T,H,d] memory order and a non-zero initial state, against the CPU fp64
oracle (which works in [B,H,T,d]; the test permutes).  Same error metric and bars as test_gpu_parity.py."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    gla.load_library()
    yield
    for opt in (gla.OPT_CHUNKS_PER_SPAN, gla.OPT_ENGINE, gla.OPT_CARRY):
        gla.gla_set_option(opt, 0)


@pytest.fixture(autouse=True)
def _reset_options():
    for opt in (gla.OPT_CHUNKS_PER_SPAN, gla.OPT_ENGINE, gla.OPT_CARRY):
        gla.gla_set_option(opt, 0)
    yield


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(rms, 1e-300))


def to_gpu(d, name, layout):
    """Upload one input tensor in the requested memory order."""
    dev = torch.device("cuda:0")
    if name != "log_alpha" and d["dtype"] == "bf16":
        t = torch.from_numpy(d[name + "_bits"].view(np.int16))
        t = t.permute(0, 2, 1, 3).contiguous() if layout == gla.LAYOUT_BTHD else t
        return t.to(dev).view(torch.bfloat16)
    t = torch.from_numpy(d[name])
    t = t.permute(0, 2, 1, 3).contiguous() if layout == gla.LAYOUT_BTHD else t
    return t.to(dev)


def run(d, gh, gw, scan, layout, init=None):
    q, k, v, la = (to_gpu(d, n, layout) for n in ("q", "k", "v", "log_alpha"))
    s0 = None if init is None else torch.from_numpy(init).to(q.device)
    out, fin = gla.gla_fwd_layout(q, k, v, la, gh, gw, scan, layout=layout, initial_state=s0)
    torch.cuda.synchronize()
    out = out.float().cpu()
    if layout == gla.LAYOUT_BTHD:
        out = out.permute(0, 2, 1, 3)
    return out.numpy(), fin.cpu().numpy()


def make_init(B, H, dk, dv, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (3.0 * rng.standard_normal((B, H, dk, dv))).astype(np.float32)


PLANS = [
    # engine, carry, chunks per span (0 = automatic)
    (gla.ENGINE_MFMA, gla.CARRY_AUTO, 0),
    (gla.ENGINE_MFMA, gla.CARRY_IN_OUTPUT_PASS, 1),
    (gla.ENGINE_MFMA, gla.CARRY_KERNEL, 2),
    (gla.ENGINE_MFMA, gla.CARRY_AUTO, 1000),     # one span per sequence
    (gla.ENGINE_RECURRENT, gla.CARRY_AUTO, 0),
    (gla.ENGINE_RECURRENT, gla.CARRY_AUTO, 1000),
]


@pytest.mark.parametrize("engine,carry,cps", PLANS)
@pytest.mark.parametrize("layout", [gla.LAYOUT_BHTD, gla.LAYOUT_BTHD])
def test_layouts_and_initial_state_agree_with_oracle(engine, carry, cps, layout):
    """Every launch plan, both memory orders, zero and non-zero initial state, ragged tail, all four scan orders."""
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv = 2, 3, 13, 23, 36, 72     # T = 299: four full chunks and 43 tokens
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=11)
    init = make_init(B, H, dk, dv, seed=12)
    gla.gla_set_option(gla.OPT_ENGINE, engine)
    gla.gla_set_option(gla.OPT_CARRY, carry)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    for scan in range(4):
        for s0 in (None, init):
            ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, scan,
                                              initial_state=None if s0 is None else s0.astype(np.float64))
            out, fin = run(d, gh, gw, scan, layout, s0)
            e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
            print(f"  layout={layout} scan={scan} init={'yes' if s0 is not None else 'no'} "
                  f"err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
            assert e_out <= TOL_BF16 and e_fin <= TOL_BF16


def test_fp32_inputs_in_token_major_order():
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv = 1, 2, 9, 14, 20, 24
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "f32", seed=13)
    init = make_init(B, H, dk, dv, seed=14)
    ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, 2,
                                      initial_state=init.astype(np.float64))
    out, fin = run(d, gh, gw, 2, gla.LAYOUT_BTHD, init)
    assert rel_err(out, ref) <= TOL_F32 and rel_err(fin, ref_fin) <= TOL_F32


def test_contract_workload_in_token_major_order():
    """DiG-XL/2 at 1024 px, column-reverse scan, [B,T,H,d] order, element by element."""
    from oracle import gla_oracle
    cfg = gi.CONFIGS["dig_xl2_1024"]
    d = gi.make_config_inputs(cfg)
    ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], cfg.grid_h, cfg.grid_w, 3)
    out, fin = run(d, cfg.grid_h, cfg.grid_w, 3, gla.LAYOUT_BTHD)
    e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
    print(f"  err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
    assert e_out <= TOL_BF16 and e_fin <= TOL_BF16


def test_sequence_fed_in_two_pieces_matches_one_call():
    """Rows 0..7 of a 16 x 32 grid, then rows 8..15 starting from the first call's final state (row-major scan):
    the same outputs and final state as one call over the whole grid, up to the engine's rounding."""
    B, H, gh, gw, dk, dv = 2, 4, 16, 32, 36, 72
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=15)
    whole, whole_fin = run(d, gh, gw, 0, gla.LAYOUT_BHTD)
    half = T // 2
    outs, state = [], None
    for piece in range(2):
        sl = slice(piece * half, (piece + 1) * half)
        dp = {"dtype": "bf16", "log_alpha": np.ascontiguousarray(d["log_alpha"][:, :, sl])}
        for n in ("q", "k", "v"):
            dp[n + "_bits"] = np.ascontiguousarray(d[n + "_bits"][:, :, sl])
        o, state = run(dp, gh // 2, gw, 0, gla.LAYOUT_BHTD, state)
        outs.append(o)
    pieces = np.concatenate(outs, axis=2)
    # (the pieces are four chunks long and run on the bf16 hi/lo kernel, the whole sequence on the fp16 kernels:
    # the two differ by the latter's rounding, a few 1e-3 of the RMS; a lost or misplaced state would be O(1))
    assert rel_err(pieces, whole) <= 1e-2
    assert rel_err(state, whole_fin) <= 1e-2
    from oracle import gla_oracle
    ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, 0)
    assert rel_err(pieces, ref) <= TOL_BF16 and rel_err(state, ref_fin) <= TOL_BF16
    assert rel_err(whole, ref) <= TOL_BF16 and rel_err(whole_fin, ref_fin) <= TOL_BF16


@pytest.mark.parametrize("z_mean", [0.0, 3.0, 6.0])
def test_long_chains_of_span_states(z_mean):
    """128 spans per head chained inside the output pass, with gates that decay fast (the chain stops after a few
    spans), slowly, or hardly at all (every span and the initial state are read); the initial state must reach
    the outputs exactly as far as the gates let it."""
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv = 1, 2, 64, 128, 36, 72        # 128 chunks
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "bf16", seed=13, z_mean=z_mean)
    init = make_init(B, H, dk, dv, seed=14)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_MFMA)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 1)
    for carry in (gla.CARRY_AUTO, gla.CARRY_KERNEL):
        gla.gla_set_option(gla.OPT_CARRY, carry)
        for scan, s0 in ((0, None), (3, init)):
            ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, scan,
                                              initial_state=None if s0 is None else s0.astype(np.float64))
            out, fin = run(d, gh, gw, scan, gla.LAYOUT_BHTD, s0)
            e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
            print(f"  z_mean={z_mean} carry={carry} scan={scan} err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
            assert e_out <= TOL_BF16 and e_fin <= TOL_BF16


@pytest.mark.parametrize("engine", [gla.ENGINE_MFMA, gla.ENGINE_AUTO])
def test_chain_behind_a_zero_tail(engine):
    """k = 0 over the last 60 chunks (a padded tail): the final state is the state after chunk 68 decayed by about
    2^-70, far below the 2^-40 at which the in-pass chain of the span states otherwise stops.  The chain has to go
    on while everything it has summed is exactly zero; the carry kernel has no cut-off and serves as second opinion."""
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv = 1, 2, 64, 128, 36, 72        # 128 chunks
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "bf16", seed=21, z_mean=1.5)
    k = d["k"].copy()
    k[:, :, 68 * 64:] = 0.0
    d["k"] = k
    d["k_bits"] = gi.round_to_bf16_bits(k)
    ref, ref_fin = gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, 0)
    assert 0.0 < np.abs(ref_fin).max() < 1e-12          # tiny, but not zero
    gla.gla_set_option(gla.OPT_ENGINE, engine)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 1)
    for carry in (gla.CARRY_IN_OUTPUT_PASS, gla.CARRY_KERNEL):
        gla.gla_set_option(gla.OPT_CARRY, carry)
        out, fin = run(d, gh, gw, 0, gla.LAYOUT_BHTD)
        e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
        print(f"  engine={engine} carry={carry} err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
        assert e_out <= TOL_BF16 and e_fin <= TOL_BF16
