"""GPU parity of the fp16 engine (producer / consumer kernels of the plain forward pass) against the CPU fp64 oracle.

The engine is what GLA_ENGINE_AUTO picks for bf16 inputs with 17..64 key channels; these tests name it
explicitly (GLA_ENGINE_MFMA_FP16), cover its three head-size classes, the span plans, both ways of chaining the
span states, and the inputs outside its range: gates that close fast, inputs scaled far up or down.  Such
sequences raise their range flags and are recomputed by the bf16 hi/lo kernel in the same call; the result has
to meet the same bar either way.  Bar for bf16 inputs and fp32 output: 2e-2 of the RMS (max norm).
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
OPTS = ("OPT_CHUNKS_PER_SPAN", "OPT_ENGINE", "OPT_CARRY", "OPT_RANGE_FALLBACK")
DEFAULTS = {"OPT_CHUNKS_PER_SPAN": 0, "OPT_ENGINE": 0, "OPT_CARRY": 0, "OPT_RANGE_FALLBACK": 1}


def _reset():
    for name in OPTS:
        gla.gla_set_option(getattr(gla, name), DEFAULTS[name])


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    gla.load_library()
    yield
    _reset()


@pytest.fixture(autouse=True)
def _reset_options():
    _reset()
    yield
    _reset()


def upload(d):
    dev = torch.device("cuda:0")
    f = lambda n: torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    return f("q"), f("k"), f("v"), torch.from_numpy(d["log_alpha"]).to(dev)


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(rms, 1e-300))


def oracle(d, gh, gw, scan):
    from oracle import gla_oracle
    return gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, scan)


def run(d, gh, gw, scan, engine, cps=0, carry=0, fallback=1):
    gla.gla_set_option(gla.OPT_ENGINE, engine)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    gla.gla_set_option(gla.OPT_CARRY, carry)
    gla.gla_set_option(gla.OPT_RANGE_FALLBACK, fallback)
    q, k, v, la = upload(d)
    out, fin = gla.gla_fwd_ex(q, k, v, la, gh, gw, scan)
    torch.cuda.synchronize()
    return out.cpu().numpy(), fin.cpu().numpy()


def scaled(d, name, factor):
    """The inputs with tensor `name` multiplied by a power of two (exact in bf16)."""
    e = dict(d)
    e[name] = (d[name] * np.float32(factor)).astype(np.float32)
    e[name + "_bits"] = gi.round_to_bf16_bits(e[name])
    assert np.array_equal(gi.bf16_bits_to_f32(e[name + "_bits"]), e[name])
    return e


# (B, H, grid_h, grid_w, dk, dv): the three head-size classes (17..32 / 33..48 / 49..64 key channels), ragged
# last chunks, sequences shorter than a chunk, grids that are not square
SHAPES = [
    (2, 3, 16, 16, 32, 64),
    (1, 2, 13, 11, 20, 24),
    (1, 2, 30, 30, 36, 72),
    (1, 3, 17, 9, 40, 80),
    (1, 2, 7, 5, 48, 40),
    (1, 2, 16, 24, 64, 128),
    (1, 2, 21, 13, 52, 96),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("cps", [0, 1, 3])
def test_shapes_plans_scans(shape, cps):
    B, H, gh, gw, dk, dv = shape
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "bf16", seed=11)
    for scan in range(4):
        ref, ref_fin = oracle(d, gh, gw, scan)
        out, fin = run(d, gh, gw, scan, gla.ENGINE_MFMA_FP16, cps=cps)
        e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
        print(f"  {shape} cps={cps} scan={scan}: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
        assert np.isfinite(out).all() and np.isfinite(fin).all()
        assert e_out <= TOL_BF16 and e_fin <= TOL_BF16


@pytest.mark.parametrize("carry", [gla.CARRY_KERNEL, gla.CARRY_IN_OUTPUT_PASS])
def test_both_ways_of_chaining_the_span_states(carry):
    B, H, gh, gw, dk, dv = 1, 3, 40, 24, 36, 72
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "bf16", seed=5, z_mean=2.0)   # slow decay: every span matters
    for scan in (0, 3):
        ref, ref_fin = oracle(d, gh, gw, scan)
        out, fin = run(d, gh, gw, scan, gla.ENGINE_MFMA_FP16, cps=2, carry=carry)
        assert rel_err(out, ref) <= TOL_BF16 and rel_err(fin, ref_fin) <= TOL_BF16


def test_auto_is_this_engine_and_hi_lo_engine_is_still_there():
    B, H, gh, gw, dk, dv = 1, 2, 32, 32, 36, 72
    d = gi.make_inputs(B, H, gh * gw, dk, dv, "bf16", seed=2)
    ref, ref_fin = oracle(d, gh, gw, 0)
    auto = run(d, gh, gw, 0, gla.ENGINE_AUTO)
    fp16 = run(d, gh, gw, 0, gla.ENGINE_MFMA_FP16)
    hilo = run(d, gh, gw, 0, gla.ENGINE_MFMA)
    assert np.array_equal(auto[0], fp16[0]) and np.array_equal(auto[1], fp16[1])
    e_fp16, e_hilo = rel_err(fp16[0], ref), rel_err(hilo[0], ref)
    print(f"  fp16 operands {e_fp16:.3e}, bf16 hi/lo operands {e_hilo:.3e}", flush=True)
    assert e_hilo <= 5e-4 and e_hilo < e_fp16 <= TOL_BF16


def test_engine_refuses_what_it_does_not_cover():
    d = gi.make_inputs(1, 1, 64, 8, 16, "bf16", seed=1)     # 8 key channels: below the engine's classes
    q, k, v, la = upload(d)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_MFMA_FP16)
    with pytest.raises(Exception):
        gla.gla_fwd_ex(q, k, v, la, 8, 8, 0)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)     # AUTO takes the bf16 hi/lo engine there
    out, fin = gla.gla_fwd_ex(q, k, v, la, 8, 8, 0)
    torch.cuda.synchronize()
    ref, ref_fin = oracle(d, 8, 8, 0)
    assert rel_err(out.cpu().numpy(), ref) <= TOL_BF16


# ---------------------------------------------------------------------------
# outside the range of the fp16 operands: flagged and recomputed in the same call
# ---------------------------------------------------------------------------
def _in_range_inputs(seed=7, H=3):
    gh, gw, dk, dv = 32, 24, 36, 72
    return gi.make_inputs(1, H, gh * gw, dk, dv, "bf16", seed=seed), gh, gw


@pytest.mark.parametrize("z_mean", [-5.0, -8.0])
def test_gates_that_close_fast(z_mean):
    """alpha = sigmoid(z)^(1/16) with z around -5 or -8: a channel decays by 2^-14 .. 2^-23 over half a chunk."""
    gh, gw, dk, dv = 32, 24, 36, 72
    d = gi.make_inputs(1, 3, gh * gw, dk, dv, "bf16", seed=9, z_mean=z_mean)
    for scan, cps in ((0, 0), (2, 2)):
        ref, ref_fin = oracle(d, gh, gw, scan)
        out, fin = run(d, gh, gw, scan, gla.ENGINE_MFMA_FP16, cps=cps)
        e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
        print(f"  z_mean={z_mean} scan={scan}: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
        assert np.isfinite(out).all() and np.isfinite(fin).all()
        assert e_out <= 5e-4 and e_fin <= 5e-4      # the hi/lo kernel's accuracy: these sequences were recomputed


@pytest.mark.parametrize("name,factor", [("k", 2.0 ** 12), ("v", 2.0 ** 16), ("q", 2.0 ** -14), ("v", 2.0 ** -20),
                                         ("q", 2.0 ** 10)])
def test_inputs_scaled_out_of_range(name, factor):
    d0, gh, gw = _in_range_inputs()
    d = scaled(d0, name, factor)
    ref, ref_fin = oracle(d, gh, gw, 0)
    out, fin = run(d, gh, gw, 0, gla.ENGINE_MFMA_FP16, cps=3)
    e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
    print(f"  {name} x {factor}: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
    assert np.isfinite(out).all() and np.isfinite(fin).all()
    assert e_out <= TOL_BF16 and e_fin <= TOL_BF16


def test_one_sequence_out_of_range_leaves_the_others_alone():
    """Head 1 gets closed gates; heads 0 and 2 keep the result of the fp16 kernels bit for bit."""
    d, gh, gw = _in_range_inputs(H=3)
    base = run(d, gh, gw, 1, gla.ENGINE_MFMA_FP16, cps=2)
    e = dict(d)
    la = d["log_alpha"].copy()
    la[:, 1] = np.float32(-0.6)
    e["log_alpha"] = la
    ref, ref_fin = oracle(e, gh, gw, 1)
    out, fin = run(e, gh, gw, 1, gla.ENGINE_MFMA_FP16, cps=2)
    assert np.array_equal(out[:, 0], base[0][:, 0]) and np.array_equal(out[:, 2], base[0][:, 2])
    assert np.array_equal(fin[:, 0], base[1][:, 0]) and np.array_equal(fin[:, 2], base[1][:, 2])
    assert rel_err(out, ref) <= TOL_BF16 and rel_err(fin, ref_fin) <= TOL_BF16
    assert rel_err(out[:, 1], ref[:, 1]) <= 5e-4


def test_fallback_launch_changes_nothing_in_range():
    d, gh, gw = _in_range_inputs()
    a = run(d, gh, gw, 0, gla.ENGINE_MFMA_FP16, cps=2, fallback=1)
    b = run(d, gh, gw, 0, gla.ENGINE_MFMA_FP16, cps=2, fallback=0)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_zero_inputs_and_open_gates():
    """All-zero k (a padded tail) and log_alpha = 0 (no decay): neither is out of range by itself."""
    d, gh, gw = _in_range_inputs()
    e = dict(d)
    la = d["log_alpha"].copy()
    la[:, 0] = 0.0
    e["log_alpha"] = la
    k = d["k"].copy()
    k[:, 2, 400:] = 0.0
    e["k"] = k
    e["k_bits"] = gi.round_to_bf16_bits(k)
    ref, ref_fin = oracle(e, gh, gw, 0)
    out, fin = run(e, gh, gw, 0, gla.ENGINE_MFMA_FP16, cps=2)
    assert rel_err(out, ref) <= TOL_BF16 and rel_err(fin, ref_fin) <= TOL_BF16


# ---------------------------------------------------------------------------
# gates from their pre-activations (gla_fwd_fused without the output epilogue) on the same engine
# ---------------------------------------------------------------------------
def run_fused(d, gh, gw, scan, engine, cps=0, tau=16.0):
    gla.gla_set_option(gla.OPT_ENGINE, engine)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    dev = torch.device("cuda:0")
    f = lambda n: torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    out, fin = gla.gla_fwd_fused(f("q"), f("k"), f("v"), f("z"), tau, gh, gw, scan)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), fin.cpu().numpy()


def oracle_fused(d, gh, gw, scan, tau=16.0):
    from oracle import gla_oracle_fused as fo
    return fo.gla_fused(d["q"], d["k"], d["v"], d["z"], tau, None, None, None, 1e-5, gh, gw, scan)


@pytest.mark.parametrize("shape", [(2, 3, 16, 16, 32, 64), (1, 2, 30, 30, 36, 72), (1, 2, 16, 24, 64, 128),
                                   (1, 2, 13, 11, 20, 24), (1, 2, 21, 13, 52, 96)])
def test_gate_prologue_shapes_plans_scans(shape):
    B, H, gh, gw, dk, dv = shape
    d = gi.make_fused_inputs(B, H, gh * gw, dk, dv, "bf16", seed=13)
    for cps in (0, 2):
        for scan in range(4):
            ref, ref_fin = oracle_fused(d, gh, gw, scan)
            out, fin = run_fused(d, gh, gw, scan, gla.ENGINE_MFMA_FP16, cps=cps)
            e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
            print(f"  {shape} cps={cps} scan={scan}: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
            assert np.isfinite(out).all() and e_out <= TOL_BF16 and e_fin <= TOL_BF16


def test_gate_prologue_auto_engine_temperature_and_closed_gates():
    gh, gw, dk, dv = 32, 24, 36, 72
    d = gi.make_fused_inputs(1, 3, gh * gw, dk, dv, "bf16", seed=4)
    ref, ref_fin = oracle_fused(d, gh, gw, 1)
    auto = run_fused(d, gh, gw, 1, gla.ENGINE_AUTO)
    fp16 = run_fused(d, gh, gw, 1, gla.ENGINE_MFMA_FP16)
    hilo = run_fused(d, gh, gw, 1, gla.ENGINE_MFMA)
    assert np.array_equal(auto[0], fp16[0]) and np.array_equal(auto[1], fp16[1])   # AUTO takes this engine
    assert rel_err(hilo[0], ref) < rel_err(fp16[0], ref) <= TOL_BF16
    # another temperature; and gates that close fast (z around -8 at tau = 16: a channel decays by 2^-23 over half a
    # chunk), which leave the fp16 range and are recomputed by the hi/lo kernel with the prologue
    ref4, fin4 = oracle_fused(d, gh, gw, 2, tau=4.0)
    out4, f4 = run_fused(d, gh, gw, 2, gla.ENGINE_MFMA_FP16, cps=2, tau=4.0)
    assert rel_err(out4, ref4) <= TOL_BF16 and rel_err(f4, fin4) <= TOL_BF16
    dc = gi.make_fused_inputs(1, 3, gh * gw, dk, dv, "bf16", seed=4, z_mean=-8.0)
    refc, finc = oracle_fused(dc, gh, gw, 0)
    outc, fc = run_fused(dc, gh, gw, 0, gla.ENGINE_MFMA_FP16, cps=2)
    e_out, e_fin = rel_err(outc, refc), rel_err(fc, finc)
    print(f"  closed gates: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
    assert np.isfinite(outc).all() and e_out <= 5e-4 and e_fin <= 5e-4


@pytest.mark.parametrize("name,scan", [("dig_xl2_1024", 2), ("dig_xl2_2048", 0)])
def test_gate_prologue_contract_workloads(name, scan):
    cfg = gi.CONFIGS[name]
    d = gi.make_fused_inputs(cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv, cfg.dtype, seed=cfg.seed, z_mean=cfg.z_mean)
    ref, ref_fin = oracle_fused(d, cfg.grid_h, cfg.grid_w, scan)
    out, fin = run_fused(d, cfg.grid_h, cfg.grid_w, scan, gla.ENGINE_AUTO)
    e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
    print(f"  {name} scan={scan}: err(out)={e_out:.3e} err(state)={e_fin:.3e}", flush=True)
    assert e_out <= TOL_BF16 and e_fin <= TOL_BF16
