"""GPU parity of gla_fwd_gates (two-sided gate alpha_t^T beta_t, Sec. 3.1 Eqs. (gate_gla), (gate_gla_2)) against the
fp64 oracle, through the C ABI.  Bars: 1e-4 x RMS (fp32 rows), 2e-2 x RMS (bf16 rows), max-norm."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi
from oracle import gla_oracle as orc
from oracle import gla_oracle_gates as og

TOL_F32, TOL_BF16 = 1e-4, 2e-2


def _err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(rms, 1e-300))


def _dev(d, dtype):
    dev = torch.device("cuda:0")
    if dtype == "bf16":
        q, k, v = (torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16) for n in "qkv")
    else:
        q, k, v = (torch.from_numpy(d[n]).to(dev) for n in "qkv")
    return q, k, v, torch.from_numpy(d["log_alpha"]).to(dev), torch.from_numpy(d["log_beta"]).to(dev)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("scan_dir", [0, 1, 2, 3])
def test_gates_parity_several_spans_ragged(dtype, scan_dir):
    B, H, gh, gw, dk, dv = 2, 3, 19, 23, 20, 33      # T = 437: seven chunks, a ragged last one, odd head sizes
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, dtype, seed=11 + scan_dir)
    q, k, v, la, lb = _dev(d, dtype)
    out, fin = gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, scan_dir)
    torch.cuda.synchronize()
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, scan_dir)
    assert _err(out.cpu().numpy(), ro) < TOL_F32
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


@pytest.mark.parametrize("dk,dv", [(8, 16), (32, 64), (36, 72), (40, 80), (64, 128)])
@pytest.mark.parametrize("scan_dir", [0, 3])
def test_gates_mfma_engine_sizes(dk, dv, scan_dir):
    """bf16 inputs with dk % 4 == 0, dv % 8 == 0, dk <= 40 and dv <= 80 run on the MFMA engine (chunk form with both
    decays factorised), larger heads on the token-by-token engine; seven chunks with a ragged last one, chained by
    the carry kernel."""
    B, H, gh, gw = 2, 2, 19, 23
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, "bf16", seed=41 + dk)
    q, k, v, la, lb = _dev(d, "bf16")
    out, fin = gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, scan_dir)
    torch.cuda.synchronize()
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, scan_dir)
    assert _err(out.cpu().numpy(), ro) < TOL_F32
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


@pytest.mark.parametrize("carry", ["kernel", "in_output"])
def test_gates_both_ways_of_chaining_the_spans(carry):
    """The spans are chained by the carry kernel or by the output pass itself; both multiply the two decays."""
    B, H, gh, gw, dk, dv = 1, 2, 30, 40, 36, 72          # 1200 tokens: 19 chunks
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, "bf16", seed=61)
    q, k, v, la, lb = _dev(d, "bf16")
    s0 = np.random.default_rng(7).standard_normal((B, H, dk, dv)).astype(np.float32)
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, 2, initial_state=s0)
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_KERNEL if carry == "kernel" else gla.CARRY_IN_OUTPUT_PASS)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 2)
    try:
        out, fin = gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, 2, initial_state=torch.from_numpy(s0).cuda())
        torch.cuda.synchronize()
    finally:
        gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)
        gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
    assert _err(out.cpu().numpy(), ro) < TOL_F32
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


def test_gates_engines_agree_and_single_span():
    """One span (T <= 256: no carry kernel, final state from the output pass) and the token-by-token engine on the
    same inputs."""
    B, H, gh, gw, dk, dv = 1, 3, 10, 20, 36, 72
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, "bf16", seed=51)
    q, k, v, la, lb = _dev(d, "bf16")
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, 1)
    for engine in (gla.ENGINE_AUTO, gla.ENGINE_RECURRENT, gla.ENGINE_MFMA):
        gla.gla_set_option(gla.OPT_ENGINE, engine)
        try:
            out, fin = gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, 1)
            torch.cuda.synchronize()
        finally:
            gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)
        assert _err(out.cpu().numpy(), ro) < TOL_F32
        assert _err(fin.cpu().numpy(), rf) < TOL_F32


def test_gates_bf16_rows_token_major_initial_state():
    B, H, gh, gw, dk, dv = 2, 4, 16, 20, 32, 64
    T = gh * gw
    d = gi.make_gate_inputs(B, H, T, dk, dv, "bf16", seed=21)
    q, k, v, la, lb = _dev(d, "bf16")
    s0 = np.random.default_rng(5).standard_normal((B, H, dk, dv)).astype(np.float32)
    tm = lambda t: t.permute(0, 2, 1, 3).contiguous()      # [B,H,T,d] -> [B,T,H,d]
    out, fin = gla.gla_fwd_gates(tm(q), tm(k), tm(v), tm(la), tm(lb), gh, gw, 2, layout=gla.LAYOUT_BTHD,
                                 initial_state=torch.from_numpy(s0).cuda(), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, 2, initial_state=s0)
    got = out.float().permute(0, 2, 1, 3).cpu().numpy()
    rms = float(np.sqrt(np.mean(ro * ro)))
    assert _err(got, ro) < TOL_BF16 + 2.0 ** -9 * float(np.abs(ro).max()) / rms
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


def test_zero_log_beta_gives_the_key_side_result():
    B, H, gh, gw, dk, dv = 1, 2, 12, 16, 36, 72
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, "bf16", seed=31)
    q, k, v, la, lb = _dev(d, "bf16")
    out, fin = gla.gla_fwd_gates(q, k, v, la, torch.zeros_like(lb), gh, gw, 0)
    torch.cuda.synchronize()
    ro, rf = orc.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, 0)
    assert _err(out.cpu().numpy(), ro) < TOL_F32
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


def test_gates_headline_shape():
    """DiG-XL/2 at 2048 x 2048 (T = 16384, H = 16, dk = 36, dv = 72): every output row against the oracle."""
    cfg = gi.CONFIGS["dig_xl2_2048"]
    d = gi.make_gate_inputs(cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv, "bf16", seed=cfg.seed)
    q, k, v, la, lb = _dev(d, "bf16")
    out, fin = gla.gla_fwd_gates(q, k, v, la, lb, cfg.grid_h, cfg.grid_w, 0)
    torch.cuda.synchronize()
    ro, rf = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], cfg.grid_h, cfg.grid_w, 0)
    assert _err(out.cpu().numpy(), ro) < TOL_F32
    assert _err(fin.cpu().numpy(), rf) < TOL_F32


def test_gates_forced_mfma_engine_rejects_what_it_cannot_run():
    d = gi.make_gate_inputs(1, 1, 64, 20, 33, "bf16", seed=1)      # dv not a multiple of 8
    q, k, v, la, lb = _dev(d, "bf16")
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_MFMA)
    try:
        with pytest.raises(gla.GlaError):
            gla.gla_fwd_gates(q, k, v, la, lb, 8, 8, 0)
    finally:
        gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)


# ---- both gates from their pre-activations, with the output epilogue (gla_fwd_fused_gates) ----

def _dev_fused(d, dtype):
    dev = torch.device("cuda:0")
    names = ("q", "k", "v", "z", "zb", "r")
    if dtype == "bf16":
        return {n: torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16) for n in names}
    return {n: torch.from_numpy(d[n]).to(dev) for n in names}


def _check_fused_gates(B, H, gh, gw, dk, dv, dtype, scan, seed, epilogue, out_dtype=None, engine=None):
    from oracle import gla_oracle_fused as fo
    d = gi.make_fused_gate_inputs(B, H, gh * gw, dk, dv, dtype, seed=seed)
    t = _dev_fused(d, dtype)
    ref, rfin = fo.gla_fused_gates(d["q"], d["k"], d["v"], d["z"], d["zb"], 16.0, d["r"] if epilogue else None,
                                   d["ln_w"], d["ln_b"], 1e-5, gh, gw, scan)
    if engine is not None:
        gla.gla_set_option(gla.OPT_ENGINE, engine)
    try:
        y, fin = gla.gla_fwd_fused_gates(t["q"], t["k"], t["v"], t["z"], t["zb"], 16.0, gh, gw, scan,
                                         r_pre=t["r"] if epilogue else None,
                                         ln_weight=torch.from_numpy(d["ln_w"]).cuda() if epilogue else None,
                                         ln_bias=torch.from_numpy(d["ln_b"]).cuda() if epilogue else None,
                                         ln_eps=1e-5, out_dtype=out_dtype)
        torch.cuda.synchronize()
    finally:
        gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)
    return _err(y.float().cpu().numpy(), ref), _err(fin.cpu().numpy(), rfin), float(np.abs(ref).max() / np.sqrt(np.mean(ref ** 2)))


@pytest.mark.parametrize("dk,dv", [(32, 64), (36, 72), (20, 33), (64, 128)])
@pytest.mark.parametrize("scan", [0, 2])
def test_fused_gates_parity(dk, dv, scan):
    """Same bars as gla_fwd_fused: 2e-2 of the RMS for bf16 inputs with the LayerNorm epilogue (LN divides by the
    row's spread), 1e-4 for fp32 inputs; the plain rows (no epilogue) of bf16 inputs to 2e-4."""
    e_y, e_f, _ = _check_fused_gates(2, 2, 19, 23, dk, dv, "bf16", scan, 71, True)
    assert e_y < TOL_BF16 and e_f < 2e-4
    e_o, e_f, _ = _check_fused_gates(2, 2, 19, 23, dk, dv, "bf16", scan, 72, False)
    assert e_o < 2e-4 and e_f < 2e-4
    if dv % 8:
        e_y, e_f, _ = _check_fused_gates(1, 2, 19, 23, dk, dv, "f32", scan, 73, True)
        assert e_y < TOL_F32 and e_f < TOL_F32


def test_fused_gates_engines_and_bf16_rows():
    for engine in (gla.ENGINE_RECURRENT, gla.ENGINE_MFMA):
        e_y, e_f, _ = _check_fused_gates(1, 3, 30, 40, 36, 72, "bf16", 1, 74, True, engine=engine)
        assert e_y < TOL_BF16 and e_f < 2e-4
    e_y, e_f, peak = _check_fused_gates(1, 3, 30, 40, 36, 72, "bf16", 3, 75, True, out_dtype=torch.bfloat16)
    assert e_y < TOL_BF16 + 2.0 ** -9 * peak


def test_fused_gates_headline_shape():
    cfg = gi.CONFIGS["dig_xl2_2048"]
    e_y, e_f, _ = _check_fused_gates(cfg.B, cfg.H, cfg.grid_h, cfg.grid_w, cfg.dk, cfg.dv, "bf16", 0, cfg.seed, True)
    assert e_y < TOL_BF16 and e_f < 2e-4


# ---- backward pass of the two-sided-gate recurrence (gla_bwd_gates) ----

def _bwd_problem(B, H, gh, gw, dk, dv, dtype, seed):
    d = gi.make_gate_inputs(B, H, gh * gw, dk, dv, dtype, seed=seed)
    w = np.random.Generator(np.random.PCG64(seed + 1000)).standard_normal((B, H, gh * gw, dv), dtype=np.float32)
    if dtype == "bf16":
        d["w_bits"] = gi.round_to_bf16_bits(w)
        d["w"] = gi.bf16_bits_to_f32(d["w_bits"])
    else:
        d["w"] = w
    return d


def _check_bwd_gates(B, H, gh, gw, dk, dv, dtype, scan, seed, tol):
    """Bars as for gla_bwd: per gradient tensor max |gpu - oracle| / RMS(oracle), the gate gradients against
    RMS(oracle) or the RMS of their summands (q * dq, o * dO), whichever is larger."""
    d = _bwd_problem(B, H, gh, gw, dk, dv, dtype, seed)
    q, k, v, la, lb = _dev(d, dtype)
    dev = torch.device("cuda:0")
    if dtype == "bf16":
        w = torch.from_numpy(d["w_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        w = torch.from_numpy(d["w"]).to(dev)
    got = gla.gla_bwd_gates(q, k, v, la, lb, w, gh, gw, scan)
    torch.cuda.synchronize()
    ref = og.gla_bwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], d["w"], gh, gw, scan)
    o, _ = og.gla_fwd_gates(d["q"], d["k"], d["v"], d["log_alpha"], d["log_beta"], gh, gw, scan)
    floors = [0.0, 0.0, 0.0, float(np.sqrt(np.mean((d["q"].astype(np.float64) * ref[0]) ** 2))),
              float(np.sqrt(np.mean((o * d["w"].astype(np.float64)) ** 2)))]
    names = ("dq", "dk", "dv", "dlog_alpha", "dlog_beta")
    for name, g, r, fl in zip(names, got, ref, floors):
        r = np.asarray(r)
        rms = max(float(np.sqrt(np.mean(r * r))), fl)
        err = float(np.abs(g.cpu().numpy().astype(np.float64) - r).max() / rms)
        assert err < tol, (name, err)


@pytest.mark.parametrize("dk,dv,dtype", [(36, 72, "bf16"), (32, 64, "bf16"), (20, 33, "bf16"), (64, 128, "bf16"),
                                         (20, 33, "f32"), (36, 72, "f32")])
@pytest.mark.parametrize("scan", [0, 3])
def test_bwd_gates_parity(dk, dv, dtype, scan):
    _check_bwd_gates(2, 2, 19, 23, dk, dv, dtype, scan, 81 + dk, TOL_BF16 if dtype == "bf16" else TOL_F32)


def test_bwd_gates_with_the_forward_outputs_given():
    """The caller may pass the outputs of gla_fwd_gates instead of having them recomputed: same gradients."""
    d = _bwd_problem(1, 2, 30, 40, 36, 72, "bf16", 97)
    q, k, v, la, lb = _dev(d, "bf16")
    w = torch.from_numpy(d["w_bits"].view(np.int16)).cuda().view(torch.bfloat16)
    out, _ = gla.gla_fwd_gates(q, k, v, la, lb, 30, 40, 1)
    a = gla.gla_bwd_gates(q, k, v, la, lb, w, 30, 40, 1)
    b = gla.gla_bwd_gates(q, k, v, la, lb, w, 30, 40, 1, out_fwd=out)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_bwd_gates_single_span_and_column_scan():
    _check_bwd_gates(1, 3, 10, 20, 36, 72, "bf16", 2, 91, TOL_BF16)
    _check_bwd_gates(1, 2, 30, 40, 36, 72, "bf16", 1, 92, TOL_BF16)


@pytest.mark.parametrize("engine,carry,split", [("auto", "in_output", 0), ("auto", "kernel", 0), ("auto", "auto", 1),
                                                ("recurrent", "auto", 0)])
def test_bwd_gates_engines_and_span_chaining(engine, carry, split):
    """The value-axis reads run in chunk form on the MFMA units (dk and dv in one walk, or split) or token by token;
    the span states are chained by the kernels themselves or by the carry kernel."""
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_RECURRENT if engine == "recurrent" else gla.ENGINE_AUTO)
    gla.gla_set_option(gla.OPT_BWD_SPLIT, split)
    gla.gla_set_option(gla.OPT_CARRY, {"in_output": gla.CARRY_IN_OUTPUT_PASS, "kernel": gla.CARRY_KERNEL,
                                       "auto": gla.CARRY_AUTO}[carry])
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 3)
    try:
        _check_bwd_gates(1, 2, 30, 40, 36, 72, "bf16", 0, 95, TOL_BF16)
        _check_bwd_gates(1, 2, 30, 40, 32, 64, "bf16", 3, 96, TOL_BF16)
    finally:
        gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)
        gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)
        gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
        gla.gla_set_option(gla.OPT_BWD_SPLIT, 0)


def test_bwd_gates_headline_shape_first_two_heads():
    """The launch configuration the benchmark times (B = 1, H = 16, T = 16384); the oracle keeps every state of a
    sequence, so it is run on the first two heads only (heads are independent) and those are compared."""
    cfg = gi.CONFIGS["dig_xl2_2048"]
    d = _bwd_problem(cfg.B, cfg.H, cfg.grid_h, cfg.grid_w, cfg.dk, cfg.dv, "bf16", cfg.seed)
    q, k, v, la, lb = _dev(d, "bf16")
    w = torch.from_numpy(d["w_bits"].view(np.int16)).cuda().view(torch.bfloat16)
    got = gla.gla_bwd_gates(q, k, v, la, lb, w, cfg.grid_h, cfg.grid_w, 0)
    torch.cuda.synchronize()
    hs = slice(0, 2)
    ref = og.gla_bwd_gates(d["q"][:, hs], d["k"][:, hs], d["v"][:, hs], d["log_alpha"][:, hs], d["log_beta"][:, hs],
                           d["w"][:, hs], cfg.grid_h, cfg.grid_w, 0)
    for name, g, r in zip(("dq", "dk", "dv", "dlog_alpha", "dlog_beta"), got, ref):
        rms = float(np.sqrt(np.mean(r * r)))
        err = float(np.abs(g[:, hs].cpu().numpy().astype(np.float64) - r).max() / rms)
        assert err < TOL_BF16, (name, err)
