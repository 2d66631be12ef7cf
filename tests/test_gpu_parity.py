"""GPU parity: the HIP path (through the C ABI) against the CPU fp64 oracle.

Error metric: max over all elements of |gpu - oracle| divided by the RMS of the
oracle tensor, separately for `out` and `final_state`.
Bars: 1e-4 for fp32 inputs, 2e-2 for bf16 inputs with fp32 accumulation and
fp32 output.  A bf16 output adds its own rounding, at most 2^-9 of the largest
|o|, so that bar is 2e-2 + 2^-9 * max|o| / rms.
"""
import functools

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
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)


@pytest.fixture(autouse=True)
def _reset_options():
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_AUTO)
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)
    yield


def upload(d):
    dev = torch.device("cuda:0")
    if d["dtype"] == "bf16":
        f = lambda n: torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        f = lambda n: torch.from_numpy(d[n]).to(dev)
    return f("q"), f("k"), f("v"), torch.from_numpy(d["log_alpha"]).to(dev)


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(rms, 1e-300))


@functools.lru_cache(maxsize=4)
def _config_inputs(name):
    return gi.make_config_inputs(gi.CONFIGS[name])


@functools.lru_cache(maxsize=8)
def _oracle(name, scan):
    from oracle import gla_oracle
    cfg = gi.CONFIGS[name]
    d = _config_inputs(name)
    return gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], cfg.grid_h, cfg.grid_w, scan)


def run_gpu(d, gh, gw, scan, out_dtype=None, simple=False):
    q, k, v, la = upload(d)
    if simple:
        out, fin = gla.gla_fwd(q, k, v, la, gh, gw, scan)
    else:
        out, fin = gla.gla_fwd_ex(q, k, v, la, gh, gw, scan, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), fin.cpu().numpy()


def check(d, gh, gw, scan, ref, ref_fin, tol, **kw):
    out, fin = run_gpu(d, gh, gw, scan, **kw)
    e_out, e_fin = rel_err(out, ref), rel_err(fin, ref_fin)
    print(f"  scan={scan} err(out)={e_out:.3e} err(state)={e_fin:.3e} tol={tol:.1e}", flush=True)
    assert np.isfinite(out).all() and np.isfinite(fin).all()
    assert e_out <= tol, f"out: {e_out} > {tol}"
    assert e_fin <= tol, f"final_state: {e_fin} > {tol}"
    return e_out, e_fin


# ---------------------------------------------------------------------------
# the five contract workloads, every listed scan order, element by element
# ---------------------------------------------------------------------------
CASES = [(name, scan) for name in gi.CONFIG_ORDER for scan in gi.CONFIGS[name].scans]
CASES.append(("dig_xl2_2048_longmem", 0))


@pytest.mark.parametrize("name,scan", CASES)
def test_contract_config(name, scan):
    cfg = gi.CONFIGS[name]
    d = _config_inputs(name)
    ref, ref_fin = _oracle(name, scan)
    tol = TOL_F32 if cfg.dtype == "f32" else TOL_BF16
    print(f"\n{name}: B={cfg.B} H={cfg.H} T={cfg.T} dk={cfg.dk} dv={cfg.dv} {cfg.dtype}", flush=True)
    check(d, cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, tol, simple=(cfg.dtype == "bf16"))


ENGINE_CARRY = [(gla.ENGINE_RECURRENT, gla.CARRY_AUTO), (gla.ENGINE_MFMA, gla.CARRY_KERNEL),
                (gla.ENGINE_MFMA, gla.CARRY_IN_OUTPUT_PASS)]


@pytest.mark.parametrize("engine,carry", ENGINE_CARRY)
@pytest.mark.parametrize("cps", [1, 2, 3, 1000])
def test_plans_and_engines_agree_with_oracle(engine, carry, cps):
    """Every launch plan (chunks per span), both engines and both places where the span states are chained, on
    DiG-XL/2 at 512 px, column-reverse scan."""
    name, scan = "dig_xl2_512", 3
    cfg = gi.CONFIGS[name]
    gla.gla_set_option(gla.OPT_ENGINE, engine)
    gla.gla_set_option(gla.OPT_CARRY, carry)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    ref, ref_fin = _oracle(name, scan)
    print(f"\nengine={engine} carry={carry} chunks_per_span={cps}", flush=True)
    check(_config_inputs(name), cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, TOL_BF16)


@pytest.mark.parametrize("cps,carry", [(1, gla.CARRY_IN_OUTPUT_PASS), (1, gla.CARRY_AUTO), (2, gla.CARRY_AUTO),
                                       (4, gla.CARRY_IN_OUTPUT_PASS), (4, gla.CARRY_AUTO), (6, gla.CARRY_AUTO),
                                       (6, gla.CARRY_KERNEL)])
def test_many_spans_per_head_at_full_size(cps, carry):
    """The 2048 px workload cut into 256, 128, 64 and 43 spans per head: long chains in the output pass (forced at
    256 spans), the carry kernel, and the automatic choice on both sides of its limit of 128 spans."""
    name, scan = "dig_xl2_2048", 1
    cfg = gi.CONFIGS[name]
    gla.gla_set_option(gla.OPT_CARRY, carry)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    ref, ref_fin = _oracle(name, scan)
    print(f"\ncarry={carry} chunks_per_span={cps}", flush=True)
    check(_config_inputs(name), cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, TOL_BF16)


@pytest.mark.parametrize("name,scan", [("dig_s2_1792", 0), ("dig_s2_1792", 3), ("dig_xl2_1792", 0), ("dig_xl2_1792", 2)])
def test_1792_px_shapes(name, scan):
    """T = 12544 (112 x 112 tokens, the 1792 px case of the paper's Fig. 1) with the head sizes of DiG-S/2 and of
    DiG-XL/2, in the launch plan the benchmark times: 196 chunks per head, which no power of two divides."""
    cfg = gi.CONFIGS[name]
    ref, ref_fin = _oracle(name, scan)
    print(f"\n{name}: B={cfg.B} H={cfg.H} T={cfg.T} dk={cfg.dk} dv={cfg.dv}", flush=True)
    check(_config_inputs(name), cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, TOL_BF16)


@pytest.mark.parametrize("cps", [4, 5, 7, 9])
def test_odd_and_even_span_lengths(cps):
    """Spans of four chunks or more run the state pass with two chunks of rows in flight (a loop over chunk pairs
    plus a last odd chunk); 1024 px has 64 chunks per head, so these span lengths also leave a shorter last span."""
    name, scan = "dig_xl2_1024", 2
    cfg = gi.CONFIGS[name]
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
    ref, ref_fin = _oracle(name, scan)
    print(f"\nchunks_per_span={cps}", flush=True)
    check(_config_inputs(name), cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, TOL_BF16)


def test_bf16_output():
    name, scan = "dig_s2_256", 2
    cfg = gi.CONFIGS[name]
    ref, ref_fin = _oracle(name, scan)
    rms = np.sqrt(np.mean(ref ** 2))
    tol = TOL_BF16 + 2.0 ** -9 * np.abs(ref).max() / rms
    check(_config_inputs(name), cfg.grid_h, cfg.grid_w, scan, ref, ref_fin, tol, out_dtype=torch.bfloat16)


# ---------------------------------------------------------------------------
# shapes that straddle tiles: ragged tails, T < chunk, T = 1, odd head sizes,
# non-square grids, both element types
# ---------------------------------------------------------------------------
SHAPES = [
    # B, H, gh, gw, dk, dv, dtype
    (1, 1, 1, 1, 36, 72, "bf16"),
    (2, 3, 1, 7, 32, 64, "bf16"),
    (1, 2, 5, 13, 36, 72, "bf16"),       # T = 65: one full chunk + 1 token
    (2, 2, 9, 21, 36, 72, "bf16"),       # T = 189: ragged tail, non-square
    (1, 3, 23, 11, 64, 128, "bf16"),     # largest head sizes
    (1, 2, 10, 13, 4, 8, "bf16"),        # smallest head sizes of the MFMA engine
    (1, 2, 10, 13, 4, 2, "bf16"),        # dv % 8 != 0 -> recurrent engine
    (1, 2, 17, 19, 40, 96, "bf16"),
    (1, 2, 9, 15, 48, 80, "bf16"),       # two channel groups in the last 32-channel step
    (1, 1, 8, 17, 56, 104, "bf16"),      # three
    (2, 1, 7, 11, 24, 40, "bf16"),
    (1, 2, 6, 11, 8, 16, "bf16"),
    (1, 2, 12, 11, 33, 65, "bf16"),      # odd head sizes -> recurrent engine
    (1, 2, 12, 11, 20, 24, "f32"),
    (2, 1, 20, 20, 64, 128, "f32"),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes_all_scans(shape):
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv, dtype = shape
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, dtype, seed=7)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    print(f"\nshape={shape}", flush=True)
    refs = [gla_oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, scan) for scan in range(4)]
    for carry in (gla.CARRY_KERNEL, gla.CARRY_IN_OUTPUT_PASS):
        gla.gla_set_option(gla.OPT_CARRY, carry)
        for cps in (0, 1, 2):
            gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
            for scan in range(4):
                check(d, gh, gw, scan, refs[scan][0], refs[scan][1], tol)


def test_strong_and_absent_decay():
    """Gates far from the synthetic recipe: alpha = 1 (no decay) and alpha near exp(-1) per token."""
    from oracle import gla_oracle
    B, H, gh, gw, dk, dv = 1, 2, 16, 12, 36, 72
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=3)
    for scale, name in ((0.0, "alpha=1"), (16.0, "log_alpha=logsigmoid(z)")):
        d2 = dict(d)
        d2["log_alpha"] = (d["log_alpha"] * np.float32(scale)).astype(np.float32)
        ref, ref_fin = gla_oracle.gla_fwd(d2["q"], d2["k"], d2["v"], d2["log_alpha"], gh, gw, 0)
        print(f"\n{name}", flush=True)
        check(d2, gh, gw, 0, ref, ref_fin, TOL_BF16)


def test_closed_gates_on_recurrent_engine():
    """alpha -> 0 wipes the state before every token: o_t = (q_t.k_t) v_t (exact engine only)."""
    B, H, gh, gw, dk, dv = 1, 2, 9, 9, 36, 72
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=4)
    d["log_alpha"] = np.full_like(d["log_alpha"], -200.0)
    gla.gla_set_option(gla.OPT_ENGINE, gla.ENGINE_RECURRENT)
    out, fin = run_gpu(d, gh, gw, 1)
    ref = (d["q"].astype(np.float64) * d["k"]).sum(-1, keepdims=True) * d["v"]
    assert rel_err(out, ref) <= 1e-5


def test_run_to_run_determinism():
    name = "dig_xl2_512"
    cfg = gi.CONFIGS[name]
    d = _config_inputs(name)
    a, fa = run_gpu(d, cfg.grid_h, cfg.grid_w, 2)
    b, fb = run_gpu(d, cfg.grid_h, cfg.grid_w, 2)
    assert np.array_equal(a, b) and np.array_equal(fa, fb)


def test_final_state_is_optional_and_streams_are_honoured():
    name = "dig_s2_256"
    cfg = gi.CONFIGS[name]
    d = _config_inputs(name)
    q, k, v, la = upload(d)
    ref, _ = _oracle(name, 0)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out, fin = gla.gla_fwd_ex(q, k, v, la, cfg.grid_h, cfg.grid_w, 0, want_final_state=False)
    s.synchronize()
    assert fin is None
    assert rel_err(out.cpu().numpy(), ref) <= TOL_BF16


def test_timed_entry_point_runs_the_same_path():
    """gla_fwd_timed (HIP events around each kernel, used by the benchmark) leaves the same outputs as gla_fwd_ex."""
    name = "dig_xl2_512"
    cfg = gi.CONFIGS[name]
    q, k, v, la = upload(_config_inputs(name))
    out, fin = gla.gla_fwd_ex(q, k, v, la, cfg.grid_h, cfg.grid_w, 1)
    out2, fin2 = torch.zeros_like(out), torch.zeros_like(fin)
    nbytes = gla.gla_fwd_workspace_bytes(cfg.B, cfg.H, cfg.T, cfg.dk, cfg.dv, gla.DT_BF16)
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=q.device)
    ms = gla.gla_fwd_timed(q, k, v, la, cfg.grid_h, cfg.grid_w, 1, out2, fin2, ws, iters=3)
    torch.cuda.synchronize()
    assert len(ms) == 4 and all(m >= 0.0 for m in ms) and ms[3] > 0.0
    assert torch.equal(out, out2) and torch.equal(fin, fin2)


def test_errors_write_nothing():
    d = gi.make_inputs(1, 1, 16, 8, 8, "bf16", seed=1)
    q, k, v, la = upload(d)
    out = torch.full((1, 1, 16, 8), 123.0, device="cuda:0")
    with pytest.raises(gla.GlaError) as ei:
        gla.gla_fwd(q, k, v, la, 3, 5, 0, out=out)          # 3*5 != 16
    assert ei.value.status == 2
    with pytest.raises(gla.GlaError) as ei:
        gla.gla_fwd(q, k, v, la, 4, 4, 9, out=out)          # bad scan order
    assert ei.value.status == 2
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(gla.GlaError) as ei:
        gla.gla_fwd_ex(q, k, v, la, 4, 4, 0, out=out, workspace=small)
    assert ei.value.status == 5
    torch.cuda.synchronize()
    assert bool((out == 123.0).all())
