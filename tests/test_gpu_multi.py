"""GPU parity of gla_fwd_multi (bidirectional and 4-directional scanning: the sum over scan orders of the forward
outputs, supplement Algorithms 2 and 3) against the CPU fp64 oracle.  Error metric and bars as for the forward pass."""
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


def upload(d, name):
    dev = torch.device("cuda:0")
    if name != "log_alpha" and d["dtype"] == "bf16":
        return torch.from_numpy(d[name + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(d[name]).to(dev)


def check(d, gh, gw, dirs, tol):
    from oracle import gla_oracle
    ref = gla_oracle.gla_fwd_multi(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, dirs)
    # `out` starts with garbage: the first scan order must overwrite it, not add to it
    out = torch.full(ref.shape, 1e30, dtype=torch.float32, device="cuda:0")
    got = gla.gla_fwd_multi(*(upload(d, n) for n in ("q", "k", "v", "log_alpha")), gh, gw, dirs, out=out)
    torch.cuda.synchronize()
    err = float(np.abs(got.cpu().numpy() - ref).max() / np.sqrt(np.mean(ref ** 2)))
    print("  dirs=%s err=%.3e" % (dirs, err), flush=True)
    assert err <= tol, err


SHAPES = [
    (1, 2, 1, 1, 36, 72, "bf16"),
    (2, 2, 5, 13, 36, 72, "bf16"),
    (1, 3, 23, 11, 64, 128, "bf16"),
    (2, 6, 16, 16, 32, 64, "bf16"),
    (1, 2, 12, 11, 33, 65, "bf16"),       # recurrent engine
    (1, 2, 12, 11, 20, 24, "f32"),
    (1, 2, 7, 9, 5, 3, "f32"),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_direction_sets_and_plans(shape):
    B, H, gh, gw, dk, dv, dtype = shape
    d = gi.make_inputs(B, H, gh * gw, dk, dv, dtype, seed=41)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    for cps in (0, 1, 2):
        gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, cps)
        for dirs in ((0, 1), (0, 1, 2, 3), (2,), (3, 1)):
            check(d, gh, gw, dirs, tol)


@pytest.mark.parametrize("name,dirs", [("dig_s2_256", (0, 1, 2, 3)), ("dig_xl2_1024", (0, 1)), ("dig_xl2_2048", (0, 1, 2, 3))])
def test_contract_workloads(name, dirs):
    cfg = gi.CONFIGS[name]
    check(gi.make_config_inputs(cfg), cfg.grid_h, cfg.grid_w, dirs, TOL_BF16)


def test_empty_direction_set_is_refused():
    d = gi.make_inputs(1, 1, 16, 8, 8, "bf16", seed=1)
    with pytest.raises(gla.GlaError):
        gla.gla_fwd_multi(*(upload(d, n) for n in ("q", "k", "v", "log_alpha")), 4, 4, ())


@pytest.mark.parametrize("schedule", [0, 1])
def test_block_by_block_schedule_against_literal_permutations(schedule):
    """Algorithm 1 / Algorithm 4: the paper flips or transposes the token sequence after every block and always scans
    it front to back.  Here the tokens stay in canonical order and block l is given gla_block_scan_dir(l): the mixer
    (gla_fwd_ex) and the SREM convolution (gla_srem_dwconv) of five consecutive blocks must equal what the literal
    route gives - permute the tensors the way the sequence has been permuted so far, run the row-major forward
    oracle (and the oracle's convolution on the reshaped matrix), undo the permutation."""
    from oracle import gla_oracle, srem_oracle
    N, B, H, dk, dv = 12, 1, 2, 36, 72
    T = N * N
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=77)
    rng = np.random.default_rng(3)
    D = 16
    x = rng.standard_normal((B, T, D)).astype(np.float32)
    w = rng.standard_normal((D, 3, 3)).astype(np.float32)
    xg = torch.from_numpy(x).cuda()
    wg = torch.from_numpy(w).cuda()
    perm = np.arange(T)                       # perm[s] = canonical token at position s of the paper's sequence
    for block in range(1, 6):
        sd = gla.gla_block_scan_dir(block, schedule)
        # the literal route on the permuted sequence
        qp, kp, vp, gp = (d[n][:, :, perm] for n in ("q", "k", "v", "log_alpha"))
        ref_p, _ = gla_oracle.gla_fwd(qp, kp, vp, gp, N, N, gla.SCAN_ROW_FWD)
        ref = np.empty_like(ref_p)
        ref[:, :, perm] = ref_p
        out, _ = gla.gla_fwd_ex(*(upload(d, n) for n in ("q", "k", "v", "log_alpha")), N, N, sd)
        torch.cuda.synchronize()
        err = float(np.abs(out.cpu().numpy() - ref).max() / np.sqrt(np.mean(ref ** 2)))
        yp = srem_oracle.srem_dwconv(x[:, perm], w, None, N, N, 0)
        yref = np.empty_like(yp)
        yref[:, perm] = yp
        y = gla.gla_srem_dwconv(xg, wg, None, N, N, orient=sd)
        torch.cuda.synchronize()
        erry = float(np.abs(y.cpu().numpy() - yref).max())
        print(f"  schedule {schedule} block {block}: scan order {sd}, mixer err {err:.3e}, conv err {erry:.3e}", flush=True)
        assert err <= TOL_BF16 and erry <= 1e-4
        # the operator the paper applies after this block
        transpose = (block % 2 == 0) if schedule == 0 else (block % 2 == 1)
        perm = perm.reshape(N, N).T.reshape(-1).copy() if transpose else perm[::-1].copy()
