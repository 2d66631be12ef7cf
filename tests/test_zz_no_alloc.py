"""gla_fwd_static (the entry point that allocates nothing: span states in a static device array) against gla_fwd
on the same inputs, and against the oracle, on two calls in a row, the second on a smaller problem."""
import numpy as np
import pytest

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2   # max |err| / RMS(oracle out), bf16 inputs with fp32 accumulation


def _device_inputs(torch, d):
    dev = torch.device("cuda:0")
    to = lambda bits: torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)
    return to(d["q_bits"]), to(d["k_bits"]), to(d["v_bits"]), torch.from_numpy(d["log_alpha"]).to(dev)


def _one_call(torch, oracle, B, H, gh, gw, dk, dv, scan, seed):
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=seed)
    q, k, v, la = _device_inputs(torch, d)
    dev = q.device
    # everything the static call touches is allocated here, before it
    out_s = torch.full((B, H, T, dv), 1e30, dtype=torch.float32, device=dev)
    fin_s = torch.full((B, H, dk, dv), 1e30, dtype=torch.float32, device=dev)
    out_r, fin_r = gla.gla_fwd(q, k, v, la, gh, gw, scan)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    gla.gla_fwd_static(q, k, v, la, gh, gw, scan, out=out_s, final_state=fin_s)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before   # (torch's allocator: not asked)
    ref, ref_fin = oracle.gla_fwd(d["q"], d["k"], d["v"], d["log_alpha"], gh, gw, scan)
    rms, rms_f = np.sqrt(np.mean(ref ** 2)), np.sqrt(np.mean(ref_fin ** 2))
    got, got_f = out_s.cpu().numpy(), fin_s.cpu().numpy()
    # against the existing entry point: the same kernels on the same plan
    assert np.abs(got - out_r.cpu().numpy()).max() <= TOL_BF16 * rms
    assert np.abs(got_f - fin_r.cpu().numpy()).max() <= TOL_BF16 * rms_f
    # and against the oracle
    assert np.abs(got - ref).max() <= TOL_BF16 * rms
    assert np.abs(got_f - ref_fin).max() <= TOL_BF16 * rms_f


def test_static_scratch_two_calls_second_smaller(oracle):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    gla.load_library()
    # several spans per head (the scratch holds span states), then a smaller problem that reuses the array
    _one_call(torch, oracle, 2, 16, 64, 64, 36, 72, gla.SCAN_COL_REV, seed=11)
    _one_call(torch, oracle, 1, 6, 28, 20, 32, 64, gla.SCAN_ROW_FWD, seed=12)
