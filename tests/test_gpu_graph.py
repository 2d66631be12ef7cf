"""The entry points that take a caller workspace enqueue kernels only (no allocation, no memset, no host
synchronisation): they can be recorded into a HIP graph and replayed.  Every replay is checked against the eager
result, with eager work and synchronisations of the same entry points between the replays."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2405_18428_amd as gla
from paper_2405_18428_amd import inputs as gi

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    gla.load_library()


def _bf16(d, n, dev):
    return torch.from_numpy(d[n + "_bits"].view(np.int16)).to(dev).view(torch.bfloat16)


def test_forward_and_backward_replay_from_a_graph():
    dev = torch.device("cuda:0")
    B, H, gh, gw, dk, dv = 2, 4, 40, 32, 36, 72
    T = gh * gw
    d = gi.make_inputs(B, H, T, dk, dv, "bf16", seed=61)
    q, k, v = (_bf16(d, n, dev) for n in ("q", "k", "v"))
    la = torch.from_numpy(d["log_alpha"]).to(dev)
    w = torch.randn((B, H, T, dv), device=dev).to(torch.bfloat16)
    out = torch.empty((B, H, T, dv), device=dev)
    fin = torch.empty((B, H, dk, dv), device=dev)
    ws = torch.empty((gla.gla_fwd_workspace_bytes(B, H, T, dk, dv),), dtype=torch.uint8, device=dev)
    ws_b = torch.empty((gla.gla_bwd_workspace_bytes(B, H, T, dk, dv),), dtype=torch.uint8, device=dev)

    # eager reference (also raises the kernels' LDS limits, which must not happen during capture)
    ref_out, ref_fin = (t.clone() for t in gla.gla_fwd_ex(q, k, v, la, gh, gw, 2, out=out, final_state=fin, workspace=ws))
    ref_grads = [t.clone() for t in gla.gla_bwd(q, k, v, la, w, gh, gw, 2, workspace=ws_b)]
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    captured = {}
    with torch.cuda.stream(side):
        # gradients are allocated by the binding: allocate through the graph's private pool
        with torch.cuda.graph(graph, stream=side):
            gla.gla_fwd_ex(q, k, v, la, gh, gw, 2, out=out, final_state=fin, workspace=ws, stream=side)
            captured["grads"] = gla.gla_bwd(q, k, v, la, w, gh, gw, 2, workspace=ws_b, stream=side)
    torch.cuda.synchronize()

    for rep in range(3):
        out.fill_(float("nan"))
        fin.fill_(float("nan"))
        for g in captured["grads"]:
            g.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(fin, ref_fin), rep
        for g, r in zip(captured["grads"], ref_grads):
            assert torch.equal(g, r), rep
        # eager work of the same library between replays (other scan order: overwrites the shared workspaces)
        gla.gla_fwd_ex(q, k, v, la, gh, gw, 1, workspace=ws)
        gla.gla_bwd(q, k, v, la, w, gh, gw, 1, workspace=ws_b)
        torch.cuda.synchronize()


@pytest.mark.parametrize("carry", ["in_output", "kernel"])
def test_two_sided_gate_call_replays_from_a_graph(carry):
    dev = torch.device("cuda:0")
    B, H, gh, gw, dk, dv = 1, 4, 24, 40, 36, 72
    T = gh * gw
    d = gi.make_gate_inputs(B, H, T, dk, dv, "bf16", seed=62)
    q, k, v = (_bf16(d, n, dev) for n in ("q", "k", "v"))
    la, lb = torch.from_numpy(d["log_alpha"]).to(dev), torch.from_numpy(d["log_beta"]).to(dev)
    out = torch.empty((B, H, T, dv), device=dev)
    fin = torch.empty((B, H, dk, dv), device=dev)
    ws = torch.empty((gla.gla_fwd_workspace_bytes(B, H, T, dk, dv),), dtype=torch.uint8, device=dev)
    gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_KERNEL if carry == "kernel" else gla.CARRY_IN_OUTPUT_PASS)
    gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 3)
    try:
        call = lambda scan, stream=None: gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, scan, out=out, final_state=fin,
                                                           workspace=ws, stream=stream)
        ref_out, ref_fin = (t.clone() for t in call(3))
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                call(3, side)
        torch.cuda.synchronize()
        for rep in range(3):
            out.fill_(float("nan"))
            fin.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref_out) and torch.equal(fin, ref_fin), rep
            tmp_o, tmp_f = torch.empty_like(out), torch.empty_like(fin)
            gla.gla_fwd_gates(q, k, v, la, lb, gh, gw, 0, out=tmp_o, final_state=tmp_f, workspace=ws)  # eager, same workspace
            torch.cuda.synchronize()
    finally:
        gla.gla_set_option(gla.OPT_CARRY, gla.CARRY_AUTO)
        gla.gla_set_option(gla.OPT_CHUNKS_PER_SPAN, 0)
