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
