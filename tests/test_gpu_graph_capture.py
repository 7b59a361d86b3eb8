"""The entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memset), so a forward + backward can be captured into a HIP graph and
replayed; every replay must reproduce the eager result bit for bit, with eager work and
synchronisations in between."""
import pytest
import torch

from paper_2507_00394_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    from paper_2507_00394_amd import binding as hx
    from tests import gpu_util as G

    cfg = I.CONFIGS[1]
    bits = I.all_inputs_bits(cfg)
    eager = G.run_fwd_bwd(bits, cfg.scale, True)
    q, k, v, g = (eager[t] for t in ("q", "k", "v", "dO"))
    B, H, S, D = q.shape
    o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")

    def run():
        hx.helix_attn_fwd(q, k, v, o, lse, cfg.scale, True)
        hx.helix_attn_bwd(q, k, v, o, lse, g, dq, dk, dv, ws, cfg.scale, True)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(4):
        for t in (o, dq, dk, dv):
            t.fill_(float("nan"))   # eager work between the replays
        lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv)):
            assert torch.equal(t.view(torch.int16), eager[n].view(torch.int16)), f"{n} differs in replay {rep}"
        assert torch.equal(lse, eager["lse"]), f"lse differs in replay {rep}"
