"""The forward entry points only enqueue kernels (no allocation, no memset, no synchronisation), so a caller can
capture them in a HIP graph - the way to run decode-sized steps, where launch overhead shows.  The graph is
replayed several times on fresh inputs, with eager work and synchronisations in between, and every replay must
reproduce the eager result bit for bit (the kernels are deterministic)."""
import pytest
import torch

from oracle import harness
from paper_2605_18643_amd import synth, zeda
from paper_2605_18643_amd.stack import EPS

pytestmark = pytest.mark.gpu

from gpu_util import desc_of, tiled_layer  # noqa: E402


@pytest.mark.parametrize("T, tiled", [(48, True), (48, False), (700, True)])
def test_captured_layer_replays_like_eager(T, tiled):
    w = synth.Workload("graph", T=T, H=256, I=128, N=12, Z=4, K=4, dtype="bf16", seed=61, recipe="zero_bias",
                       x_std=1.0, w_std=0.05, wr_std=0.05, zero_bias=0.4)
    print(w, "tiled" if tiled else "row-major", flush=True)
    L = harness.gapped_layer(w, "cuda")
    if tiled:
        L = tiled_layer(w, L)
    d = desc_of(w, weight_layout=zeda.WEIGHTS_TILED if tiled else zeda.WEIGHTS_ROW_MAJOR)
    ws = torch.empty(zeda.workspace_bytes(d), dtype=torch.uint8, device="cuda")
    x = L["x"].clone()                      # static input buffer of the graph
    out = torch.empty_like(x)
    nreal = torch.zeros(1, dtype=torch.int32, device="cuda")
    x_res = torch.zeros_like(x)             # for the residual-block entry point
    xn_next = torch.empty_like(x)

    def run():
        zeda.zeda_moe_forward(d, x, L["w_router"], L["router_bias"], L["w_gate"], L["w_up"], L["w_down"], out, nreal, ws)
        zeda.zeda_moe_block_forward(d, x, x_res, L["w_router"], L["router_bias"], L["w_gate"], L["w_up"], L["w_down"], None,
                                    EPS, xn_next, nreal, ws)

    run()  # first calls set kernel attributes: outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    gen = torch.Generator().manual_seed(3)
    for rep in range(4):
        new_x = torch.randn(w.T, w.H, generator=gen).to(torch.bfloat16).cuda()
        x.copy_(new_x)
        x_res.fill_(0.25 * rep)
        graph.replay()
        torch.cuda.synchronize()
        got = (out.clone(), x_res.clone(), xn_next.clone(), int(nreal.item()))
        # the same step eagerly, on the same buffers
        x_res.fill_(0.25 * rep)
        run()
        torch.cuda.synchronize()
        want = (out, x_res, xn_next, int(nreal.item()))
        assert got[3] == want[3] and 0 < got[3] < w.T * w.K
        for a, b in zip(got[:3], want[:3]):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {rep}"
        # eager work between the replays
        _ = (new_x.float() @ new_x.float().t()).sum().item()
