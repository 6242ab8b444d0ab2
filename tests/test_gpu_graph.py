"""The drivers enqueue kernels only (no allocation, no memset, no host synchronisation), so a caller may
capture them in a HIP graph: every replay must reproduce the eager result for the inputs then in place."""
import pytest
import torch

from paper_2510_08055_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    (inputs.Workload("graph_bf16", H=256, E=16, K=4, I=192, n_layers=3, D=7, P=150, dtype="bf16", seed=71), "group"),
    (inputs.Workload("graph_stack", H=256, E=16, K=4, I=192, n_layers=4, D=5, P=96, dtype="bf16", seed=72), "stack"),
    (inputs.Workload("graph_w4", H=192, E=8, K=2, I=128, n_layers=2, D=4, P=70, dtype="bf16", seed=73,
                     weight_format="mxfp4"), "group"),
]


@pytest.mark.parametrize("w,kind", CASES, ids=[c[0].name for c in CASES])
def test_replays_match_eager(gpu_lib, w, kind):
    layers = [{k: (v.to(DEV) if v is not None else None) for k, v in inputs.make_layer(w, l).items()}
              for l in range(w.n_layers)]
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D + w.P, residual=w.residual, device=DEV,
                          weight_format=w.weight_format)
    packed = ctx.pack_layers(layers)
    xd0, xp0 = inputs.make_hidden(w)
    xd, xp = xd0.to(DEV), xp0.to(DEV)                 # static input buffers of the graph
    yd = torch.empty((w.D, w.H), dtype=torch.bfloat16, device=DEV)
    yp = torch.empty((w.P, w.H), dtype=torch.bfloat16, device=DEV)

    def run(out_d, out_p):
        if kind == "group":
            ctx.moe_group_forward(layers, xd, xp, "chunked", 64, packed=packed, y_decode=out_d, y_prefill=out_p)
        else:
            ctx.moe_stack_forward(layers, xd, xp, chunk=48, n_groups=2, packed=packed, y_decode=out_d, y_prefill=out_p)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(yd, yp)                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(yd, yp)
    for rep in range(4):
        # new inputs in the graph's buffers, eager work and a synchronisation between the replays
        gen = torch.Generator(device="cpu").manual_seed(1000 + rep)
        xd.copy_(torch.randn(xd.shape, generator=gen).to(torch.bfloat16))
        xp.copy_(torch.randn(xp.shape, generator=gen).to(torch.bfloat16))
        ed, ep = torch.empty_like(yd), torch.empty_like(yp)
        run(ed, ep)
        torch.cuda.synchronize()
        yd.zero_()
        yp.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(yd, ed) and torch.equal(yp, ep), f"replay {rep}"
