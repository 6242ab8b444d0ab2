"""The router entry point that allocates nothing (static device scratch instead of a workspace), through the
C ABI, against the context-based moe_router_topk: two calls in a row, the second with a smaller input."""
import pytest
import torch

from paper_2510_08055_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_router_topk_noalloc_equals_the_workspace_call(gpu_lib):
    H, E, K = 512, 128, 8
    wr = inputs.randn((E, H), 0.02, 71, "w_router", 0, "bf16").to(DEV)
    bias = inputs.randn((E,), 0.5, 71, "bias", 0, "f32").to(DEV)
    ctx = gpu_lib.Context(H, E, K, 64, torch.bfloat16, max_tokens=4096, device=DEV)
    for T in (4096, 333):       # the largest batch the static scratch takes for 128 experts, then a smaller one
        x = inputs.randn((T, H), 1.0, 71 + T, "x", 0, "bf16").to(DEV)
        ref_idx, ref_w = ctx.moe_router_topk(x, wr, bias)
        idx = torch.full((T, K), -1, dtype=torch.int32, device=DEV)
        w = torch.full((T, K), -1.0, dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        gpu_lib.moe_router_topk_noalloc(x, wr, bias, K, topk_idx=idx, topk_w=w)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(idx, ref_idx) and torch.equal(w, ref_w)
    # one row more than the scratch holds is refused before anything is launched
    x = torch.zeros((4097, H), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(gpu_lib.MoeError) as e:
        gpu_lib.moe_router_topk_noalloc(x, wr, bias, K)
    assert e.value.status == 5
    # fp32 inputs, no bias, no renormalisation
    xf = inputs.randn((100, 256), 1.0, 72, "x", 0, "f32").to(DEV)
    wf = inputs.randn((8, 256), 0.02, 72, "w_router", 0, "f32").to(DEV)
    c2 = gpu_lib.Context(256, 8, 2, 64, torch.float32, max_tokens=100, renormalize=False, device=DEV)
    a = c2.moe_router_topk(xf, wf)
    b = gpu_lib.moe_router_topk_noalloc(xf, wf, None, 2, renormalize=False)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
