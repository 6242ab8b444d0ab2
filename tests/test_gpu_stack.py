"""GPU parity of the whole-stack schedules (Sec. 4.1-4.4) through the C ABI.

Outputs: the plain pass over all layers is checked layer by layer against the oracle (teacher-forced: the
oracle is fed the GPU's own input to each layer), and every stack schedule must reproduce that pass bit
for bit.  Counters: compared with the oracle's stack schedule
where the activated-expert count does not depend on rounding (full coverage; a lone decode token activates
exactly k experts) and with the closed forms.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

STACK = inputs.Workload("stack", H=256, E=16, K=4, I=320, n_layers=6, D=9, P=200, dtype="bf16", chunk=64, seed=43)


def dev_layer(layer):
    return {k: (v.to(DEV) if v is not None else None) for k, v in layer.items()}


def make_ctx(lib, w, max_tokens):
    return lib.Context(w.H, w.E, w.K, w.I, inputs.torch_dtype(w.dtype), max_tokens=max_tokens, residual=w.residual,
                       device=DEV)


def test_group_count_rule_and_groups_match_the_oracle(gpu_lib):
    for L in (0, 1, 511, 512, 513, 8192, 8193, 100000):
        for n_layers in (1, 16, 48):
            for gran in (256, 512):
                assert gpu_lib.moe_num_layer_groups(L, n_layers, gran) == oracle.num_layer_groups(L, n_layers, gran)
    assert gpu_lib.moe_num_layer_groups(8192, 48, 512) == 16 and gpu_lib.moe_num_layer_groups(512, 48, 512) == 1
    for n_layers, g in ((48, 16), (10, 4), (7, 7), (5, 1), (24, 5)):
        assert gpu_lib.moe_layer_groups(n_layers, g) == oracle.layer_groups(n_layers, g).tolist()
    with pytest.raises(gpu_lib.MoeError):
        gpu_lib.moe_layer_groups(4, 5)


@pytest.mark.parametrize("D", [9, 0])
def test_every_stack_schedule_gives_the_plain_pass(gpu_lib, D):
    w = inputs.scaled(STACK, D=D)
    layers = [inputs.make_layer(w, l) for l in range(w.n_layers)]
    dl = [dev_layer(L) for L in layers]
    nl = [inputs.layer_to_numpy(L) for L in layers]
    xd, xp = inputs.make_hidden(w)
    xd_d = xd.to(DEV) if D else None
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    ref_d, ref_p = ctx.moe_group_forward(dl, xd_d, xp.to(DEV), "layered")
    # teacher-forced: layer by layer, the oracle is fed the GPU's own bf16 input to each layer
    x = torch.cat([xd.to(DEV), xp.to(DEV)]) if D else xp.to(DEV)
    for l in range(w.n_layers):
        yd, yp = ctx.moe_group_forward([dl[l]], x[:w.D] if D else None, x[w.D:], "layered")
        y = torch.cat([yd, yp]) if D else yp
        o_y, o_idx, _ = oracle.moe_layer(inputs.to_numpy(x), nl[l]["w_router"], None, nl[l]["w_gate_up"],
                                         nl[l]["w_down"], w.K, residual=True)
        idx, _ = ctx.moe_router_topk(x, dl[l]["w_router"])
        assert (idx.cpu().numpy() == o_idx).all()
        assert_close(y, o_y, "bf16", f"stack layer {l}")
        x = y
    assert torch.equal(x[w.D:], ref_p) and (not D or torch.equal(x[:w.D], ref_d))
    # free running against the oracle's own stack schedule: six layers of bf16 rounding apart, so only
    # the relative L2 error is held to the bound
    o_d, o_p, _ = oracle.stack_forward(nl, inputs.to_numpy(xd), inputs.to_numpy(xp), w.K, chunk=0, n_groups=3)
    rel = np.linalg.norm(ref_p.double().cpu().numpy() - o_p) / np.linalg.norm(o_p)
    assert rel <= 5e-3, rel
    for chunk, n_groups, granule in ((0, 1, 0), (0, 2, 0), (0, 6, 0), (0, 4, 0), (64, 1, 0), (64, 3, 0), (33, 6, 0),
                                     (0, 0, 64), (128, 0, 32), (500, 2, 0)):
        ctx.moe_reset_counters()
        yd, yp = ctx.moe_stack_forward(dl, xd_d, xp.to(DEV), chunk=chunk, n_groups=n_groups, granule=granule)
        c = ctx.moe_read_counters()
        assert torch.equal(yp, ref_p), (chunk, n_groups, granule)
        if D:
            assert torch.equal(yd, ref_d), (chunk, n_groups, granule)
        _, _, oc = oracle.stack_forward(nl, inputs.to_numpy(xd), inputs.to_numpy(xp), w.K, chunk=chunk,
                                        n_groups=n_groups, granule=max(granule, 1))
        assert (c.iterations, c.layer_passes, c.tokens_processed, c.router_bytes) == \
               (oc.iterations, oc.layer_passes, oc.tokens_processed, oc.router_bytes), (chunk, n_groups, granule)


def test_stack_counters_follow_the_traffic_model(gpu_lib):
    # one decode token + 192 prompt tokens, E = 16, top-4: a decode-only pass activates exactly 4 experts,
    # a pass with (a share of) the prompt all 16
    w = inputs.scaled(STACK, D=1, P=192, n_layers=4)
    layers = [inputs.make_layer(w, l) for l in range(w.n_layers)]
    dl = [dev_layer(L) for L in layers]
    nl = [inputs.layer_to_numpy(L) for L in layers]
    xd, xp = inputs.make_hidden(w)
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    We = 3 * w.H * w.I * 2
    G = 4
    got = {}
    for name, kw in (("layered", dict(chunk=0, n_groups=G)), ("chunked", dict(chunk=w.P // G, n_groups=1)),
                     ("hybrid", dict(chunk=w.P // 2, n_groups=2))):
        ctx.moe_reset_counters()
        ctx.moe_stack_forward(dl, xd.to(DEV), xp.to(DEV), **kw)
        c = ctx.moe_read_counters()
        _, _, oc = oracle.stack_forward(nl, inputs.to_numpy(xd), inputs.to_numpy(xp), w.K, **kw)
        assert c.iterations == G and c == gpu_lib.Counters(oc.expert_bytes, oc.router_bytes, oc.active_experts_total,
                                                           oc.tokens_processed, oc.iterations, oc.layer_passes), name
        got[name] = c
    assert got["layered"].active_experts_total == w.n_layers * (w.E + (G - 1) * w.K)
    assert got["chunked"].active_experts_total == G * w.n_layers * w.E
    assert got["hybrid"].active_experts_total == w.n_layers * (2 * w.E + 2 * w.K)
    assert got["layered"].expert_bytes == got["layered"].active_experts_total * We
    saving = 1 - got["layered"].expert_bytes / got["chunked"].expert_bytes
    assert abs(saving - (1 - (1 + (G - 1) * w.K / w.E) / G)) < 1e-12


def test_stack_forward_argument_errors(gpu_lib):
    w = STACK
    dl = [dev_layer(inputs.make_layer(w, l)) for l in range(2)]
    xd, xp = (t.to(DEV) for t in inputs.make_hidden(w))
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    for kw, status in ((dict(chunk=-1, n_groups=1), 6), (dict(n_groups=-1), 6), (dict(n_groups=3), 6),
                       (dict(n_groups=0, granule=0), 6)):
        with pytest.raises(gpu_lib.MoeError) as e:
            ctx.moe_stack_forward(dl, xd, xp, **kw)
        assert e.value.status == status, kw
    with pytest.raises(gpu_lib.MoeError) as e:                  # an output may not be its own input
        ctx.moe_stack_forward(dl, xd, xp, n_groups=2, y_prefill=xp)
    assert e.value.status == 2
    small = make_ctx(gpu_lib, w, 64)
    with pytest.raises(gpu_lib.MoeError) as e:
        small.moe_stack_forward(dl, xd, xp, n_groups=2)
    assert e.value.status == 2
    yd, yp = small.moe_stack_forward(dl, xd, xp, chunk=50, n_groups=2)          # 9 + 50 rows fit
    ref = ctx.moe_group_forward(dl, xd, xp, "layered")
    assert torch.equal(yd, ref[0]) and torch.equal(yp, ref[1])
    ctx.moe_stack_forward(dl, None, None, n_groups=1)                           # nothing at all is a no-op
