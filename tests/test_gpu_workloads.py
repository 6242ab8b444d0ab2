"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (same context
size, same schedule, same kernel variants).  Routing, counts and permutation are checked bit for bit for
EVERY token; floating-point outputs on sampled rows the oracle can compute one by one (tokens are
independent in an MoE layer, so a row's value does not depend on the rest of the batch).  Layer groups
are checked teacher-forced: for each layer the oracle is fed the GPU's own bf16 input to that layer.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check_layer(ctx, w, L, x, y, rows, what):
    """Layer output y = layer(x) on the GPU: routing of all rows bit-exact, sampled rows within tolerance."""
    Ln = inputs.layer_to_numpy(L)
    xn = inputs.to_numpy(x)
    idx, wt = ctx.moe_router_topk(x, L["w_router"], L["router_bias"])
    counts, offsets, perm, inv, _ = ctx.moe_permute(x, idx, want_x_perm=False)
    o_idx, o_w, gap = oracle.router_topk(xn, Ln["w_router"], Ln["router_bias"], w.K, want_gap=True)
    assert gap.min() > 1e-9, f"{what}: a token sits on a routing tie"
    assert (idx.cpu().numpy() == o_idx).all(), what
    np.testing.assert_allclose(wt.cpu().numpy(), o_w, rtol=2e-6, atol=1e-9)
    oc, oo, op, oi = oracle.permute(o_idx, w.E)
    assert (counts.cpu().numpy() == oc).all() and (offsets.cpu().numpy() == oo).all(), what
    assert (perm.cpu().numpy() == op).all() and (inv.cpu().numpy() == oi).all(), what
    o_y, _, _, mag = oracle.moe_layer(xn[rows], Ln["w_router"], Ln["router_bias"], Ln["w_gate_up"], Ln["w_down"],
                                      w.K, residual=w.residual, want_mag=True)
    assert_close(y[torch.from_numpy(rows).to(DEV)], o_y, w.dtype, what, mag=np.abs(o_y) + mag)
    return oc


def sample_rows(T, n, seed):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([[0, T - 1], rng.choice(T, size=min(n, T), replace=False)]))


def test_qwen3_group8_layered_and_chunked(gpu_lib):
    w = inputs.WORKLOADS["qwen3_group8"]
    layers = [inputs.make_layer(w, l, device=DEV) for l in range(w.n_layers)]
    xd, xp = inputs.make_hidden(w, device=DEV)
    T = w.D + w.P
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=T, residual=w.residual, device=DEV)
    # layer by layer (teacher-forced check of every layer at T = 8320 rows, ~520 rows per expert)
    x = torch.cat([xd, xp])
    for l, L in enumerate(layers):
        yd, yp = ctx.moe_group_forward([L], x[:w.D], x[w.D:], "layered")
        y = torch.cat([yd, yp])
        oc = check_layer(ctx, w, L, x, y, sample_rows(T, 10, l), f"qwen3_group8 layer {l}")
        assert oc.sum() == T * w.K and oc.mean() == 520        # Sec. 4.3: ~512 tokens per expert: compute-bound
        x = y
    # the group in one call, layered: one pass over every expert's weights per layer
    ctx.moe_reset_counters()
    yd_l, yp_l = ctx.moe_group_forward(layers, xd, xp, "layered")
    c_l = ctx.moe_read_counters()
    assert torch.equal(torch.cat([yd_l, yp_l]), x)
    per_pass = w.E * 3 * w.H * w.I * 2
    assert c_l.expert_bytes == w.n_layers * per_pass and c_l.iterations == 1
    # chunked(512): 16 iterations, every chunk re-streams every expert (Fig. 2: load = per-chunk load x chunks)
    cc = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D + w.chunk, residual=w.residual,
                         device=DEV)
    yd_c, yp_c = cc.moe_group_forward(layers, xd, xp, "chunked", w.chunk)
    c_c = cc.moe_read_counters()
    assert c_c.iterations == 16 and c_c.expert_bytes == 16 * c_l.expert_bytes
    assert torch.equal(yd_c, yd_l) and torch.equal(yp_c, yp_l)      # a scheduling change is not a model change
    # determinism: a second run gives the same bits
    yd_2, yp_2 = ctx.moe_group_forward(layers, xd, xp, "layered")
    assert torch.equal(yd_2, yd_l) and torch.equal(yp_2, yp_l)


def test_mixtral_zipf_layer(gpu_lib):
    w = inputs.WORKLOADS["mixtral_zipf"]
    L = inputs.make_layer(w, 0, device=DEV)
    xd, xp = inputs.make_hidden(w, device=DEV)
    T = w.D + w.P
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=T, residual=w.residual, device=DEV)
    yd, yp = ctx.moe_group_forward([L], xd, xp, "layered")
    oc = check_layer(ctx, w, L, torch.cat([xd, xp]), torch.cat([yd, yp]), sample_rows(T, 14, 3), "mixtral_zipf")
    share = oc / oc.sum()
    assert np.abs(share - inputs.zipf_shares(w.E, w.zipf_s)).max() < 2e-3       # load-imbalanced on purpose
    assert oc.max() > 10 * oc.min()
    yd_c, yp_c = ctx.moe_group_forward([L], xd, xp, "chunked", w.chunk)
    assert torch.equal(yd_c, yd) and torch.equal(yp_c, yp)


def test_decode_large_group(gpu_lib):
    w = inputs.WORKLOADS["decode_large"]
    xd, _ = inputs.make_hidden(w, device=DEV)
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D, residual=w.residual, device=DEV)
    x = xd
    layers = []
    active = 0
    for l in range(w.n_layers):
        L = inputs.make_layer(w, l, device=DEV)
        layers.append(L)
        y, _ = ctx.moe_group_forward([L], x, None, "layered")
        oc = check_layer(ctx, w, L, x, y, sample_rows(w.D, 6, l), f"decode_large layer {l}")
        active += int((oc > 0).sum())
        x = y
    ctx.moe_reset_counters()
    y_all, _ = ctx.moe_group_forward(layers, xd, None, "layered")
    c = ctx.moe_read_counters()
    assert torch.equal(y_all, x)
    assert c.active_experts_total == active and c.expert_bytes == active * 3 * w.H * w.I * 2
    assert active >= 0.99 * w.n_layers * w.E        # 256 tokens x top-4 over 128 experts touch (nearly) all of them


def test_gptoss_layer(gpu_lib):
    # the second model family of Table 3: 32 experts, top-4, hidden size 2880 (264 rows per expert here)
    w = inputs.WORKLOADS["gptoss_layer"]
    L = inputs.make_layer(w, 0, device=DEV)
    xd, xp = inputs.make_hidden(w, device=DEV)
    T = w.D + w.P
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=T, residual=w.residual, device=DEV)
    yd, yp = ctx.moe_group_forward([L], xd, xp, "layered")
    oc = check_layer(ctx, w, L, torch.cat([xd, xp]), torch.cat([yd, yp]), sample_rows(T, 12, 5), "gptoss_layer")
    assert oc.sum() == T * w.K and oc.min() > 0
    yd_c, yp_c = ctx.moe_group_forward([L], xd, xp, "chunked", w.chunk)
    assert torch.equal(yd_c, yd) and torch.equal(yp_c, yp)
