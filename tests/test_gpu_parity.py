"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Routing indices, per-expert counts, offsets and the permutation must agree bit
for bit; floating-point outputs within the tolerance of tests/parity.py of the oracle's UNROUNDED
fp64 value (bf16: max-abs <= 2e-2, relative L2 <= 5e-3; fp32: max-abs <= 1e-4, relative L2 <= 1e-5).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
def make_ctx(gpu_lib, w, max_tokens, residual=None):
    return gpu_lib.Context(w.H, w.E, w.K, w.I, inputs.torch_dtype(w.dtype), max_tokens=max_tokens,
                           residual=w.residual if residual is None else residual, device=DEV)


def dev_layer(layer):
    return {k: (v.to(DEV) if v is not None else None) for k, v in layer.items()}


# --------------------------------------------------------------------------- router
@pytest.mark.parametrize("T,H,E,K,dtype,bias", [
    (64, 256, 8, 2, "f32", False),
    (77, 256, 8, 2, "bf16", True),
    (300, 2048, 128, 8, "bf16", False),
    (33, 2880, 32, 4, "bf16", False),
    (50, 512, 128, 4, "bf16", True),
    (19, 64, 1, 1, "bf16", False),
    (40, 128, 200, 5, "bf16", False),       # E not a multiple of 16 or 64
    (5, 72, 16, 16, "f32", False),          # K = E, H not a multiple of 32
    (45, 128, 300, 12, "bf16", True),       # more than 256 experts: 32 logits per lane in the 16-lane-row kernel
    (30, 128, 64, 24, "bf16", True),        # K > 16: the one-token-per-wave kernel
    (9, 256, 512, 64, "bf16", False),       # the largest E and K the library takes
])
def test_router_topk_bit_exact(gpu_lib, T, H, E, K, dtype, bias):
    w = inputs.Workload("r", H=H, E=E, K=K, I=64, n_layers=1, D=0, P=T, dtype=dtype, seed=T + E)
    x = inputs.randn((T, H), 1.0, w.seed, "x", 0, dtype)
    wr = inputs.randn((E, H), 0.02, w.seed, "w_router", 0, dtype)
    b = inputs.randn((E,), 0.5, w.seed, "bias", 0, "f32") if bias else None
    for renorm in (True, False):
        c2 = gpu_lib.Context(H, E, K, 64, inputs.torch_dtype(dtype), max_tokens=T, renormalize=renorm, device=DEV)
        idx, wt = c2.moe_router_topk(x.to(DEV), wr.to(DEV), None if b is None else b.to(DEV))
        o_idx, o_w, gap = oracle.router_topk(inputs.to_numpy(x), inputs.to_numpy(wr),
                                             None if b is None else b.numpy(), K, renormalize=renorm, want_gap=True)
        assert gap.min() > 1e-9, "seed produced a near-tie; routing order would be ill-defined"
        assert (idx.cpu().numpy() == o_idx).all()
        np.testing.assert_allclose(wt.cpu().numpy(), o_w, rtol=2e-6, atol=1e-9)


def test_router_ties_go_to_the_lower_index(gpu_lib):
    H, E, K = 64, 16, 5
    ctx = gpu_lib.Context(H, E, K, 64, torch.bfloat16, max_tokens=64, device=DEV)
    wr = inputs.randn((E, H), 0.02, 3, "w_router", 0, "bf16")
    wr[9] = wr[3]
    idx, w = ctx.moe_router_topk(torch.zeros((8, H), dtype=torch.bfloat16, device=DEV), wr.to(DEV))
    assert (idx.cpu().numpy() == np.arange(K)[None, :]).all()
    np.testing.assert_allclose(w.cpu().numpy(), 1.0 / K, rtol=1e-6)
    x = inputs.randn((64, H), 1.0, 3, "x", 0, "bf16")
    idx, _ = ctx.moe_router_topk(x.to(DEV), wr.to(DEV))
    o_idx, _ = oracle.router_topk(inputs.to_numpy(x), inputs.to_numpy(wr), None, K)
    assert (idx.cpu().numpy() == o_idx).all()           # experts 3 and 9 tie exactly in every token


# -------------------------------------------------------------------------- permute
@pytest.mark.parametrize("T,K,E", [(1, 1, 1), (7, 2, 8), (64, 2, 8), (1024, 8, 128), (1025, 8, 128),
                                   (2112, 8, 128), (8320, 8, 128), (4128, 2, 8), (256, 4, 128), (999, 5, 300),
                                   (3000, 3, 512)])
def test_permute_bit_exact(gpu_lib, T, K, E):
    rng = np.random.default_rng(T * 7 + E)
    # K distinct experts per token, skewed popularity so that per-expert counts differ widely
    pop = rng.random(E) ** 3 + 1e-3
    idx = np.stack([rng.choice(E, size=K, replace=False, p=pop / pop.sum()) for _ in range(T)]).astype(np.int32)
    H = 64
    x = inputs.randn((T, H), 1.0, T, "x", 0, "bf16")
    ctx = gpu_lib.Context(H, E, K, 64, torch.bfloat16, max_tokens=T, device=DEV)
    counts, offsets, perm, inv, x_perm = ctx.moe_permute(x.to(DEV), torch.from_numpy(idx).to(DEV))
    oc, oo, op, oi = oracle.permute(idx, E)
    assert (counts.cpu().numpy() == oc).all() and (offsets.cpu().numpy() == oo).all()
    assert (perm.cpu().numpy() == op).all() and (inv.cpu().numpy() == oi).all()
    assert torch.equal(x_perm.cpu(), x[torch.from_numpy(op // K).long()])
    # run twice: the order never depends on timing
    again = ctx.moe_permute(x.to(DEV), torch.from_numpy(idx).to(DEV))
    assert torch.equal(again[2], perm) and torch.equal(again[3], inv)


def test_step_calls_on_an_empty_batch(gpu_lib):
    """No rows: every step call is a no-op, except that the permutation still reports E zero counts and E + 1 zero
    offsets (written by a fill kernel, so that the call stays capturable)."""
    H, E, K, I = 128, 8, 2, 64
    ctx = gpu_lib.Context(H, E, K, I, torch.bfloat16, max_tokens=16, device=DEV)
    x = torch.zeros((0, H), dtype=torch.bfloat16, device=DEV)
    wr = inputs.randn((E, H), 0.02, 5, "wr", 0, "bf16").to(DEV)
    idx, w = ctx.moe_router_topk(x, wr)
    assert idx.shape == (0, K) and w.shape == (0, K)
    counts, offsets, perm, inv, x_perm = ctx.moe_permute(x, idx)
    assert counts.shape == (E,) and offsets.shape == (E + 1,)
    assert int(counts.abs().sum()) == 0 and int(offsets.abs().sum()) == 0
    assert perm.numel() == 0 and inv.numel() == 0 and x_perm.shape == (0, H)
    wg = torch.zeros((E, 2 * I, H), dtype=torch.bfloat16, device=DEV)
    wd = torch.zeros((E, H, I), dtype=torch.bfloat16, device=DEV)
    y_perm = ctx.moe_grouped_ffn(x_perm, offsets, wg, wd)
    assert y_perm.shape == (0, H)
    y = ctx.moe_combine(y_perm, inv, w)
    assert y.shape == (0, H)


# ------------------------------------------------------------- grouped FFN and combine
@pytest.mark.parametrize("H,I,E,rows,dtype", [
    (256, 512, 4, [130, 0, 1, 64], "bf16"),       # an empty expert, a 1-row expert, a ragged tile
    (256, 512, 3, [5, 200, 33], "f32"),
    (192, 72, 2, [257, 31], "bf16"),              # N and K tails: I = 72, H = 192
    (256, 320, 5, [3, 0, 70, 1, 33], "bf16"),     # mean 21 rows/expert: streaming variant, one 32-row block per pass
    (2880, 2880, 3, [8, 5, 11], "bf16"),          # decode-like: H = I = 2880 (tails in N), 8 rows per expert
    (256, 328, 5, [40, 64, 65, 0, 100], "bf16"),  # mean 54 rows/expert: streaming variant, two row blocks per pass
])
def test_grouped_ffn_is_the_dense_swiglu_of_each_expert(gpu_lib, H, I, E, rows, dtype):
    A = sum(rows)
    w = inputs.Workload("f", H=H, E=E, K=1, I=I, n_layers=1, D=0, P=A, dtype=dtype, seed=11)
    L = inputs.make_layer(w, 0)
    x_perm = inputs.randn((A, H), 1.0, 11, "x_perm", 0, dtype)
    offsets = torch.tensor(np.concatenate([[0], np.cumsum(rows)]), dtype=torch.int32)
    ctx = make_ctx(gpu_lib, w, A)
    y = ctx.moe_grouped_ffn(x_perm.to(DEV), offsets.to(DEV), L["w_gate_up"].to(DEV), L["w_down"].to(DEV))
    ref = np.zeros((A, H))
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:   # a one-expert MoE layer is that expert's dense FFN with weight 1
            ones = inputs.to_numpy(torch.ones((1, H), dtype=inputs.torch_dtype(dtype)))
            ref[lo:hi], _, _ = oracle.moe_layer(inputs.to_numpy(x_perm[lo:hi]), ones, None,
                                                inputs.to_numpy(L["w_gate_up"][e:e + 1]),
                                                inputs.to_numpy(L["w_down"][e:e + 1]), 1)
    assert_close(y, ref, dtype, "grouped_ffn")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_combine_weighted_sum_and_residual(gpu_lib, dtype):
    T, K, H, E = 37, 3, 136, 8
    ctx = gpu_lib.Context(H, E, K, 64, inputs.torch_dtype(dtype), max_tokens=T, device=DEV)
    rng = np.random.default_rng(5)
    y_perm = inputs.randn((T * K, H), 1.0, 5, "y_perm", 0, dtype)
    res = inputs.randn((T, H), 1.0, 5, "res", 0, dtype)
    inv = torch.from_numpy(rng.permutation(T * K).astype(np.int32))
    wt = torch.from_numpy(rng.random((T, K)).astype(np.float32))
    yp64 = y_perm.double().numpy()
    ref = (wt.double().numpy()[:, :, None] * yp64[inv.numpy().reshape(T, K)]).sum(1)
    y = ctx.moe_combine(y_perm.to(DEV), inv.to(DEV), wt.to(DEV))
    assert_close(y, ref, dtype, "combine")
    r_dev = res.to(DEV)
    y2 = ctx.moe_combine(y_perm.to(DEV), inv.to(DEV), wt.to(DEV), residual=r_dev, out=r_dev)   # in place
    assert_close(y2, ref + res.double().numpy(), dtype, "combine+residual")


# --------------------------------------------------------------- one layer, step by step
def _layer_steps(ctx, x, L):
    idx, wt = ctx.moe_router_topk(x, L["w_router"], L["router_bias"])
    counts, offsets, perm, inv, x_perm = ctx.moe_permute(x, idx)
    y_perm = ctx.moe_grouped_ffn(x_perm, offsets, L["w_gate_up"], L["w_down"])
    y = ctx.moe_combine(y_perm, inv, wt)
    return idx, wt, counts, offsets, perm, inv, y


SMALL_LAYERS = [
    inputs.Workload("s_bf16", H=256, E=8, K=2, I=512, n_layers=1, D=11, P=300, dtype="bf16", seed=31, residual=False),
    inputs.Workload("s_f32", H=256, E=8, K=2, I=512, n_layers=1, D=0, P=64, dtype="f32", seed=0, residual=False),
    inputs.Workload("s_many", H=512, E=128, K=8, I=192, n_layers=1, D=64, P=333, dtype="bf16", seed=32, residual=False),
    inputs.Workload("s_dense", H=320, E=1, K=1, I=136, n_layers=1, D=0, P=150, dtype="bf16", seed=33, residual=False),
    inputs.Workload("s_kE", H=128, E=4, K=4, I=64, n_layers=1, D=3, P=70, dtype="bf16", seed=34, residual=False),
]


@pytest.mark.parametrize("w", SMALL_LAYERS, ids=lambda w: w.name)
def test_single_layer_steps_and_group_call(gpu_lib, w):
    L = inputs.make_layer(w, 0)
    xd, xp = inputs.make_hidden(w)
    x = torch.cat([xd, xp])
    T = w.D + w.P
    ctx = make_ctx(gpu_lib, w, T)
    Ld = dev_layer(L)
    idx, wt, counts, offsets, perm, inv, y = _layer_steps(ctx, x.to(DEV), Ld)
    Ln = inputs.layer_to_numpy(L)
    o_y, o_idx, o_w = oracle.moe_layer(inputs.to_numpy(x), Ln["w_router"], None, Ln["w_gate_up"], Ln["w_down"], w.K)
    _, _, gap = oracle.router_topk(inputs.to_numpy(x), Ln["w_router"], None, w.K, want_gap=True)
    assert gap.min() > 1e-9
    oc, oo, op, oi = oracle.permute(o_idx, w.E)
    assert (idx.cpu().numpy() == o_idx).all()
    assert (counts.cpu().numpy() == oc).all() and (offsets.cpu().numpy() == oo).all()
    assert (perm.cpu().numpy() == op).all() and (inv.cpu().numpy() == oi).all()
    assert_close(y, o_y, w.dtype, "layer")
    # the fused driver (gathers rows inside the GEMM instead of materialising x_perm) gives the same bits
    for sched, chunk in (("layered", 0), ("chunked", 64), ("chunked", 7)):
        yd, yp = ctx.moe_group_forward([Ld], xd.to(DEV), xp.to(DEV), sched, chunk)
        assert torch.equal(torch.cat([yd, yp]), y), (sched, chunk)


# ---------------------------------------------------------------- layer group, schedules
GROUP = inputs.Workload("g", H=256, E=16, K=4, I=320, n_layers=3, D=9, P=200, dtype="bf16", chunk=64, seed=41)


def test_group_forward_teacher_forced_and_schedules(gpu_lib):
    w = GROUP
    layers = [inputs.make_layer(w, l) for l in range(w.n_layers)]
    dl = [dev_layer(L) for L in layers]
    nl = [inputs.layer_to_numpy(L) for L in layers]
    xd, xp = inputs.make_hidden(w)
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    # layer by layer on the GPU; the oracle is fed the GPU's own input to each layer
    x = torch.cat([xd, xp]).to(DEV)
    for l in range(w.n_layers):
        ctx.moe_reset_counters()
        yd, yp = ctx.moe_group_forward([dl[l]], x[:w.D], x[w.D:], "layered")
        y = torch.cat([yd, yp])
        o_y, o_idx, _ = oracle.moe_layer(inputs.to_numpy(x), nl[l]["w_router"], None, nl[l]["w_gate_up"],
                                         nl[l]["w_down"], w.K, residual=True)
        idx, _ = ctx.moe_router_topk(x, dl[l]["w_router"])
        assert (idx.cpu().numpy() == o_idx).all()
        assert_close(y, o_y, "bf16", f"layer {l}")
        assert ctx.moe_read_counters().active_experts_total == len(set(o_idx.reshape(-1).tolist()))
        x = y
    # the whole group in one call equals the chain of single-layer calls, under either schedule
    ctx.moe_reset_counters()
    yd_l, yp_l = ctx.moe_group_forward(dl, xd.to(DEV), xp.to(DEV), "layered")
    c_l = ctx.moe_read_counters()
    assert torch.equal(torch.cat([yd_l, yp_l]), x)
    ctx.moe_reset_counters()
    yd_c, yp_c = ctx.moe_group_forward(dl, xd.to(DEV), xp.to(DEV), "chunked", w.chunk)
    c_c = ctx.moe_read_counters()
    assert torch.equal(yd_c, yd_l) and torch.equal(yp_c, yp_l)
    # counters follow the traffic model: chunked re-streams the experts once per chunk
    n_it = -(-w.P // w.chunk)
    assert (c_l.iterations, c_l.layer_passes, c_l.tokens_processed) == (1, w.n_layers, w.D + w.P)
    assert (c_c.iterations, c_c.layer_passes, c_c.tokens_processed) == (n_it, n_it * w.n_layers, n_it * w.D + w.P)
    per_expert = 3 * w.H * w.I * 2
    assert c_l.expert_bytes == c_l.active_experts_total * per_expert
    assert c_l.expert_bytes == w.n_layers * w.E * per_expert          # full coverage at this batch size
    assert c_c.expert_bytes == n_it * c_l.expert_bytes                # C-fold
    assert c_c.router_bytes == n_it * w.n_layers * w.E * w.H * 2
    # free-running oracle agrees with the GPU's counters
    _, _, oc = oracle.group_forward(nl, inputs.to_numpy(xd), inputs.to_numpy(xp), w.K, "chunked", w.chunk)
    assert (oc.iterations, oc.layer_passes, oc.tokens_processed) == (c_c.iterations, c_c.layer_passes,
                                                                     c_c.tokens_processed)


def test_group_forward_edge_cases(gpu_lib):
    w = GROUP
    layers = [dev_layer(inputs.make_layer(w, l)) for l in range(2)]
    xd, xp = (t.to(DEV) for t in inputs.make_hidden(w))
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    full_d, full_p = ctx.moe_group_forward(layers, xd, xp, "layered")
    # decode only: one iteration under either schedule, same rows as in the hybrid batch
    ctx.moe_reset_counters()
    d1, _ = ctx.moe_group_forward(layers, xd, None, "layered")
    d2, _ = ctx.moe_group_forward(layers, xd, None, "chunked", 16)
    assert ctx.moe_read_counters().iterations == 2
    assert torch.equal(d1, full_d) and torch.equal(d2, full_d)
    # prefill only, chunk not dividing P, chunk larger than P
    for chunk in (1000, 64, 33):
        _, p = ctx.moe_group_forward(layers, None, xp, "chunked", chunk)
        assert torch.equal(p, full_p)
    # nothing at all is a no-op
    ctx.moe_group_forward(layers, None, None, "layered")
    # argument errors come back as status codes
    with pytest.raises(gpu_lib.MoeError) as e:
        ctx.moe_group_forward(layers, xd, xp, "chunked", 0)
    assert e.value.status == 6
    small = make_ctx(gpu_lib, w, 32)
    with pytest.raises(gpu_lib.MoeError) as e:
        small.moe_group_forward(layers, xd, xp, "layered")
    assert e.value.status == 2
    small.moe_group_forward(layers, xd, xp, "chunked", 16)        # fits: 9 + 16 rows per iteration


# ------------------------------------------------ output-side formats and kernel shapes
FORMATS = [dict(), dict(y_perm_f32=True), dict(y_perm_f32=True, act_split=True)]
FORMAT_LAYERS = [
    SMALL_LAYERS[0], SMALL_LAYERS[2],
    inputs.Workload("s_tail", H=192, E=4, K=2, I=72, n_layers=1, D=7, P=290, dtype="bf16", seed=35, residual=False),   # k tails: tile kernel only
    inputs.Workload("s_wide", H=128, E=2, K=1, I=1216, n_layers=1, D=0, P=330, dtype="bf16", seed=36, residual=True),   # 19 + 19 k-stages in the down GEMM
]


@pytest.mark.parametrize("fmt", range(len(FORMATS)), ids=["bf16", "y_perm_f32", "act_split"])
@pytest.mark.parametrize("w", FORMAT_LAYERS, ids=lambda w: w.name)
def test_output_side_formats_on_every_kernel_shape(gpu_lib, w, fmt):
    """Expert outputs in fp32 and the intermediate as a bf16 pair: every grouped-GEMM shape gives the same bits,
    the step calls equal the fused driver, and the result stays within tolerance of the oracle (closer to it
    the more is kept: checked on the relative L2 error)."""
    L = inputs.make_layer(w, 0)
    Ld, Ln = dev_layer(L), inputs.layer_to_numpy(L)
    xd, xp = inputs.make_hidden(w)
    x = torch.cat([xd, xp]).to(DEV)
    o_y, _, _ = oracle.moe_layer(inputs.to_numpy(x), Ln["w_router"], None, Ln["w_gate_up"], Ln["w_down"], w.K,
                                 residual=w.residual)
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D + w.P, residual=w.residual, device=DEV,
                          **FORMATS[fmt])
    outs = {}
    for variant in ("tile128", "small", "big", "auto"):
        ctx.moe_set_ffn_variant(variant)
        idx, wt = ctx.moe_router_topk(x, Ld["w_router"])
        _, offsets, _, inv, x_perm = ctx.moe_permute(x, idx)
        y_perm = ctx.moe_grouped_ffn(x_perm, offsets, Ld["w_gate_up"], Ld["w_down"])
        assert y_perm.dtype == (torch.float32 if fmt else torch.bfloat16)
        y = ctx.moe_combine(y_perm, inv, wt, residual=x if w.residual else None)
        yd, yp = ctx.moe_group_forward([Ld], x[:w.D] if w.D else None, x[w.D:], "layered")
        assert torch.equal(torch.cat([t for t in (yd, yp) if t.shape[0]]), y), variant
        yd, yp = ctx.moe_group_forward([Ld], x[:w.D] if w.D else None, x[w.D:], "chunked", 100)
        assert torch.equal(torch.cat([t for t in (yd, yp) if t.shape[0]]), y), variant
        outs[variant] = y
    for variant in ("small", "big", "auto"):
        assert torch.equal(outs[variant], outs["tile128"]), variant
    st = assert_close(outs["auto"], o_y, "bf16", f"{w.name} {FORMATS[fmt]}")
    # what each format is for: the error that is left
    base = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D + w.P, residual=w.residual, device=DEV)
    yd, yp = base.moe_group_forward([Ld], x[:w.D] if w.D else None, x[w.D:], "layered")
    st0 = assert_close(torch.cat([t for t in (yd, yp) if t.shape[0]]), o_y, "bf16", w.name)
    if fmt:
        assert st["rel_l2"] < st0["rel_l2"]


def test_config_rejects_bad_output_side_formats(gpu_lib):
    for kw in (dict(act_split=True), dict(y_perm_f32=True, act_split=True, weight_format="mxfp4")):
        with pytest.raises(gpu_lib.MoeError) as e:
            gpu_lib.Context(128, 4, 2, 64, torch.bfloat16, max_tokens=8, device=DEV, **kw)
        assert e.value.status == 3
    with pytest.raises(gpu_lib.MoeError) as e:
        gpu_lib.Context(128, 4, 2, 64, torch.float32, max_tokens=8, device=DEV, y_perm_f32=True, act_split=True)
    assert e.value.status == 3
    ctx = gpu_lib.Context(128, 4, 2, 64, torch.bfloat16, max_tokens=8, device=DEV)
    with pytest.raises(gpu_lib.MoeError) as e:
        ctx.moe_set_ffn_variant(9)
    assert e.value.status == 2


# ------------------------------------------------------------ fp32 layer group
GROUP_F32 = inputs.Workload("g_f32", H=256, E=8, K=2, I=512, n_layers=3, D=5, P=59, dtype="f32", chunk=16, seed=42)


def test_fp32_group_teacher_forced_and_free_running(gpu_lib):
    """The fp32 path between layers: per layer against the oracle fed the GPU's own fp32 input, the group call
    against the chain of single-layer calls (bit for bit, both schedules), and the whole group against the
    oracle's own free-running pass, which rounds to fp32 between layers."""
    w = GROUP_F32
    layers = [inputs.make_layer(w, l) for l in range(w.n_layers)]
    dl = [dev_layer(L) for L in layers]
    nl = [inputs.layer_to_numpy(L) for L in layers]
    xd, xp = inputs.make_hidden(w)
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    x = torch.cat([xd, xp]).to(DEV)
    for l in range(w.n_layers):
        yd, yp = ctx.moe_group_forward([dl[l]], x[:w.D], x[w.D:], "layered")
        y = torch.cat([yd, yp])
        o_y, o_idx, _ = oracle.moe_layer(inputs.to_numpy(x), nl[l]["w_router"], None, nl[l]["w_gate_up"],
                                         nl[l]["w_down"], w.K, residual=True)
        idx, _ = ctx.moe_router_topk(x, dl[l]["w_router"])
        assert (idx.cpu().numpy() == o_idx).all()
        assert_close(y, o_y, "f32", f"fp32 layer {l}")
        x = y
    yd_l, yp_l = ctx.moe_group_forward(dl, xd.to(DEV), xp.to(DEV), "layered")
    assert torch.equal(torch.cat([yd_l, yp_l]), x)
    yd_c, yp_c = ctx.moe_group_forward(dl, xd.to(DEV), xp.to(DEV), "chunked", w.chunk)
    assert torch.equal(yd_c, yd_l) and torch.equal(yp_c, yp_l)
    o_d, o_p, _ = oracle.group_forward(nl, inputs.to_numpy(xd), inputs.to_numpy(xp), w.K, "layered")
    assert_close(torch.cat([yd_l, yp_l]), np.concatenate([o_d, o_p]), "f32", "fp32 group, free-running")
