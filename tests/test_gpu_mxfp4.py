"""GPU parity of the 4-bit expert-weight path (MXFP4 weights, bf16 activations) through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_layer(layer):
    return {k: (v.to(DEV) if v is not None else None) for k, v in layer.items()}


def make_ctx(lib, w, max_tokens):
    return lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=max_tokens, residual=w.residual, device=DEV,
                       weight_format=w.weight_format)


def oracle_layer(w, Ln, xn, residual, rows=None):
    x = xn if rows is None else xn[rows]
    return oracle.moe_layer(x, Ln["w_router"], Ln["router_bias"], Ln["w_gate_up"], Ln["w_down"], w.K,
                            residual=residual, s_gate_up=Ln["s_gate_up"], s_down=Ln["s_down"])


SHAPES = [
    inputs.Workload("w4_small", H=128, E=4, K=2, I=64, n_layers=1, D=5, P=60, dtype="bf16", seed=61, residual=False,
                    weight_format="mxfp4"),
    inputs.Workload("w4_ragged", H=192, E=16, K=4, I=320, n_layers=1, D=9, P=333, dtype="bf16", seed=62,
                    residual=False, weight_format="mxfp4"),           # 5 and 3 k-stages, ragged n-tiles, 64+ rows per expert
    inputs.Workload("w4_sparse", H=2880, E=32, K=4, I=2880 // 5 * 1 // 64 * 64, n_layers=1, D=7, P=0, dtype="bf16",
                    seed=63, residual=False, weight_format="mxfp4"),  # 45 k-stages, most experts with 0-2 rows
    inputs.Workload("w4_deep", H=4160, E=4, K=2, I=128, n_layers=1, D=3, P=20, dtype="bf16", seed=65, residual=False,
                    weight_format="mxfp4"),   # 65 k-stages: more than 128 scale bytes per row; rows of 2080 bytes (odd multiple of 32)
    inputs.Workload("w4_deep_even", H=4224, E=4, K=2, I=192, n_layers=1, D=0, P=37, dtype="bf16", seed=66,
                    residual=False, weight_format="mxfp4"),   # 66 k-stages, rows of 2112 bytes (phases 0 and 64 only)
]


# both kernel shapes on every case (the library would pick one by the batch's rows per expert)
@pytest.mark.parametrize("variant", ["w4_tile64", "w4_stream"])
@pytest.mark.parametrize("w", SHAPES, ids=[w.name for w in SHAPES])
def test_single_layer_steps(gpu_lib, w, variant):
    L = inputs.make_layer(w, 0)
    Ld, Ln = dev_layer(L), inputs.layer_to_numpy(L)
    xd, xp = inputs.make_hidden(w)
    x = torch.cat([xd, xp]).to(DEV)
    xn = inputs.to_numpy(x)
    T = w.D + w.P
    ctx = make_ctx(gpu_lib, w, T)
    ctx.moe_set_ffn_variant(variant)
    o_y, o_idx, o_w = oracle_layer(w, Ln, xn, False)
    # the grouped FFN step alone, on the oracle's routing
    idx, wt = ctx.moe_router_topk(x, Ld["w_router"])
    assert (idx.cpu().numpy() == o_idx).all()
    counts, offsets, perm, inv, x_perm = ctx.moe_permute(x, idx)
    y_perm = ctx.moe_grouped_ffn_mxfp4(x_perm, offsets, Ld["w_gate_up"], Ld["s_gate_up"], Ld["w_down"], Ld["s_down"])
    y = ctx.moe_combine(y_perm, inv, wt)
    assert_close(y, o_y, "bf16", w.name + " steps")
    # the bf16 entry point refuses a 4-bit context
    with pytest.raises(gpu_lib.MoeError) as e:
        ctx.moe_grouped_ffn(x_perm, offsets, Ld["w_gate_up"], Ld["w_down"])
    assert e.value.status == 3
    # the whole layer in one call, both schedules, bit-identical
    ctx.moe_reset_counters()
    yd, yp = ctx.moe_group_forward([Ld], x[:w.D] if w.D else None, x[w.D:] if w.P else None, "layered")
    c = ctx.moe_read_counters()
    full = torch.cat([t for t in (yd, yp) if t.shape[0]])
    assert torch.equal(full, y)
    active = len(set(o_idx.reshape(-1).tolist()))
    assert c.active_experts_total == active
    assert c.expert_bytes == active * (3 * w.H * w.I // 2 + 3 * w.H * w.I // 32)      # codes + scale bytes
    if w.P:
        yd2, yp2 = ctx.moe_group_forward([Ld], x[:w.D] if w.D else None, x[w.D:], "chunked", 50)
        assert torch.equal(torch.cat([yd2, yp2]), y)


def test_kernel_shapes_bit_identical(gpu_lib):
    """Chunked and layered passes may pick different kernel shapes: their results must not differ by a bit."""
    for w in SHAPES[1:3]:
        L = dev_layer(inputs.make_layer(w, 0))
        xd, xp = inputs.make_hidden(w)
        x = torch.cat([xd, xp]).to(DEV)
        ctx = make_ctx(gpu_lib, w, w.D + w.P)
        idx, _ = ctx.moe_router_topk(x, L["w_router"])
        _, offsets, _, _, x_perm = ctx.moe_permute(x, idx)
        out = {}
        for variant in ("w4_tile64", "w4_stream"):
            ctx.moe_set_ffn_variant(variant)
            out[variant] = ctx.moe_grouped_ffn_mxfp4(x_perm, offsets, L["w_gate_up"], L["s_gate_up"], L["w_down"],
                                                     L["s_down"]).clone()
        assert torch.equal(out["w4_tile64"], out["w4_stream"]), w.name


def test_group_with_residual_teacher_forced(gpu_lib):
    w = inputs.Workload("w4_group", H=256, E=8, K=2, I=192, n_layers=3, D=6, P=90, dtype="bf16", seed=64,
                        weight_format="mxfp4")
    layers = [inputs.make_layer(w, l) for l in range(w.n_layers)]
    dl = [dev_layer(L) for L in layers]
    nl = [inputs.layer_to_numpy(L) for L in layers]
    xd, xp = inputs.make_hidden(w)
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    x = torch.cat([xd, xp]).to(DEV)
    for l in range(w.n_layers):
        yd, yp = ctx.moe_group_forward([dl[l]], x[:w.D], x[w.D:], "layered")
        y = torch.cat([yd, yp])
        o_y, o_idx, _ = oracle_layer(w, nl[l], inputs.to_numpy(x), True)
        idx, _ = ctx.moe_router_topk(x, dl[l]["w_router"])
        assert (idx.cpu().numpy() == o_idx).all()
        assert_close(y, o_y, "bf16", f"w4 group layer {l}")
        x = y
    yd, yp = ctx.moe_group_forward(dl, xd.to(DEV), xp.to(DEV), "layered")
    assert torch.equal(torch.cat([yd, yp]), x)
    yd, yp = ctx.moe_stack_forward(dl, xd.to(DEV), xp.to(DEV), chunk=40, n_groups=3)
    assert torch.equal(torch.cat([yd, yp]), x)
    # a layer without scale bytes is rejected before anything is launched
    broken = dict(dl[0]); broken["s_down"] = None
    with pytest.raises(gpu_lib.MoeError) as e:
        ctx.moe_group_forward([broken], xd.to(DEV), xp.to(DEV), "layered")
    assert e.value.status == 1


def test_config_errors(gpu_lib):
    with pytest.raises(gpu_lib.MoeError) as e:       # 4-bit weights need bf16 activations
        gpu_lib.Context(128, 4, 2, 64, torch.float32, max_tokens=8, device=DEV, weight_format="mxfp4")
    assert e.value.status == 3
    with pytest.raises(gpu_lib.MoeError) as e:       # and H, I multiples of 64
        gpu_lib.Context(96, 4, 2, 64, torch.bfloat16, max_tokens=8, device=DEV, weight_format="mxfp4")
    assert e.value.status == 4


@pytest.mark.parametrize("variant", ["w4_tile64", "w4_stream"])
@pytest.mark.parametrize("H,I,E,rows", [
    (128, 192, 6, [32, 0, 33, 1, 64, 65]),        # whole and just-over row blocks, an empty expert, one row
    (448, 64, 3, [0, 0, 70]),                     # leading empty experts; 224-byte rows (phases 0 / 96 / 64 / 32)
    (2880, 2880, 2, [9, 40]),                     # the decode shape: 45 stages, ragged last n-tile
])
def test_grouped_ffn_is_the_dense_swiglu_of_each_expert(gpu_lib, H, I, E, rows, variant):
    A = sum(rows)
    w = inputs.Workload("f4", H=H, E=E, K=1, I=I, n_layers=1, D=0, P=A, dtype="bf16", seed=67, weight_format="mxfp4")
    L = inputs.make_layer(w, 0)
    # (rows of spread 0.5: uniformly drawn FP4 codes make heavier weights than the N(0, 0.02) of the bf16
    # recipe, and with unit rows the 2880-wide case has outputs of magnitude ~10, where bf16 rounding of
    # the intermediate alone exceeds the absolute bound)
    x_perm = inputs.randn((A, H), 0.5, 67, "x_perm", 0, "bf16")
    offsets = torch.tensor(np.concatenate([[0], np.cumsum(rows)]), dtype=torch.int32)
    ctx = make_ctx(gpu_lib, w, A)
    ctx.moe_set_ffn_variant(variant)
    y = ctx.moe_grouped_ffn_mxfp4(x_perm.to(DEV), offsets.to(DEV), L["w_gate_up"].to(DEV), L["s_gate_up"].to(DEV),
                                  L["w_down"].to(DEV), L["s_down"].to(DEV))
    ref = np.zeros((A, H))
    ones = inputs.to_numpy(torch.ones((1, H), dtype=torch.bfloat16))
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:   # a one-expert MoE layer is that expert's dense FFN with weight 1
            ref[lo:hi], _, _ = oracle.moe_layer(
                inputs.to_numpy(x_perm[lo:hi]), ones, None, inputs.to_numpy(L["w_gate_up"][e:e + 1]),
                inputs.to_numpy(L["w_down"][e:e + 1]), 1,
                s_gate_up=inputs.to_numpy(L["s_gate_up"][e:e + 1]), s_down=inputs.to_numpy(L["s_down"][e:e + 1]))
    assert_close(y, ref, "bf16", "grouped_ffn_mxfp4")


# ------------------------------------------------------------------ alignment of the packed codes
def _view_at(t: torch.Tensor, offset: int) -> torch.Tensor:
    """A copy of the uint8 tensor t that starts `offset` bytes into a larger (256-byte aligned) allocation."""
    buf = torch.zeros(t.numel() + 512, dtype=torch.uint8, device=DEV)
    base = (-buf.data_ptr()) % 256
    v = buf[base + offset: base + offset + t.numel()].view(t.shape)
    v.copy_(t)
    assert v.data_ptr() % 256 == offset and v.is_contiguous()
    return v


ALIGN_SHAPES = [
    inputs.Workload("w4_al_odd", H=192, E=6, K=2, I=320, n_layers=1, D=4, P=75, dtype="bf16", seed=68, residual=False,
                    weight_format="mxfp4"),      # rows of 96 and 160 bytes: odd multiples of 32, all four line phases
    inputs.Workload("w4_al_even", H=256, E=4, K=2, I=128, n_layers=1, D=0, P=50, dtype="bf16", seed=69, residual=False,
                    weight_format="mxfp4"),      # rows of 128 and 64 bytes: one or two phases
]


@pytest.mark.parametrize("variant", ["w4_tile64", "w4_stream"])
@pytest.mark.parametrize("w", ALIGN_SHAPES, ids=[w.name for w in ALIGN_SHAPES])
def test_code_tensors_inside_a_larger_allocation(gpu_lib, w, variant):
    """Weights handed over as views into a packed buffer: 32-byte aligned code tensors must give the same bits
    as 256-byte aligned ones (and the oracle's values); 16-byte aligned ones are refused before any launch."""
    L = inputs.make_layer(w, 0)
    Ld, Ln = dev_layer(L), inputs.layer_to_numpy(L)
    xd, xp = inputs.make_hidden(w)
    x = torch.cat([xd, xp]).to(DEV)
    ctx = make_ctx(gpu_lib, w, w.D + w.P)
    ctx.moe_set_ffn_variant(variant)
    idx, wt = ctx.moe_router_topk(x, Ld["w_router"])
    _, offsets, _, inv, x_perm = ctx.moe_permute(x, idx)
    ref = ctx.moe_grouped_ffn_mxfp4(x_perm, offsets, Ld["w_gate_up"], Ld["s_gate_up"], Ld["w_down"], Ld["s_down"]).clone()
    o_y, _, _ = oracle_layer(w, Ln, inputs.to_numpy(x), False)
    assert_close(ctx.moe_combine(ref, inv, wt), o_y, "bf16", w.name)
    for off in (32, 64, 96, 160):
        gu, dn = _view_at(Ld["w_gate_up"], off), _view_at(Ld["w_down"], (off + 64) % 256)
        sgu, sdn = _view_at(Ld["s_gate_up"], 16), _view_at(Ld["s_down"], 48)       # scale bytes: 16-byte alignment
        y = ctx.moe_grouped_ffn_mxfp4(x_perm, offsets, gu, sgu, dn, sdn)
        assert torch.equal(y, ref), (variant, off)
        lay = dict(Ld, w_gate_up=gu, w_down=dn, s_gate_up=sgu, s_down=sdn)
        yd, yp = ctx.moe_group_forward([lay], x[:w.D] if w.D else None, x[w.D:], "layered")
        assert_close(torch.cat([t for t in (yd, yp) if t.shape[0]]), o_y, "bf16", f"{w.name} +{off}")
    for bad in (dict(w_gate_up=_view_at(Ld["w_gate_up"], 16)), dict(w_down=_view_at(Ld["w_down"], 48)),
                dict(s_gate_up=_view_at(Ld["s_gate_up"], 8)), dict(s_down=_view_at(Ld["s_down"], 4))):
        lay = dict(Ld, **bad)
        with pytest.raises(gpu_lib.MoeError) as e:
            ctx.moe_grouped_ffn_mxfp4(x_perm, offsets, lay["w_gate_up"], lay["s_gate_up"], lay["w_down"], lay["s_down"])
        assert e.value.status == 4
        with pytest.raises(gpu_lib.MoeError) as e:
            ctx.moe_group_forward([lay], x[:w.D] if w.D else None, x[w.D:], "layered")
        assert e.value.status == 4
