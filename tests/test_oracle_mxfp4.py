"""Pins for the oracle's 4-bit expert-weight format (CPU only).

The format is the published OCP Microscaling MXFP4 (FP4 E2M1 elements, E8M0 scale per 32 elements); the
paper's Table 7 reports a model with fp4 expert weights.  Pins: the element and scale values written out
from the specification (tests/golden/mxfp4_format.json), a look-up-table dequantiser written here in numpy
(a third implementation), and the layer with MXFP4 weights against the layer on the dequantised weights.
"""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2510_08055_amd import inputs

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "mxfp4_format.json")))


def lut_dequant(codes, scales):
    lut = np.array(GOLDEN["e2m1_values"])
    lo, hi = codes & 15, codes >> 4
    el = np.stack([lut[lo], lut[hi]], axis=-1).reshape(codes.shape[:-1] + (codes.shape[-1] * 2,))
    sc = np.exp2(scales.astype(np.float64) - 127.0)
    return el * np.repeat(sc, 32, axis=-1)


def test_element_and_scale_values_match_the_specification():
    # one block of 32 elements holding every code twice, scale 1: low nibble is the even element
    codes = np.array([[(2 * i % 16) | (((2 * i + 1) % 16) << 4) for i in range(16)]], dtype=np.uint8)
    out = oracle.mxfp4_dequant(codes, np.array([[127]], dtype=np.uint8))
    want = np.array(GOLDEN["e2m1_values"] * 2)
    assert (out[0] == want).all() and (np.signbit(out[0]) == np.signbit(want)).all()
    for ex in GOLDEN["e8m0_examples"]:
        one = oracle.mxfp4_dequant(np.full((1, 16), 0x22, dtype=np.uint8), np.array([[ex["s"]]], dtype=np.uint8))
        assert (one == ex["value"]).all()          # code 2 is 1.0


def test_dequant_matches_a_lookup_table_implementation():
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 256, size=(3, 7, 48), dtype=np.uint8)           # 96 elements per row = 3 blocks
    scales = rng.integers(100, 140, size=(3, 7, 3), dtype=np.uint8)
    got = oracle.mxfp4_dequant(codes, scales)
    assert got.shape == (3, 7, 96)
    assert (got == lut_dequant(codes, scales)).all()
    # the scale is shared by 32 consecutive elements of a row and changes at the block border
    c1 = np.full((1, 32), 0x22, dtype=np.uint8)
    got = oracle.mxfp4_dequant(c1, np.array([[127, 129]], dtype=np.uint8))
    assert (got[0, :32] == 1.0).all() and (got[0, 32:] == 4.0).all()


W4 = inputs.Workload("w4", H=64, E=4, K=2, I=128, n_layers=1, D=3, P=10, dtype="bf16", seed=51, residual=False,
                     weight_format="mxfp4")


def test_generated_mxfp4_weights_have_the_stated_shape_and_scale():
    L = inputs.layer_to_numpy(inputs.make_layer(W4, 0))
    assert L["w_gate_up"].shape == (W4.E, 2 * W4.I, W4.H // 2) and L["s_gate_up"].shape == (W4.E, 2 * W4.I, W4.H // 32)
    assert L["w_down"].shape == (W4.E, W4.H, W4.I // 2) and L["s_down"].shape == (W4.E, W4.H, W4.I // 32)
    assert L["s_gate_up"].min() >= 118 and L["s_gate_up"].max() <= 120
    w = oracle.mxfp4_dequant(L["w_gate_up"], L["s_gate_up"])
    assert 0.012 < w.std() < 0.02                  # just under the N(0, 0.02) weights of the other workloads


@pytest.mark.parametrize("residual", [False, True])
def test_layer_with_mxfp4_weights_is_the_layer_on_the_dequantised_weights(residual):
    L = inputs.layer_to_numpy(inputs.make_layer(W4, 0))
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(W4))
    x = np.concatenate([xd, xp])
    y, idx, w = oracle.moe_layer(x, L["w_router"], None, L["w_gate_up"], L["w_down"], W4.K, residual=residual,
                                 s_gate_up=L["s_gate_up"], s_down=L["s_down"])
    wgu = lut_dequant(L["w_gate_up"], L["s_gate_up"])
    wd = lut_dequant(L["w_down"], L["s_down"])
    wr = oracle.round_bf16(inputs.make_layer(W4, 0)["w_router"].double().numpy())      # bf16 values as fp64
    xf = np.concatenate([t.double().numpy() for t in inputs.make_hidden(W4)])
    y2, idx2, w2 = oracle.moe_layer(xf, wr, None, wgu, wd, W4.K, residual=residual)
    assert (idx == idx2).all() and (w == w2).all() and (y == y2).all()
    assert np.abs(y).max() > 1e-3


def test_invalid_mxfp4_arguments_are_rejected():
    L = inputs.layer_to_numpy(inputs.make_layer(W4, 0))
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(W4))
    bad = L["s_down"].copy()
    bad[1, 2, 3] = 255                       # the format's not-a-number scale
    with pytest.raises(oracle.OracleError):
        oracle.moe_layer(xp, L["w_router"], None, L["w_gate_up"], L["w_down"], W4.K, s_gate_up=L["s_gate_up"],
                         s_down=bad)
