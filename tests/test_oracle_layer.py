"""Pins for the oracle's MoE layer and for the two schedules (CPU only).

The layer is pinned by hand-derived closed forms, by special cases that reduce
to a dense SwiGLU FFN computed with library matmuls, by a brute-force per-token
loop in plain Python/numpy, and by equivariances of the definition.  The
schedules are pinned by their defining property (a scheduling change is not a
model change: Sec. 4.1-4.2) and by the closed-form traffic model (Fig. 2
caption: total load = per-pass load x number of chunks; Sec. 4.1: each layer is
crossed once under layered prefill; Sec. 5.4: what counts as a load byte).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")


def _ev(expr_rows):
    env = {"exp": math.exp}
    return np.array([[eval(e, {"__builtins__": {}}, env) for e in row] for row in expr_rows])


def _dense_swiglu(x, wg, wu, wd):
    g = x @ wg.T
    u = x @ wu.T
    return (g / (1.0 + np.exp(-g)) * u) @ wd.T


def _rand_layer(rng, E, H, I, std=0.3):
    return (rng.standard_normal((E, H)) * std, rng.standard_normal((E, 2 * I, H)) * std,
            rng.standard_normal((E, H, I)) * std)


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["layer"], ids=lambda c: c["name"])
def test_layer_closed_forms(case):
    x = np.array(case["x"], dtype=np.float64)
    args = (x, np.array(case["w_router"]), None, np.array(case["w_gate_up"]), np.array(case["w_down"]), case["k"])
    y, _, _ = oracle.moe_layer(*args)
    np.testing.assert_allclose(y, _ev(case["y_expr"]), rtol=1e-14)
    y_res, _, _ = oracle.moe_layer(*args, residual=True)
    np.testing.assert_allclose(y_res, _ev(case["y_expr"]) + x, rtol=1e-14)


def test_single_expert_is_a_dense_swiglu_ffn():
    rng = np.random.default_rng(10)
    T, H, I = 17, 24, 40                      # H != I so a transposed operand cannot pass
    wr, wgu, wd = _rand_layer(rng, 1, H, I)
    x = rng.standard_normal((T, H))
    y, idx, w = oracle.moe_layer(x, wr, None, wgu, wd, 1)
    assert (idx == 0).all() and (w == 1.0).all()
    np.testing.assert_allclose(y, _dense_swiglu(x, wgu[0, :I], wgu[0, I:], wd[0]), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("k", [1, 3, 6])
def test_identical_experts_make_routing_irrelevant(k):
    rng = np.random.default_rng(11)
    T, H, I, E = 9, 16, 12, 6
    wr, wgu, wd = _rand_layer(rng, E, H, I)
    wgu[:] = wgu[0]
    wd[:] = wd[0]
    x = rng.standard_normal((T, H))
    y, _, _ = oracle.moe_layer(x, wr, None, wgu, wd, k)          # weights sum to 1 -> dense FFN
    np.testing.assert_allclose(y, _dense_swiglu(x, wgu[0, :I], wgu[0, I:], wd[0]), rtol=1e-12, atol=1e-13)


def test_brute_force_per_token_loop():
    rng = np.random.default_rng(12)
    T, H, I, E, k = 11, 10, 7, 5, 3
    wr, wgu, wd = _rand_layer(rng, E, H, I)
    b = rng.standard_normal(E).astype(np.float32)
    x = rng.standard_normal((T, H))
    y, idx, w = oracle.moe_layer(x, wr, b, wgu, wd, k)
    for t in range(T):
        z = [sum(x[t, h] * wr[e, h] for h in range(H)) + float(b[e]) for e in range(E)]
        order = sorted(range(E), key=lambda e: (-z[e], e))[:k]
        assert idx[t].tolist() == order
        ex = [math.exp(v - max(z)) for v in z]
        ws = [ex[e] / sum(ex) for e in order]
        ws = [v / sum(ws) for v in ws]
        out = [0.0] * H
        for j, e in enumerate(order):
            act = []
            for i in range(I):
                g = sum(wgu[e, i, h] * x[t, h] for h in range(H))
                u = sum(wgu[e, I + i, h] * x[t, h] for h in range(H))
                act.append(g / (1.0 + math.exp(-g)) * u)
            for h in range(H):
                out[h] += ws[j] * sum(wd[e, h, i] * act[i] for i in range(I))
        np.testing.assert_allclose(y[t], out, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(w[t], ws, rtol=1e-13)


def test_equivariances():
    rng = np.random.default_rng(13)
    T, H, I, E, k = 20, 12, 9, 8, 3
    wr, wgu, wd = _rand_layer(rng, E, H, I)
    x = rng.standard_normal((T, H))
    y, idx, w = oracle.moe_layer(x, wr, None, wgu, wd, k)
    # shuffling tokens shuffles outputs (tokens are independent), bit for bit
    p = rng.permutation(T)
    y2, idx2, _ = oracle.moe_layer(x[p], wr, None, wgu, wd, k)
    assert (y2 == y[p]).all() and (idx2 == idx[p]).all()
    # relabelling experts leaves y unchanged (no ties here) and relabels idx
    q = rng.permutation(E)
    y3, idx3, w3 = oracle.moe_layer(x, wr[q], None, wgu[q], wd[q], k)
    np.testing.assert_allclose(y3, y, rtol=1e-13, atol=1e-15)
    assert (q[idx3] == idx).all()
    # the MoE branch is linear in the down projection
    y4, _, _ = oracle.moe_layer(x, wr, None, wgu, 2.5 * wd, k)
    np.testing.assert_allclose(y4, 2.5 * y, rtol=1e-13, atol=1e-15)
    # k = E is the dense softmax mixture of all experts
    yE, _, wE = oracle.moe_layer(x, wr, None, wgu, wd, E)
    z = x @ wr.T
    pz = np.exp(z - z.max(1, keepdims=True))
    pz /= pz.sum(1, keepdims=True)
    dense = sum(pz[:, [e]] * _dense_swiglu(x, wgu[e, :I], wgu[e, I:], wd[e]) for e in range(E))
    np.testing.assert_allclose(yE, dense, rtol=1e-12, atol=1e-14)


def test_magnitude_output_is_the_weighted_abs_sum():
    rng = np.random.default_rng(16)
    T, H, I, E, k = 6, 9, 5, 4, 2
    wr, wgu, wd = _rand_layer(rng, E, H, I)
    x = rng.standard_normal((T, H))
    y, idx, w, mag = oracle.moe_layer(x, wr, None, wgu, wd, k, residual=True, want_mag=True)
    ref = np.abs(x).copy()
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            ref[t] += w[t, j] * np.abs(_dense_swiglu(x[t:t + 1], wgu[e, :I], wgu[e, I:], wd[e])[0])
    np.testing.assert_allclose(mag, ref, rtol=1e-12)
    assert (mag >= np.abs(y) - 1e-12).all()          # triangle inequality


def test_layer_routing_agrees_with_router_call():
    rng = np.random.default_rng(14)
    wr, wgu, wd = _rand_layer(rng, 8, 16, 8)
    x = rng.standard_normal((30, 16))
    _, idx, w = oracle.moe_layer(x, wr, None, wgu, wd, 2)
    idx_r, w_r = oracle.router_topk(x, wr, None, 2)
    assert (idx == idx_r).all() and (w == w_r).all()


# ------------------------------------------------------------------- rounding

def test_round_bf16_matches_the_library_cast_and_hand_cases():
    # hand cases: ties go to the even 8-bit significand
    got = oracle.round_bf16([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -40])
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, -1.0, 1.0 + 2.0 ** -7]
    # values that are exactly fp32: torch's fp32 -> bf16 cast (round to nearest even) must agree
    rng = np.random.default_rng(15)
    v = (rng.standard_normal(5000) * np.exp(rng.uniform(-30, 30, 5000))).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).double().numpy()
    assert (oracle.round_bf16(v.astype(np.float64)) == ref).all()
    # a double just above a bf16 tie must round up although its fp32 rounding sits on the tie
    tie_plus = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert oracle.round_bf16([tie_plus])[0] == 1.0 + 2.0 ** -7


def test_round_f32_matches_numpy_casts_hand_ties_and_subnormals():
    """The fp32 rounding used between the layers of an fp32 group, pinned to numpy's double -> float32 cast
    (IEEE round to nearest even, done by the hardware conversion) and to hand-derived cases."""
    # hand cases: exact ties between neighbouring binary32 values go to the even 24-bit significand
    ulp = 2.0 ** -23
    cases = [1.0 + ulp / 2, 1.0 + 3 * ulp / 2, -(1.0 + ulp / 2), 1.0 + ulp / 2 + 2.0 ** -50, 1.0 + ulp / 4,
             2.0 ** 127 * (2 - 2.0 ** -24),           # halfway between the largest finite float and 2^128: overflows
             2.0 ** -149 * 0.5, 2.0 ** -149 * 1.5, 2.0 ** -149 * 0.75,           # subnormals: spacing 2^-149 throughout
             2.0 ** -127 + 2.0 ** -150, 2.0 ** -127 + 2.0 ** -150 + 2.0 ** -170]      # a tie (2^-127 = even 2^22 steps) and just above it
    want = [1.0, 1.0 + 2 * ulp, -1.0, 1.0 + ulp, 1.0, float("inf"), 0.0, 2.0 ** -148, 2.0 ** -149, 2.0 ** -127,
            2.0 ** -127 + 2.0 ** -149]
    assert oracle.round_f32(cases).tolist() == want
    # ~5000 random doubles over the whole binary32 exponent range, subnormals included, plus exact floats
    rng = np.random.default_rng(16)
    v = rng.standard_normal(5000) * np.exp2(rng.uniform(-152, 127, 5000))
    with np.errstate(over="ignore"):
        ref = v.astype(np.float32).astype(np.float64)
    assert np.isfinite(ref).all() and (np.abs(ref) < 2.0 ** -126).sum() > 50      # the sample does reach the subnormals
    assert (oracle.round_f32(v) == ref).all()
    f = (rng.standard_normal(1000) * np.exp2(rng.uniform(-100, 100, 1000))).astype(np.float32).astype(np.float64)
    assert (oracle.round_f32(f) == f).all()                                       # representable values are fixed points
    # the array form is the scalar function applied element by element
    one = np.array([oracle.lib().orc_round_f32(float(t)) for t in v[:200]])
    assert (one == ref[:200]).all()


def test_fp32_group_rounds_between_layers_only():
    """A group whose activations are held in fp32 between layers: the oracle's group driver must equal the
    chain layer -> round_f32 -> layer written out here, and differ from the unrounded chain."""
    rng = np.random.default_rng(17)
    layers = []
    for _ in range(3):
        wr, wgu, wd = _rand_layer(rng, 6, 24, 16)
        layers.append({"w_router": wr.astype(np.float32), "router_bias": None,
                       "w_gate_up": wgu.astype(np.float32), "w_down": wd.astype(np.float32)})
    x = rng.standard_normal((11, 24)).astype(np.float32)
    yd, yp, _ = oracle.group_forward(layers, x[:3], x[3:], 2, "layered")
    cur = x.astype(np.float64)
    plain = x.astype(np.float64)
    for l, L in enumerate(layers):
        y, _, _ = oracle.moe_layer(cur, L["w_router"].astype(np.float64), None, L["w_gate_up"].astype(np.float64),
                                   L["w_down"].astype(np.float64), 2, residual=True)
        cur = y.astype(np.float32).astype(np.float64) if l + 1 < len(layers) else y
        plain, _, _ = oracle.moe_layer(plain, L["w_router"].astype(np.float64), None, L["w_gate_up"].astype(np.float64),
                                       L["w_down"].astype(np.float64), 2, residual=True)
    got = np.concatenate([yd, yp])
    assert (got == cur).all()
    assert (got != plain).any() and np.abs(got - plain).max() < 1e-3


# ------------------------------------------------------------------ schedules

def _np_layers(w, n_layers=None):
    n = w.n_layers if n_layers is None else n_layers
    return [inputs.layer_to_numpy(inputs.make_layer(w, l)) for l in range(n)]


SMALL = inputs.scaled(inputs.WORKLOADS["qwen3_group8"], name="small_group", H=32, E=8, K=2, I=24,
                      n_layers=3, D=5, P=37, chunk=16, seed=21)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("chunk", [1, 16, 37, 38, 7])
def test_chunked_equals_layered_bit_for_bit(dtype, chunk):
    w = inputs.scaled(SMALL, dtype=dtype)
    layers = _np_layers(w)
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(w))
    yd_l, yp_l, c_l = oracle.group_forward(layers, xd, xp, w.K, "layered")
    yd_c, yp_c, c_c = oracle.group_forward(layers, xd, xp, w.K, "chunked", chunk)
    assert yd_l.tobytes() == yd_c.tobytes() and yp_l.tobytes() == yp_c.tobytes()
    n_iter = -(-w.P // chunk)
    assert (c_l.iterations, c_l.layer_passes) == (1, w.n_layers)
    assert (c_c.iterations, c_c.layer_passes) == (n_iter, n_iter * w.n_layers)
    assert c_l.tokens_processed == w.D + w.P
    assert c_c.tokens_processed == n_iter * w.D + w.P


def test_schedule_edge_cases():
    w = SMALL
    layers = _np_layers(w)
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(w))
    none = np.zeros((0, w.H), dtype=xd.dtype)
    # no prefill: exactly one decode-only iteration under either schedule
    a = oracle.group_forward(layers, xd, none, w.K, "layered")
    b = oracle.group_forward(layers, xd, none, w.K, "chunked", 16)
    assert a[0].tobytes() == b[0].tobytes() and a[2] == b[2] and a[2].iterations == 1
    assert a[2].tokens_processed == w.D
    # no decode rows
    c = oracle.group_forward(layers, none, xp, w.K, "layered")
    d = oracle.group_forward(layers, none, xp, w.K, "chunked", 16)
    assert c[1].tobytes() == d[1].tobytes() and d[2].iterations == 3
    # decode rows do not depend on what rides along with them
    full = oracle.group_forward(layers, xd, xp, w.K, "layered")
    assert full[0].tobytes() == a[0].tobytes() and full[1].tobytes() == c[1].tobytes()
    # nothing at all
    e = oracle.group_forward(layers, none, none, w.K, "layered")
    assert e[2].iterations == 0 and e[2].expert_bytes == 0
    with pytest.raises(oracle.OracleError):
        oracle.group_forward(layers, xd, xp, w.K, "chunked", 0)


def test_group_is_the_composition_of_layers_with_rounding_between():
    w = SMALL
    layers = _np_layers(w)
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(w))
    yd, yp, _ = oracle.group_forward(layers, xd, xp, w.K, "layered")
    x = torch.cat([torch.from_numpy(xd.view(np.int16)).view(torch.bfloat16),
                   torch.from_numpy(xp.view(np.int16)).view(torch.bfloat16)]).double().numpy()
    for l, L in enumerate(layers):
        y, _, _ = oracle.moe_layer(x, L["w_router"], None, L["w_gate_up"], L["w_down"], w.K, residual=True)
        x = oracle.round_bf16(y) if l + 1 < len(layers) else y
    assert (x[:w.D] == yd).all() and (x[w.D:] == yp).all()
    # the residual is what links the layers: without it the result is different
    yd0, _, _ = oracle.group_forward(layers, xd, xp, w.K, "layered", residual=False)
    assert not np.allclose(yd0, yd)


def test_tiny_fp32_workload_chunk16_vs_layered():
    w = inputs.WORKLOADS["tiny_f32"]
    layers = _np_layers(w)
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(w))
    a = oracle.group_forward(layers, xd, xp, w.K, "layered", residual=w.residual)
    b = oracle.group_forward(layers, xd, xp, w.K, "chunked", w.chunk, residual=w.residual)
    assert a[1].tobytes() == b[1].tobytes()
    assert b[2].iterations == 4 and a[2].iterations == 1
    sz, We = 4, 3 * w.H * w.I
    # 16 tokens x top-2 over 8 experts: every expert is hit in each chunk for this seed
    assert b[2].expert_bytes == b[2].active_experts_total * We * sz
    assert a[2].expert_bytes == w.E * We * sz
    assert b[2].expert_bytes <= 4 * a[2].expert_bytes


def test_traffic_model_closed_forms():
    # Full coverage (T*k >> E): bytes = iterations x layers x E x 3*H*I*sz; layered: one iteration.
    w = inputs.scaled(SMALL, D=8, P=96, chunk=24, n_layers=2)
    layers = _np_layers(w)
    xd, xp = (inputs.to_numpy(t) for t in inputs.make_hidden(w))
    per_pass = w.E * 3 * w.H * w.I * 2
    _, _, cl, tl = oracle.group_forward(layers, xd, xp, w.K, "layered", want_trace=True)
    _, _, cc, tc = oracle.group_forward(layers, xd, xp, w.K, "chunked", w.chunk, want_trace=True)
    assert cl.expert_bytes == 1 * w.n_layers * per_pass
    assert cc.expert_bytes == 4 * w.n_layers * per_pass            # C-fold more for C chunks
    assert cc.router_bytes == 4 * w.n_layers * w.E * w.H * 2
    assert cl.active_experts_total == w.n_layers * w.E
    # the counter is "experts with at least one token", recomputed here from the routing trace
    T = w.D + w.P
    tl = tl.reshape(w.n_layers, T, w.K)
    assert cl.active_experts_total == sum(len(set(tl[l].reshape(-1).tolist())) for l in range(w.n_layers))
    # sparse case: one decode token per iteration touches exactly k experts per layer (k/E coverage)
    one = np.ascontiguousarray(xd[:1])
    _, _, c1 = oracle.group_forward(layers, one, np.zeros((0, w.H), xd.dtype), w.K, "layered")
    assert c1.active_experts_total == w.n_layers * w.K
    assert c1.expert_bytes == w.n_layers * w.K * 3 * w.H * w.I * 2


def test_iid_coverage_curve_matches_expectation():
    # For iid-uniform routing the expected coverage at batch B is 1-(1-k/E)^B; synthetic N(0,.02)
    # routers are close to that (the paper's Table 1 lies below it: real routing is correlated).
    rng = np.random.default_rng(17)
    E, k, H = 128, 8, 64
    wr = rng.standard_normal((E, H)) * 0.02
    for B in (2, 8, 32):
        cov = []
        for rep in range(40):
            idx, _ = oracle.router_topk(rng.standard_normal((B, H)), wr, None, k)
            cov.append(len(set(idx.reshape(-1).tolist())) / E)
        expect = 1 - (1 - k / E) ** B
        assert abs(np.mean(cov) - expect) < 0.04


def test_stored_zipf_bias_gives_zipf_shares():
    # Mixtral-shaped workload: the stored router bias makes the experts' assignment shares follow Zipf(1.2)
    w = inputs.WORKLOADS["mixtral_zipf"]
    xd, xp = inputs.make_hidden(w)
    x = inputs.to_numpy(torch.cat([xd, xp]))
    wr = inputs.to_numpy(inputs.randn((w.E, w.H), 0.02, w.seed, "w_router", 0, w.dtype, "cpu"))
    b = inputs.stored_router_bias(w, 0).numpy()
    idx, wt = oracle.router_topk(x, wr, b, w.K)
    share = np.bincount(idx.reshape(-1), minlength=w.E) / idx.size
    target = inputs.zipf_shares(w.E, w.zipf_s)
    assert np.abs(share - target).max() < 2e-3
    assert abs(target[0] - 0.4286) < 1e-3 and abs(target[-1] - 0.0353) < 1e-3     # Zipf(1.2) over 8 experts
    np.testing.assert_allclose(wt.sum(1), 1.0, rtol=1e-13)
