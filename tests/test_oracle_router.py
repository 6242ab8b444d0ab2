"""Pins for the oracle's router / top-k / mixing weights and its permutation (CPU only).

Nothing here compares the oracle with itself: each test checks it against a
closed form, a library routine used as a whole (scipy softmax, numpy stable
sort), brute force in plain Python, or an invariant of the definition.
"""
import json
import math
import os

import numpy as np
import pytest
from scipy.special import softmax

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")


def _ev(expr_rows):
    env = {"exp": math.exp}
    return np.array([[eval(e, {"__builtins__": {}}, env) for e in row] for row in expr_rows])


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["router"], ids=lambda c: c["name"])
def test_router_closed_forms(case):
    x = np.array(case["x"], dtype=np.float64)
    wr = np.array(case["w_router"], dtype=np.float64)
    b = None if case["bias"] is None else np.array(case["bias"], dtype=np.float32)
    idx, w = oracle.router_topk(x, wr, b, case["k"], renormalize=True)
    assert idx.tolist() == case["idx"]
    np.testing.assert_allclose(w, _ev(case["w_renorm_expr"]), rtol=1e-14)
    idx2, w2 = oracle.router_topk(x, wr, b, case["k"], renormalize=False)
    assert idx2.tolist() == case["idx"]
    np.testing.assert_allclose(w2, _ev(case["w_plain_expr"]), rtol=1e-14)


def test_zero_input_all_logits_equal():
    # all logits equal -> the k lowest indices in order, equal weights
    E, H, k = 16, 8, 5
    wr = np.random.default_rng(0).standard_normal((E, H))
    idx, w = oracle.router_topk(np.zeros((3, H)), wr, None, k)
    assert (idx == np.arange(k)[None, :]).all()
    np.testing.assert_allclose(w, 1.0 / k, rtol=1e-15)
    # negative zero compares equal to zero: still the lowest indices
    x = np.zeros((1, H))
    x[0, 0] = -0.0
    idx, _ = oracle.router_topk(x, wr, None, k)
    assert idx[0].tolist() == list(range(k))


def test_duplicate_router_rows_lower_index_first():
    rng = np.random.default_rng(1)
    E, H, k = 12, 32, 4
    wr = rng.standard_normal((E, H))
    wr[9] = wr[3]            # experts 3 and 9 always tie
    x = rng.standard_normal((200, H))
    idx, _ = oracle.router_topk(x, wr, None, k)
    seen_both = 0
    for row in idx.tolist():
        if 3 in row and 9 in row:
            seen_both += 1
            assert row.index(9) == row.index(3) + 1
        assert not (9 in row and 3 not in row)      # 9 can never beat 3
    assert seen_both > 10


@pytest.mark.parametrize("E,k", [(8, 2), (128, 8), (32, 4), (5, 5), (7, 1)])
def test_selection_is_sorted_prefix_and_weights_are_softmax(E, k):
    rng = np.random.default_rng(E * 100 + k)
    T, H = 64, 48
    x = rng.standard_normal((T, H))
    wr = rng.standard_normal((E, H)) * 0.3
    b = (rng.standard_normal(E) * 0.5).astype(np.float32)
    idx, w, logits, gap = oracle.router_topk(x, wr, b, k, want_logits=True, want_gap=True)
    z = x @ wr.T + b.astype(np.float64)[None, :]
    np.testing.assert_allclose(logits, z, rtol=0, atol=1e-12)
    # library sort as the reference order: by (-logit, index), on the oracle's own logits
    order = np.lexsort((np.broadcast_to(np.arange(E), (T, E)), -logits), axis=1)[:, :k]
    assert (idx == order).all()
    # k distinct experts per token (Table 1: one token covers k/E of the experts)
    assert all(len(set(r)) == k for r in idx.tolist())
    p = softmax(logits, axis=1)
    sel = np.take_along_axis(p, idx, axis=1)
    np.testing.assert_allclose(w, sel / sel.sum(1, keepdims=True), rtol=1e-13)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)
    _, w_plain = oracle.router_topk(x, wr, b, k, renormalize=False)
    np.testing.assert_allclose(w_plain, sel, rtol=1e-13)
    if k == E:
        np.testing.assert_allclose(np.sort(w, axis=1), np.sort(p, axis=1), rtol=1e-13)
    # gap = smallest spacing among the sorted top-(k+1) logits
    srt = -np.sort(-logits, axis=1)[:, :min(k + 1, E)]
    if srt.shape[1] > 1:
        np.testing.assert_allclose(gap, (srt[:, :-1] - srt[:, 1:]).min(1), rtol=0, atol=1e-13)


def test_single_token_coverage_is_k_over_E():
    # Table 1, batch size 1: 6.25 % = 8/128 of the experts are touched by one token.
    rng = np.random.default_rng(5)
    E, k, H = 128, 8, 64
    idx, _ = oracle.router_topk(rng.standard_normal((1, H)), rng.standard_normal((E, H)), None, k)
    counts, offsets, perm, inv = oracle.permute(idx, E)
    assert (counts > 0).sum() / E == 0.0625


@pytest.mark.parametrize("T,mean", [(2048, 128), (128, 8), (8192, 512)])
def test_mean_tokens_per_expert(T, mean):
    # Sec. 2.5 / 3.1 / 4.3: with E=128 and top-8, T tokens give T*8/128 tokens per expert on average.
    rng = np.random.default_rng(T)
    E, k, H = 128, 8, 16
    idx, _ = oracle.router_topk(rng.standard_normal((T, H)), rng.standard_normal((E, H)), None, k)
    counts, offsets, _, _ = oracle.permute(idx, E)
    assert counts.sum() == T * k and offsets[-1] == T * k
    assert counts.mean() == mean


def test_nonfinite_logit_is_an_error():
    x = np.ones((2, 4))
    wr = np.ones((3, 4))
    wr[1, 2] = np.inf
    with pytest.raises(oracle.OracleError):
        oracle.router_topk(x, wr, None, 2)


def test_bf16_and_f32_inputs_are_widened_exactly():
    import torch
    rng = np.random.default_rng(7)
    x32 = rng.standard_normal((9, 24)).astype(np.float32)
    w32 = rng.standard_normal((6, 24)).astype(np.float32)
    xb = torch.from_numpy(x32).to(torch.bfloat16)
    wb = torch.from_numpy(w32).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    i1, w1, z1 = oracle.router_topk(bits(xb), bits(wb), None, 3, want_logits=True)
    i2, w2, z2 = oracle.router_topk(xb.double().numpy(), wb.double().numpy(), None, 3, want_logits=True)
    assert (i1 == i2).all() and (z1 == z2).all() and (w1 == w2).all()
    i3, _, z3 = oracle.router_topk(x32, w32, None, 3, want_logits=True)
    _, _, z4 = oracle.router_topk(x32.astype(np.float64), w32.astype(np.float64), None, 3, want_logits=True)
    assert (z3 == z4).all()


# ----------------------------------------------------------------- permutation

def _brute_perm(idx, E):
    T, k = idx.shape
    triples = sorted((int(idx[t, j]), t, j) for t in range(T) for j in range(k))
    perm = [t * k + j for (_, t, j) in triples]
    counts = [sum(1 for tr in triples if tr[0] == e) for e in range(E)]
    return counts, perm


@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (7, 2, 8), (64, 2, 8), (33, 8, 128), (50, 4, 4), (0, 2, 8)])
def test_permute_against_brute_force_and_stable_sort(T, k, E):
    rng = np.random.default_rng(T * 31 + k)
    # k distinct experts per token, as a router would produce
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32) if T else np.zeros((0, k), np.int32)
    counts, offsets, perm, inv = oracle.permute(idx, E)
    bc, bp = _brute_perm(idx, E)
    assert counts.tolist() == bc and perm.tolist() == bp
    # a library stable sort of the flat expert ids gives the same order
    assert perm.tolist() == np.argsort(idx.reshape(-1), kind="stable").tolist()
    assert offsets.tolist() == [0] + np.cumsum(bc).tolist()
    A = T * k
    assert sorted(perm.tolist()) == list(range(A))                 # a permutation of [0, A)
    assert (inv[perm] == np.arange(A)).all() and (perm[inv] == np.arange(A)).all()
    for e in range(E):                                             # rows inside an expert rise with the token
        seg = perm[offsets[e]:offsets[e + 1]]
        assert (idx.reshape(-1)[seg] == e).all()
        assert (np.diff(seg) > 0).all()


def test_permute_then_unpermute_is_identity_on_rows():
    rng = np.random.default_rng(3)
    T, k, E, H = 40, 4, 16, 5
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    _, _, perm, inv = oracle.permute(idx, E)
    x = rng.standard_normal((T, H))
    x_perm = x[perm // k]                 # gather rows into expert order
    back = x_perm[inv].reshape(T, k, H)   # and back
    assert (back == x[:, None, :]).all()


def test_permute_rejects_out_of_range_expert():
    with pytest.raises(oracle.OracleError):
        oracle.permute(np.array([[0, 8]], dtype=np.int32), 8)
