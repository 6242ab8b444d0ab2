"""A seeded sweep of small layer shapes through the C ABI: every case is checked against the oracle and its
chunked and stack schedules against its layered pass, bit for bit.  The shapes are drawn, not hand-picked, so
that tile borders, k tails, line phases of the 4-bit rows and expert loads fall where nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_08055_amd import inputs
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw_case(i):
    rng = np.random.default_rng(9000 + i)
    fmt = "mxfp4" if i % 2 else ""
    E = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 40]))
    K = int(rng.integers(1, min(E, 6) + 1))
    H = 64 * int(rng.integers(1, 13))              # 64 .. 768
    I = 64 * int(rng.integers(1, 9)) if fmt else 8 * int(rng.integers(2, 60))
    D = int(rng.choice([0, 1, 3, 17, 40]))
    P = int(rng.choice([0, 1, 31, 64, 129, 300]))
    if D + P == 0:
        P = 5
    skew = float(rng.choice([0.0, 0.0, 1.0]))      # some cases with a few popular experts
    return inputs.Workload(f"sweep{i}", H=H, E=E, K=K, I=I, n_layers=1, D=D, P=P, dtype="bf16", seed=9100 + i,
                           residual=bool(i % 3 == 0), weight_format=fmt, route_skew=skew)


CASES = [draw_case(i) for i in range(28)]


@pytest.mark.parametrize("w", CASES, ids=[f"{c.name}-H{c.H}-I{c.I}-E{c.E}-K{c.K}-D{c.D}-P{c.P}-{c.weight_format or 'bf16'}"
                                          for c in CASES])
def test_layer_against_oracle_and_schedules(gpu_lib, w):
    L = inputs.make_layer(w, 0)
    Ld = {k: (v.to(DEV) if v is not None else None) for k, v in L.items()}
    Ln = inputs.layer_to_numpy(L)
    xd, xp = inputs.make_hidden(w)
    x = torch.cat([xd, xp])
    ctx = gpu_lib.Context(w.H, w.E, w.K, w.I, torch.bfloat16, max_tokens=w.D + w.P, residual=w.residual, device=DEV,
                          weight_format=w.weight_format)
    xdd, xpd = (xd.to(DEV) if w.D else None), (xp.to(DEV) if w.P else None)
    yd, yp = ctx.moe_group_forward([Ld], xdd, xpd, "layered")
    y = torch.cat([t for t in (yd, yp) if t.shape[0]])
    o_y, o_idx, _ = oracle.moe_layer(inputs.to_numpy(x), Ln["w_router"], Ln["router_bias"], Ln["w_gate_up"],
                                     Ln["w_down"], w.K, residual=w.residual,
                                     s_gate_up=Ln.get("s_gate_up"), s_down=Ln.get("s_down"))
    idx, _ = ctx.moe_router_topk(x.to(DEV), Ld["w_router"], Ld["router_bias"])
    assert (idx.cpu().numpy() == o_idx).all()
    assert_close(y, o_y, "bf16", w.name)
    if w.P:
        for chunk in (7, 64):
            yd2, yp2 = ctx.moe_group_forward([Ld], xdd, xpd, "chunked", chunk)
            assert torch.equal(torch.cat([t for t in (yd2, yp2) if t.shape[0]]), y), f"chunk {chunk}"
        yd3, yp3 = ctx.moe_stack_forward([Ld], xdd, xpd, chunk=50, n_groups=1)
        assert torch.equal(torch.cat([t for t in (yd3, yp3) if t.shape[0]]), y)
