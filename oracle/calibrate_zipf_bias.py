"""Write the stored router bias of a skewed-routing workload (calls only the oracle and the input generators).

For the Mixtral-shaped workload the baseline asks for a per-expert router bias such that the experts'
token shares follow Zipf(s = 1.2).  Starting from b_e = ln(p_e), the bias is refined by the fixed point
b_e += ln(target_e / observed_e), the observed shares being those of the oracle's router on the workload's
own (CPU-drawn) hidden states and router weights.  Top-2 routing caps any share at 0.5; Zipf(1.2) over 8
experts tops out at 0.429, so the target is feasible.

    python oracle/calibrate_zipf_bias.py mixtral_zipf
"""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2510_08055_amd import inputs  # noqa: E402


def calibrate(name: str, rounds: int = 40):
    w = inputs.WORKLOADS[name]
    target = inputs.zipf_shares(w.E, w.zipf_s)
    xd, xp = inputs.make_hidden(w)
    x = inputs.to_numpy(torch.cat([xd, xp]))
    out = []
    for layer in range(w.n_layers):
        wr = inputs.to_numpy(inputs.randn((w.E, w.H), 0.02, w.seed, "w_router", layer, w.dtype, "cpu"))
        b = np.log(target)
        for it in range(rounds):
            idx, _ = oracle.router_topk(x, wr, b.astype(np.float32), w.K)
            share = np.bincount(idx.reshape(-1), minlength=w.E) / idx.size
            err = np.abs(share - target).max()
            if err < 2e-4:
                break
            b = b + 0.7 * np.log(target / np.maximum(share, 1e-6))
            b -= b.max()
        b32 = b.astype(np.float32)
        idx, _ = oracle.router_topk(x, wr, b32, w.K)
        share = np.bincount(idx.reshape(-1), minlength=w.E) / idx.size
        print(f"layer {layer}: {it + 1} rounds, max share error {np.abs(share - target).max():.2e}")
        print("  target  ", np.round(target, 4))
        print("  observed", np.round(share, 4), "rows", np.bincount(idx.reshape(-1), minlength=w.E))
        out.append([float(v) for v in b32])
    path = os.path.join(ROOT, "paper_2510_08055_amd", "data", f"router_bias_{name}.json")
    with open(path, "w") as f:
        json.dump({"workload": name, "E": w.E, "seed": w.seed, "zipf_s": w.zipf_s,
                   "target_shares": [float(v) for v in target], "bias": out}, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    calibrate(sys.argv[1] if len(sys.argv) > 1 else "mixtral_zipf")
