"""Seeded synthetic inputs shaped like the layered-prefill paper's workloads.

This module only draws random tensors and names workload shapes.  It holds none
of the MoE layer's arithmetic, so both the CPU oracle's tests and the GPU
library's tests can take their inputs from it without sharing method code.

Recipe (the paper's traces and trained weights are not available; Table 3 gives
the shapes E / top-k / hidden size, Sec. 3.2 the 8192-token prompt, Sec. 4.4 the
512-token chunk, Sec. 3.1 the decode batch sizes):
  hidden states  ~ N(0, 1)
  router, gate_up and down weights ~ N(0, 0.02)
each drawn in fp32 from a generator seeded by (seed, tensor name, layer) and
then rounded ONCE to the workload dtype; every consumer sees those exact bits.
Tensors can be drawn on the CPU or directly on the GPU (large weights); the two
devices give different, individually reproducible, streams.
"""
import json
import os
import zlib
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    H: int            # hidden size
    E: int            # experts
    K: int            # experts per token (top-k)
    I: int            # expert intermediate size
    n_layers: int
    D: int            # decode tokens
    P: int            # prefill tokens
    dtype: str        # "bf16" | "f32"
    chunk: int = 0    # chunk size used when the chunked schedule is run
    seed: int = 0
    zipf_s: float = 0.0   # > 0: router bias shaped so expert shares follow Zipf(s)
    residual: bool = True
    weight_format: str = ""   # "" = expert weights in `dtype`; "mxfp4" = 4-bit codes + scale bytes (Table 7)
    route_skew: float = 0.0   # > 0: per-expert router bias ~ N(0, route_skew): some experts are popular, so a
                              # decode batch covers fewer experts than under iid routing (Table 1 lies below
                              # the iid curve 1 - (1 - k/E)^B for the same reason)
    y_perm_f32: bool = False  # the GPU context keeps the expert outputs in fp32 between down GEMM and combine
                              # (layers whose expert outputs are large against the absolute tolerance)
    act_split: bool = False   # ... and the SwiGLU intermediate as a pair of bf16 values (very wide experts)


# The five benchmark workloads, in the order of the baseline description, and a second model family.
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", H=256, E=8, K=2, I=512, n_layers=1, D=0, P=64, dtype="f32",
                         chunk=16, seed=0, residual=False),
    "qwen3_layer": Workload("qwen3_layer", H=2048, E=128, K=8, I=768, n_layers=1, D=64, P=2048,
                            dtype="bf16", chunk=512, seed=1, residual=False),
    "qwen3_group8": Workload("qwen3_group8", H=2048, E=128, K=8, I=768, n_layers=8, D=128, P=8192,
                             dtype="bf16", chunk=512, seed=2),
    # (expert outputs of magnitude up to ~10 from a 14336-wide intermediate: the bf16 rounding of the
    # intermediate alone is worth ~3e-3 rms per output, so the context holds it as a bf16 pair)
    "mixtral_zipf": Workload("mixtral_zipf", H=4096, E=8, K=2, I=14336, n_layers=1, D=32, P=4096,
                             dtype="bf16", chunk=512, seed=3, zipf_s=1.2, residual=False, y_perm_f32=True,
                             act_split=True),
    # the same layer with the intermediate in plain bf16 (what a serving stack would run): faster, and short of
    # the absolute tolerance on a few elements in ten thousand
    "mixtral_zipf_bf16act": Workload("mixtral_zipf_bf16act", H=4096, E=8, K=2, I=14336, n_layers=1, D=32, P=4096,
                                     dtype="bf16", chunk=512, seed=3, zipf_s=1.2, residual=False, y_perm_f32=True),
    "decode_large": Workload("decode_large", H=2880, E=128, K=4, I=2880, n_layers=4, D=256, P=0,
                             dtype="bf16", chunk=512, seed=4, y_perm_f32=True),
    # the second model family of Table 3 (32 experts, top-4, hidden size 2880; the intermediate size is not
    # printed there: 2880 is the value the baseline's decode-heavy configuration gives for this hidden
    # size), one layer, 64 decode tokens + a 2048-token chunk
    "gptoss_layer": Workload("gptoss_layer", H=2880, E=32, K=4, I=2880, n_layers=1, D=64, P=2048,
                             dtype="bf16", chunk=512, seed=5, residual=False),
    # 4-bit expert weights (Table 7 runs a model with fp4 expert weights): the decode-heavy shape again, the
    # expert weights in MXFP4, so a pass streams 17/64 of the bf16 bytes
    # the second model family as it ships: MXFP4 expert weights under the hybrid batch of gptoss_layer
    "gptoss_layer_w4": Workload("gptoss_layer_w4", H=2880, E=32, K=4, I=2880, n_layers=1, D=64, P=2048,
                                dtype="bf16", chunk=512, seed=7, residual=False, weight_format="mxfp4"),
    "decode_large_w4": Workload("decode_large_w4", H=2880, E=128, K=4, I=2880, n_layers=4, D=256, P=0,
                                dtype="bf16", chunk=512, seed=6, weight_format="mxfp4", y_perm_f32=True),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller test versions)."""
    return replace(w, **kw)


def torch_dtype(name: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f32": torch.float32}[name]


def _stream_seed(seed: int, name: str, layer: int) -> int:
    return (zlib.crc32(f"{name}/{layer}".encode()) ^ (seed * 0x9E3779B1)) & 0x7FFFFFFF


def randn(shape, std: float, seed: int, name: str, layer: int = 0, dtype: str = "bf16",
          device: str = "cpu") -> torch.Tensor:
    """N(0, std) drawn in fp32 on `device`, rounded once to `dtype`."""
    g = torch.Generator(device=device)
    g.manual_seed(_stream_seed(seed, name, layer))
    numel = int(np.prod(shape)) if len(shape) else 1
    out = torch.empty(shape, dtype=torch_dtype(dtype), device=device)
    flat = out.view(-1)
    step = 1 << 27      # draw in slices so the fp32 temporary stays small
    for s in range(0, numel, step):
        n = min(step, numel - s)
        flat[s:s + n] = (torch.randn(n, generator=g, device=device, dtype=torch.float32) * std).to(out.dtype)
    return out


def zipf_shares(E: int, s: float) -> np.ndarray:
    """Target per-expert assignment shares p_e proportional to rank^-s, rank = e+1."""
    p = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    return p / p.sum()


def stored_router_bias(w: Workload, layer: int) -> Optional[torch.Tensor]:
    """Per-expert router bias of a skewed-routing workload (fp32 [E], CPU), or None.

    The values were calibrated once, against the CPU-drawn router weights and hidden states of the
    workload, so that the experts' assignment shares follow Zipf(zipf_s); they are stored as data in
    data/router_bias_<workload>.json (written by oracle/calibrate_zipf_bias.py).
    """
    if w.zipf_s <= 0:
        if w.route_skew > 0:
            return randn((w.E,), w.route_skew, w.seed, "route_skew_bias", layer, "f32", "cpu")
        return None
    # (variants of a workload that differ only in how the GPU context holds its intermediates share the data)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data",
                        f"router_bias_{w.name.replace('_bf16act', '')}.json")
    with open(path) as f:
        rec = json.load(f)
    assert rec["E"] == w.E and rec["seed"] == w.seed and abs(rec["zipf_s"] - w.zipf_s) < 1e-12
    return torch.tensor(rec["bias"][layer], dtype=torch.float32)


def rand_bytes(shape, lo: int, hi: int, seed: int, name: str, layer: int = 0, device: str = "cpu") -> torch.Tensor:
    """uint8 tensor, uniform over [lo, hi], from the stream of (seed, name, layer) on `device`."""
    g = torch.Generator(device=device)
    g.manual_seed(_stream_seed(seed, name, layer))
    numel = int(np.prod(shape))
    out = torch.empty(shape, dtype=torch.uint8, device=device)
    flat = out.view(-1)
    step = 1 << 28
    for s in range(0, numel, step):
        n = min(step, numel - s)
        flat[s:s + n] = torch.randint(lo, hi + 1, (n,), generator=g, device=device, dtype=torch.uint8)
    return out


def make_layer(w: Workload, layer: int, device: str = "cpu", with_bias: bool = True):
    """Random weights of one MoE layer: dict of w_router [E,H], router_bias, w_gate_up [E,2I,H], w_down [E,H,I].

    The (small) router tensors are always drawn on the CPU, so that they are the same bits wherever the
    (large) expert weights are drawn; everything is returned on `device`.

    weight_format "mxfp4": the expert weights are drawn directly in their storage format (no quantiser is
    involved): code bytes uniform over 0..255, i.e. every FP4 E2M1 value equally likely (rms 2.93), and
    scale bytes uniform over 118..120 (2^-9 .. 2^-7), which gives weights of rms 0.015, just under the
    N(0, 0.02) weights of the other workloads (one step up, 119..121, gives rms 0.030: a branch gain above
    one at H = I = 2880, and a residual stream that grows 2.5-fold per layer).  w_gate_up is uint8 [E,2I,H/2] with s_gate_up uint8
    [E,2I,H/32]; w_down uint8 [E,H,I/2] with s_down uint8 [E,H,I/32].
    """
    bias = stored_router_bias(w, layer) if with_bias else None
    if w.weight_format == "mxfp4":
        assert w.dtype == "bf16" and w.H % 64 == 0 and w.I % 64 == 0
        return {
            "w_router": randn((w.E, w.H), 0.02, w.seed, "w_router", layer, w.dtype, "cpu").to(device),
            "router_bias": None if bias is None else bias.to(device),
            "w_gate_up": rand_bytes((w.E, 2 * w.I, w.H // 2), 0, 255, w.seed, "w_gate_up_codes", layer, device),
            "s_gate_up": rand_bytes((w.E, 2 * w.I, w.H // 32), 118, 120, w.seed, "w_gate_up_scales", layer, device),
            "w_down": rand_bytes((w.E, w.H, w.I // 2), 0, 255, w.seed, "w_down_codes", layer, device),
            "s_down": rand_bytes((w.E, w.H, w.I // 32), 118, 120, w.seed, "w_down_scales", layer, device),
        }
    return {
        "w_router": randn((w.E, w.H), 0.02, w.seed, "w_router", layer, w.dtype, "cpu").to(device),
        "router_bias": None if bias is None else bias.to(device),
        "w_gate_up": randn((w.E, 2 * w.I, w.H), 0.02, w.seed, "w_gate_up", layer, w.dtype, device),
        "w_down": randn((w.E, w.H, w.I), 0.02, w.seed, "w_down", layer, w.dtype, device),
    }


def make_hidden(w: Workload, device: str = "cpu"):
    """(x_decode [D,H], x_prefill [P,H]) ~ N(0,1); drawn on the CPU (same bits everywhere), returned on `device`."""
    xd = randn((w.D, w.H), 1.0, w.seed, "x_decode", 0, w.dtype, "cpu").to(device)
    xp = randn((w.P, w.H), 1.0, w.seed, "x_prefill", 0, w.dtype, "cpu").to(device)
    return xd, xp


def to_numpy(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """Host copy for the oracle: float32/float64 as they are, bfloat16 as uint16 bit patterns."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def layer_to_numpy(layer: dict) -> dict:
    return {k: to_numpy(v) for k, v in layer.items()}
