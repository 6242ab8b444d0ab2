#!/usr/bin/env python3
"""Benchmark of the MoE expert-FFN hot path on one MI355X.

A "step" is one pass of the whole path (router -> top-k -> permutation -> grouped gate_up/SwiGLU
-> grouped down -> combine, for every layer and iteration of the chosen schedule) over one batch
of seeded synthetic input that is already resident in HBM.

With no --workload the headline is the largest single-GPU configuration of the baseline, the
8-layer Qwen3-30B-A3B-shaped group under layered prefill (one 8192-token prompt + 128 decode
tokens, bf16; Sec. 4.1-4.2 against Sec. 2.3), and the same run also measures every other baseline
configuration under the schedules it names (a `workloads` list in the same JSON line: ms/step,
tokens/s, the gate_up and down kernels' time and roofline fraction, and the whole step's fraction
of its roofline).  With --workload only that workload is measured.

Prints ONE JSON line: tokens/s of the whole job, the roofline fraction of the dominant kernel
(the gate_up grouped GEMM, timed live with HIP events on the launch stream), and the fp64 CPU
oracle timed on this host's cores as a reported baseline.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
RIDGE_ROWS = 312.0             # 2.5 PFLOP/s / 8 TB/s: rows per expert above which a bf16 layer is compute bound (Sec. 2.5)
# which roofline prices a workload (None: by schedule; the hybrid Qwen-shaped batches sit below the ridge
# with ~130 rows per expert, the 8192-token layered pass above it with ~520: Sec. 2.5, 4.3)
BOUND = {"qwen3_layer": "hbm", "decode_large": "hbm", "qwen3_group8": None, "mixtral_zipf": "mfma",
         "mixtral_zipf_bf16act": "mfma", "tiny_f32": "hbm",
         "gptoss_layer": "hbm",       # 264 rows per expert: below the ridge
         "decode_large_w4": "hbm",
         "gptoss_layer_w4": "mfma"}   # 17/32 byte per weight moves the ridge to ~83 rows per expert
# the default run: the headline first, then every other baseline configuration x the schedules it names
HEADLINE = ("qwen3_group8", "layered")
ALSO = [("qwen3_group8", "chunked"), ("qwen3_layer", "layered"), ("mixtral_zipf", "layered"),
        ("mixtral_zipf_bf16act", "layered"), ("decode_large", "layered"), ("tiny_f32", "layered"),
        ("tiny_f32", "chunked")]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="",
                    help="measure this workload only (default: the headline plus a `workloads` list of the others)")
    ap.add_argument("--schedule", default="layered", choices=["layered", "chunked", "stack"],
                    help="layered / chunked: the workload's layers as ONE layer group (moe_group_forward); "
                         "stack: the workload's layers as a whole stack cut into --groups layer groups, one group "
                         "per iteration carrying the prompt, with --chunk prompt tokens per outer pass "
                         "(moe_stack_forward)")
    ap.add_argument("--chunk", type=int, default=0,
                    help="chunk size (chunked: default the workload's; stack: default 0 = the whole prompt)")
    ap.add_argument("--groups", type=int, default=0,
                    help="--schedule stack: number of layer groups (0 = max(1, ceil(slice / --granule)), at most layers)")
    ap.add_argument("--granule", type=int, default=512, help="--schedule stack: tokens per iteration the group rule aims for")
    ap.add_argument("--per-iteration", action="store_true",
                    help="stack schedule with --chunk 0: also time every iteration of the step on its own (the "
                         "iteration whose designated layer group carries the prompt, Sec. 4.1-4.2), rebuilt from "
                         "group calls and checked against the stack driver's result")
    ap.add_argument("--decode", type=int, default=-1, help="override the workload's number of decode tokens")
    ap.add_argument("--route-skew", type=float, default=-1.0,
                    help="override the workload's router popularity skew (std of a per-expert logit bias)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--time-all-kernels", action="store_true",
                    help="bracket all six kernels of a layer with events (default: the two grouped GEMMs)")
    ap.add_argument("--ffn-variant", default="auto",
                    choices=["auto", "tile128", "small", "big", "w4_tile64", "w4_stream"],
                    help="tuning aid: pin the grouped-GEMM kernel shape (moe_set_ffn_variant); auto = the library's own choice")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy kernel a few times (reference for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    return ap.parse_args()


def traffic_from_profiles(workload, schedule, variant):
    """(HBM bytes per gate_up launch, file) as measured once with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE,
    scaled by a copy kernel) and committed under profiles/, when a summary for this workload, schedule and
    kernel variant exists; else (None, None).  The figure is read from that file: it is not measured by this run."""
    rel = os.path.join("profiles", f"gate_up_traffic_{workload}_{schedule}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    if f"variant: {variant}" not in text:
        return None, None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    return (float(m.group(1)), rel) if m else (None, None)


def measure(args, name, schedule, steps, warmup, cpu_baseline):
    """One workload under one schedule: timed steps, kernel timings, counters -> the fields of a JSON entry."""
    import torch
    from paper_2510_08055_amd import binding, inputs

    dev = "cuda:0"
    w = inputs.WORKLOADS[name]
    if args.decode >= 0:
        w = inputs.scaled(w, D=args.decode)
    if args.route_skew >= 0:
        w = inputs.scaled(w, route_skew=args.route_skew)
    stack = schedule == "stack"
    chunk = args.chunk if stack else (args.chunk or w.chunk)
    dt = inputs.torch_dtype(w.dtype)
    esz = 2 if w.dtype == "bf16" else 4

    layers = [inputs.make_layer(w, l, device=dev) for l in range(w.n_layers)]
    xd, xp = inputs.make_hidden(w, device=dev)
    if stack:
        T_iter = w.D + (w.P if chunk == 0 else min(w.P, chunk))
    else:
        T_iter = w.D + (w.P if schedule == "layered" else min(w.P, chunk))
    ctx = binding.Context(w.H, w.E, w.K, w.I, dt, max_tokens=T_iter, residual=w.residual, device=dev,
                          weight_format=w.weight_format, y_perm_f32=w.y_perm_f32, act_split=w.act_split)
    wsz = 17.0 / 32.0 if w.weight_format == "mxfp4" else esz       # bytes per expert-weight element (codes + scales)
    act_sz = esz * (2 if w.act_split else 1)                        # bytes per element of the intermediate
    y_sz = 4 if (w.y_perm_f32 or w.dtype == "f32") else 2           # bytes per element of y_perm
    if args.ffn_variant != "auto":
        ctx.moe_set_ffn_variant(args.ffn_variant)
    packed = ctx.pack_layers(layers)
    yd = torch.empty((w.D, w.H), dtype=dt, device=dev)
    yp = torch.empty((w.P, w.H), dtype=dt, device=dev)

    def step():
        if stack:
            ctx.moe_stack_forward(layers, xd if w.D else None, xp if w.P else None, chunk=chunk, n_groups=args.groups,
                                  granule=args.granule, packed=packed, y_decode=yd, y_prefill=yp)
        else:
            ctx.moe_group_forward(layers, xd if w.D else None, xp if w.P else None, schedule, chunk,
                                  packed=packed, y_decode=yd, y_prefill=yp)

    timed = list(binding.KERNELS) if args.time_all_kernels else ["gate_up", "down"]
    ctx.moe_kernel_timing(timed)            # the warm-up also fills the context's pool of event pairs
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ctx.moe_reset_counters()
    ctx.moe_kernel_timing(timed)            # forget the warm-up's records; event pairs per launch, on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    k_time = {k: ctx.moe_read_kernel_timing(k) for k in timed}
    ctr = ctx.moe_read_counters()
    ctx.moe_kernel_timing([])

    tokens_per_step = w.D + w.P                 # distinct tokens served by one step
    ms_per_step = elapsed / steps * 1e3
    value = tokens_per_step * steps / elapsed

    # ---- algorithmic work per launch of the two GEMMs and per step ----
    # (launches differ in size when decode-only passes mix with prompt passes: the figures are means over
    # the launches; every layer sees the decode rows once per iteration and each prompt row once per step)
    launches_per_step = ctr.layer_passes / steps
    active_per_launch = ctr.active_experts_total / ctr.layer_passes
    iters_per_step = ctr.iterations / steps
    rows_per_launch = w.n_layers * (iters_per_step * w.D + w.P) / launches_per_step
    A = rows_per_launch * w.K
    gu_bytes = active_per_launch * 2 * w.I * w.H * wsz + rows_per_launch * w.H * esz + A * w.I * act_sz
    gu_flops = 2.0 * A * w.H * 2 * w.I
    dn_bytes = active_per_launch * w.I * w.H * wsz + A * w.I * act_sz + A * w.H * y_sz
    dn_flops = 2.0 * A * w.I * w.H
    # the rest of a layer pass at its least traffic: router reads x and its weights, writes and re-reads the
    # fp64 logits; the combine reads y_perm (and x as the residual) and writes the layer's output
    rest_bytes = (rows_per_launch * w.H * esz + w.E * w.H * esz + 2 * rows_per_launch * w.E * 8 + A * w.H * y_sz
                  + (rows_per_launch * w.H * esz if w.residual else 0) + rows_per_launch * w.H * esz + 6 * A * 4)
    step_bytes = launches_per_step * (gu_bytes + dn_bytes + rest_bytes)
    step_flops = launches_per_step * (gu_flops + dn_flops + 2.0 * rows_per_launch * w.E * w.H)
    if stack:
        bound = "mfma" if A / w.E > RIDGE_ROWS else "hbm"      # mean rows per expert against the ridge
    else:
        bound = BOUND.get(name) or ("mfma" if schedule == "layered" else "hbm")
    variant = ctx.moe_ffn_variant(int(rows_per_launch))

    def priced(nbytes, nflops, seconds):
        if bound == "hbm":
            return nbytes / seconds / 1e9, HBM_PEAK_GBS, "GB/s"
        return nflops / seconds / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"

    kernels = {}
    for k, (ms, n) in k_time.items():
        kernels[k] = {"avg_us": round(ms / max(n, 1) * 1e3, 2), "launches": n}
    for k, (nb, nf) in (("gate_up", (gu_bytes, gu_flops)), ("down", (dn_bytes, dn_flops))):
        ach, peak, unit = priced(nb, nf, kernels[k]["avg_us"] * 1e-6)
        kernels[k].update(achieved=round(ach, 2), unit=unit, frac=round(ach / peak, 4),
                          algorithmic_bytes_per_launch=int(nb), algorithmic_flops_per_launch=int(nf))
    s_ach, s_peak, s_unit = priced(step_bytes, step_flops, ms_per_step * 1e-3)
    traffic, traffic_file = traffic_from_profiles(name, schedule, variant)
    g = kernels["gate_up"]
    roofline = {"bound": bound, "achieved": g["achieved"], "peak": s_peak, "unit": g["unit"], "frac": g["frac"],
                "traffic": traffic, "traffic_source": (f"{traffic_file} (rocprofv3 --pmc summary committed with the "
                                                       "sources; not measured by this run)") if traffic_file else None,
                "kernel": variant, "kernel_avg_us": g["avg_us"], "kernel_launches": g["launches"],
                "algorithmic_bytes_per_launch": g["algorithmic_bytes_per_launch"],
                "algorithmic_flops_per_launch": g["algorithmic_flops_per_launch"]}

    # ---- iteration-time balance of the layered schedule over the stack (one slice only) ----
    iteration_ms = None
    if stack and args.per_iteration and chunk == 0 and w.D and w.P:
        G = args.groups if args.groups > 0 else binding.moe_num_layer_groups(w.P, w.n_layers, args.granule)
        first = binding.moe_layer_groups(w.n_layers, G)
        big = binding.Context(w.H, w.E, w.K, w.I, dt, max_tokens=w.D + w.P, residual=w.residual, device=dev,
                              weight_format=w.weight_format, y_perm_f32=w.y_perm_f32, act_split=w.act_split)
        p_state = [xp, torch.empty_like(xp)]
        d_buf = [torch.empty_like(xd), torch.empty_like(xd)]

        def iteration(g_, src):       # iteration g_: group g_ carries the prompt rows, every group the decode rows
            d_in = xd
            for h in range(G):
                sub = layers[first[h]:first[h + 1]]
                d_out = d_buf[h % 2]
                if h == g_:
                    big.moe_group_forward(sub, d_in, p_state[src], "layered", y_decode=d_out, y_prefill=p_state[1 - src])
                else:
                    big.moe_group_forward(sub, d_in, None, "layered", y_decode=d_out)
                d_in = d_out
            return d_in

        def whole_step():
            src, d_last = 0, None
            for g_ in range(G):
                d_last = iteration(g_, src)
                src = 1 - src
            return d_last, p_state[src]

        d_last, p_last = whole_step()
        torch.cuda.synchronize()
        if not (torch.equal(d_last, yd) and torch.equal(p_last, yp)):
            print("bench.py: the iterations rebuilt from group calls do not reproduce the stack driver", file=sys.stderr)
            sys.exit(3)
        reps = 3
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(G)]
              for _ in range(reps)]
        for r in range(reps):
            src = 0
            for g_ in range(G):
                ev[r][g_][0].record()
                iteration(g_, src)
                ev[r][g_][1].record()
                src = 1 - src
        torch.cuda.synchronize()
        iteration_ms = [round(min(ev[r][g_][0].elapsed_time(ev[r][g_][1]) for r in range(reps)), 4) for g_ in range(G)]
        big.close()

    # ---- the oracle as it stands, on this host's cores, on a bounded sample of the same workload ----
    cpu = None
    if cpu_baseline:
        import oracle
        n_sample = min(tokens_per_step, 8320)        # ~12 s of the oracle on 16 cores for the headline's layer shape
        x = torch.cat([xd, xp])[:n_sample]
        L0 = inputs.layer_to_numpy(layers[0])
        xn = inputs.to_numpy(x)
        t1 = time.perf_counter()
        oracle.moe_layer(xn, L0["w_router"], L0["router_bias"], L0["w_gate_up"], L0["w_down"], w.K,
                         residual=w.residual, s_gate_up=L0.get("s_gate_up"), s_down=L0.get("s_down"))
        cpu_s = time.perf_counter() - t1
        # one layer over n_sample tokens; a step crosses n_layers layers per token
        cpu = {"value": round(n_sample / cpu_s / w.n_layers, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"first {n_sample} rows of the batch through layer 0 (fp64 C, {cpu_s:.1f} s), "
                         f"scaled by 1/{w.n_layers} layers"}

    out = {
        "value": round(value, 1), "ms_per_step": round(ms_per_step, 4), "steps": steps, "warmup": warmup, "dtype": w.dtype,
        "config": {"workload": name, "schedule": schedule,
                   "chunk": chunk if schedule != "layered" else None,
                   "groups": args.groups if stack else None, "granule": args.granule if stack else None, "H": w.H, "E": w.E,
                   "top_k": w.K, "I": w.I, "layers": w.n_layers, "decode_tokens": w.D, "prefill_tokens": w.P, "seed": w.seed,
                   "route_skew": w.route_skew, "weight_format": w.weight_format or w.dtype,
                   "y_perm": "f32" if y_sz == 4 else "bf16", "intermediate": "bf16 pair" if w.act_split else w.dtype,
                   "ffn_variant": args.ffn_variant},
        "roofline": roofline,
        "kernels": kernels,
        "step": {"bound": bound, "achieved": round(s_ach, 2), "unit": s_unit, "frac": round(s_ach / s_peak, 4),
                 "algorithmic_bytes": int(step_bytes), "algorithmic_flops": int(step_flops)},
        "cpu_baseline": cpu,
        "expert_bytes_per_step": ctr.expert_bytes // steps,
        "expert_bytes_per_prompt_token": (ctr.expert_bytes / steps / w.P) if w.P else None,
        "iterations_per_step": ctr.iterations // steps,
        "gate_up_launches_per_step": launches_per_step,
    }
    if iteration_ms is not None:
        out["iteration_ms"] = iteration_ms      # one entry per iteration of the step; group sizes differ by at most one layer
    ctx.close()
    del layers, packed, xd, xp, yd, yp, ctx
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures the single-GPU hot path only: this build has no multi-GPU path "
              "(run with --gpus 1; value is the one GPU's throughput)", file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 5}))
        return

    single = bool(args.workload)
    name, schedule = (args.workload, args.schedule) if single else HEADLINE
    head = measure(args, name, schedule, args.steps, args.warmup, cpu_baseline=not args.no_cpu_baseline)
    out = {"metric": "MoE layer tokens/s", "value": head.pop("value"), "unit": "tokens/s", "n_gpus": 1,
           "steps": head.pop("steps"), "warmup": head.pop("warmup"), "ms_per_step": head.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": head.pop("dtype"),
           "data": "synthetic"}
    out.update(head)
    if not single:
        # every other baseline configuration, fewer steps each (the long ones are tens of milliseconds a step)
        others = []
        for wl, sc in ALSO:
            n_steps = min(args.steps, 10)
            e = measure(args, wl, sc, n_steps, min(args.warmup, 3), cpu_baseline=False)
            e.pop("cpu_baseline", None)
            e["tokens_per_s"] = e.pop("value")
            e["workload"], e["schedule"] = wl, sc
            others.append(e)
        out["workloads"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
