#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2] [--no-cpu-baseline]

One "step" is one whole moe_layer_forward call (gate -> capacity routing ->
dispatch -> expert FFNs -> combine [+ dense branch]) over one batch of seeded
synthetic input that is already resident in HBM.  Prints ONE JSON line.

  value / unit     tokens/s of the whole call (input tokens, dropped ones included)
  roofline         the dominant kernel (the longer of the two expert GEMMs):
                   algorithmic bytes per launch / its mean duration, measured with
                   HIP events recorded by the library on the launch stream inside
                   the timed region; `traffic` is the rocprofv3 FETCH_SIZE+WRITE_SIZE
                   figure for the same launch (see profiles/), or null
  layer_roofline   the same for the whole call against the layer's algorithmic bytes
  cpu_baseline     the fp64 NumPy oracle on the host cores, one full step of the
                   same workload (reported baseline, not the target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
# scaled by a copy kernel of known size; keyed by workload.  Filled from profiles/*.md.
MEASURED_TRAFFIC_BYTES = {
    ("c2", "expert_gemm1"): 1161762918,   # profiles/wsgemm_expert_gemm_c2.md
    ("c2", "expert_gemm2"): 1162602291,
    ("c4", "expert_gemm1"): 1627605606,   # profiles/wsgemm_decode_c4.md
    ("c4", "expert_gemm2"): 1613486490,
}


# What a kernel that only reads the same weights in the same access pattern reaches (GB/s), measured with
# paper_2201_05596_amd/hbm_rate (profiles/hbm_read_ceiling.md): context for roofline.frac, not its denominator.
MEASURED_READ_CEILING_GBS = {
    ("c2", "expert_gemm1"): 6850.0,
    ("c2", "expert_gemm2"): 6910.0,
}


def algorithmic_bytes(cfg, rows):
    """Bytes the method itself has to move, from the actual per-expert row counts."""
    d, f, T = cfg.d_model, cfg.d_ffn, cfg.T
    wb = 4 if cfg.dtype == "f32" else 2
    touched = int((rows > 0).sum())
    kept = int(rows.sum())
    g1 = touched * (d * f + f) * wb + kept * d * wb + kept * f * wb        # W1,b1 once; rows in; h out
    g2 = touched * (f * d + d) * wb + kept * f * wb + kept * d * wb        # W2,b2 once; h in; rows out
    layer = touched * (2 * d * f + f + d) * wb + 2 * T * d * wb + d * cfg.E * 4
    flops = 4 * d * f * kept + 2 * T * d * cfg.E
    if cfg.residual:
        layer += (2 * d * f + f + d) * wb
        flops += 4 * d * f * T
    return {"expert_gemm1": g1, "expert_gemm2": g2, "layer": layer, "flops": flops,
            "touched_experts": touched, "kept_rows": kept}


def cpu_baseline(inp, cfg):
    """The oracle as it stands, one full step of the workload on the host cores."""
    import numpy as np
    from oracle import moe_oracle as orc
    from workloads.generate import to_f32_numpy
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    h = {k: to_f32_numpy(v) for k, v in inp.tensors().items()}
    steps, total = 0, 0.0
    while total < 10.0 and steps < 8:          # about 10-20 s of CPU work
        t0 = time.perf_counter()
        orc.moe_layer_forward(h["x"], h["Wg"], h.get("bg"), h["W1"], h["b1"], h["W2"], h["b2"], cfg.top_k,
                              cfg.capacity, Wd1=h.get("Wd1"), bd1=h.get("bd1"), Wd2=h.get("Wd2"), bd2=h.get("bd2"))
        total += time.perf_counter() - t0
        steps += 1
    return {"value": cfg.T * steps / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{steps} full step(s) of {cfg.name} ({cfg.T} tokens each), fp64 NumPy, {total:.2f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--capacity-factor", type=float, default=None, help="experiment: override the workload's capacity factor")
    ap.add_argument("--no-gate-bias", action="store_true",
                    help="experiment: drop the workload's gate bias (c5 without its skew: ~512 rows per expert)")
    ap.add_argument("--no-stage-events", action="store_true",
                    help="experiment: time the steps without the library's per-stage events (no roofline then)")
    ap.add_argument("--all-stage-events", action="store_true", help="time every stage (more events, slower step)")
    ap.add_argument("--event-stride", type=int, default=5,
                    help="stage events are recorded in every n-th timed step only (the first, the (n+1)-th, ...)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "traffic that scales the FETCH_SIZE / WRITE_SIZE counters in rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    import paper_2201_05596_amd as moe
    from workloads import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    if args.capacity_factor is not None:
        cfg = cfg.scaled(name=f"{cfg.name}-cf{args.capacity_factor}", capacity_factor=args.capacity_factor)
    if args.no_gate_bias:
        cfg = cfg.scaled(name=f"{cfg.name}-nobias", gate_bias_zipf=None)
    inp = make_inputs(cfg, "cuda:0")
    layer = moe.MoELayer(cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, cfg.capacity, cfg.dtype, inp.Wg, inp.bg,
                         inp.W1, inp.b1, inp.W2, inp.b2, inp.Wd1, inp.bd1, inp.Wd2, inp.bd2)
    for _ in range(args.warmup):
        layer(inp.x)
    torch.cuda.synchronize()

    if not args.no_stage_events:
        # events only around the two expert GEMMs (the roofline kernel is the longer one): three per timed step, and
        # only every --event-stride-th step is timed that way (1.5 us per event is 1.5 % of a c2 step)
        moe.moe_profile_select(None if args.all_stage_events else ["expert_gemm1", "expert_gemm2"])
        moe.moe_profile_stride(args.event_stride)
        moe.moe_profile_enable((args.steps + args.event_stride - 1) // args.event_stride)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer(inp.x)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    names = moe.moe_profile_stage_names()
    sums = [0.0] * len(names)
    ncalls = moe.moe_profile_calls()
    for c in range(ncalls):
        for i, v in enumerate(moe.moe_profile_elapsed(c)):
            sums[i] += v
    moe.moe_profile_enable(0)
    stage_ms = {n: s / max(ncalls, 1) for n, s in zip(names, sums) if s > 0}

    if args.calibration_copy_mib > 0:
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    rows = layer.routing["expert_rows"].cpu().numpy()
    alg = algorithmic_bytes(cfg, rows)
    dom = max(("expert_gemm1", "expert_gemm2"), key=lambda n: stage_ms.get(n, 0.0))
    dom_ms = stage_ms.get(dom, 0.0)
    achieved = alg[dom] / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, dom)),
                "algorithmic_bytes": alg[dom], "avg_ms": dom_ms}
    ceiling = MEASURED_READ_CEILING_GBS.get((cfg.name, dom))
    if ceiling:
        roofline["read_only_kernel_GBps"] = ceiling
        roofline["frac_of_read_only_kernel"] = achieved / ceiling
    layer_gbs = alg["layer"] / (ms_per_step * 1e-3) / 1e9
    layer_tflops = alg["flops"] / (ms_per_step * 1e-3) / 1e12

    out = {
        "metric": "MoE-layer tokens/s at 1 GPU",
        "value": cfg.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_layer": ms_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d_model={cfg.d_model} d_ffn={cfg.d_ffn} E={cfg.E} "
                               f"top_k={cfg.top_k} capacity={cfg.capacity} residual={int(cfg.residual)} seed={cfg.seed}",
                   "kept_rows": alg["kept_rows"], "touched_experts": alg["touched_experts"]},
        "roofline": roofline,
        "layer_roofline": {"hbm_GBps": layer_gbs, "hbm_frac": layer_gbs / HBM_PEAK_GBS,
                           "mfma_TFLOPs": layer_tflops, "mfma_frac": layer_tflops / MFMA_BF16_PEAK_TFLOPS,
                           "algorithmic_bytes": alg["layer"], "algorithmic_flops": alg["flops"]},
        "stage_ms": stage_ms,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
