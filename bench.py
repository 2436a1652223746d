#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c5] [--only] [--no-cpu-baseline]

One "step" is one whole moe_layer_forward call (gate -> capacity routing ->
dispatch -> expert FFNs -> combine [+ dense branch]) over one batch of seeded
synthetic input that is already resident in HBM.  Prints ONE JSON line.

The headline workload (--config, default c5: the largest single-GPU
configuration) is timed for exactly K steps after W warm-up steps; the same
line carries one sub-record per benchmark configuration (c2, c3a, c3b, c4, c5)
under "configs" unless --only is given.  Before the W warm-up steps every
workload runs RAMP untimed steps: the matrix-core-bound ones are 5-10 % slower
while the engine clock is still settling.

  value / unit     tokens/s of the whole call (input tokens, dropped ones included)
  roofline         which roofline binds the workload (the larger of algorithmic
                   bytes / 8 TB/s and algorithmic flops / 2.5 PFLOP/s), and the
                   longest kernel of the call against that roofline: its
                   algorithmic bytes (weights and biases of the experts it
                   touches) or flops per launch / its mean duration, from HIP
                   events the library records on the launch stream inside the
                   timed region.  `traffic` is the HBM traffic of that kernel
                   from separate rocprofv3 --pmc runs (see profiles/), or null.
  layer_roofline   the whole call against the layer's algorithmic bytes and flops
  cpu_baseline     the fp64 NumPy oracle on the host cores on a bounded sample of
                   the headline workload (reported baseline, not the target)
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

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
RAMP_STEPS = 100                # untimed steps before the warm-up steps (clock settling)
EVENT_STRIDE = 5                # stage events are recorded in every 5th timed step only
SUB_STEPS = 40                  # timed steps of a sub-record
ALL_CONFIGS = ("c2", "c3a", "c3b", "c4", "c5")

# HBM traffic per launch (bytes) of a workload's longest kernel: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE,
# each scaled by what the same counter reads for a plain copy of known size.  Measured in separate runs
# (profiles/*.md name the commands), not in this process.
PROFILED_TRAFFIC = {          # profiles/hbm_traffic_all_configs.md
    ("c2", "expert_gemm1"): 1161700000, ("c2", "expert_gemm2"): 1162500000,
    ("c3a", "expert_gemm2"): 500000000, ("c3a", "expert_gemm1"): 583500000,       # experts + dense branch, one launch
    ("c3b", "expert_gemm1"): 617200000, ("c3b", "expert_gemm2"): 769000000,       # GEMM-2: experts + dense branch
    ("c4", "expert_gemm1"): 1628100000, ("c4", "expert_gemm2"): 1613400000,
    ("c5", "expert_gemm1"): 9341700000, ("c5", "expert_gemm2"): 11142800000,
}


def algorithmic_work(cfg, rows):
    """Bytes and flops the method itself has to move and compute, from the actual per-expert row counts.
    Per kernel: the weights and biases it has to read once (unit = one expert with at least one row) and
    the multiply-adds of its rows (unit = one kept row)."""
    d, f, T, E = cfg.d_model, cfg.d_ffn, cfg.T, cfg.E
    wb = 4 if cfg.dtype == "f32" else 2
    touched = int((rows > 0).sum())
    kept = int(rows.sum())
    stage_bytes = {"expert_gemm1": touched * (d * f + f) * wb, "expert_gemm2": touched * (f * d + d) * wb,
                   "gate_logits": T * d * wb + d * E * 4, "dense_gemm1": (d * f + f) * wb, "dense_gemm2": (f * d + d) * wb}
    stage_flops = {"expert_gemm1": 2 * d * f * kept, "expert_gemm2": 2 * d * f * kept, "gate_logits": 2 * T * d * E,
                   "dense_gemm1": 2 * d * f * T, "dense_gemm2": 2 * d * f * T}
    layer_bytes = touched * (2 * d * f + f + d) * wb + 2 * T * d * wb + d * E * 4
    layer_flops = 4 * d * f * kept + 2 * T * d * E
    if cfg.residual:
        layer_bytes += (2 * d * f + f + d) * wb
        layer_flops += 4 * d * f * T
    return {"stage_bytes": stage_bytes, "stage_flops": stage_flops, "layer_bytes": layer_bytes, "layer_flops": layer_flops,
            "touched_experts": touched, "kept_rows": kept}


def describe(cfg):
    return (f"{cfg.name}: T={cfg.T} d_model={cfg.d_model} d_ffn={cfg.d_ffn} E={cfg.E} top_k={cfg.top_k} "
            f"capacity={cfg.capacity} residual={int(cfg.residual)} seed={cfg.seed}")


def time_config(cfg, steps, warmup, pack):
    """RAMP + warmup untimed steps, then exactly `steps` timed ones.  Returns (record, inputs)."""
    import torch
    import paper_2201_05596_amd as moe
    from workloads import make_inputs

    inp = make_inputs(cfg, "cuda:0")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    layer = moe.MoELayer(cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, cfg.capacity, cfg.dtype, inp.Wg, inp.bg,
                         inp.W1, inp.b1, inp.W2, inp.b2, inp.Wd1, inp.bd1, inp.Wd2, inp.bd2, pack_weights=pack)
    torch.cuda.synchronize()
    setup_ms = (time.perf_counter() - t0) * 1e3       # buffers + (packed) the one-time moe_pack_weights calls
    for _ in range(RAMP_STEPS + warmup):
        layer(inp.x)
    torch.cuda.synchronize()

    moe.moe_profile_select(None)                 # every stage gets its own pair of events ...
    moe.moe_profile_stride(EVENT_STRIDE)         # ... in every EVENT_STRIDE-th timed step
    moe.moe_profile_enable((steps + EVENT_STRIDE - 1) // EVENT_STRIDE)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        layer(inp.x)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    names = moe.moe_profile_stage_names()
    sums = [0.0] * len(names)
    ncalls = moe.moe_profile_calls()
    for c in range(ncalls):
        for i, v in enumerate(moe.moe_profile_elapsed(c)):
            sums[i] += v
    moe.moe_profile_enable(0)
    moe.moe_profile_stride(1)
    stage_ms = {n: s / max(ncalls, 1) for n, s in zip(names, sums) if s > 0}

    rows = layer.routing["expert_rows"].cpu().numpy()
    alg = algorithmic_work(cfg, rows)
    paired = []    # stages in which the dense branch's product ran inside the experts' launch: its work belongs there
    for e, dn in (("expert_gemm1", "dense_gemm1"), ("expert_gemm2", "dense_gemm2")):
        if cfg.residual and dn not in stage_ms and e in stage_ms:
            alg["stage_flops"][e] += alg["stage_flops"][dn]
            alg["stage_bytes"][e] += alg["stage_bytes"][dn]
            paired.append(e)
    t_hbm = alg["layer_bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = alg["layer_flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12) if cfg.dtype == "bf16" else 0.0
    bound = "mfma" if t_mfma > t_hbm else "hbm"
    dom = max(stage_ms, key=stage_ms.get) if stage_ms else None
    dom_ms = stage_ms.get(dom, 0.0) if dom else 0.0
    if bound == "hbm":
        work, peak, unit = alg["stage_bytes"].get(dom, 0), HBM_PEAK_GBS, "GB/s"
        achieved = work / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    else:
        work, peak, unit = alg["stage_flops"].get(dom, 0), MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        achieved = work / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    traffic = PROFILED_TRAFFIC.get((cfg.name, dom))
    roofline = {"bound": bound, "kernel": dom + (" (experts + dense branch in one launch)" if dom in paired else "") if dom else dom, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                "traffic": traffic, "traffic_source": "rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, separate runs on packed weights "
                                  "(profiles/hbm_traffic_all_configs.md); not measured in this process" if traffic else None,
                "algorithmic_work_per_launch": work, "avg_ms": dom_ms, "timed_launches": ncalls,
                "t_floor_hbm_us": t_hbm * 1e6, "t_floor_mfma_us": t_mfma * 1e6}
    layer_gbs = alg["layer_bytes"] / (ms_per_step * 1e-3) / 1e9
    layer_tflops = alg["layer_flops"] / (ms_per_step * 1e-3) / 1e12
    rec = {
        "workload": describe(cfg), "us_per_layer": ms_per_step * 1e3, "tokens_per_s": cfg.T / (ms_per_step * 1e-3),
        "steps": steps, "warmup": warmup,
        "weights": f"packed once by moe_pack_weights, outside the timed region (layer set-up {setup_ms:.1f} ms)" if pack
                   else "plain [E,d,f] / [E,f,d]",
        "kept_rows": alg["kept_rows"], "touched_experts": alg["touched_experts"],
        "expert_rows": [int(r) for r in rows],
        "roofline": roofline,
        "layer_roofline": {"hbm_GBps": layer_gbs, "hbm_frac": layer_gbs / HBM_PEAK_GBS, "mfma_TFLOPs": layer_tflops,
                           "mfma_frac": layer_tflops / MFMA_BF16_PEAK_TFLOPS, "binding_frac":
                           (layer_tflops / MFMA_BF16_PEAK_TFLOPS) if bound == "mfma" else layer_gbs / HBM_PEAK_GBS,
                           "algorithmic_bytes": alg["layer_bytes"], "algorithmic_flops": alg["layer_flops"]},
        "stage_ms": stage_ms,
    }
    return rec, inp, rows


def time_decode_block(steps, warmup, pack):
    """One decode step of a whole decoder block at the decode workload's shape (c4: 64 sequences, hidden 2048,
    16 heads, 128 experts) with a full 2048-token key/value cache: extra record, not the headline metric."""
    import torch
    import paper_2201_05596_amd as moe
    from workloads import CONFIGS, make_block_inputs

    cfg, heads, max_len = CONFIGS["c4"], 16, 2048
    bi = make_block_inputs(cfg, heads, max_len, "cuda:0", bias_std=0.0, pos_mode="full")
    lay = bi.layer
    T, d, f, E = cfg.T, cfg.d_model, cfg.d_ffn, cfg.E
    packed_gate = moe.moe_pack_gate(lay.Wg) if pack else None
    flags = (moe.MOE_FLAG_PACKED_WEIGHTS if pack else 0) | (moe.MOE_FLAG_PACKED_GATE if packed_gate is not None else 0)
    shape = moe.make_shape(T, d, f, E, cfg.top_k, cfg.capacity, "bf16", flags=flags)
    block = moe.MoeBlockShape(heads, max_len)
    ws = torch.empty(moe.moe_decode_block_workspace_bytes(shape, block), dtype=torch.uint8, device="cuda:0")
    pk = moe.moe_pack_weights if pack else (lambda w: w)
    weights = dict(ln1_gamma=bi.ln1_gamma, ln1_beta=bi.ln1_beta, Wqkv=bi.Wqkv, bqkv=bi.bqkv, Wo=bi.Wo, bo=bi.bo,
                   ln2_gamma=bi.ln2_gamma, ln2_beta=bi.ln2_beta, Wg=packed_gate if packed_gate is not None else lay.Wg, bg=lay.bg, W1=pk(lay.W1), b1=lay.b1,
                   W2=pk(lay.W2), b2=lay.b2)
    out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda:0")
    logits = torch.empty((T, E), dtype=torch.float32, device="cuda:0")

    def step():
        moe.moe_decode_block_forward(shape, block, weights, lay.x, bi.k_cache, bi.v_cache, bi.pos, out, None, None, logits, ws)

    for _ in range(RAMP_STEPS + warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) * 1e6 / steps
    touched = int(torch.unique(logits.argmax(dim=1)).numel())          # top-1: experts that win at least one token
    cache_bytes = 2 * T * heads * max_len * (d // heads) * 2
    bytes_alg = cache_bytes + (4 * d * d + 4 * d) * 2 + touched * (2 * d * f + f + d) * 2 + 2 * T * d * 2 + d * E * 4
    return {"workload": f"decode block: {describe(cfg)}, {heads} heads, key/value cache of {max_len} positions, all full",
            "us_per_block": us, "tokens_per_s": T / (us * 1e-6), "steps": steps, "algorithmic_bytes": bytes_alg,
            "kv_cache_bytes": cache_bytes, "touched_experts": touched, "hbm_GBps": bytes_alg / (us * 1e-6) / 1e9,
            "hbm_frac": bytes_alg / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}


def time_library_gemm(steps, warmup):
    """Context only, never part of a step: the vendor's bf16 GEMM (torch.matmul) on the dense products whose shapes
    the prefill workloads' FFN halves have, on this GPU and at the same clock state as the timed layers.  What this
    library reaches on a product is the practical mark for a hand-written tile kernel on the same machine."""
    import torch
    out = []
    for M, K, N in ((8192, 4096, 4096), (8192, 1024, 4096), (8192, 4096, 1024), (16384, 4096, 16384)):
        a = torch.randn(M, K, device="cuda:0", dtype=torch.bfloat16)
        b = torch.randn(K, N, device="cuda:0", dtype=torch.bfloat16) * 0.02
        c = torch.empty(M, N, device="cuda:0", dtype=torch.bfloat16)
        for _ in range(RAMP_STEPS + warmup):
            torch.matmul(a, b, out=c)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            torch.matmul(a, b, out=c)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        out.append({"M": M, "K": K, "N": N, "us": us, "TFLOPs": 2.0 * M * K * N / us / 1e6,
                    "mfma_frac": 2.0 * M * K * N / us / 1e6 / MFMA_BF16_PEAK_TFLOPS})
        del a, b, c
    return out


def cpu_baseline(inp, cfg, rows, budget_s=12.0):
    """The oracle as it stands on the host cores, on a bounded sample of the workload: the gate, the dispatch and
    the combine on all tokens, the expert FFNs on every n-th touched expert (by row count, busiest first) until the
    time budget is used; the FFN time is scaled by kept rows / sampled rows, the dense branch is timed in full."""
    import numpy as np
    from oracle import moe_oracle as orc
    from workloads.generate import to_f32_numpy
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    x = to_f32_numpy(inp.x)
    Wg, bg = to_f32_numpy(inp.Wg), to_f32_numpy(inp.bg)
    t0 = time.perf_counter()
    r = orc.gate(orc.gate_logits(x, Wg, bg), cfg.top_k, cfg.capacity)
    xe = orc.dispatch(x, r["slot_token"])
    t_front = time.perf_counter() - t0
    order = [int(e) for e in np.argsort(-r["expert_rows"], kind="stable") if r["expert_rows"][e] > 0]
    stride = max(1, len(order) // 8)
    ye = np.zeros((cfg.E, cfg.capacity, cfg.d_model))
    t_ffn, sampled_rows, sampled = 0.0, 0, []
    for e in order[::stride] + [e for i, e in enumerate(order) if i % stride]:
        if t_ffn > budget_s and sampled:
            break
        n = int(r["expert_rows"][e])
        w = [to_f32_numpy(t[e]) for t in (inp.W1, inp.b1, inp.W2, inp.b2)]       # widening is not timed
        t0 = time.perf_counter()
        ye[e, :n] = orc.ffn(xe[e, :n], *w)
        t_ffn += time.perf_counter() - t0
        sampled_rows += n
        sampled.append(e)
    kept = int(r["expert_rows"].sum())
    t0 = time.perf_counter()
    dense = None
    if cfg.residual:
        dense = orc.ffn(x, *[to_f32_numpy(t) for t in (inp.Wd1, inp.bd1, inp.Wd2, inp.bd2)])
    orc.combine(ye, r["expert_idx"], r["slot_idx"], r["gate_w"], dense)
    t_back = time.perf_counter() - t0
    total = t_front + t_ffn * kept / max(sampled_rows, 1) + t_back
    return {"value": cfg.T / total, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{cfg.name}: gate, dispatch, combine{' and dense branch' if cfg.residual else ''} on all {cfg.T} "
                      f"tokens ({t_front + t_back:.2f} s); expert FFNs of {len(sampled)} of {len(order)} touched experts "
                      f"= {sampled_rows} of {kept} kept rows ({t_ffn:.2f} s), scaled by rows to {total:.2f} s per step; "
                      f"fp64 NumPy"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c5", help="headline workload")
    ap.add_argument("--only", action="store_true", help="time the headline workload only (no sub-records)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain-weights", action="store_true",
                    help="hand the plain [E,d,f] / [E,f,d] weights to every call instead of packing them once")
    ap.add_argument("--capacity-factor", type=float, default=None,
                    help="headline workload with another capacity factor (capacity is an input of the library)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="after the timed region, run one plain device copy of this many MiB (a kernel of known "
                         "traffic that scales the FETCH_SIZE / WRITE_SIZE counters in rocprofv3 --pmc runs)")
    ap.add_argument("--decode-block", action="store_true",
                    help="with --only: time the decode block (extras.decode_block_c4) as well")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor library's bf16 GEMM on the prefill workloads' dense product shapes "
                         "(extras.library_gemm: context for the tiled kernel's rate, not part of any step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    from workloads import CONFIGS

    head_cfg = CONFIGS[args.config]
    if args.capacity_factor is not None:
        head_cfg = head_cfg.scaled(name=f"{head_cfg.name}-cf{args.capacity_factor}", capacity_factor=args.capacity_factor)

    configs = {}
    if not args.only:
        for name in ALL_CONFIGS:
            if name == head_cfg.name:
                continue
            rec, inp, _ = time_config(CONFIGS[name], SUB_STEPS, args.warmup, not args.plain_weights)
            configs[name] = rec
            del inp
            torch.cuda.empty_cache()
        extras = {"decode_block_c4": time_decode_block(SUB_STEPS, args.warmup, not args.plain_weights)}
        torch.cuda.empty_cache()
    else:
        extras = {}
        if args.decode_block:
            extras["decode_block_c4"] = time_decode_block(SUB_STEPS, args.warmup, not args.plain_weights)
            torch.cuda.empty_cache()
    head, inp, rows = time_config(head_cfg, args.steps, args.warmup, not args.plain_weights)
    configs[head_cfg.name] = head

    if args.library_gemm:
        extras["library_gemm"] = time_library_gemm(SUB_STEPS, args.warmup)
    if args.calibration_copy_mib > 0:
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "MoE-layer tokens/s + us/layer at 1 GPU; % HBM roofline (decode) / % MFMA (prefill)",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_ramp_steps": RAMP_STEPS,
        "ms_per_step": head["us_per_layer"] * 1e-3, "us_per_layer": head["us_per_layer"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head_cfg.dtype, "data": "synthetic",
        "config": {"workload": head["workload"], "weights": head["weights"], "kept_rows": head["kept_rows"], "touched_experts": head["touched_experts"]},
        "roofline": head["roofline"],
        "layer_roofline": head["layer_roofline"],
        "stage_ms": head["stage_ms"], "expert_rows": head["expert_rows"],
        "configs": {n: configs[n] for n in ALL_CONFIGS if n in configs},
        "extras": extras,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, head_cfg, rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
