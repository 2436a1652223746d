"""Times the stand-alone entry points of the library (the layer as four calls instead of one) on one workload.

    python -m paper_2201_05596_amd.bench_entry_points [--config c2] [--steps 30] [--warmup 5]

bench.py measures moe_layer_forward, where dispatch and (for top-1) combine are fused into the expert GEMMs and
never run as kernels of their own.  This script times moe_gate, moe_dispatch, moe_expert_ffn and moe_combine one
by one (torch.cuda.Event on the stream the binding launches on, inputs resident in HBM) and sets each against
its own bound: the data-layout transforms and the gate against the bytes they must move, the FFN as in bench.py.
Prints one JSON object per entry point.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def _time(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / steps          # microseconds


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    import paper_2201_05596_amd as moe
    from workloads import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    dev = "cuda:0"
    inp = make_inputs(cfg, dev)
    T, d, f, E, k, C = cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, cfg.capacity
    eb = 4 if cfg.dtype == "f32" else 2
    el = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    shape = moe.make_shape(T, d, f, E, k, C, cfg.dtype, residual=cfg.residual)
    ws = moe.alloc_workspace(shape, dev)
    i32 = torch.int32
    logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    expert_idx = torch.empty((T, k), dtype=i32, device=dev)
    slot_idx = torch.empty((T, k), dtype=i32, device=dev)
    gate_w = torch.empty((T, k), dtype=torch.float32, device=dev)
    rows = torch.empty((E,), dtype=i32, device=dev)
    slot_token = torch.empty((E, C), dtype=i32, device=dev)
    xe = torch.zeros((E, C, d), dtype=el, device=dev)
    ye = torch.zeros((E, C, d), dtype=el, device=dev)
    out = torch.empty((T, d), dtype=el, device=dev)

    def gate():
        moe.moe_gate(shape, inp.x, inp.Wg, inp.bg, logits, expert_idx, slot_idx, gate_w, rows, slot_token, ws)

    def dispatch():
        moe.moe_dispatch(shape, inp.x, slot_token, rows, xe)

    def ffn():
        moe.moe_expert_ffn(shape, xe, rows, inp.W1, inp.b1, inp.W2, inp.b2, ye, ws)

    def combine():
        moe.moe_combine(shape, ye, expert_idx, slot_idx, gate_w, None, out)

    gate()
    torch.cuda.synchronize()
    r = rows.cpu().numpy()
    kept, touched = int(r.sum()), int((r > 0).sum())
    kept_pairs = int((slot_idx.cpu().numpy() >= 0).sum())
    bytes_of = {
        # x and Wg in, logits and the tables out
        "moe_gate": T * d * eb + d * E * 4 + T * E * 4 + 3 * T * k * 4 + E * C * 4,
        # kept rows read and written once, the table read
        "moe_dispatch": 2 * kept * d * eb + E * C * 4,
        # both weight matrices of the touched experts once, rows in, h out and in again, rows out
        "moe_expert_ffn": touched * (2 * d * f + f + d) * eb + 2 * kept * d * eb + 2 * kept * f * eb,
        # kept expert rows in, every token row out
        "moe_combine": kept_pairs * d * eb + T * d * eb + 3 * T * k * 4,
    }
    for name, fn in (("moe_gate", gate), ("moe_dispatch", dispatch), ("moe_expert_ffn", ffn), ("moe_combine", combine)):
        us = _time(fn, args.steps, args.warmup)
        gbs = bytes_of[name] / (us * 1e-6) / 1e9
        print(json.dumps({"entry_point": name, "workload": cfg.name, "us": round(us, 2), "algorithmic_bytes": bytes_of[name],
                          "achieved_GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
                          "kept_rows": kept, "touched_experts": touched}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
