"""Helpers shared by the GPU parity tests: run the HIP path through the binding,
run the oracle on host copies of the very same tensors, compare."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from oracle import moe_oracle as orc
from workloads import LayerInputs, MoEConfig
from workloads.generate import to_f32_numpy

TOL = {"f32": 1e-4, "bf16": 1.5e-2}        # max|delta| <= TOL * max|ref|
GATE_W_ATOL = 1e-6
LOGIT_RTOL = 1e-5                          # max|delta l| <= LOGIT_RTOL * max|l|


def amd():
    import paper_2201_05596_amd as m
    return m


class LazyHost:
    """Indexable view of a [E, ...] device tensor that widens one expert at a time to a host float32
    array, so that the oracle never needs a full host copy of the expert weights."""

    def __init__(self, t: torch.Tensor):
        self.t = t

    def __getitem__(self, e):
        return to_f32_numpy(self.t[int(e)])


_PER_EXPERT = ("W1", "b1", "W2", "b2")


def host(inp: LayerInputs, lazy_experts: bool = False) -> Dict[str, Optional[np.ndarray]]:
    out = {}
    for k, v in inp.tensors().items():
        out[k] = LazyHost(v) if (lazy_experts and k in _PER_EXPERT) else to_f32_numpy(v)
    return out


CANARY_ROWS = 16
CANARY = 12345.0                            # exactly representable in bf16 and fp32


def gpu_forward(inp: LayerInputs, capacity: Optional[int] = None, pack: bool = False) -> Dict[str, torch.Tensor]:
    """One moe_layer_forward call.  The output buffer sits between two bands of canary rows, which
    must come back untouched (a write past either end of `out` shows here)."""
    m = amd()
    cfg = inp.cfg
    C = cfg.capacity if capacity is None else capacity
    layer = m.MoELayer(cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, C, cfg.dtype, inp.Wg, inp.bg, inp.W1, inp.b1,
                       inp.W2, inp.b2, inp.Wd1, inp.bd1, inp.Wd2, inp.bd2, pack_weights=pack)
    padded = torch.full((cfg.T + 2 * CANARY_ROWS, cfg.d_model), CANARY, dtype=layer.out.dtype, device=layer.out.device)
    layer.out = padded[CANARY_ROWS:CANARY_ROWS + cfg.T]
    out = layer(inp.x)
    torch.cuda.synchronize()
    assert bool((padded[:CANARY_ROWS] == CANARY).all()), "write in front of out"
    assert bool((padded[CANARY_ROWS + cfg.T:] == CANARY).all()), "write behind out"
    res = dict(layer.routing)
    res["out"] = out
    return res


def gpu_route(logits: torch.Tensor, k: int, C: int) -> Dict[str, torch.Tensor]:
    """moe_gate with x == NULL: routing from given fp32 logits."""
    m = amd()
    T, E = logits.shape
    dev = logits.device
    shape = m.make_shape(T, 8, 8, E, k, C, "bf16")
    ws = m.alloc_workspace(shape, dev)
    i32 = torch.int32
    r = dict(expert_idx=torch.full((T, k), -7, dtype=i32, device=dev),
             slot_idx=torch.full((T, k), -7, dtype=i32, device=dev),
             gate_w=torch.full((T, k), -7.0, dtype=torch.float32, device=dev),
             expert_rows=torch.full((E,), -7, dtype=i32, device=dev),
             slot_token=torch.full((E, C), -7, dtype=i32, device=dev))
    m.moe_gate(shape, None, None, None, logits, r["expert_idx"], r["slot_idx"], r["gate_w"], r["expert_rows"],
               r["slot_token"], ws)
    torch.cuda.synchronize()
    return r


def assert_routing_equal(gpu: Dict[str, torch.Tensor], ref: Dict[str, np.ndarray]) -> None:
    for name in ("expert_idx", "slot_idx", "expert_rows", "slot_token"):
        g = gpu[name].cpu().numpy()
        assert g.shape == ref[name].shape, name
        assert np.array_equal(g, ref[name]), f"{name} differs at {np.argwhere(g != ref[name])[:5].tolist()}"
    gw = gpu["gate_w"].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(gw - ref["gate_w"])) <= GATE_W_ATOL


def assert_close(gpu_out: torch.Tensor, ref: np.ndarray, dtype: str, what: str = "out") -> float:
    g = gpu_out.detach().to("cpu").to(torch.float64).numpy()
    scale = float(np.max(np.abs(ref)))
    err = float(np.max(np.abs(g - ref)))
    assert np.all(np.isfinite(g)), f"{what}: non-finite values"
    assert err <= TOL[dtype] * scale, f"{what}: max|delta|={err:.3e} > {TOL[dtype]:.1e} * {scale:.3e}"
    return err / scale if scale > 0 else 0.0


def check_layer(inp: LayerInputs, capacity: Optional[int] = None, lazy_experts: bool = False,
                packed_too: Optional[bool] = None) -> Dict[str, float]:
    """Full-layer parity: logits within tolerance of the oracle's own; then the
    oracle evaluates the rest of the layer on the GPU's fp32 logits, routing must
    match bit for bit and the output within the dtype's tolerance.  bf16 layers
    run a second time on packed weights (moe_pack_weights) against the same
    oracle result: the gate does not depend on the weights' layout."""
    cfg = inp.cfg
    C = cfg.capacity if capacity is None else capacity
    if packed_too is None:
        packed_too = cfg.dtype == "bf16"
    res = gpu_forward(inp, C)
    h = host(inp, lazy_experts)
    own = orc.gate_logits(h["x"], h["Wg"], h.get("bg"))
    gl = res["logits"].cpu().numpy()
    lerr = float(np.max(np.abs(gl.astype(np.float64) - own)))
    assert lerr <= LOGIT_RTOL * float(np.max(np.abs(own))), f"logits off by {lerr:.3e}"
    ref = orc.moe_layer_forward(h["x"], h["Wg"], h.get("bg"), h["W1"], h["b1"], h["W2"], h["b2"], cfg.top_k, C,
                                Wd1=h.get("Wd1"), bd1=h.get("bd1"), Wd2=h.get("Wd2"), bd2=h.get("bd2"), logits=gl)
    assert_routing_equal(res, ref)
    rel = assert_close(res["out"], ref["out"], cfg.dtype)
    runs = [res]
    rel_packed = None
    if packed_too:
        resp = gpu_forward(inp, C, pack=True)
        assert torch.equal(resp["logits"], res["logits"])
        assert_routing_equal(resp, ref)
        rel_packed = assert_close(resp["out"], ref["out"], cfg.dtype, "out (packed weights)")
        runs.append(resp)
    if not cfg.residual:
        dropped = np.all(ref["slot_idx"] < 0, axis=1)
        if dropped.any():
            for r in runs:
                go = r["out"].cpu().to(torch.float32).numpy()
                assert np.all(go[dropped] == 0.0), "fully dropped tokens must be exactly zero"
    own_route = orc.gate(own, cfg.top_k, C)
    flips = int(np.sum(np.any(own_route["expert_idx"] != ref["expert_idx"], axis=1)))
    return {"rel_err": rel, "rel_err_packed": rel_packed, "logit_err": lerr, "route_flips_vs_own_logits": flips,
            "kept": int(ref["expert_rows"].sum()), "dropped_tokens": int(np.all(ref["slot_idx"] < 0, axis=1).sum())}
