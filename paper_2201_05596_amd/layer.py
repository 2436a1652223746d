"""Buffer holder around moe_layer_forward: owns the workspace, the output and the
exported routing tensors so that repeated calls allocate nothing."""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as B


class MoELayer:
    """One MoE layer's weights (device tensors, shaped as in include/moe.h) plus
    preallocated buffers.  ``forward(x)`` enqueues one moe_layer_forward call on
    the current stream and returns the output tensor (reused between calls)."""

    def __init__(self, T: int, d_model: int, d_ffn: int, E: int, top_k: int, capacity: int, dtype,
                 Wg, bg, W1, b1, W2, b2, Wd1=None, bd1=None, Wd2=None, bd2=None, export_routing: bool = True,
                 pack_weights: bool = False):
        residual = Wd1 is not None
        if pack_weights:          # one-time re-tiling; the layer then holds the packed copies only
            W1, W2 = B.moe_pack_weights(W1), B.moe_pack_weights(W2)
            if residual:
                Wd1, Wd2 = B.moe_pack_weights(Wd1), B.moe_pack_weights(Wd2)
        flags = B.MOE_FLAG_PACKED_WEIGHTS if pack_weights else 0
        if pack_weights:
            packed_gate = B.moe_pack_gate(Wg)           # None: shape outside the bf16 gate kernel, Wg stays plain
            if packed_gate is not None:
                Wg, flags = packed_gate, flags | B.MOE_FLAG_PACKED_GATE
        self.shape = B.make_shape(T, d_model, d_ffn, E, top_k, capacity, dtype, residual, flags)
        self.weights = (Wg, bg, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2)
        dev = W1.device
        el = torch.float32 if self.shape.dtype == B.MOE_F32 else torch.bfloat16
        self.ws = B.alloc_workspace(self.shape, dev)
        self.out = torch.empty((T, d_model), dtype=el, device=dev)
        self.routing: Dict[str, Optional[torch.Tensor]] = dict(
            logits=None, expert_idx=None, slot_idx=None, gate_w=None, expert_rows=None, slot_token=None)
        if export_routing:
            i32, f32 = torch.int32, torch.float32
            self.routing = dict(
                logits=torch.empty((T, E), dtype=f32, device=dev),
                expert_idx=torch.empty((T, top_k), dtype=i32, device=dev),
                slot_idx=torch.empty((T, top_k), dtype=i32, device=dev),
                gate_w=torch.empty((T, top_k), dtype=f32, device=dev),
                expert_rows=torch.empty((E,), dtype=i32, device=dev),
                slot_token=torch.empty((E, capacity), dtype=i32, device=dev))

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        r = self.routing
        B.moe_layer_forward(self.shape, x, *self.weights, self.out, r["logits"], r["expert_idx"], r["slot_idx"],
                            r["gate_w"], r["expert_rows"], r["slot_token"], self.ws)
        return self.out

    __call__ = forward
