"""Shapes of the synthetic MoE layers.

The shapes follow the model family of the paper's Table 1 (hidden sizes 1024,
2048 and 4096; 128 experts for Standard-MoE, 32/64 for PR-MoE) and Sec. 3.1
(top-1 gating, an MoE FFN on every other layer).  The paper gives neither the
FFN width nor the capacity formula; d_ffn = 4*d_model and
C = ceil(cf * k * T / E) are this build's readings.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional


def capacity_from_factor(T: int, E: int, top_k: int, capacity_factor: float) -> int:
    """Rows per expert for a capacity factor: ceil(cf * k * T / E), at least 1.

    With cf = 1 and perfectly uniform routing nothing is dropped for any k.
    The library itself only ever sees the resulting integer.
    """
    return max(1, int(math.ceil(capacity_factor * top_k * T / E - 1e-9)))


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int                 # tokens (batch * sequence, flattened)
    d_model: int
    d_ffn: int
    E: int                 # experts resident on the GPU
    top_k: int             # 1 or 2
    capacity_factor: float
    dtype: str             # "f32" or "bf16": x, expert/dense weights, out
    residual: bool         # Residual-MoE: out = dense MLP(x) + gate * expert(x)
    seed: int
    gate_bias_zipf: Optional[float] = None   # bg[e] = s * ln(1/(e+1)) when set

    @property
    def capacity(self) -> int:
        return capacity_from_factor(self.T, self.E, self.top_k, self.capacity_factor)

    def scaled(self, **kw) -> "MoEConfig":
        """A copy with some fields replaced (reduced-size parity cases)."""
        return replace(self, **kw)


CONFIGS: Dict[str, MoEConfig] = {
    # Tiny Standard-MoE, fp32 throughout.
    "c1": MoEConfig("c1", T=256, d_model=64, d_ffn=256, E=8, top_k=1,
                    capacity_factor=1.0, dtype="f32", residual=False, seed=0),
    # 350M+MoE-128 shaped prefill batch (8 sequences x 1024 tokens).
    "c2": MoEConfig("c2", T=8192, d_model=1024, d_ffn=4096, E=128, top_k=1,
                    capacity_factor=1.0, dtype="bf16", residual=False, seed=1),
    # PR-MoE layer pair: shallow layer 32 experts, deep layer 64 experts.
    "c3a": MoEConfig("c3a", T=8192, d_model=1024, d_ffn=4096, E=32, top_k=1,
                     capacity_factor=1.0, dtype="bf16", residual=True, seed=2),
    "c3b": MoEConfig("c3b", T=8192, d_model=1024, d_ffn=4096, E=64, top_k=1,
                     capacity_factor=1.0, dtype="bf16", residual=True, seed=2),
    # 1.3B+MoE-128 shaped decode step (64 sequences x 1 new token).
    "c4": MoEConfig("c4", T=64, d_model=2048, d_ffn=8192, E=128, top_k=1,
                    capacity_factor=2.0, dtype="bf16", residual=False, seed=3),
    # One GPU's share of a 6.7B-class expert-parallel model, skewed top-2.
    "c5": MoEConfig("c5", T=16384, d_model=4096, d_ffn=16384, E=64, top_k=2,
                    capacity_factor=1.25, dtype="bf16", residual=False, seed=4,
                    gate_bias_zipf=1.5),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]
