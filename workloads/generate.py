"""Seeded input generator shared by the oracle's callers and the HIP path's callers.

Recipe (stand-in for the paper's training data and trained weights, which are
not needed to exercise the layer): x ~ N(0,1); gate weights Wg ~ N(0,0.02^2)
kept in fp32; expert and dense-branch weights ~ N(0,0.02^2); biases zero unless
``bias_std`` is given; optional Zipf gate bias bg[e] = s*ln(1/(e+1)).  For bf16
configs x and the FFN weights are rounded to bf16 once, here, so both sides
consume identical bits.  Tensors are drawn from one ``torch.Generator`` in the
fixed order x, Wg, W1, W2, [Wd1, Wd2], [b1, b2, bd1, bd2].

Nothing in this file computes any part of the MoE layer.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from .configs import MoEConfig

_WEIGHT_STD = 0.02


@dataclass
class LayerInputs:
    cfg: MoEConfig
    x: torch.Tensor                      # [T, d]      f32 | bf16
    Wg: torch.Tensor                     # [d, E]      f32
    bg: Optional[torch.Tensor]           # [E]         f32 or None
    W1: torch.Tensor                     # [E, d, f]
    b1: torch.Tensor                     # [E, f]
    W2: torch.Tensor                     # [E, f, d]
    b2: torch.Tensor                     # [E, d]
    Wd1: Optional[torch.Tensor] = None   # [d, f]      residual branch only
    bd1: Optional[torch.Tensor] = None   # [f]
    Wd2: Optional[torch.Tensor] = None   # [f, d]
    bd2: Optional[torch.Tensor] = None   # [d]

    def tensors(self):
        return {k: v for k, v in self.__dict__.items() if isinstance(v, torch.Tensor)}


def _normal(shape, std, dtype, device, gen):
    """N(0, std^2) drawn slice by slice along dim 0 so that no fp32 temporary
    larger than one slice is ever alive (config c5 holds 17 GB of weights)."""
    out = torch.empty(shape, dtype=dtype, device=device)
    if out.dim() >= 3:
        for i in range(shape[0]):
            out[i].normal_(0.0, std, generator=gen)
    else:
        out.normal_(0.0, std, generator=gen)
    return out


def make_inputs(cfg: MoEConfig, device: str = "cpu", bias_std: float = 0.0) -> LayerInputs:
    """Draw every tensor of one layer.  The stream depends on (seed, device type,
    shapes); a CPU draw and a GPU draw of the same config differ, which is fine
    because each test hands the *same* tensors to both sides."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    wdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    T, d, f, E = cfg.T, cfg.d_model, cfg.d_ffn, cfg.E

    x = _normal((T, d), 1.0, wdt, dev, gen)
    Wg = _normal((d, E), _WEIGHT_STD, torch.float32, dev, gen)
    bg = None
    if cfg.gate_bias_zipf is not None:
        e = torch.arange(E, dtype=torch.float64)
        bg = (cfg.gate_bias_zipf * torch.log(1.0 / (e + 1.0))).to(torch.float32).to(dev)
    W1 = _normal((E, d, f), _WEIGHT_STD, wdt, dev, gen)
    W2 = _normal((E, f, d), _WEIGHT_STD, wdt, dev, gen)
    Wd1 = Wd2 = bd1 = bd2 = None
    if cfg.residual:
        Wd1 = _normal((d, f), _WEIGHT_STD, wdt, dev, gen)
        Wd2 = _normal((f, d), _WEIGHT_STD, wdt, dev, gen)
    if bias_std > 0.0:
        b1 = _normal((E, f), bias_std, wdt, dev, gen)
        b2 = _normal((E, d), bias_std, wdt, dev, gen)
        if cfg.residual:
            bd1 = _normal((f,), bias_std, wdt, dev, gen)
            bd2 = _normal((d,), bias_std, wdt, dev, gen)
    else:
        b1 = torch.zeros((E, f), dtype=wdt, device=dev)
        b2 = torch.zeros((E, d), dtype=wdt, device=dev)
        if cfg.residual:
            bd1 = torch.zeros((f,), dtype=wdt, device=dev)
            bd2 = torch.zeros((d,), dtype=wdt, device=dev)
    return LayerInputs(cfg, x, Wg, bg, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2)


@dataclass
class BlockInputs:
    """One decode step of a decoder block: the MoE layer's inputs plus the attention half's."""
    layer: LayerInputs                   # x [T, d] is the block's input; the MoE weights
    n_heads: int
    max_len: int
    ln1_gamma: torch.Tensor              # [d] f32
    ln1_beta: torch.Tensor
    ln2_gamma: torch.Tensor
    ln2_beta: torch.Tensor
    Wqkv: torch.Tensor                   # [d, 3d]
    bqkv: torch.Tensor                   # [3d]
    Wo: torch.Tensor                     # [d, d]
    bo: torch.Tensor                     # [d]
    k_cache: torch.Tensor                # [T, H, max_len, dh]
    v_cache: torch.Tensor
    pos: torch.Tensor                    # [T] int32: cached positions per sequence


def make_block_inputs(cfg: MoEConfig, n_heads: int, max_len: int, device: str = "cpu", bias_std: float = 0.02,
                      pos_mode: str = "mixed") -> BlockInputs:
    """Attention-half tensors around make_inputs(cfg): LayerNorm gains ~ N(1, 0.1^2), shifts ~ N(0, 0.1^2);
    projection weights ~ N(0, 0.02^2) (Wqkv scaled up so that attention is not uniform); caches ~ N(0,1);
    pos: "mixed" = uniform over 0..max_len-1 with the two extremes forced in, "full" = max_len-1 everywhere."""
    layer = make_inputs(cfg, device, bias_std=bias_std)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed + 1000)
    T, d = cfg.T, cfg.d_model
    dh = d // n_heads
    wdt = torch.bfloat16
    f32 = torch.float32
    ln = lambda mean: (mean + 0.1 * torch.randn((d,), generator=gen, device=dev, dtype=f32))
    ln1_gamma, ln1_beta, ln2_gamma, ln2_beta = ln(1.0), ln(0.0), ln(1.0), ln(0.0)
    Wqkv = _normal((d, 3 * d), 4 * _WEIGHT_STD, wdt, dev, gen)
    Wo = _normal((d, d), _WEIGHT_STD, wdt, dev, gen)
    bqkv = _normal((3 * d,), bias_std, wdt, dev, gen) if bias_std > 0 else torch.zeros((3 * d,), dtype=wdt, device=dev)
    bo = _normal((d,), bias_std, wdt, dev, gen) if bias_std > 0 else torch.zeros((d,), dtype=wdt, device=dev)
    k_cache = _normal((T, n_heads, max_len, dh), 1.0, wdt, dev, gen)
    v_cache = _normal((T, n_heads, max_len, dh), 1.0, wdt, dev, gen)
    if pos_mode == "full":
        pos = torch.full((T,), max_len - 1, dtype=torch.int32, device=dev)
    else:
        pos = torch.randint(0, max_len, (T,), generator=gen, device=dev).to(torch.int32)
        pos[0] = 0
        pos[-1] = max_len - 1
    return BlockInputs(layer, n_heads, max_len, ln1_gamma, ln1_beta, ln2_gamma, ln2_beta, Wqkv, bqkv, Wo, bo, k_cache,
                       v_cache, pos)


def make_logits(T: int, E: int, seed: int, kind: str = "normal", device: str = "cpu") -> torch.Tensor:
    """fp32 gate logits for routing-only tests.

    kinds: "normal" (N(0,1)); "ties" (values from a 3-level grid, so equal
    logits abound); "equal" (all zero); "hot" (expert 0 wins every token);
    "zipf" (N(0,1) + 1.5*ln(1/(e+1)))."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    if kind == "normal":
        l = torch.randn((T, E), generator=gen, dtype=torch.float32)
    elif kind == "ties":
        l = torch.randint(0, 3, (T, E), generator=gen).to(torch.float32) * 0.5
    elif kind == "equal":
        l = torch.zeros((T, E), dtype=torch.float32)
    elif kind == "hot":
        l = torch.randn((T, E), generator=gen, dtype=torch.float32)
        l[:, 0] += 100.0
    elif kind == "zipf":
        l = torch.randn((T, E), generator=gen, dtype=torch.float32)
        e = torch.arange(E, dtype=torch.float64)
        l += (1.5 * torch.log(1.0 / (e + 1.0))).to(torch.float32)
    else:
        raise ValueError(kind)
    return l.to(device)


def to_f32_numpy(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """Exact widening of an f32/bf16 tensor to a host float32 array."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float32).numpy()
