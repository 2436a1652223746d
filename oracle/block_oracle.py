"""CPU oracle for one decode step of a transformer block whose feed-forward part is an MoE layer.

TEST INFRASTRUCTURE ONLY (see moe_oracle.py): plain fp64 NumPy, shares no code with the HIP path; only tests, the
smoke check and the benchmark's cpu_baseline leg may import it.

What is computed.  The paper's models are GPT-like decoders (Sec. 3.1: 24 layers, hidden size 1024/2048, 16 heads;
experts on every other feed-forward layer); at inference the non-expert part of a layer runs beside the MoE kernels
(Sec. 5.4, first paragraph).  One block, one new token per sequence, with a key/value cache:

    a   = LayerNorm(x; g1, b1)
    q,k,v = split(a Wqkv + bqkv)                       per head h: columns h*dh .. (h+1)*dh of each third
    K_b = [cache_k[b, :, :pos[b]] ; k_b],  V_b likewise     (the new token's key/value join the cached ones)
    s   = q_b,h . K_b,h^T / sqrt(dh);  p = softmax(s);  o_b,h = p V_b,h      (the newest token sees all earlier ones)
    x1  = x + concat_h(o) Wo + bo
    out = x1 + MoE(LayerNorm(x1; g2, b2))              the MoE layer of moe_oracle.moe_layer_forward

Readings where the paper is silent: pre-LayerNorm residual blocks with eps = 1e-5 (GPT-3-style decoder, whose
hyper-parameters Sec. 3.2 says were followed), biases on every projection, scaled dot-product attention with
1/sqrt(dh), no dropout at inference.

Pins (tests/test_oracle_block.py): LayerNorm and attention against torch's fp64 library routines; a decode step
with a cache equals the last row of full causal attention over the whole sequence; closed forms (equal scores give
the mean of the values, a one-token context returns its value, softmax shift invariance); a block whose attention
and MoE weights are zero returns x.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import moe_oracle as moe

_F64 = np.float64


def layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """(x - mean) / sqrt(var + eps) * gamma + beta over the last axis, biased variance."""
    x = np.asarray(x, _F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, _F64) + np.asarray(beta, _F64)


def linear(x: np.ndarray, W: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    y = np.asarray(x, _F64) @ np.asarray(W, _F64)
    return y if b is None else y + np.asarray(b, _F64)


def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query vector q [dh] over keys K [n, dh] and values V [n, dh]: softmax(q K^T / sqrt(dh)) V."""
    q, K, V = np.asarray(q, _F64), np.asarray(K, _F64), np.asarray(V, _F64)
    s = K @ q / np.sqrt(q.shape[0])
    p = np.exp(s - s.max())
    p = p / p.sum()
    return p @ V


def decode_attention(q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, cache_k: np.ndarray, cache_v: np.ndarray,
                     pos: np.ndarray) -> np.ndarray:
    """q, k_new, v_new [B, H, dh]; caches [B, H, Lmax, dh] of which the first pos[b] positions are valid.
    Returns o [B, H, dh]: the new token attends to its sequence's cached positions and to itself."""
    B, H, dh = q.shape
    o = np.zeros((B, H, dh), dtype=_F64)
    for b in range(B):
        n = int(pos[b])
        for h in range(H):
            K = np.concatenate([np.asarray(cache_k[b, h, :n], _F64), np.asarray(k_new[b, h], _F64)[None, :]], axis=0)
            V = np.concatenate([np.asarray(cache_v[b, h, :n], _F64), np.asarray(v_new[b, h], _F64)[None, :]], axis=0)
            o[b, h] = attend(q[b, h], K, V)
    return o


def attention_half(x, g1, be1, Wqkv, bqkv, cache_k, cache_v, pos, Wo, bo, n_heads: int) -> Dict[str, np.ndarray]:
    """x1 = x + Attention(LayerNorm(x)) for one new token per sequence; also the new key/value rows."""
    x = np.asarray(x, _F64)
    B, d = x.shape
    dh = d // n_heads
    a = layer_norm(x, g1, be1)
    qkv = linear(a, Wqkv, bqkv)
    q = qkv[:, :d].reshape(B, n_heads, dh)
    k = qkv[:, d:2 * d].reshape(B, n_heads, dh)
    v = qkv[:, 2 * d:].reshape(B, n_heads, dh)
    o = decode_attention(q, k, v, cache_k, cache_v, pos)
    x1 = x + linear(o.reshape(B, d), Wo, bo)
    return {"x1": x1, "k_new": k, "v_new": v, "attn": o.reshape(B, d)}


def moe_half(x1, g2, be2, Wg, bg, W1, b1, W2, b2, top_k: int, capacity: int, Wd1=None, bd1=None, Wd2=None, bd2=None,
             moe_input: Optional[np.ndarray] = None, logits: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """out = x1 + MoE(LayerNorm(x1)).  `moe_input` / `logits` replace LayerNorm(x1) / the gate logits (to evaluate
    the rest on the very values another implementation produced, as moe_oracle.moe_layer_forward allows)."""
    x1 = np.asarray(x1, _F64)
    xn = layer_norm(x1, g2, be2) if moe_input is None else np.asarray(moe_input, _F64)
    r = moe.moe_layer_forward(xn, Wg, bg, W1, b1, W2, b2, top_k, capacity, Wd1=Wd1, bd1=bd1, Wd2=Wd2, bd2=bd2,
                              logits=logits)
    r["moe_input"] = xn
    r["moe_out"] = r["out"]
    r["out"] = x1 + r["moe_out"]
    return r


def decode_block(x, g1, be1, Wqkv, bqkv, cache_k, cache_v, pos, Wo, bo, n_heads, g2, be2, Wg, bg, W1, b1, W2, b2,
                 top_k, capacity, Wd1=None, bd1=None, Wd2=None, bd2=None) -> Dict[str, np.ndarray]:
    """The whole block for one decode step."""
    a = attention_half(x, g1, be1, Wqkv, bqkv, cache_k, cache_v, pos, Wo, bo, n_heads)
    r = moe_half(a["x1"], g2, be2, Wg, bg, W1, b1, W2, b2, top_k, capacity, Wd1, bd1, Wd2, bd2)
    r.update({"x1": a["x1"], "k_new": a["k_new"], "v_new": a["v_new"], "attn": a["attn"]})
    return r
