"""CPU oracle for the forward pass of one Mixture-of-Experts layer.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 NumPy statement of what
the layer computes, used to check the HIP kernels.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import it; the product path never
does.  It shares no code with the HIP path and imports nothing from it.

What is computed (paper Sec. 5.4: the MoE-related computation is a gating
function producing one-hot assignments, a sparse einsum that sorts tokens by
expert, the expert FFNs, and a final einsum that scales and re-sorts tokens
back; Sec. 3.1: top-1 gating, top-2 also tried; Sec. 4.1.1: Residual-MoE adds a
fixed dense MLP branch to the chosen expert's output).  The paper's optimised
kernels reach exactly this result, so the oracle is the definition itself:
``moe_layer_einsum`` builds the dense one-hot tensors and calls einsum
literally; ``moe_layer_forward`` evaluates the same sums over the non-zero
entries only, so that it finishes on the larger configurations.

Precision: gate logits are formed in fp64 and rounded to fp32 (the layer's
routing is defined on fp32 logits); argmax decisions are taken on those fp32
logits; everything else is fp64.  bf16 inputs arrive already widened (exactly)
to float32/float64 arrays; no intermediate bf16 rounding is emulated.

Readings where the paper is silent (each also listed in the design notes):
  * gate = softmax over all E logits, no noise (Sec. 5.4: the gate's logits
    are turned into probabilities before they scale the expert output).
  * top-k by logit value, lowest expert index wins ties.
  * top-1 weight = softmax probability of the chosen expert; top-2 weights =
    the two chosen probabilities renormalised to sum to one, before any drop.
  * capacity: position of a token within its expert = exclusive running count
    in token order (the cumsum of Sec. 5.4); all first choices rank ahead of
    all second choices of the same expert; a choice whose position is >= C is
    dropped and contributes zero.
  * expert FFN = gelu_tanh(x W1 + b1) W2 + b2.
  * Residual-MoE output = dense_mlp(x) + gate_weight * expert(x), plain sum.

Pins (see tests/test_oracle_*.py): hand-worked 4-token routing examples,
closed forms (top-2 weight = logistic of the logit gap), invariants of the
slot assignment, library routines on special cases (E=1 layer == dense FFN via
torch fp64; softmax/topk/gelu against torch), and an independent pure-Python
loop implementation on tiny inputs.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

_F64 = np.float64


# --------------------------------------------------------------------------- gate

def gate_logits(x: np.ndarray, Wg: np.ndarray, bg: Optional[np.ndarray] = None) -> np.ndarray:
    """l[t,e] = bg[e] + sum_i x[t,i] Wg[i,e]  (Sec. 3.1 gating function; Sec. 5.4
    first component).  fp64 accumulation, result rounded to fp32."""
    l = np.asarray(x, _F64) @ np.asarray(Wg, _F64)
    if bg is not None:
        l = l + np.asarray(bg, _F64)[None, :]
    return l.astype(np.float32)


def softmax(logits: np.ndarray) -> np.ndarray:
    """p[t,:] = exp(l - max) / sum exp(l - max), fp64, from fp32 logits."""
    l = np.asarray(logits, _F64)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def top_k_experts(logits: np.ndarray, k: int) -> np.ndarray:
    """The k experts with the k highest logits per token (Sec. 5.4 top-k),
    chosen one after another; ``np.argmax`` returns the first (lowest-index)
    maximum, which is the tie rule."""
    l = np.array(logits, dtype=np.float32, copy=True)
    T, E = l.shape
    assert 1 <= k <= E
    idx = np.empty((T, k), dtype=np.int32)
    rows = np.arange(T)
    for j in range(k):
        e = np.argmax(l, axis=1)
        idx[:, j] = e
        l[rows, e] = -np.inf
    return idx


def gate_weights(logits: np.ndarray, expert_idx: np.ndarray) -> np.ndarray:
    """Top-1: the chosen expert's softmax probability.  Top-k (k>=2): the chosen
    probabilities divided by their sum."""
    p = softmax(logits)
    T, k = expert_idx.shape
    g = p[np.arange(T)[:, None], expert_idx]
    if k > 1:
        g = g / g.sum(axis=1, keepdims=True)
    return g


def capacity_slots(expert_idx: np.ndarray, E: int, C: int) -> Dict[str, np.ndarray]:
    """Position of every (token, choice) inside its expert, via one-hot masks and
    an exclusive cumulative sum over tokens (Sec. 5.4 cumsum), then the capacity
    cut.  Choice j of any token ranks after every choice j' < j of all tokens.

    Returns slot_idx [T,k] (-1 = dropped), expert_rows [E], slot_token [E,C]
    (-1 = empty) and loc [T,k] (the untruncated positions)."""
    T, k = expert_idx.shape
    loc = np.empty((T, k), dtype=np.int64)
    offset = np.zeros(E, dtype=np.int64)          # choices of earlier rank come first
    rows_t = np.arange(T)
    for j in range(k):
        mask = np.zeros((T, E), dtype=np.int64)   # one-hot m_j[t,e]
        mask[rows_t, expert_idx[:, j]] = 1
        excl = np.cumsum(mask, axis=0) - mask     # tokens t' < t that chose e
        loc[:, j] = offset[expert_idx[:, j]] + excl[rows_t, expert_idx[:, j]]
        offset = offset + mask.sum(axis=0)
    keep = loc < C
    slot_idx = np.where(keep, loc, -1).astype(np.int32)
    expert_rows = np.zeros(E, dtype=np.int32)
    slot_token = np.full((E, C), -1, dtype=np.int32)
    for j in range(k):
        for t in range(T):
            if keep[t, j]:
                e = expert_idx[t, j]
                slot_token[e, loc[t, j]] = t
                expert_rows[e] += 1
    return {"slot_idx": slot_idx, "expert_rows": expert_rows,
            "slot_token": slot_token, "loc": loc}


def gate(logits: np.ndarray, k: int, C: int) -> Dict[str, np.ndarray]:
    """Routing from given fp32 logits: mapping table, weights, slots."""
    logits = np.asarray(logits, np.float32)
    assert np.all(np.isfinite(logits)), "non-finite gate logits"
    E = logits.shape[1]
    expert_idx = top_k_experts(logits, k)
    out = {"logits": logits, "expert_idx": expert_idx,
           "gate_w": gate_weights(logits, expert_idx)}
    out.update(capacity_slots(expert_idx, E, C))
    return out


# ------------------------------------------------------------------ expert FFN

def gelu_tanh(z: np.ndarray) -> np.ndarray:
    """0.5 z (1 + tanh( sqrt(2/pi) (z + 0.044715 z^3) ))."""
    z = np.asarray(z, _F64)
    return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))


def ffn(x_rows: np.ndarray, W1: np.ndarray, b1: Optional[np.ndarray],
        W2: np.ndarray, b2: Optional[np.ndarray]) -> np.ndarray:
    """gelu_tanh(x W1 + b1) W2 + b2 for a block of rows, fp64.  Used for one
    expert (Sec. 3.1: an expert is an FFN of the base model's size) and for the
    dense branch of Residual-MoE (Sec. 4.1.1)."""
    h = np.asarray(x_rows, _F64) @ np.asarray(W1, _F64)
    if b1 is not None:
        h = h + np.asarray(b1, _F64)[None, :]
    y = gelu_tanh(h) @ np.asarray(W2, _F64)
    if b2 is not None:
        y = y + np.asarray(b2, _F64)[None, :]
    return y


# ------------------------------------------------- dispatch / experts / combine

def dispatch(x: np.ndarray, slot_token: np.ndarray) -> np.ndarray:
    """xe[e,c,:] = x[t,:] where token t holds slot c of expert e; empty slots are
    zero (what the one-hot einsum "tec,tm->ecm" yields; Sec. 5.4 second
    component)."""
    E, C = slot_token.shape
    x = np.asarray(x, _F64)
    xe = np.zeros((E, C, x.shape[1]), dtype=_F64)
    for e in range(E):
        for c in range(C):
            t = slot_token[e, c]
            if t >= 0:
                xe[e, c, :] = x[t, :]
    return xe


def expert_ffn(xe: np.ndarray, expert_rows: np.ndarray, W1, b1, W2, b2) -> np.ndarray:
    """ye[e,c,:] = FFN_e(xe[e,c,:]) for c < expert_rows[e]; other rows zero."""
    E, C, d = xe.shape
    ye = np.zeros((E, C, d), dtype=_F64)
    for e in range(E):
        r = int(expert_rows[e])
        if r > 0:
            ye[e, :r, :] = ffn(xe[e, :r, :], W1[e], None if b1 is None else b1[e],
                               W2[e], None if b2 is None else b2[e])
    return ye


def combine(ye: np.ndarray, expert_idx: np.ndarray, slot_idx: np.ndarray,
            gate_w: np.ndarray, addend: Optional[np.ndarray] = None) -> np.ndarray:
    """out[t,:] = sum_j [slot_j(t) >= 0] g_j(t) ye[e_j(t), slot_j(t), :] (+ addend)
    (Sec. 5.4 third component: scale by the gate probability and restore token
    order).  A token all of whose choices were dropped gets zero."""
    T, k = expert_idx.shape
    out = np.zeros((T, ye.shape[2]), dtype=_F64)
    for t in range(T):
        for j in range(k):
            s = slot_idx[t, j]
            if s >= 0:
                out[t, :] += gate_w[t, j] * ye[expert_idx[t, j], s, :]
    if addend is not None:
        out = out + np.asarray(addend, _F64)
    return out


# ---------------------------------------------------------------- whole layer

def moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, top_k: int, capacity: int,
                      Wd1=None, bd1=None, Wd2=None, bd2=None,
                      logits: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """One MoE layer: gate -> capacity -> dispatch -> expert FFNs -> combine, plus
    the dense branch when Wd1/Wd2 are given (Residual-MoE, Sec. 4.1.1).  When
    ``logits`` is given it replaces x.Wg+bg (used to evaluate the rest of the
    layer on the very logits another implementation produced)."""
    if logits is None:
        logits = gate_logits(x, Wg, bg)
    r = gate(logits, top_k, capacity)
    xe = dispatch(x, r["slot_token"])
    ye = expert_ffn(xe, r["expert_rows"], W1, b1, W2, b2)
    dense = None
    if Wd1 is not None:
        dense = ffn(x, Wd1, bd1, Wd2, bd2)
    out = combine(ye, r["expert_idx"], r["slot_idx"], r["gate_w"], dense)
    r.update({"xe": xe, "ye": ye, "out": out})
    if dense is not None:
        r["dense"] = dense
    return r


def moe_layer_einsum(x, Wg, bg, W1, b1, W2, b2, top_k: int, capacity: int,
                     Wd1=None, bd1=None, Wd2=None, bd2=None) -> np.ndarray:
    """The same layer written as the sparse-einsum formulation the paper starts
    from (Sec. 5.4): dense one-hot dispatch mask D[t,e,c] and combine weights
    G[t,e,c], einsum "tec,tm->ecm", every expert applied to all C rows, einsum
    "tec,ecm->tm".  Cost grows with T*E*C*d, so small inputs only."""
    x64 = np.asarray(x, _F64)
    logits = gate_logits(x, Wg, bg)
    T, E = logits.shape
    C = capacity
    expert_idx = top_k_experts(logits, top_k)
    g = gate_weights(logits, expert_idx)
    D = np.zeros((T, E, C), dtype=_F64)
    G = np.zeros((T, E, C), dtype=_F64)
    count = np.zeros(E, dtype=np.int64)              # running per-expert position
    for j in range(top_k):                           # earlier choices rank first
        for t in range(T):
            e = expert_idx[t, j]
            if count[e] < C:
                D[t, e, count[e]] = 1.0
                G[t, e, count[e]] = g[t, j]
            count[e] += 1
    xe = np.einsum("tec,tm->ecm", D, x64)
    ye = np.stack([ffn(xe[e], W1[e], None if b1 is None else b1[e],
                       W2[e], None if b2 is None else b2[e]) for e in range(E)])
    out = np.einsum("tec,ecm->tm", G, ye)
    if Wd1 is not None:
        out = out + ffn(x64, Wd1, bd1, Wd2, bd2)
    return out
