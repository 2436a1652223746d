"""Pure-Python loop implementation of the MoE layer for tiny inputs.

Written independently of oracle/moe_oracle.py (scalar loops, sequential
per-expert counters, math.* functions, no NumPy linear algebra) so that the two
can be checked against each other.  Follows paper Sec. 5.4 (gate, sort by
expert, scale and re-sort) and Sec. 4.1.1 (dense branch added)."""
import math


def logits_loops(x, Wg, bg):
    T, d, E = len(x), len(x[0]), len(Wg[0])
    out = []
    for t in range(T):
        row = []
        for e in range(E):
            s = math.fsum(float(x[t][i]) * float(Wg[i][e]) for i in range(d))
            if bg is not None:
                s += float(bg[e])
            row.append(s)
        out.append(row)
    return out


def route_loops(logits, k, C):
    """logits: list of lists of python floats (already fp32-rounded)."""
    T, E = len(logits), len(logits[0])
    choices, weights = [], []
    for t in range(T):
        row = list(logits[t])
        order = sorted(range(E), key=lambda e: (-row[e], e))[:k]   # high logit first, low index on ties
        m = max(row)
        z = [math.exp(v - m) for v in row]
        s = math.fsum(z)
        p = [z[e] / s for e in order]
        if k > 1:
            ps = math.fsum(p)
            p = [v / ps for v in p]
        choices.append(order)
        weights.append(p)
    filled = [0] * E
    slot = [[-1] * k for _ in range(T)]
    slot_token = [[-1] * C for _ in range(E)]
    for j in range(k):                      # every first choice before any second choice
        for t in range(T):
            e = choices[t][j]
            if filled[e] < C:
                slot[t][j] = filled[e]
                slot_token[e][filled[e]] = t
            filled[e] += 1
    rows = [min(n, C) for n in filled]
    return choices, weights, slot, rows, slot_token


def _gelu(z):
    return 0.5 * z * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z * z * z)))


def ffn_row(xrow, W1, b1, W2, b2):
    d, f = len(W1), len(W1[0])
    h = []
    for n in range(f):
        s = math.fsum(float(xrow[i]) * float(W1[i][n]) for i in range(d)) + (float(b1[n]) if b1 is not None else 0.0)
        h.append(_gelu(s))
    dout = len(W2[0])
    y = []
    for m in range(dout):
        s = math.fsum(h[n] * float(W2[n][m]) for n in range(f)) + (float(b2[m]) if b2 is not None else 0.0)
        y.append(s)
    return y


def layer_loops(x, logits, k, C, W1, b1, W2, b2, dense=None):
    """Per token: sum over its kept choices of weight * FFN_expert(x_t); plus the
    dense branch.  No dispatch buffer at all: the definition applied token by token."""
    choices, weights, slot, rows, slot_token = route_loops(logits, k, C)
    T, d = len(x), len(x[0])
    out = []
    for t in range(T):
        acc = [0.0] * d
        for j in range(k):
            if slot[t][j] >= 0:
                e = choices[t][j]
                y = ffn_row(x[t], W1[e], None if b1 is None else b1[e], W2[e], None if b2 is None else b2[e])
                acc = [a + weights[t][j] * v for a, v in zip(acc, y)]
        if dense is not None:
            y = ffn_row(x[t], *dense)
            acc = [a + v for a, v in zip(acc, y)]
        out.append(acc)
    return out, (choices, weights, slot, rows, slot_token)
