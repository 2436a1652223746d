"""Pins for the oracle's routing (gate, top-k, capacity slots): hand examples,
closed forms, invariants, library routines on tie-free inputs, brute force."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from tests import bruteforce as bf
from workloads import make_logits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "routing_hand_examples.json")


def _golden():
    with open(GOLDEN) as fh:
        g = json.load(fh)
    return {k: v for k, v in g.items() if not k.startswith("_")}


@pytest.mark.parametrize("name", sorted(_golden().keys()))
def test_hand_examples(name):
    ex = _golden()[name]
    r = orc.gate(np.array(ex["logits"], np.float32), ex["k"], ex["C"])
    assert r["expert_idx"].tolist() == ex["expert_idx"]
    assert r["loc"].tolist() == ex["loc"]
    assert r["slot_idx"].tolist() == ex["slot_idx"]
    assert r["expert_rows"].tolist() == ex["expert_rows"]
    assert r["slot_token"].tolist() == ex["slot_token"]
    np.testing.assert_allclose(r["gate_w"], np.array(ex["gate_w"]), rtol=0, atol=1e-15)


def test_hand_example_dropped_token_outputs_zero():
    # H1: token 2 is over capacity; a Standard-MoE layer outputs exactly 0 for it.
    ex = _golden()["H1_top1"]
    rng = np.random.default_rng(0)
    d, f = 4, 8
    x = rng.standard_normal((4, d))
    W1 = rng.standard_normal((2, d, f)); b1 = rng.standard_normal((2, f))
    W2 = rng.standard_normal((2, f, d)); b2 = rng.standard_normal((2, d))
    r = orc.moe_layer_forward(x, None, None, W1, b1, W2, b2, 1, 2,
                              logits=np.array(ex["logits"], np.float32))
    assert np.all(r["out"][2] == 0.0)
    # token 0 went to expert 0 with weight sigma(2)
    y0 = orc.ffn(x[0:1], W1[0], b1[0], W2[0], b2[0])[0]
    np.testing.assert_allclose(r["out"][0], 0.8807970779778823 * y0, rtol=1e-14)


@pytest.mark.parametrize("E", [1, 2, 3, 8, 64, 128])
@pytest.mark.parametrize("k", [1, 2])
def test_softmax_topk_against_torch_no_ties(E, k):
    if k > E:
        pytest.skip("k > E")
    l = make_logits(97, E, seed=E * 10 + k, kind="normal")       # continuous: no ties
    ln = l.numpy()
    p = orc.softmax(ln)
    np.testing.assert_allclose(p, torch.softmax(l.double(), dim=1).numpy(), rtol=1e-13, atol=0)
    idx = orc.top_k_experts(ln, k)
    tv, ti = torch.topk(l, k, dim=1)                               # sorted descending
    assert np.array_equal(idx, ti.numpy().astype(np.int32))


@pytest.mark.parametrize("kind", ["normal", "ties", "equal", "hot", "zipf"])
@pytest.mark.parametrize("k", [1, 2])
def test_weights_closed_forms(kind, k):
    E = 8
    l = make_logits(200, E, seed=3, kind=kind).numpy()
    r = orc.gate(l, k, 1000)
    g, idx = r["gate_w"], r["expert_idx"]
    rows = np.arange(l.shape[0])
    if k == 1:
        # weight = max of the softmax, hence >= 1/E, = 1/sum exp(l - lmax)
        lm = l.astype(np.float64)
        closed = 1.0 / np.exp(lm - lm.max(1, keepdims=True)).sum(1)
        np.testing.assert_allclose(g[:, 0], closed, rtol=1e-14)
        assert np.all(g[:, 0] >= 1.0 / E - 1e-15)
        assert np.all(l[rows, idx[:, 0]] == l.max(1))
    else:
        gap = l[rows, idx[:, 0]].astype(np.float64) - l[rows, idx[:, 1]].astype(np.float64)
        assert np.all(gap >= 0)
        np.testing.assert_allclose(g[:, 0], 1.0 / (1.0 + np.exp(-gap)), rtol=1e-13)
        np.testing.assert_allclose(g.sum(1), 1.0, rtol=1e-15)
        assert np.all(g[:, 0] >= 0.5 - 1e-15)
        assert np.all(idx[:, 0] != idx[:, 1])


def test_tie_rule_lowest_index():
    l = np.array([[1, 1, 1], [0, 2, 2], [3, 0, 3], [0, 0, 5]], np.float32)
    assert orc.top_k_experts(l, 1)[:, 0].tolist() == [0, 1, 0, 2]
    assert orc.top_k_experts(l, 2).tolist() == [[0, 1], [1, 2], [0, 2], [2, 0]]


def test_shift_invariance_of_routing():
    l = make_logits(300, 16, seed=5, kind="normal").numpy()
    r0 = orc.gate(l, 2, 20)
    shift = np.float32(2.0)            # power of two, |l| < 8: l + 2 is exact enough to keep order
    r1 = orc.gate((l.astype(np.float64) + 2.0).astype(np.float32), 2, 20)
    # ordering could only change where rounding merges two logits; weights move by rounding only
    same = np.all(r0["expert_idx"] == r1["expert_idx"], axis=1)
    assert same.mean() > 0.99
    np.testing.assert_allclose(r0["gate_w"][same], r1["gate_w"][same], atol=1e-6)


def _check_invariants(r, k, E, C, T):
    idx, slot, rows, st, loc = r["expert_idx"], r["slot_idx"], r["expert_rows"], r["slot_token"], r["loc"]
    seen = set()
    for t in range(T):
        for j in range(k):
            s = slot[t, j]
            if s >= 0:
                e = idx[t, j]
                assert (e, s) not in seen
                seen.add((e, s))
                assert st[e, s] == t
                assert s < rows[e] <= C
    assert len(seen) == rows.sum()
    for e in range(E):
        assert np.all(st[e, : rows[e]] >= 0)
        assert np.all(st[e, rows[e]:] == -1)
    n = [np.bincount(idx[:, j], minlength=E) for j in range(k)]
    if k == 1:
        assert np.array_equal(rows, np.minimum(n[0], C))
    else:
        assert np.array_equal(rows, np.minimum(n[0], C) + np.minimum(np.maximum(C - n[0], 0), n[1]))
    # first-choice slots in an expert are increasing in token order (cumsum semantics)
    for e in range(E):
        toks = [t for t in range(T) if idx[t, 0] == e and slot[t, 0] >= 0]
        assert [slot[t, 0] for t in toks] == list(range(len(toks)))
        dropped = [t for t in range(T) if idx[t, 0] == e and slot[t, 0] < 0]
        if toks and dropped:
            assert min(dropped) > max(toks)          # lower token index wins


@pytest.mark.parametrize("kind", ["normal", "ties", "equal", "hot", "zipf"])
@pytest.mark.parametrize("k,E,C,T", [(1, 8, 32, 256), (1, 128, 1, 64), (2, 8, 10, 61), (2, 64, 5, 333),
                                     (1, 1, 7, 9), (2, 2, 3, 10), (1, 3, 1000, 50)])
def test_slot_invariants(kind, k, E, C, T):
    l = make_logits(T, E, seed=T + E, kind=kind).numpy()
    r = orc.gate(l, k, C)
    _check_invariants(r, k, E, C, T)


def test_prefix_property_top1():
    # routing of tokens < t does not depend on tokens >= t (cumsum in token order)
    l = make_logits(128, 8, seed=9, kind="normal").numpy()
    r = orc.gate(l, 1, 12)
    l2 = l.copy()
    l2[70:] = make_logits(58, 8, seed=10, kind="hot").numpy()
    r2 = orc.gate(l2, 1, 12)
    assert np.array_equal(r["slot_idx"][:70], r2["slot_idx"][:70])
    assert np.array_equal(r["expert_idx"][:70], r2["expert_idx"][:70])


def test_no_drop_when_capacity_large():
    l = make_logits(100, 4, seed=11, kind="zipf").numpy()
    r = orc.gate(l, 2, 200)
    assert np.all(r["slot_idx"] >= 0)
    assert r["expert_rows"].sum() == 200


@pytest.mark.parametrize("kind", ["normal", "ties", "equal"])
@pytest.mark.parametrize("k,E,C,T", [(1, 4, 3, 16), (2, 4, 5, 16), (2, 3, 2, 11), (1, 2, 1, 5)])
def test_routing_against_bruteforce(kind, k, E, C, T):
    l = make_logits(T, E, seed=100 + T, kind=kind).numpy()
    r = orc.gate(l, k, C)
    ch, w, slot, rows, st = bf.route_loops([[float(v) for v in row] for row in l], k, C)
    assert r["expert_idx"].tolist() == ch
    assert r["slot_idx"].tolist() == slot
    assert r["expert_rows"].tolist() == rows
    assert r["slot_token"].tolist() == st
    np.testing.assert_allclose(r["gate_w"], np.array(w), rtol=1e-13)


def test_gate_logits_against_loops_and_fp32_rounding():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 13)).astype(np.float32)
    Wg = (0.02 * rng.standard_normal((13, 5))).astype(np.float32)
    bg = rng.standard_normal(5).astype(np.float32)
    l = orc.gate_logits(x, Wg, bg)
    assert l.dtype == np.float32
    ref = np.array(bf.logits_loops(x.tolist(), Wg.tolist(), bg.tolist()))
    assert np.array_equal(l, ref.astype(np.float32))
    # transposed operand or dropped bias would fail:
    assert not np.allclose(l, orc.gate_logits(x, Wg, None))


def test_nonfinite_logits_rejected():
    l = np.zeros((2, 2), np.float32)
    l[0, 0] = np.nan
    with pytest.raises(AssertionError):
        orc.gate(l, 1, 1)
