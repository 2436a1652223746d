"""Pins for the oracle's floating-point side: library routines on special cases,
the literal one-hot einsum formulation, pure-Python loops, structural identities."""
import math

import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from tests import bruteforce as bf
from workloads import CONFIGS, make_inputs
from workloads.generate import to_f32_numpy


def _small(rng, T, d, f, E, residual=False, bias=True, gate_scale=1.0):
    x = rng.standard_normal((T, d))
    Wg = gate_scale * rng.standard_normal((d, E))
    bg = rng.standard_normal(E)
    W1 = 0.3 * rng.standard_normal((E, d, f)); W2 = 0.3 * rng.standard_normal((E, f, d))
    b1 = rng.standard_normal((E, f)) if bias else None
    b2 = rng.standard_normal((E, d)) if bias else None
    dense = None
    if residual:
        dense = (0.3 * rng.standard_normal((d, f)), rng.standard_normal(f),
                 0.3 * rng.standard_normal((f, d)), rng.standard_normal(d))
    return x, Wg, bg, W1, b1, W2, b2, dense


def test_gelu_tanh_against_torch_and_values():
    z = np.linspace(-6, 6, 1001)
    ref = torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    np.testing.assert_allclose(orc.gelu_tanh(z), ref, rtol=1e-13, atol=1e-15)
    assert orc.gelu_tanh(np.array([0.0]))[0] == 0.0
    # value worked from the formula: z=1 -> 0.5*(1+tanh(0.7978845608*1.044715))
    assert abs(orc.gelu_tanh(np.array([1.0]))[0] - 0.5 * (1 + math.tanh(0.7978845608028654 * 1.044715))) < 1e-15
    assert abs(orc.gelu_tanh(np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(orc.gelu_tanh(np.array([-10.0]))[0]) < 1e-12


def test_ffn_against_torch_fp64():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((9, 6)); W1 = rng.standard_normal((6, 10)); b1 = rng.standard_normal(10)
    W2 = rng.standard_normal((10, 6)); b2 = rng.standard_normal(6)
    tx, tW1, tb1, tW2, tb2 = map(torch.from_numpy, (x, W1, b1, W2, b2))
    ref = torch.nn.functional.gelu(tx @ tW1 + tb1, approximate="tanh") @ tW2 + tb2
    np.testing.assert_allclose(orc.ffn(x, W1, b1, W2, b2), ref.numpy(), rtol=1e-12, atol=1e-13)
    # a transposed weight or dropped bias must not pass
    assert not np.allclose(orc.ffn(x, W1, None, W2, b2), ref.numpy())


def test_single_expert_layer_is_dense_ffn():
    # E=1, k=1, C=T: softmax over one logit is 1, nothing dropped -> layer == FFN.
    rng = np.random.default_rng(2)
    x, Wg, bg, W1, b1, W2, b2, _ = _small(rng, 12, 5, 7, 1)
    r = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, 1, 12)
    tx = torch.from_numpy(x)
    ref = torch.nn.functional.gelu(tx @ torch.from_numpy(W1[0]) + torch.from_numpy(b1[0]),
                                   approximate="tanh") @ torch.from_numpy(W2[0]) + torch.from_numpy(b2[0])
    np.testing.assert_allclose(r["out"], ref.numpy(), rtol=1e-12, atol=1e-13)
    assert np.all(r["gate_w"] == 1.0)


@pytest.mark.parametrize("k,E,C,T,residual", [(1, 4, 3, 16, False), (2, 4, 5, 16, False), (1, 3, 4, 16, True),
                                               (2, 3, 100, 9, True), (1, 8, 2, 40, False), (2, 6, 7, 33, False)])
def test_forward_equals_literal_einsum(k, E, C, T, residual):
    rng = np.random.default_rng(T * 7 + E)
    x, Wg, bg, W1, b1, W2, b2, dense = _small(rng, T, 6, 10, E, residual)
    dk = {} if dense is None else dict(Wd1=dense[0], bd1=dense[1], Wd2=dense[2], bd2=dense[3])
    r = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, k, C, **dk)
    ein = orc.moe_layer_einsum(x, Wg, bg, W1, b1, W2, b2, k, C, **dk)
    np.testing.assert_allclose(r["out"], ein, rtol=1e-12, atol=1e-12)
    if C < T:      # the case must really exercise drops
        assert (r["slot_idx"] < 0).any() or k * T <= E * C


@pytest.mark.parametrize("k,E,C,T,residual", [(1, 3, 2, 8, False), (2, 3, 3, 8, False), (1, 2, 3, 7, True)])
def test_forward_equals_python_loops(k, E, C, T, residual):
    rng = np.random.default_rng(31 + T + k)
    x, Wg, bg, W1, b1, W2, b2, dense = _small(rng, T, 4, 6, E, residual)
    dk = {} if dense is None else dict(Wd1=dense[0], bd1=dense[1], Wd2=dense[2], bd2=dense[3])
    r = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, k, C, **dk)
    logits = [[float(v) for v in row] for row in r["logits"]]
    ref, _ = bf.layer_loops(x.tolist(), logits, k, C, W1.tolist(), b1.tolist(), W2.tolist(), b2.tolist(),
                            None if dense is None else [a.tolist() for a in dense])
    np.testing.assert_allclose(r["out"], np.array(ref), rtol=1e-11, atol=1e-12)


def test_zero_experts_identities():
    rng = np.random.default_rng(5)
    x, Wg, bg, W1, b1, W2, b2, dense = _small(rng, 20, 6, 8, 4, residual=True)
    Z = lambda a: np.zeros_like(a)
    r = orc.moe_layer_forward(x, Wg, bg, Z(W1), Z(b1), Z(W2), Z(b2), 1, 3,
                              Wd1=dense[0], bd1=dense[1], Wd2=dense[2], bd2=dense[3])
    assert np.array_equal(r["out"], orc.ffn(x, *dense))          # Residual-MoE == dense MLP, exactly
    r = orc.moe_layer_forward(x, Wg, bg, Z(W1), Z(b1), Z(W2), Z(b2), 1, 3)
    assert np.all(r["out"] == 0.0)                                # Standard-MoE == 0


def test_residual_is_sum_of_branches():
    rng = np.random.default_rng(6)
    x, Wg, bg, W1, b1, W2, b2, dense = _small(rng, 20, 6, 8, 4, residual=True)
    a = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, 1, 4)["out"]
    b = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, 1, 4,
                              Wd1=dense[0], bd1=dense[1], Wd2=dense[2], bd2=dense[3])["out"]
    np.testing.assert_allclose(b - a, orc.ffn(x, *dense), rtol=1e-12, atol=1e-12)


def test_permutation_equivariance_without_drops():
    rng = np.random.default_rng(7)
    x, Wg, bg, W1, b1, W2, b2, _ = _small(rng, 24, 6, 8, 4)
    perm = rng.permutation(24)
    a = orc.moe_layer_forward(x, Wg, bg, W1, b1, W2, b2, 2, 48)["out"]
    b = orc.moe_layer_forward(x[perm], Wg, bg, W1, b1, W2, b2, 2, 48)["out"]
    np.testing.assert_allclose(a[perm], b, rtol=1e-12, atol=1e-13)


def test_dispatch_combine_roundtrip():
    rng = np.random.default_rng(8)
    T, d, E, C, k = 30, 5, 4, 6, 2
    x = rng.standard_normal((T, d))
    r = orc.gate(rng.standard_normal((T, E)).astype(np.float32), k, C)
    xe = orc.dispatch(x, r["slot_token"])
    assert np.all(xe[r["slot_token"] < 0] == 0.0)
    ones = np.ones_like(r["gate_w"])
    back = orc.combine(xe, r["expert_idx"], r["slot_idx"], ones)
    kept = (r["slot_idx"] >= 0).sum(1)
    np.testing.assert_allclose(back, x * kept[:, None], rtol=1e-15)


def test_tiny_config_runs_and_is_self_consistent():
    # workload c1 (fp32, T=256, E=8, C=32): the oracle finishes well under a second.
    cfg = CONFIGS["c1"]
    inp = make_inputs(cfg, "cpu", bias_std=0.02)
    a = {k: to_f32_numpy(v) for k, v in inp.tensors().items()}
    r = orc.moe_layer_forward(a["x"], a["Wg"], None, a["W1"], a["b1"], a["W2"], a["b2"], 1, cfg.capacity)
    assert cfg.capacity == 32
    ein = orc.moe_layer_einsum(a["x"], a["Wg"], None, a["W1"], a["b1"], a["W2"], a["b2"], 1, cfg.capacity)
    np.testing.assert_allclose(r["out"], ein, rtol=1e-11, atol=1e-14)
    dropped = r["slot_idx"][:, 0] < 0
    assert dropped.any() and np.all(r["out"][dropped] == 0.0)


def test_capacities_of_the_five_configs():
    caps = {n: c.capacity for n, c in CONFIGS.items()}
    assert caps == {"c1": 32, "c2": 64, "c3a": 256, "c3b": 128, "c4": 1, "c5": 640}
