"""Seeded sweep of moe_layer_forward over shapes inside the documented limits that no hand-picked case covers:
every combination drawn here of token count (1 .. 4500), widths that are multiples of 8 but of nothing larger,
expert counts off the XCD count, top-1 / top-2, with and without the dense branch, capacity factors from 0.5 to 4
and skewed or even routing runs through the same check as the named workloads (routing bit for bit on the
kernel's logits, output within tolerance, plain and packed weights)."""
import random

import pytest

from tests import gpu_util as U
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def _cases(seed, n):
    rng = random.Random(seed)
    out = []
    for i in range(n):
        k = rng.choice([1, 2])
        E = rng.choice([1, 2, 3, 5, 8, 9, 16, 17, 31, 40, 64, 70])
        if k > E:
            k = 1
        residual = rng.random() < 0.4
        T = rng.choice([1, 7, 64, 100, 129, 256, 257, 600, 1000, 2048, 2300, 3000, 4500])
        d = rng.choice([32, 64, 72, 96, 128, 200, 256, 264, 512])
        f = rng.choice([32, 40, 64, 128, 136, 256, 520, 1024])
        cf = rng.choice([0.5, 0.9, 1.0, 1.25, 2.0, 4.0])
        zipf = rng.choice([None, None, 1.0, 1.5])
        out.append(CONFIGS["c2"].scaled(name=f"sweep{seed}-{i}", T=T, d_model=d, d_ffn=f, E=E, top_k=k,
                                        capacity_factor=cf, residual=residual, seed=100 + i, gate_bias_zipf=zipf))
    return out


CASES = _cases(1, 30)


@pytest.mark.parametrize("cfg", CASES, ids=[c.name for c in CASES])
def test_layer_random_shape(cfg):
    print(f"case {cfg.name}: T={cfg.T} d={cfg.d_model} f={cfg.d_ffn} E={cfg.E} k={cfg.top_k} C={cfg.capacity} "
          f"residual={cfg.residual} zipf={cfg.gate_bias_zipf}", flush=True)
    U.check_layer(make_inputs(cfg, "cuda", bias_std=0.05))
