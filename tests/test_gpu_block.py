"""GPU parity of moe_decode_block_forward (one decode step of a decoder block with an MoE feed-forward part) against
oracle/block_oracle.py, through the C ABI.

The block is compared in two halves, because its MoE layer routes on logits of a bf16 input that the GPU has
rounded: (1) x1 = x + attention against the oracle on the same inputs, the new key/value rows in the cache, every
other cache entry untouched; (2) the MoE input against the oracle's LayerNorm of the GPU's own x1; (3) the block
output against x1 + the oracle's MoE layer evaluated on the GPU's MoE input and fp32 logits (as the layer tests do),
with the logits themselves checked against the oracle's."""
import numpy as np
import pytest
import torch

from oracle import block_oracle as blk
from oracle import moe_oracle as orc
from tests import gpu_util as U
from workloads import CONFIGS, make_block_inputs
from workloads.generate import to_f32_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run_block(bi, pack=False):
    m = U.amd()
    lay, cfg = bi.layer, bi.layer.cfg
    T, d, E = cfg.T, cfg.d_model, cfg.E
    shape = m.make_shape(T, d, cfg.d_ffn, E, cfg.top_k, cfg.capacity, "bf16", residual=cfg.residual,
                         flags=m.MOE_FLAG_PACKED_WEIGHTS if pack else 0)
    block = m.MoeBlockShape(bi.n_heads, bi.max_len)
    nbytes = m.moe_decode_block_workspace_bytes(shape, block)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    pk = (lambda w: m.moe_pack_weights(w)) if pack else (lambda w: w)
    weights = dict(ln1_gamma=bi.ln1_gamma, ln1_beta=bi.ln1_beta, Wqkv=bi.Wqkv, bqkv=bi.bqkv, Wo=bi.Wo, bo=bi.bo,
                   ln2_gamma=bi.ln2_gamma, ln2_beta=bi.ln2_beta, Wg=lay.Wg, bg=lay.bg, W1=pk(lay.W1), b1=lay.b1,
                   W2=pk(lay.W2), b2=lay.b2, Wd1=None if lay.Wd1 is None else pk(lay.Wd1), bd1=lay.bd1,
                   Wd2=None if lay.Wd2 is None else pk(lay.Wd2), bd2=lay.bd2)
    bf = torch.bfloat16
    canary = 12345.0
    pad = torch.full((T + 32, d), canary, dtype=bf, device=DEV)
    out = pad[16:16 + T]
    x1 = torch.empty((T, d), dtype=bf, device=DEV)
    moe_in = torch.empty((T, d), dtype=bf, device=DEV)
    logits = torch.empty((T, E), dtype=torch.float32, device=DEV)
    kc, vc = bi.k_cache.clone(), bi.v_cache.clone()
    m.moe_decode_block_forward(shape, block, weights, lay.x, kc, vc, bi.pos, out, x1, moe_in, logits, ws)
    torch.cuda.synchronize()
    assert bool((pad[:16] == canary).all()) and bool((pad[16 + T:] == canary).all()), "write outside out"
    return dict(out=out, x1=x1, moe_in=moe_in, logits=logits, k_cache=kc, v_cache=vc)


def _check_block(bi, lazy_experts=False, packed_too=True):
    lay, cfg = bi.layer, bi.layer.cfg
    T, H = cfg.T, bi.n_heads
    tol = U.TOL["bf16"]
    f = to_f32_numpy
    pos = bi.pos.cpu().numpy()
    ref_a = blk.attention_half(f(lay.x), f(bi.ln1_gamma), f(bi.ln1_beta), f(bi.Wqkv), f(bi.bqkv), f(bi.k_cache),
                               f(bi.v_cache), pos, f(bi.Wo), f(bi.bo), H)
    h = U.host(lay, lazy_experts)
    stats = {}
    for pack in ([False, True] if packed_too else [False]):
        print(f"block {cfg.name} pack={pack}", flush=True)
        res = _run_block(bi, pack)
        U.assert_close(res["x1"], ref_a["x1"], "bf16", "x1")
        # the cache: row pos[b] holds the new key/value, nothing else changed
        kc, vc = f(res["k_cache"]), f(res["v_cache"])
        k0, v0 = f(bi.k_cache), f(bi.v_cache)
        rows = np.arange(T)
        kn, vn = kc[rows, :, pos, :], vc[rows, :, pos, :]
        assert np.max(np.abs(kn - ref_a["k_new"])) <= tol * np.max(np.abs(ref_a["k_new"]))
        assert np.max(np.abs(vn - ref_a["v_new"])) <= tol * np.max(np.abs(ref_a["v_new"]))
        kc[rows, :, pos, :] = k0[rows, :, pos, :]
        vc[rows, :, pos, :] = v0[rows, :, pos, :]
        assert np.array_equal(kc, k0) and np.array_equal(vc, v0), "cache rows other than pos[b] changed"
        # LayerNorm of the GPU's own x1
        x1g = f(res["x1"])
        U.assert_close(res["moe_in"], blk.layer_norm(x1g, f(bi.ln2_gamma), f(bi.ln2_beta)), "bf16", "moe input")
        # the MoE half on the GPU's MoE input and logits
        xin = f(res["moe_in"])
        gl = res["logits"].cpu().numpy()
        own = orc.gate_logits(xin, h["Wg"], h.get("bg"))
        assert np.max(np.abs(gl.astype(np.float64) - own)) <= U.LOGIT_RTOL * np.max(np.abs(own))
        ref = blk.moe_half(x1g, None, None, h["Wg"], h.get("bg"), h["W1"], h["b1"], h["W2"], h["b2"], cfg.top_k,
                           cfg.capacity, h.get("Wd1"), h.get("bd1"), h.get("Wd2"), h.get("bd2"), moe_input=xin, logits=gl)
        stats[f"rel_err_pack{int(pack)}"] = U.assert_close(res["out"], ref["out"], "bf16", "block out")
        stats["kept"] = int(ref["expert_rows"].sum())
    return stats


SMALL = {
    # name: (config, heads, max_len)
    "dh64": (CONFIGS["c4"].scaled(name="b-dh64", T=64, d_model=256, d_ffn=512, E=8, capacity_factor=2.0), 4, 300),
    "dh128": (CONFIGS["c4"].scaled(name="b-dh128", T=33, d_model=512, d_ffn=1024, E=16, capacity_factor=4.0), 4, 700),
    "top2": (CONFIGS["c5"].scaled(name="b-top2", T=40, d_model=256, d_ffn=512, E=6, capacity_factor=1.5), 2, 257),
    "residual": (CONFIGS["c3a"].scaled(name="b-res", T=48, d_model=256, d_ffn=512, E=4, capacity_factor=1.0), 4, 64),
    "one": (CONFIGS["c4"].scaled(name="b-one", T=1, d_model=128, d_ffn=256, E=4, capacity_factor=4.0), 2, 1),
    "dense_ffn": (CONFIGS["c4"].scaled(name="b-dense", T=20, d_model=256, d_ffn=1024, E=1, capacity_factor=1.0), 4, 513),
    "many_rows": (CONFIGS["c3a"].scaled(name="b-rows", T=300, d_model=256, d_ffn=512, E=4, capacity_factor=1.0), 4, 40),
}


@pytest.mark.parametrize("name", sorted(SMALL))
def test_decode_block_reduced(name):
    cfg, heads, max_len = SMALL[name]
    stats = _check_block(make_block_inputs(cfg, heads, max_len, DEV))
    print(name, stats, flush=True)


def test_decode_block_full_context():
    """Every sequence at the last cache position: all chunks of the attention kernel are full."""
    cfg, heads, max_len = SMALL["dh128"]
    _check_block(make_block_inputs(cfg, heads, 1024, DEV, pos_mode="full"))


def test_decode_block_1p3b_shape():
    """The decode workload's shape (64 sequences, hidden 2048, 16 heads, 128 experts of 2048 x 8192) with a 2048-token cache."""
    print("case block c4-shaped", flush=True)
    stats = _check_block(make_block_inputs(CONFIGS["c4"], 16, 2048, DEV, bias_std=0.0), lazy_experts=True, packed_too=False)
    print("c4 block", stats, flush=True)


def test_decode_block_rejects_bad_arguments():
    m = U.amd()
    shape = m.make_shape(8, 256, 512, 4, 1, 2, "bf16")
    assert m.moe_decode_block_workspace_bytes(shape, m.MoeBlockShape(3, 16)) == 0          # 256/3 is no head size
    assert m.moe_decode_block_workspace_bytes(shape, m.MoeBlockShape(8, 16)) == 0          # head size 32
    assert m.moe_decode_block_workspace_bytes(m.make_shape(8, 256, 512, 4, 1, 2, "f32"), m.MoeBlockShape(4, 16)) == 0
    assert m.moe_decode_block_workspace_bytes(shape, m.MoeBlockShape(4, 16)) > 0
