"""Pins of the decode-block oracle (oracle/block_oracle.py): library routines, the equivalence of a cached decode
step with full causal attention, closed forms and structural identities.  CPU only."""
import numpy as np
import torch

from oracle import block_oracle as blk
from oracle import moe_oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


def test_layer_norm_matches_torch():
    r = _rng(0)
    x, g, b = r.normal(size=(7, 48)) * 3 + 1, r.normal(size=48), r.normal(size=48)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), eps=1e-5)
    assert np.allclose(blk.layer_norm(x, g, b), ref.numpy(), rtol=0, atol=1e-12)
    # rows end up with mean beta-weighted 0 and unit variance when gamma = 1, beta = 0 (up to eps)
    y = blk.layer_norm(x, np.ones(48), np.zeros(48))
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12) and np.allclose(y.var(axis=1), 1, atol=1e-4)
    # a constant shift of the row changes nothing, a positive scale neither (up to eps)
    assert np.allclose(blk.layer_norm(x + 5.0, g, b), blk.layer_norm(x, g, b), atol=1e-9)


def test_attend_closed_forms():
    r = _rng(1)
    V = r.normal(size=(9, 16))
    q = r.normal(size=16)
    # equal scores (all keys identical): the mean of the values
    K = np.tile(r.normal(size=(1, 16)), (9, 1))
    assert np.allclose(blk.attend(q, K, V), V.mean(axis=0), atol=1e-12)
    # one position: its value, whatever the key
    assert np.allclose(blk.attend(q, K[:1], V[:1]), V[0], atol=1e-15)
    # one key far better than the rest: its value
    K2 = r.normal(size=(9, 16))
    K2[4] = q * 50.0
    assert np.allclose(blk.attend(q, K2, V), V[4], atol=1e-9)
    # the scale is 1/sqrt(dh): two positions with scores 0 and ln(3)*sqrt(dh)/|q|^2 ... -> weights 1/4, 3/4
    q1 = np.zeros(16)
    q1[0] = 1.0
    K3 = np.zeros((2, 16))
    K3[1, 0] = np.log(3.0) * np.sqrt(16)
    assert np.allclose(blk.attend(q1, K3, V[:2]), 0.25 * V[0] + 0.75 * V[1], atol=1e-12)


def test_attend_matches_torch_sdpa():
    r = _rng(2)
    q, K, V = r.normal(size=24), r.normal(size=(13, 24)), r.normal(size=(13, 24))
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[None, None, None, :],
                                                           torch.from_numpy(K)[None, None], torch.from_numpy(V)[None, None])
    assert np.allclose(blk.attend(q, K, V), ref.numpy()[0, 0, 0], atol=1e-12)


def test_decode_step_equals_last_row_of_causal_attention():
    """Sequences of different lengths: the cached decode step for the newest token equals row n of causal attention
    over the whole sequence (torch's library routine with is_causal), per head."""
    r = _rng(3)
    B, H, dh, Lmax = 3, 2, 8, 12
    pos = np.array([0, 5, 11])
    ck, cv = r.normal(size=(B, H, Lmax, dh)), r.normal(size=(B, H, Lmax, dh))
    q, kn, vn = r.normal(size=(B, H, dh)), r.normal(size=(B, H, dh)), r.normal(size=(B, H, dh))
    o = blk.decode_attention(q, kn, vn, ck, cv, pos)
    for b in range(B):
        n = pos[b]
        Kf = np.concatenate([ck[b, :, :n], kn[b][:, None, :]], axis=1)          # [H, n+1, dh]
        Vf = np.concatenate([cv[b, :, :n], vn[b][:, None, :]], axis=1)
        Qf = r.normal(size=(H, n + 1, dh))
        Qf[:, n] = q[b]
        ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(Qf)[None], torch.from_numpy(Kf)[None],
                                                               torch.from_numpy(Vf)[None], is_causal=True)
        assert np.allclose(o[b], ref.numpy()[0, :, n], atol=1e-12)
    # positions at and beyond pos[b] of the cache are never read
    ck2, cv2 = ck.copy(), cv.copy()
    for b in range(B):
        ck2[b, :, pos[b]:] = 1e6
        cv2[b, :, pos[b]:] = -1e6
    assert np.array_equal(blk.decode_attention(q, kn, vn, ck2, cv2, pos), o)


def _block_inputs(seed, B=5, d=16, H=2, Lmax=6, f=32, E=3):
    r = _rng(seed)
    return dict(x=r.normal(size=(B, d)), g1=r.normal(size=d), be1=r.normal(size=d), Wqkv=r.normal(size=(d, 3 * d)) * 0.2,
                bqkv=r.normal(size=3 * d) * 0.1, cache_k=r.normal(size=(B, H, Lmax, d // H)),
                cache_v=r.normal(size=(B, H, Lmax, d // H)), pos=r.integers(0, Lmax, size=B), Wo=r.normal(size=(d, d)) * 0.2,
                bo=r.normal(size=d) * 0.1, n_heads=H, g2=r.normal(size=d), be2=r.normal(size=d),
                Wg=r.normal(size=(d, E)).astype(np.float32), bg=None, W1=r.normal(size=(E, d, f)) * 0.2,
                b1=r.normal(size=(E, f)) * 0.1, W2=r.normal(size=(E, f, d)) * 0.2, b2=r.normal(size=(E, d)) * 0.1,
                top_k=1, capacity=3)


def test_block_is_the_composition_written_out_with_torch():
    """The whole block against the same computation spelled with torch's library routines (layer_norm, linear,
    scaled_dot_product_attention on the concatenated keys) and the MoE oracle, on fp64."""
    p = _block_inputs(4)
    r = blk.decode_block(**p)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    B, d = p["x"].shape
    H = p["n_heads"]
    dh = d // H
    a = torch.nn.functional.layer_norm(t(p["x"]), (d,), t(p["g1"]), t(p["be1"]), eps=1e-5)
    qkv = torch.nn.functional.linear(a, t(p["Wqkv"]).T, t(p["bqkv"]))
    q, k, v = (z.reshape(B, H, dh) for z in qkv.split(d, dim=1))
    o = torch.zeros(B, H, dh, dtype=torch.float64)
    for b in range(B):
        n = int(p["pos"][b])
        K = torch.cat([t(p["cache_k"][b, :, :n]), k[b][:, None, :]], dim=1)
        V = torch.cat([t(p["cache_v"][b, :, :n]), v[b][:, None, :]], dim=1)
        o[b] = torch.nn.functional.scaled_dot_product_attention(q[b][None, :, None, :], K[None], V[None])[0, :, 0]
    x1 = t(p["x"]) + torch.nn.functional.linear(o.reshape(B, d), t(p["Wo"]).T, t(p["bo"]))
    assert np.allclose(r["x1"], x1.numpy(), atol=1e-11)
    xn = torch.nn.functional.layer_norm(x1, (d,), t(p["g2"]), t(p["be2"]), eps=1e-5).numpy()
    m = orc.moe_layer_forward(xn, p["Wg"], None, p["W1"], p["b1"], p["W2"], p["b2"], 1, p["capacity"])
    assert np.allclose(r["out"], x1.numpy() + m["out"], atol=1e-10)
    assert np.allclose(r["k_new"], k.numpy(), atol=1e-12) and np.allclose(r["v_new"], v.numpy(), atol=1e-12)


def test_block_with_zero_projections_is_identity():
    p = _block_inputs(5)
    for n in ("Wo", "bo", "W2", "b2"):
        p[n] = np.zeros_like(p[n])
    r = blk.decode_block(**p)
    assert np.array_equal(r["out"], p["x"])


def test_moe_half_accepts_foreign_moe_input():
    p = _block_inputs(6)
    a = blk.attention_half(p["x"], p["g1"], p["be1"], p["Wqkv"], p["bqkv"], p["cache_k"], p["cache_v"], p["pos"],
                           p["Wo"], p["bo"], p["n_heads"])
    args = (p["g2"], p["be2"], p["Wg"], None, p["W1"], p["b1"], p["W2"], p["b2"], 1, p["capacity"])
    own = blk.moe_half(a["x1"], *args)
    same = blk.moe_half(a["x1"], *args, moe_input=own["moe_input"], logits=own["logits"])
    assert np.array_equal(own["out"], same["out"])
