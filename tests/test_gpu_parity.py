"""GPU parity tests: every C-ABI entry point against the CPU oracle on the same
seeded inputs.  Routing is compared bit for bit on identical fp32 logits;
floating-point outputs within max|delta| <= tol * max|ref| (1e-4 fp32, 1.5e-2
bf16)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as orc
from tests import gpu_util as U
from workloads import CONFIGS, make_inputs, make_logits

pytestmark = pytest.mark.gpu
DEV = "cuda"


# ------------------------------------------------------------------ routing from logits

@pytest.mark.parametrize("kind", ["normal", "ties", "equal", "hot", "zipf"])
@pytest.mark.parametrize("k,E,C,T", [
    (1, 8, 32, 256), (1, 128, 64, 8192), (1, 128, 1, 64), (2, 64, 640, 16384),
    (1, 1, 5, 9), (2, 2, 3, 10), (1, 3, 7, 63), (2, 3, 7, 65), (1, 64, 3, 257), (2, 128, 2, 1000),
    (1, 200, 4, 777), (2, 1024, 1, 300), (1, 32, 256, 8192), (2, 8, 100000, 513), (1, 4, 2, 1), (2, 5, 1, 2),
])
def test_gate_routing_bit_exact(kind, k, E, C, T):
    print(f"case kind={kind} k={k} E={E} C={C} T={T}", flush=True)
    logits = make_logits(T, E, seed=T + 3 * E + k, kind=kind, device=DEV)
    res = U.gpu_route(logits, k, C)
    ref = orc.gate(logits.cpu().numpy(), k, C)
    U.assert_routing_equal(res, ref)


def test_gate_routing_deterministic():
    logits = make_logits(5000, 64, seed=1, kind="zipf", device=DEV)
    a = U.gpu_route(logits, 2, 50)
    b = U.gpu_route(logits, 2, 50)
    for n in a:
        assert torch.equal(a[n], b[n]), n


# ------------------------------------------------------------------ gate logits

@pytest.mark.parametrize("dtype,T,d,E,bias", [("f32", 256, 64, 8, False), ("bf16", 1000, 1024, 128, False),
                                              ("bf16", 77, 2048, 128, True), ("bf16", 300, 520, 64, True),
                                              ("f32", 33, 100, 3, True), ("bf16", 129, 256, 300, False)])
def test_gate_logits(dtype, T, d, E, bias):
    m = U.amd()
    g = torch.Generator(device=DEV).manual_seed(T + d)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.randn((T, d), generator=g, device=DEV).to(tdt)
    Wg = 0.02 * torch.randn((d, E), generator=g, device=DEV)
    bg = torch.randn((E,), generator=g, device=DEV) if bias else None
    shape = m.make_shape(T, d, 8, E, 1, 4, dtype)
    ws = m.alloc_workspace(shape, DEV)
    i32 = torch.int32
    logits = torch.empty((T, E), dtype=torch.float32, device=DEV)
    outs = [torch.empty((T, 1), dtype=i32, device=DEV), torch.empty((T, 1), dtype=i32, device=DEV),
            torch.empty((T, 1), dtype=torch.float32, device=DEV), torch.empty((E,), dtype=i32, device=DEV),
            torch.empty((E, 4), dtype=i32, device=DEV)]
    m.moe_gate(shape, x, Wg, bg, logits, *outs, ws)
    torch.cuda.synchronize()
    ref = orc.gate_logits(x.float().cpu().numpy(), Wg.cpu().numpy(), None if bg is None else bg.cpu().numpy())
    err = np.max(np.abs(logits.cpu().numpy().astype(np.float64) - ref))
    assert err <= U.LOGIT_RTOL * np.max(np.abs(ref)), err


# ------------------------------------------------------------------ the whole gate from tokens

# >= 2048 bf16 tokens with d % 32 == 0 and E <= 128 take the fused kernel (logits + top-k + tile ranks), fewer
# tokens the split one (logits over expert groups, then routing), everything else the fp32-MFMA logits kernel.
# dup: two pairs of experts get identical weight columns, so their logits tie exactly for every token;
# "hot": in addition all tokens are equal, so every token makes the same choice.
@pytest.mark.parametrize("dtype,T,d,E,k,C,bias,dup", [
    ("bf16", 2048, 64, 128, 1, 20, False, False), ("bf16", 3001, 64, 16, 2, 37, True, "hot"),
    ("bf16", 20000, 32, 128, 1, 5000, False, "hot"), ("bf16", 1, 32, 4, 1, 1, True, False), ("bf16", 2085, 96, 48, 2, 100, True, False),
    ("bf16", 4096, 32, 8, 2, 600, True, True), ("bf16", 3000, 256, 64, 1, 40, False, True),
    ("bf16", 2500, 128, 20, 2, 300, True, False), ("bf16", 2111, 64, 30, 1, 64, True, True),
    ("bf16", 16448, 64, 16, 1, 1100, False, False), ("bf16", 16500, 32, 100, 2, 250, True, True),
    ("bf16", 77, 2048, 128, 1, 1, True, False), ("bf16", 1000, 64, 30, 2, 50, True, True),
    ("bf16", 300, 520, 64, 1, 5, False, False), ("bf16", 500, 64, 200, 2, 4, False, True),
    # at most 256 bf16 tokens, d % 32 == 0, E <= 128: the one-launch decode gate (1 to 64 work-groups)
    ("bf16", 256, 64, 128, 2, 5, True, True), ("bf16", 33, 512, 16, 1, 9, False, False),
    ("bf16", 255, 96, 17, 2, 40, True, True), ("bf16", 64, 2048, 128, 1, 1, False, "hot"), ("bf16", 2, 32, 3, 2, 1, True, False),
    ("bf16", 31, 64, 100, 1, 2, True, True), ("bf16", 257, 64, 128, 1, 3, False, False),
    ("f32", 300, 100, 12, 2, 40, True, True)])
def test_gate_from_tokens(dtype, T, d, E, k, C, bias, dup):
    m = U.amd()
    g = torch.Generator(device=DEV).manual_seed(T + 3 * d + 7 * E)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.randn((T, d), generator=g, device=DEV).to(tdt)
    if dup == "hot":                # every token is the same row: one expert (pair) takes them all
        x = x[:1].repeat(T, 1).contiguous()
    Wg = 0.05 * torch.randn((d, E), generator=g, device=DEV)
    if dup:
        Wg[:, E - 1] = Wg[:, 1]
        Wg[:, E // 2] = Wg[:, 0]
    bg = None
    if bias:
        bg = 0.3 * torch.randn((E,), generator=g, device=DEV)
        if dup:
            bg[E - 1] = bg[1]
            bg[E // 2] = bg[0]
    shape = m.make_shape(T, d, 8, E, k, C, dtype)
    ws = m.alloc_workspace(shape, DEV)
    i32 = torch.int32
    logits = torch.full((T, E), 7.0, dtype=torch.float32, device=DEV)
    r = dict(expert_idx=torch.full((T, k), -7, dtype=i32, device=DEV), slot_idx=torch.full((T, k), -7, dtype=i32, device=DEV),
             gate_w=torch.full((T, k), -7.0, dtype=torch.float32, device=DEV),
             expert_rows=torch.full((E,), -7, dtype=i32, device=DEV), slot_token=torch.full((E, C), -7, dtype=i32, device=DEV))
    for rep in range(2):            # twice on one workspace: nothing may depend on what the previous call left
        m.moe_gate(shape, x, Wg, bg, logits, r["expert_idx"], r["slot_idx"], r["gate_w"], r["expert_rows"],
                   r["slot_token"], ws)
    torch.cuda.synchronize()
    lg = logits.cpu().numpy()
    ref_l = orc.gate_logits(x.float().cpu().numpy(), Wg.cpu().numpy(), None if bg is None else bg.cpu().numpy())
    err = np.max(np.abs(lg.astype(np.float64) - ref_l))
    assert err <= U.LOGIT_RTOL * np.max(np.abs(ref_l)), err
    if dup:                         # the tie is exact on the GPU too, and the lower index wins
        assert np.array_equal(lg[:, E - 1], lg[:, 1]) and np.array_equal(lg[:, E // 2], lg[:, 0])
    U.assert_routing_equal(r, orc.gate(lg, k, C))     # routing bit-exact on the GPU's own fp32 logits
    packed = m.moe_pack_gate(Wg) if dtype == "bf16" else None
    if packed is not None:          # the same call on gate weights split once beforehand: identical bits everywhere
        pshape = m.make_shape(T, d, 8, E, k, C, dtype, flags=m.MOE_FLAG_PACKED_GATE)
        logits2 = torch.full((T, E), 7.0, dtype=torch.float32, device=DEV)
        r2 = {n: torch.full_like(v, -7) for n, v in r.items()}
        m.moe_gate(pshape, x, packed, bg, logits2, r2["expert_idx"], r2["slot_idx"], r2["gate_w"], r2["expert_rows"],
                   r2["slot_token"], ws)
        torch.cuda.synchronize()
        assert torch.equal(logits2, logits)
        for n in r:
            assert torch.equal(r2[n], r[n]), n


# ------------------------------------------------------------------ dispatch / ffn / combine

def _routing_on_device(ref, dev=DEV):
    return {k: torch.from_numpy(np.ascontiguousarray(ref[k])).to(dev) for k in
            ("expert_idx", "slot_idx", "expert_rows", "slot_token")}


@pytest.mark.parametrize("dtype,T,d,E,k,C", [("f32", 256, 64, 8, 1, 32), ("bf16", 1000, 1024, 16, 2, 70),
                                             ("bf16", 64, 2048, 128, 1, 1), ("bf16", 300, 264, 5, 2, 1000)])
def test_dispatch_exact_and_combine(dtype, T, d, E, k, C):
    m = U.amd()
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=DEV).manual_seed(T)
    x = torch.randn((T, d), generator=g, device=DEV).to(tdt)
    ref = orc.gate(make_logits(T, E, seed=T, kind="zipf").numpy(), k, C)
    r = _routing_on_device(ref)
    shape = m.make_shape(T, d, 8, E, k, C, dtype)
    canary = 123.0
    xe = torch.full((E, C, d), canary, dtype=tdt, device=DEV)
    m.moe_dispatch(shape, x, r["slot_token"], r["expert_rows"], xe)
    torch.cuda.synchronize()
    xe_ref = orc.dispatch(x.float().cpu().numpy(), ref["slot_token"])
    xe_h = xe.float().cpu().numpy()
    filled = ref["slot_token"] >= 0
    assert np.array_equal(xe_h[filled], xe_ref[filled].astype(np.float32))         # data movement: exact
    assert np.all(xe_h[~filled] == canary)                                          # untouched rows stay untouched
    # combine on a random ye, with and without addend
    ye = torch.randn((E, C, d), generator=g, device=DEV).to(tdt)
    gw = torch.rand((T, k), generator=g, device=DEV)
    addend = torch.randn((T, d), generator=g, device=DEV).to(tdt)
    for add in (None, addend):
        out = torch.empty((T, d), dtype=tdt, device=DEV)
        m.moe_combine(shape, ye, r["expert_idx"], r["slot_idx"], gw, add, out)
        torch.cuda.synchronize()
        oref = orc.combine(ye.float().cpu().numpy(), ref["expert_idx"], ref["slot_idx"],
                           gw.cpu().numpy().astype(np.float64), None if add is None else add.float().cpu().numpy())
        U.assert_close(out, oref, dtype, "combine")
        drop = np.all(ref["slot_idx"] < 0, axis=1)
        if drop.any():
            expect = np.zeros((int(drop.sum()), d), np.float32) if add is None else add.float().cpu().numpy()[drop]
            assert np.array_equal(out.float().cpu().numpy()[drop], expect)


@pytest.mark.parametrize("dtype,d,f,E,C,bias", [("f32", 64, 256, 8, 32, True), ("bf16", 256, 1024, 6, 70, True),
                                                ("bf16", 1024, 4096, 4, 64, False), ("bf16", 2048, 8192, 6, 1, True),
                                                ("bf16", 264, 520, 3, 130, True), ("bf16", 288, 544, 9, 300, True),
                                                ("bf16", 512, 96, 8, 100, False),
                                                # many groups, few output columns in the second product: 256 x 128 tiles
                                                ("bf16", 1024, 128, 32, 200, True), ("bf16", 1000, 160, 33, 250, True)])
def test_expert_ffn(dtype, d, f, E, C, bias):
    _check_expert_ffn(dtype, d, f, E, C, bias, None)
    if dtype == "bf16":
        _check_expert_ffn(dtype, d, f, E, C, bias, None, pack=True)


def test_expert_ffn_unequal_experts():
    """Two full experts among nearly empty ones (and a group count that is not a multiple of 8): the tiled kernel
    deals the column tiles of every expert over the XCDs instead of whole experts."""
    for pack in (False, True):
        _check_expert_ffn("bf16", 256, 2048, 9, 300, True, [300, 3, 2, 1, 280, 5, 0, 2, 1], pack=pack)
        _check_expert_ffn("bf16", 128, 4096, 16, 200, False, [200, 1, 1, 0, 2, 1, 150, 1, 3, 1, 0, 1, 2, 1, 1, 70], pack=pack)


@pytest.mark.parametrize("dtype,d,f,E,C", [("f32", 64, 256, 4, 40), ("bf16", 64, 256, 4, 40), ("bf16", 128, 512, 3, 150)])
def test_expert_ffn_saturating_gelu(dtype, d, f, E, C):
    """Pre-activations far into both tails of the tanh-GELU (|z| up to about 40): the kernels evaluate it as
    z / (1 + exp2(.)), whose exponential overflows to infinity for z << 0 and underflows for z >> 0; the result must
    still be the oracle's (-0 and z)."""
    _check_expert_ffn(dtype, d, f, E, C, True, None, w1_std=1.0, b1_std=5.0)
    if dtype == "bf16":
        _check_expert_ffn(dtype, d, f, E, C, True, None, w1_std=1.0, b1_std=5.0, pack=True)


@pytest.mark.parametrize("d,f,E,C,cuts,pack", [(256, 1024, 6, 70, (0, 384, 1024), False), (256, 1024, 6, 70, (0, 512, 1024), True),
                                               (512, 768, 5, 40, (0, 256, 512, 768), False), (2048, 1024, 9, 3, (0, 640, 1024), True),
                                               (264, 520, 4, 150, (0, 200, 520), False)])
def test_expert_ffn_slices_sum_to_the_expert(d, f, E, C, cuts, pack):
    """Expert-slicing on one device: every slice of the inner dimension gives an fp32 partial output; their sum in
    slice order plus b2 is the expert FFN of the oracle."""
    m = U.amd()
    tdt = torch.bfloat16
    g = torch.Generator(device=DEV).manual_seed(d + f + C)
    rows = torch.randint(0, C + 1, (E,), generator=g, device=DEV).to(torch.int32)
    rows[0], rows[1] = C, 0
    xe = torch.randn((E, C, d), generator=g, device=DEV).to(tdt)
    W1 = (0.02 * torch.randn((E, d, f), generator=g, device=DEV)).to(tdt)
    W2 = (0.02 * torch.randn((E, f, d), generator=g, device=DEV)).to(tdt)
    b1 = (0.1 * torch.randn((E, f), generator=g, device=DEV)).to(tdt)
    b2 = (0.1 * torch.randn((E, d), generator=g, device=DEV)).to(tdt)
    n = len(cuts) - 1
    canary = 99.0
    partials = torch.full((n, E, C, d), canary, dtype=torch.float32, device=DEV)
    for s_ in range(n):
        f0, f1 = cuts[s_], cuts[s_ + 1]
        print(f"slice {s_}: columns {f0}..{f1}", flush=True)
        shape = m.make_shape(8, d, f1 - f0, E, 1, C, "bf16", flags=m.MOE_FLAG_PACKED_WEIGHTS if pack else 0)
        ws = m.alloc_workspace(shape, DEV)
        W1s, W2s = W1[:, :, f0:f1].contiguous(), W2[:, f0:f1, :].contiguous()
        if pack:
            W1s, W2s = m.moe_pack_weights(W1s), m.moe_pack_weights(W2s)
        m.moe_expert_ffn_slice(shape, xe, rows, W1s, b1[:, f0:f1].contiguous(), W2s, partials[s_], ws)
    shape = m.make_shape(8, d, f, E, 1, C, "bf16")
    ye = torch.full((E, C, d), 77.0, dtype=tdt, device=DEV)
    m.moe_expert_ffn_slice_reduce(shape, n, partials, rows, b2, ye)
    torch.cuda.synchronize()
    f32 = lambda t: t.float().cpu().numpy()
    rows_h = rows.cpu().numpy()
    ref = orc.expert_ffn(f32(xe).astype(np.float64), rows_h, f32(W1), f32(b1), f32(W2), f32(b2))
    valid = np.arange(C)[None, :] < rows_h[:, None]
    ye_h, ph = f32(ye), partials.cpu().numpy()
    assert np.all(ye_h[~valid] == 77.0) and np.all(ph[:, ~valid] == canary)
    scale = np.max(np.abs(ref[valid]))
    assert np.max(np.abs(ye_h[valid] - ref[valid])) <= U.TOL["bf16"] * scale
    # the partials themselves: their fp64 sum plus b2 is the reference before any bf16 rounding of the output
    total = ph.astype(np.float64).sum(axis=0) + f32(b2).astype(np.float64)[:, None, :]
    assert np.max(np.abs(total[valid] - ref[valid])) <= U.TOL["bf16"] * scale


def _check_expert_ffn(dtype, d, f, E, C, bias, fixed_rows, w1_std=0.02, b1_std=0.1, pack=False):
    m = U.amd()
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=DEV).manual_seed(d + f)
    rows = torch.randint(0, C + 1, (E,), generator=g, device=DEV).to(torch.int32)
    rows[0] = C
    if E > 2:
        rows[1] = 0
    if fixed_rows is not None:
        rows = torch.tensor(fixed_rows, dtype=torch.int32, device=DEV)
    xe = torch.randn((E, C, d), generator=g, device=DEV).to(tdt)
    W1 = (w1_std * torch.randn((E, d, f), generator=g, device=DEV)).to(tdt)
    W2 = (0.02 * torch.randn((E, f, d), generator=g, device=DEV)).to(tdt)
    b1 = (b1_std * torch.randn((E, f), generator=g, device=DEV)).to(tdt) if bias else None
    b2 = (0.1 * torch.randn((E, d), generator=g, device=DEV)).to(tdt) if bias else None
    shape = m.make_shape(8, d, f, E, 1, C, dtype, flags=m.MOE_FLAG_PACKED_WEIGHTS if pack else 0)
    ws = m.alloc_workspace(shape, DEV)
    canary = 77.0
    ye = torch.full((E, C, d), canary, dtype=tdt, device=DEV)
    if pack:
        m.moe_expert_ffn(shape, xe, rows, m.moe_pack_weights(W1), b1, m.moe_pack_weights(W2), b2, ye, ws)
    else:
        m.moe_expert_ffn(shape, xe, rows, W1, b1, W2, b2, ye, ws)
    torch.cuda.synchronize()
    f32 = lambda t: None if t is None else t.float().cpu().numpy()
    rows_h = rows.cpu().numpy()
    ref = orc.expert_ffn(f32(xe).astype(np.float64), rows_h, f32(W1), f32(b1), f32(W2), f32(b2))
    ye_h = ye.float().cpu().numpy()
    valid = np.arange(C)[None, :] < rows_h[:, None]
    assert np.all(ye_h[~valid] == canary)
    scale = np.max(np.abs(ref[valid]))
    assert np.max(np.abs(ye_h[valid] - ref[valid])) <= U.TOL[dtype] * scale


# ------------------------------------------------------------------ whole layer

def test_layer_c1_full():
    stats = U.check_layer(make_inputs(CONFIGS["c1"], DEV, bias_std=0.0))
    print("c1", stats, flush=True)
    assert stats["dropped_tokens"] > 0


def test_layer_c1_with_biases():
    U.check_layer(make_inputs(CONFIGS["c1"], DEV, bias_std=0.05))


REDUCED = {
    # same structure as the full configurations, fewer experts/tokens so the fp64 oracle stays fast
    "c2r": CONFIGS["c2"].scaled(name="c2r", T=1000, E=16, capacity_factor=1.0),
    "c3r": CONFIGS["c3a"].scaled(name="c3r", T=900, E=8, d_ffn=2048),
    # Residual-MoE whose expert and dense products pair up on 256 x 128 tiles (48 row tiles of 256: too few for 256 x 256)
    "c3p": CONFIGS["c3a"].scaled(name="c3p", T=4100, E=16, d_ffn=2048),
    "c4r": CONFIGS["c4"].scaled(name="c4r", E=32, d_ffn=4096),
    "c5r": CONFIGS["c5"].scaled(name="c5r", T=1100, E=8, d_model=512, d_ffn=2048),
}


@pytest.mark.parametrize("name", sorted(REDUCED))
@pytest.mark.parametrize("bias_std", [0.0, 0.05])
def test_layer_reduced(name, bias_std):
    print(f"case {name} bias_std={bias_std}", flush=True)
    stats = U.check_layer(make_inputs(REDUCED[name], DEV, bias_std=bias_std))
    print(name, stats, flush=True)


# >= 2048 bf16 tokens: the layer's gate runs as the fused kernel (logits + top-k + tile ranks); narrow models keep
# the fp64 oracle fast
WIDE = {
    "c2w": CONFIGS["c2"].scaled(name="c2w", T=2500, d_model=128, d_ffn=256, E=40, capacity_factor=1.0),
    "c3w": CONFIGS["c3a"].scaled(name="c3w", T=2100, d_model=64, d_ffn=128, E=16),
    "c5w": CONFIGS["c5"].scaled(name="c5w", T=2300, d_model=96, d_ffn=160, E=24),
    "c5x": CONFIGS["c5"].scaled(name="c5x", T=16400, d_model=32, d_ffn=64, E=8),
}


@pytest.mark.parametrize("name", sorted(WIDE))
def test_layer_fused_gate(name):
    print(f"case {name}", flush=True)
    stats = U.check_layer(make_inputs(WIDE[name], DEV, bias_std=0.05))
    print(name, stats, flush=True)


def test_layer_ragged_sizes():
    cfg = CONFIGS["c2"].scaled(name="ragged", T=333, d_model=264, d_ffn=520, E=5, top_k=2, capacity_factor=0.9)
    U.check_layer(make_inputs(cfg, DEV, bias_std=0.05))


def test_layer_single_expert_is_dense_ffn():
    cfg = CONFIGS["c2"].scaled(name="e1", T=200, d_model=256, d_ffn=512, E=1, capacity_factor=1.0)
    stats = U.check_layer(make_inputs(cfg, DEV, bias_std=0.05))
    assert stats["dropped_tokens"] == 0


@pytest.mark.parametrize("top_k", [1, 2])
def test_layer_no_drop_mode(top_k):
    """Capacity large enough for every choice of every token (C = T): nothing is dropped, whatever the skew."""
    cfg = CONFIGS["c5"].scaled(name="nodrop", T=300, E=6, d_model=256, d_ffn=512, top_k=top_k, capacity_factor=6.0 / top_k)
    assert cfg.capacity == cfg.T
    stats = U.check_layer(make_inputs(cfg, DEV, bias_std=0.05))
    assert stats["dropped_tokens"] == 0 and stats["kept"] == cfg.T * top_k


def test_layer_deterministic():
    inp = make_inputs(REDUCED["c5r"], DEV)
    a = U.gpu_forward(inp)["out"].clone()
    b = U.gpu_forward(inp)["out"].clone()
    assert torch.equal(a, b)


def test_residual_with_zero_experts_equals_dense_branch():
    cfg = REDUCED["c3r"]
    inp = make_inputs(cfg, DEV, bias_std=0.05)
    for t in (inp.W1, inp.b1, inp.W2, inp.b2):
        t.zero_()
    res = U.gpu_forward(inp)
    h = U.host(inp)
    ref = orc.ffn(h["x"], h["Wd1"], h["bd1"], h["Wd2"], h["bd2"])
    U.assert_close(res["out"], ref, cfg.dtype)


# ------------------------------------------------------------------ full sizes, as benchmarked

@pytest.mark.parametrize("name", ["c2", "c3a", "c3b", "c4", "c5"])
def test_layer_full_size(name):
    """The five benchmark workloads at full size, in the launch configuration bench.py times: routing bit for bit,
    every output element against the oracle (expert weights widened one expert at a time on the host; config 5
    holds 17 GB of them, of which the oracle touches the experts that have rows)."""
    print(f"case full {name}", flush=True)
    stats = U.check_layer(make_inputs(CONFIGS[name], DEV), lazy_experts=True)
    print(name, stats, flush=True)
    assert stats["kept"] > 0
    if name == "c5":
        assert stats["dropped_tokens"] > 0


def test_stage_timing_api():
    """moe_profile_*: events around selected stages of moe_layer_forward give positive times."""
    m = U.amd()
    inp = make_inputs(REDUCED["c2r"], DEV)
    cfg = inp.cfg
    layer = m.MoELayer(cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, cfg.capacity, cfg.dtype, inp.Wg, inp.bg, inp.W1,
                       inp.b1, inp.W2, inp.b2)
    names = m.moe_profile_stage_names()
    try:
        m.moe_profile_select(None)
        m.moe_profile_enable(3)
        for _ in range(4):                       # one call more than there are slots: silently untimed
            layer(inp.x)
        torch.cuda.synchronize()
        assert m.moe_profile_calls() == 3
        ms = dict(zip(names, m.moe_profile_elapsed(2)))
        for n in ("gate_logits", "gate_route", "expert_gemm1", "expert_gemm2"):
            assert 0.0 < ms[n] < 50.0, (n, ms)
        assert ms["dense_gemm1"] == 0.0
        m.moe_profile_enable(0)
        m.moe_profile_select(["expert_gemm1"])
        m.moe_profile_enable(1)
        layer(inp.x)
        torch.cuda.synchronize()
        ms = dict(zip(names, m.moe_profile_elapsed(0)))
        assert ms["expert_gemm1"] > 0.0 and ms["expert_gemm2"] == 0.0 and ms["gate_logits"] == 0.0
        m.moe_profile_enable(0)
        m.moe_profile_stride(3)                  # calls 0, 3, 6 of the next seven are timed
        m.moe_profile_enable(5)
        for _ in range(7):
            layer(inp.x)
        torch.cuda.synchronize()
        assert m.moe_profile_calls() == 3
        assert dict(zip(names, m.moe_profile_elapsed(2)))["expert_gemm1"] > 0.0
    finally:
        m.moe_profile_enable(0)
        m.moe_profile_select(None)
        m.moe_profile_stride(1)
