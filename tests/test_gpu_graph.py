"""moe_layer_forward under HIP graph capture: the library only enqueues kernels on the caller's stream (no
allocation, no synchronisation, no memset), so a captured call must replay to exactly what the eager call gives,
every time and with new tokens in the same buffers.  The decode gate hands its logits over between work-groups
through flags that hold a per-call number: a replay carries the number of the captured call again, which the
kernel has to survive (it puts the flags back after use).  Eager work of the library runs between the replays."""
import pytest
import torch

from tests import gpu_util as U
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda"

# name -> reduced workload: decode gate (at most 256 tokens), fused prefill gate + tiled experts, Residual-MoE with the
# paired launches, skewed top-2 with drops
CASES = {
    "decode": CONFIGS["c4"].scaled(name="g-decode", T=64, d_model=256, d_ffn=512, E=16),
    "decode_top2": CONFIGS["c5"].scaled(name="g-decode2", T=200, d_model=128, d_ffn=256, E=8),
    "prefill": CONFIGS["c2"].scaled(name="g-prefill", T=2304, d_model=256, d_ffn=512, E=8),
    "residual": CONFIGS["c3a"].scaled(name="g-residual", T=2304, d_model=256, d_ffn=512, E=8),
    "skewed_top2": CONFIGS["c5"].scaled(name="g-skew", T=2200, d_model=128, d_ffn=256, E=16),
}


@pytest.mark.parametrize("case", sorted(CASES))
@pytest.mark.parametrize("pack", [False, True])
def test_layer_forward_replays_like_eager(case, pack):
    print(f"case {case} pack={pack}", flush=True)
    m = U.amd()
    cfg = CASES[case]
    inp = make_inputs(cfg, device=DEV)
    args = (cfg.T, cfg.d_model, cfg.d_ffn, cfg.E, cfg.top_k, cfg.capacity, cfg.dtype, inp.Wg, inp.bg, inp.W1, inp.b1,
            inp.W2, inp.b2, inp.Wd1, inp.bd1, inp.Wd2, inp.bd2)
    eager = m.MoELayer(*args, pack_weights=pack)
    graphed = m.MoELayer(*args, pack_weights=pack)
    g = torch.Generator(device=DEV).manual_seed(17)
    xs = [inp.x] + [torch.randn(inp.x.shape, generator=g, device=DEV).to(inp.x.dtype) for _ in range(3)]
    x_static = xs[0].clone()

    side = torch.cuda.Stream()                       # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graphed(x_static)                            # kernel attributes and occupancy are looked up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        graphed(x_static)
    torch.cuda.synchronize()

    for i, x in enumerate(xs + xs[:2]):              # six replays, the first tokens again at the end
        x_static.copy_(x)
        graph.replay()
        torch.cuda.synchronize()
        want = eager(x).clone()                      # the library's eager work between two replays
        torch.cuda.synchronize()
        assert torch.equal(graphed.out, want), f"replay {i}: output differs from the eager call"
        for name in ("logits", "expert_idx", "slot_idx", "gate_w", "expert_rows", "slot_token"):
            assert torch.equal(graphed.routing[name], eager.routing[name]), f"replay {i}: {name}"


@pytest.mark.parametrize("pack", [False, True])
def test_decode_block_replays_like_eager(pack):
    """One decode step of the whole block, captured: twelve launches per replay, the decode gate among them.  A replay
    writes the same key/value rows into the cache again (same positions), so cache and outputs must equal the eager
    call's bit for bit."""
    from workloads import make_block_inputs
    m = U.amd()
    cfg = CONFIGS["c4"].scaled(name="g-block", T=48, d_model=256, d_ffn=512, E=16)
    bi = make_block_inputs(cfg, n_heads=4, max_len=600, device=DEV, pos_mode="mixed")
    lay = bi.layer
    T, d, E = cfg.T, cfg.d_model, cfg.E
    shape = m.make_shape(T, d, cfg.d_ffn, E, cfg.top_k, cfg.capacity, "bf16",
                         flags=m.MOE_FLAG_PACKED_WEIGHTS if pack else 0)
    block = m.MoeBlockShape(bi.n_heads, bi.max_len)
    pk = (lambda w: m.moe_pack_weights(w)) if pack else (lambda w: w)
    weights = dict(ln1_gamma=bi.ln1_gamma, ln1_beta=bi.ln1_beta, Wqkv=bi.Wqkv, bqkv=bi.bqkv, Wo=bi.Wo, bo=bi.bo,
                   ln2_gamma=bi.ln2_gamma, ln2_beta=bi.ln2_beta, Wg=lay.Wg, bg=lay.bg, W1=pk(lay.W1), b1=lay.b1,
                   W2=pk(lay.W2), b2=lay.b2)

    def buffers():
        bf = torch.bfloat16
        return dict(ws=torch.empty(m.moe_decode_block_workspace_bytes(shape, block), dtype=torch.uint8, device=DEV),
                    out=torch.empty((T, d), dtype=bf, device=DEV), x1=torch.empty((T, d), dtype=bf, device=DEV),
                    moe_in=torch.empty((T, d), dtype=bf, device=DEV),
                    logits=torch.empty((T, E), dtype=torch.float32, device=DEV),
                    kc=bi.k_cache.clone(), vc=bi.v_cache.clone())

    def run(b, x):
        m.moe_decode_block_forward(shape, block, weights, x, b["kc"], b["vc"], bi.pos, b["out"], b["x1"], b["moe_in"],
                                   b["logits"], b["ws"])

    e, g_ = buffers(), buffers()
    gen = torch.Generator(device=DEV).manual_seed(5)
    xs = [lay.x] + [torch.randn(lay.x.shape, generator=gen, device=DEV).to(lay.x.dtype) for _ in range(2)]
    x_static = xs[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(g_, x_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(g_, x_static)
    torch.cuda.synchronize()
    for i, x in enumerate(xs + xs[:1]):
        print(f"block replay {i} pack={pack}", flush=True)
        x_static.copy_(x)
        graph.replay()
        torch.cuda.synchronize()
        run(e, x)
        torch.cuda.synchronize()
        for name in ("out", "x1", "moe_in", "logits", "kc", "vc"):
            assert torch.equal(g_[name], e[name]), f"replay {i}: {name}"
