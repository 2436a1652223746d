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
