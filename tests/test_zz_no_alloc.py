"""moe_gate_noalloc (the entry point for callers that cannot allocate: scratch in a fixed array inside the
library) against moe_gate (scratch in the caller's workspace): same kernels, so every result must be identical,
on two calls in a row, the second with a smaller input."""
import pytest
import torch

from tests import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _outputs(T, E, k, C):
    i32 = torch.int32
    return dict(logits=torch.full((T, E), 7.0, dtype=torch.float32, device=DEV),
                expert_idx=torch.full((T, k), -7, dtype=i32, device=DEV),
                slot_idx=torch.full((T, k), -7, dtype=i32, device=DEV),
                gate_w=torch.full((T, k), -7.0, dtype=torch.float32, device=DEV),
                expert_rows=torch.full((E,), -7, dtype=i32, device=DEV),
                slot_token=torch.full((E, C), -7, dtype=i32, device=DEV))


def _both(m, dtype, T, d, E, k, C, seed, export_logits):
    g = torch.Generator(device=DEV).manual_seed(seed)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.randn((T, d), generator=g, device=DEV).to(tdt)
    Wg = 0.05 * torch.randn((d, E), generator=g, device=DEV)
    bg = 0.3 * torch.randn((E,), generator=g, device=DEV)
    shape = m.make_shape(T, d, 8, E, k, C, dtype)
    assert 0 < m.moe_gate_noalloc_bytes(shape) <= m.moe_gate_noalloc_max_bytes()
    ws = m.alloc_workspace(shape, DEV)
    a, b = _outputs(T, E, k, C), _outputs(T, E, k, C)
    la = a["logits"] if export_logits else None
    lb = b["logits"] if export_logits else None
    m.moe_gate(shape, x, Wg, bg, la, a["expert_idx"], a["slot_idx"], a["gate_w"], a["expert_rows"], a["slot_token"], ws)
    m.moe_gate_noalloc(shape, x, Wg, bg, lb, b["expert_idx"], b["slot_idx"], b["gate_w"], b["expert_rows"],
                       b["slot_token"])
    torch.cuda.synchronize()
    for n in a:
        assert torch.equal(a[n], b[n]), (n, T, E, k)
    assert int(a["expert_rows"].sum()) > 0


def test_gate_noalloc_matches_gate_twice():
    m = U.amd()
    print("case noalloc large bf16 T=4096 E=64 k=2", flush=True)
    _both(m, "bf16", 4096, 256, 64, 2, 150, seed=1, export_logits=False)     # fused kernel, logits kept in the scratch
    print("case noalloc small bf16 T=300 E=24 k=1", flush=True)
    _both(m, "bf16", 300, 128, 24, 1, 20, seed=2, export_logits=True)        # smaller: few-token path on the same array
    print("case noalloc small f32 T=77 E=5 k=2", flush=True)
    _both(m, "f32", 77, 100, 5, 2, 40, seed=3, export_logits=False)


def test_gate_noalloc_rejects_shapes_beyond_its_scratch():
    m = U.amd()
    T, E = 65536, 128                                                         # 32 MiB of logits alone
    shape = m.make_shape(T, 64, 8, E, 1, 4, "bf16")
    assert m.moe_gate_noalloc_bytes(shape) > m.moe_gate_noalloc_max_bytes()
    i32 = torch.int32
    outs = [torch.empty((T, 1), dtype=i32, device=DEV), torch.empty((T, 1), dtype=i32, device=DEV),
            torch.empty((T, 1), dtype=torch.float32, device=DEV), torch.empty((E,), dtype=i32, device=DEV),
            torch.empty((E, 4), dtype=i32, device=DEV)]
    x = torch.zeros((T, 64), dtype=torch.bfloat16, device=DEV)
    Wg = torch.zeros((64, E), dtype=torch.float32, device=DEV)
    with pytest.raises(m.MoeError) as ei:
        m.moe_gate_noalloc(shape, x, Wg, None, None, *outs)
    assert ei.value.status == -5
