"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, sizes its workspace sanely, and rejects bad
arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2201_05596_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = _declared()
    assert set(names) == set(B.ENTRY_POINTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    lib = B.load_library()
    assert B.moe_version() == "0.2"
    assert lib.moe_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, 99):
        assert len(lib.moe_status_string(code)) > 0


def test_workspace_bytes():
    s = B.make_shape(8192, 1024, 4096, 128, 1, 64, "bf16")
    n = B.moe_workspace_bytes(s)
    # at least logits + h + ye
    assert n >= 8192 * 128 * 4 + 128 * 64 * (1024 + 4096) * 2
    assert n % 256 == 0
    r = B.make_shape(8192, 1024, 4096, 32, 1, 256, "bf16", residual=True)
    assert B.moe_workspace_bytes(r) > B.moe_workspace_bytes(B.make_shape(8192, 1024, 4096, 32, 1, 256, "bf16"))
    assert B.moe_workspace_bytes(B.make_shape(0, 1024, 4096, 128, 1, 64, "bf16")) == 0


BAD_SHAPES = [
    (dict(T=0), -1), (dict(E=0), -1), (dict(capacity=0), -1), (dict(top_k=0), -1), (dict(top_k=200), -1),
    (dict(dtype=5), -1), (dict(residual=2), -1), (dict(flags=4), -1), (dict(flags=1, dtype=0), -2), (dict(flags=2, dtype=0), -2), (dict(flags=2, E=200), -2),
    (dict(top_k=3), -2), (dict(E=2048), -2), (dict(d_model=1028), -2), (dict(d_ffn=4100), -2),
]


@pytest.mark.parametrize("patch,code", BAD_SHAPES)
def test_bad_shapes_rejected_without_launch(patch, code):
    lib = B.load_library()
    base = dict(T=8192, d_model=1024, d_ffn=4096, E=128, top_k=1, capacity=64, dtype=1, residual=0, flags=0)
    base.update(patch)
    s = B.MoeShape(**base)
    fake = 0x1000          # aligned, never dereferenced: the call must fail before any launch
    assert lib.moe_gate(ctypes.byref(s), *([fake] * 9), fake, 1 << 40, None) == code
    assert lib.moe_dispatch(ctypes.byref(s), fake, fake, fake, fake, None) == code
    assert lib.moe_expert_ffn(ctypes.byref(s), *([fake] * 7), fake, 1 << 40, None) == code
    assert lib.moe_combine(ctypes.byref(s), *([fake] * 6), None) == code
    assert lib.moe_layer_forward(ctypes.byref(s), *([fake] * 18), fake, 1 << 40, None) == code


def test_null_misaligned_and_short_workspace():
    lib = B.load_library()
    s = B.make_shape(256, 64, 256, 8, 1, 32, "f32")
    fake, odd = 0x1000, 0x1004
    need = B.moe_workspace_bytes(s)
    assert lib.moe_gate(None, *([fake] * 9), fake, need, None) == -1
    assert lib.moe_gate(ctypes.byref(s), fake, fake, None, fake, None, fake, fake, fake, fake, fake, need, None) == -1
    assert lib.moe_gate(ctypes.byref(s), None, None, None, None, fake, fake, fake, fake, fake, fake, need, None) == -1
    assert lib.moe_gate(ctypes.byref(s), odd, *([fake] * 8), fake, need, None) == -1
    assert lib.moe_gate(ctypes.byref(s), *([fake] * 9), fake, need - 1, None) == -3
    assert lib.moe_gate(ctypes.byref(s), *([fake] * 9), None, need, None) == -3
    assert lib.moe_expert_ffn(ctypes.byref(s), *([fake] * 7), fake, 16, None) == -3
    assert lib.moe_combine(ctypes.byref(s), fake, fake, fake, fake, odd, fake, None) == -1
    # dense-branch weights must come with residual = 1 and only then
    assert lib.moe_layer_forward(ctypes.byref(s), *([fake] * 7), fake, None, fake, None, *([fake] * 7), fake, need, None) == -1
    r = B.make_shape(256, 64, 256, 8, 1, 32, "f32", residual=True)
    args = [fake] * 7 + [None, None, None, None] + [fake] * 7
    assert lib.moe_layer_forward(ctypes.byref(r), *args, fake, B.moe_workspace_bytes(r), None) == -1


def test_binding_refuses_host_tensors():
    import torch
    s = B.make_shape(4, 8, 8, 2, 1, 2, "f32")
    x = torch.zeros((4, 8))
    with pytest.raises(ValueError):
        B.moe_dispatch(s, x, x, x, x)


class _FakeDeviceTensor:
    """Stands in for a CUDA tensor so that the binding's argument checks can run without a GPU."""

    def __init__(self, numel, dtype, contiguous=True):
        import torch
        self._n, self.dtype, self._c, self.is_cuda = numel, dtype, contiguous, True
        self._torch = torch

    def is_contiguous(self):
        return self._c

    def numel(self):
        return self._n

    def element_size(self):
        return {self._torch.float32: 4, self._torch.int32: 4, self._torch.bfloat16: 2, self._torch.uint8: 1}[self.dtype]

    def data_ptr(self):
        return 0x1000


def test_binding_checks_element_counts_before_calling_the_library():
    """A buffer sized for another shape must be refused on the host: the kernels index by T/E/C/d/f."""
    import torch
    s = B.make_shape(64, 256, 512, 8, 1, 16, "bf16")
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    ok = dict(x=_FakeDeviceTensor(64 * 256, bf), slot_token=_FakeDeviceTensor(8 * 16, i32),
              expert_rows=_FakeDeviceTensor(8, i32), xe=_FakeDeviceTensor(8 * 16 * 256, bf))
    for bad_name, bad in (("slot_token", _FakeDeviceTensor(8 * 32, i32)),       # a table built for another capacity
                          ("xe", _FakeDeviceTensor(8 * 16 * 128, bf)), ("x", _FakeDeviceTensor(64 * 256, f32)),
                          ("expert_rows", _FakeDeviceTensor(8, i32, contiguous=False))):
        args = dict(ok)
        args[bad_name] = bad
        with pytest.raises(ValueError, match=bad_name):
            B.moe_dispatch(s, args["x"], args["slot_token"], args["expert_rows"], args["xe"])
    # a workspace allocated for a smaller shape
    small = B.moe_workspace_bytes(B.make_shape(8, 256, 512, 8, 1, 2, "bf16"))
    assert small < B.moe_workspace_bytes(s)
    with pytest.raises(ValueError, match="workspace"):
        B.moe_expert_ffn(s, _FakeDeviceTensor(8 * 16 * 256, bf), ok["expert_rows"], _FakeDeviceTensor(8 * 256 * 512, bf), None,
                         _FakeDeviceTensor(8 * 512 * 256, bf), None, _FakeDeviceTensor(8 * 16 * 256, bf),
                         _FakeDeviceTensor(small, torch.uint8))
    # packed weights have their own element count
    sp = B.make_shape(64, 256, 520, 8, 1, 16, "bf16", flags=B.MOE_FLAG_PACKED_WEIGHTS)
    assert B._w(sp, 8, 256, 520) == 8 * 8 * 5 * 4096 and B._w(s, 8, 256, 512) == 8 * 256 * 512
