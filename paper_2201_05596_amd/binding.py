"""ctypes binding of libmoe_hip.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point
declared in include/moe.h and does nothing but check tensor device, dtype and
contiguity, and pass raw device pointers plus the current HIP stream.  PyTorch
is used for device memory and streams only; every step of the layer runs in the
library's kernels.  There is no fallback: if the shared library is missing, or
a call returns a non-zero status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_OK = 0
MOE_FLAG_PACKED_WEIGHTS = 1
MOE_FLAG_PACKED_GATE = 2
ENTRY_POINTS = ("moe_workspace_bytes", "moe_status_string", "moe_version", "moe_packed_weights_bytes",
                "moe_pack_weights", "moe_packed_gate_bytes", "moe_pack_gate", "moe_gate", "moe_gate_noalloc",
                "moe_gate_noalloc_bytes", "moe_gate_noalloc_max_bytes", "moe_dispatch",
                "moe_expert_ffn", "moe_expert_ffn_slice", "moe_expert_ffn_slice_reduce", "moe_combine", "moe_layer_forward", "moe_decode_block_workspace_bytes",
                "moe_decode_block_forward", "moe_profile_enable", "moe_profile_select",
                "moe_profile_stride", "moe_profile_calls",
                "moe_profile_stage_count", "moe_profile_stage_name", "moe_profile_elapsed")


class MoeShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "d_model", "d_ffn", "E", "top_k", "capacity", "dtype", "residual", "flags")]


class MoeBlockShape(ctypes.Structure):
    _fields_ = [("n_heads", ctypes.c_int32), ("max_len", ctypes.c_int32)]


BLOCK_WEIGHT_FIELDS = ("ln1_gamma", "ln1_beta", "Wqkv", "bqkv", "Wo", "bo", "ln2_gamma", "ln2_beta", "Wg", "bg",
                       "W1", "b1", "W2", "b2", "Wd1", "bd1", "Wd2", "bd2")


class MoeBlockWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in BLOCK_WEIGHT_FIELDS]


class MoeError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed: status {status} ({text})")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmoe_hip.so (built by ``python -m paper_2201_05596_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2201_05596_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, st = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sp = ctypes.POINTER(MoeShape)
    lib.moe_workspace_bytes.restype = st
    lib.moe_workspace_bytes.argtypes = [sp]
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [i32]
    lib.moe_version.restype = ctypes.c_char_p
    lib.moe_version.argtypes = []
    lib.moe_packed_weights_bytes.restype = st
    lib.moe_packed_weights_bytes.argtypes = [i32, i32, i32]
    lib.moe_pack_weights.restype = i32
    lib.moe_pack_weights.argtypes = [i32, i32, i32, vp, vp, vp]
    lib.moe_packed_gate_bytes.restype = st
    lib.moe_packed_gate_bytes.argtypes = [i32, i32]
    lib.moe_pack_gate.restype = i32
    lib.moe_pack_gate.argtypes = [i32, i32, vp, vp, vp]
    lib.moe_gate.restype = i32
    lib.moe_gate.argtypes = [sp] + [vp] * 9 + [vp, st, vp]
    lib.moe_gate_noalloc.restype = i32
    lib.moe_gate_noalloc.argtypes = [sp] + [vp] * 9 + [vp]
    lib.moe_gate_noalloc_bytes.restype = st
    lib.moe_gate_noalloc_bytes.argtypes = [sp]
    lib.moe_gate_noalloc_max_bytes.restype = st
    lib.moe_gate_noalloc_max_bytes.argtypes = []
    lib.moe_dispatch.restype = i32
    lib.moe_dispatch.argtypes = [sp] + [vp] * 4 + [vp]
    lib.moe_expert_ffn.restype = i32
    lib.moe_expert_ffn.argtypes = [sp] + [vp] * 7 + [vp, st, vp]
    lib.moe_expert_ffn_slice.restype = i32
    lib.moe_expert_ffn_slice.argtypes = [sp] + [vp] * 6 + [vp, st, vp]
    lib.moe_expert_ffn_slice_reduce.restype = i32
    lib.moe_expert_ffn_slice_reduce.argtypes = [sp, i32] + [vp] * 4 + [vp]
    lib.moe_combine.restype = i32
    lib.moe_combine.argtypes = [sp] + [vp] * 6 + [vp]
    lib.moe_layer_forward.restype = i32
    lib.moe_layer_forward.argtypes = [sp] + [vp] * 18 + [vp, st, vp]
    lib.moe_decode_block_workspace_bytes.restype = st
    lib.moe_decode_block_workspace_bytes.argtypes = [sp, ctypes.POINTER(MoeBlockShape)]
    lib.moe_decode_block_forward.restype = i32
    lib.moe_decode_block_forward.argtypes = [sp, ctypes.POINTER(MoeBlockShape), ctypes.POINTER(MoeBlockWeights)] + \
        [vp] * 8 + [vp, st, vp]
    lib.moe_profile_enable.restype = i32
    lib.moe_profile_enable.argtypes = [i32]
    lib.moe_profile_select.restype = i32
    lib.moe_profile_select.argtypes = [ctypes.c_uint]
    lib.moe_profile_stride.restype = i32
    lib.moe_profile_stride.argtypes = [i32]
    lib.moe_profile_calls.restype = i32
    lib.moe_profile_calls.argtypes = []
    lib.moe_profile_stage_count.restype = i32
    lib.moe_profile_stage_count.argtypes = []
    lib.moe_profile_stage_name.restype = ctypes.c_char_p
    lib.moe_profile_stage_name.argtypes = [i32]
    lib.moe_profile_elapsed.restype = i32
    lib.moe_profile_elapsed.argtypes = [i32, ctypes.POINTER(ctypes.c_float)]
    _lib = lib
    return lib


def make_shape(T: int, d_model: int, d_ffn: int, E: int, top_k: int, capacity: int, dtype, residual: bool = False,
               flags: int = 0) -> MoeShape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: MOE_F32, torch.bfloat16: MOE_BF16}[dtype]
    elif isinstance(dtype, str):
        dtype = {"f32": MOE_F32, "bf16": MOE_BF16}[dtype]
    return MoeShape(T, d_model, d_ffn, E, top_k, capacity, int(dtype), int(bool(residual)), int(flags))


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None, numel: Optional[int] = None,
         name: str = "tensor") -> Optional[int]:
    """Device address of a tensor argument after checking what the C ABI cannot: device, contiguity, dtype and, when
    `numel` is given, the element count (a buffer sized for another shape would be indexed out of bounds on the GPU)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name}: device tensor required")
    if not t.is_contiguous():
        raise ValueError(f"{name}: contiguous tensor required")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: expected {dtype}, got {t.dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name}: expected {numel} elements for this shape, got {t.numel()}")
    return t.data_ptr()


def _ws(shape, ws, need: Optional[int] = None):
    """(address, bytes) of a workspace tensor; `need`: the byte count the call requires (checked here as well)."""
    if ws is None:
        return None, 0
    nbytes = ws.numel() * ws.element_size()
    if need is not None and nbytes < need:
        raise ValueError(f"workspace: {nbytes} bytes, this shape needs {need}")
    return _ptr(ws, name="ws"), nbytes


def _w(shape, G: int, K: int, N: int) -> int:
    """Elements of an FFN weight array [G,K,N]: plain, or as moe_pack_weights lays it out."""
    if shape.flags & MOE_FLAG_PACKED_WEIGHTS:
        return G * ((K + 31) // 32) * ((N + 127) // 128) * 4096
    return G * K * N


def _wg(shape) -> int:
    """float32 elements of the gate weights: plain [d,E], or the buffer moe_pack_gate returns."""
    if shape.flags & MOE_FLAG_PACKED_GATE:
        return (moe_packed_gate_bytes(shape.d_model, shape.E) + 3) // 4
    return shape.d_model * shape.E


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, status: int) -> None:
    if status != MOE_OK:
        raise MoeError(fn, status, load_library().moe_status_string(status).decode())


def _elem(shape: MoeShape) -> torch.dtype:
    return torch.float32 if shape.dtype == MOE_F32 else torch.bfloat16


def moe_workspace_bytes(shape: MoeShape) -> int:
    return int(load_library().moe_workspace_bytes(ctypes.byref(shape)))


def moe_version() -> str:
    return load_library().moe_version().decode()


def alloc_workspace(shape: MoeShape, device="cuda") -> torch.Tensor:
    """Device memory for the `ws` argument (plumbing: torch owns the allocation)."""
    n = moe_workspace_bytes(shape)
    if n == 0:
        raise MoeError("moe_workspace_bytes", -1, "invalid shape")
    return torch.empty(n, dtype=torch.uint8, device=device)


def moe_packed_weights_bytes(G: int, K: int, N: int) -> int:
    return int(load_library().moe_packed_weights_bytes(int(G), int(K), int(N)))


def moe_pack_weights(W: torch.Tensor) -> torch.Tensor:
    """Packed copy of bf16 weights [G,K,N] (or [K,N]) for MOE_FLAG_PACKED_WEIGHTS; torch owns the new buffer."""
    G, K, N = (1, *W.shape) if W.dim() == 2 else W.shape
    nbytes = moe_packed_weights_bytes(G, K, N)
    if nbytes == 0:
        raise MoeError("moe_packed_weights_bytes", -2, "unsupported size")
    packed = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=W.device)
    _check("moe_pack_weights", load_library().moe_pack_weights(G, K, N, _ptr(W, torch.bfloat16), _ptr(packed), _stream()))
    return packed


def moe_packed_gate_bytes(d_model: int, E: int) -> int:
    return int(load_library().moe_packed_gate_bytes(int(d_model), int(E)))


def moe_pack_gate(Wg: torch.Tensor) -> Optional[torch.Tensor]:
    """Packed copy of the float gate weights [d,E] for MOE_FLAG_PACKED_GATE, or None when the shape is not covered.
    The buffer is typed float32 only so that it passes where Wg is expected; its contents are bf16 triples."""
    d, E = Wg.shape
    nbytes = moe_packed_gate_bytes(d, E)
    if nbytes == 0:
        return None
    packed = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=Wg.device)
    _check("moe_pack_gate", load_library().moe_pack_gate(d, E, _ptr(Wg, torch.float32), _ptr(packed), _stream()))
    return packed


def _gate_args(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token):
    i32, f32 = torch.int32, torch.float32
    T, d, E, k, C = shape.T, shape.d_model, shape.E, shape.top_k, shape.capacity
    return (_ptr(x, _elem(shape) if x is not None else None, T * d, "x"),
            _ptr(Wg, f32, _wg(shape) if x is not None else None, "Wg"), _ptr(bg, f32, E, "bg"),
            _ptr(logits, f32, T * E, "logits"), _ptr(expert_idx, i32, T * k, "expert_idx"),
            _ptr(slot_idx, i32, T * k, "slot_idx"), _ptr(gate_w, f32, T * k, "gate_w"),
            _ptr(expert_rows, i32, E, "expert_rows"), _ptr(slot_token, i32, E * C, "slot_token"))


def moe_gate(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token, ws) -> None:
    wsp, wsn = _ws(shape, ws, moe_workspace_bytes(shape))
    rc = load_library().moe_gate(ctypes.byref(shape), *_gate_args(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w,
                                                                 expert_rows, slot_token), wsp, wsn, _stream())
    _check("moe_gate", rc)


def moe_gate_noalloc(shape, x, Wg, bg, logits, expert_idx, slot_idx, gate_w, expert_rows, slot_token) -> None:
    rc = load_library().moe_gate_noalloc(ctypes.byref(shape), *_gate_args(shape, x, Wg, bg, logits, expert_idx, slot_idx,
                                                                         gate_w, expert_rows, slot_token), _stream())
    _check("moe_gate_noalloc", rc)


def moe_gate_noalloc_bytes(shape: MoeShape) -> int:
    return int(load_library().moe_gate_noalloc_bytes(ctypes.byref(shape)))


def moe_gate_noalloc_max_bytes() -> int:
    return int(load_library().moe_gate_noalloc_max_bytes())


def moe_dispatch(shape, x, slot_token, expert_rows, xe) -> None:
    el = _elem(shape)
    T, d, E, C = shape.T, shape.d_model, shape.E, shape.capacity
    rc = load_library().moe_dispatch(ctypes.byref(shape), _ptr(x, el, T * d, "x"),
                                     _ptr(slot_token, torch.int32, E * C, "slot_token"),
                                     _ptr(expert_rows, torch.int32, E, "expert_rows"), _ptr(xe, el, E * C * d, "xe"), _stream())
    _check("moe_dispatch", rc)


def moe_expert_ffn(shape, xe, expert_rows, W1, b1, W2, b2, ye, ws) -> None:
    el = _elem(shape)
    d, f, E, C = shape.d_model, shape.d_ffn, shape.E, shape.capacity
    wsp, wsn = _ws(shape, ws, moe_workspace_bytes(shape))
    rc = load_library().moe_expert_ffn(
        ctypes.byref(shape), _ptr(xe, el, E * C * d, "xe"), _ptr(expert_rows, torch.int32, E, "expert_rows"),
        _ptr(W1, el, _w(shape, E, d, f), "W1"), _ptr(b1, el, E * f, "b1"), _ptr(W2, el, _w(shape, E, f, d), "W2"),
        _ptr(b2, el, E * d, "b2"), _ptr(ye, el, E * C * d, "ye"), wsp, wsn, _stream())
    _check("moe_expert_ffn", rc)


def moe_expert_ffn_slice(shape, xe, expert_rows, W1s, b1s, W2s, ye_partial, ws) -> None:
    el = _elem(shape)
    d, f, E, C = shape.d_model, shape.d_ffn, shape.E, shape.capacity
    wsp, wsn = _ws(shape, ws, moe_workspace_bytes(shape))
    rc = load_library().moe_expert_ffn_slice(
        ctypes.byref(shape), _ptr(xe, el, E * C * d, "xe"), _ptr(expert_rows, torch.int32, E, "expert_rows"),
        _ptr(W1s, el, _w(shape, E, d, f), "W1s"), _ptr(b1s, el, E * f, "b1s"), _ptr(W2s, el, _w(shape, E, f, d), "W2s"),
        _ptr(ye_partial, torch.float32, E * C * d, "ye_partial"), wsp, wsn, _stream())
    _check("moe_expert_ffn_slice", rc)


def moe_expert_ffn_slice_reduce(shape, n_slices, ye_partials, expert_rows, b2, ye) -> None:
    el = _elem(shape)
    d, E, C = shape.d_model, shape.E, shape.capacity
    rc = load_library().moe_expert_ffn_slice_reduce(
        ctypes.byref(shape), int(n_slices), _ptr(ye_partials, torch.float32, int(n_slices) * E * C * d, "ye_partials"),
        _ptr(expert_rows, torch.int32, E, "expert_rows"), _ptr(b2, el, E * d, "b2"), _ptr(ye, el, E * C * d, "ye"), _stream())
    _check("moe_expert_ffn_slice_reduce", rc)


def moe_combine(shape, ye, expert_idx, slot_idx, gate_w, addend, out) -> None:
    el = _elem(shape)
    T, d, E, k, C = shape.T, shape.d_model, shape.E, shape.top_k, shape.capacity
    rc = load_library().moe_combine(ctypes.byref(shape), _ptr(ye, el, E * C * d, "ye"),
                                    _ptr(expert_idx, torch.int32, T * k, "expert_idx"),
                                    _ptr(slot_idx, torch.int32, T * k, "slot_idx"), _ptr(gate_w, torch.float32, T * k, "gate_w"),
                                    _ptr(addend, el, T * d, "addend"), _ptr(out, el, T * d, "out"), _stream())
    _check("moe_combine", rc)


def _ffn_weight_args(shape, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2):
    el = _elem(shape)
    d, f, E = shape.d_model, shape.d_ffn, shape.E
    return (_ptr(W1, el, _w(shape, E, d, f), "W1"), _ptr(b1, el, E * f, "b1"), _ptr(W2, el, _w(shape, E, f, d), "W2"),
            _ptr(b2, el, E * d, "b2"), _ptr(Wd1, el, _w(shape, 1, d, f), "Wd1"), _ptr(bd1, el, f, "bd1"),
            _ptr(Wd2, el, _w(shape, 1, f, d), "Wd2"), _ptr(bd2, el, d, "bd2"))


def moe_layer_forward(shape, x, Wg, bg, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2, out,
                      logits_out, expert_idx_out, slot_idx_out, gate_w_out, expert_rows_out, slot_token_out, ws) -> None:
    el, i32, f32 = _elem(shape), torch.int32, torch.float32
    T, d, E, k, C = shape.T, shape.d_model, shape.E, shape.top_k, shape.capacity
    wsp, wsn = _ws(shape, ws, moe_workspace_bytes(shape))
    rc = load_library().moe_layer_forward(
        ctypes.byref(shape), _ptr(x, el, T * d, "x"), _ptr(Wg, f32, _wg(shape), "Wg"), _ptr(bg, f32, E, "bg"),
        *_ffn_weight_args(shape, W1, b1, W2, b2, Wd1, bd1, Wd2, bd2), _ptr(out, el, T * d, "out"),
        _ptr(logits_out, f32, T * E, "logits_out"), _ptr(expert_idx_out, i32, T * k, "expert_idx_out"),
        _ptr(slot_idx_out, i32, T * k, "slot_idx_out"), _ptr(gate_w_out, f32, T * k, "gate_w_out"),
        _ptr(expert_rows_out, i32, E, "expert_rows_out"), _ptr(slot_token_out, i32, E * C, "slot_token_out"),
        wsp, wsn, _stream())
    _check("moe_layer_forward", rc)


def moe_decode_block_workspace_bytes(shape: MoeShape, block: MoeBlockShape) -> int:
    return int(load_library().moe_decode_block_workspace_bytes(ctypes.byref(shape), ctypes.byref(block)))


def moe_decode_block_forward(shape, block, weights: dict, x, k_cache, v_cache, pos, out, x1_out, moe_in_out, logits_out,
                             ws) -> None:
    """`weights`: name -> tensor (or None) for the fields of moe_block_weights_t."""
    el, f32 = _elem(shape), torch.float32
    T, d, f, E = shape.T, shape.d_model, shape.d_ffn, shape.E
    cache = T * d * block.max_len                      # [T, H, max_len, d/H]
    sizes = {"ln1_gamma": (f32, d), "ln1_beta": (f32, d), "ln2_gamma": (f32, d), "ln2_beta": (f32, d),
             "Wqkv": (el, 3 * d * d), "bqkv": (el, 3 * d), "Wo": (el, d * d), "bo": (el, d),
             "Wg": (f32, _wg(shape)), "bg": (f32, E), "W1": (el, _w(shape, E, d, f)), "b1": (el, E * f),
             "W2": (el, _w(shape, E, f, d)), "b2": (el, E * d), "Wd1": (el, _w(shape, 1, d, f)), "bd1": (el, f),
             "Wd2": (el, _w(shape, 1, f, d)), "bd2": (el, d)}
    w = MoeBlockWeights(**{n: _ptr(weights.get(n), sizes[n][0], sizes[n][1], n) for n in BLOCK_WEIGHT_FIELDS})
    wsp, wsn = _ws(shape, ws, moe_decode_block_workspace_bytes(shape, block))
    rc = load_library().moe_decode_block_forward(
        ctypes.byref(shape), ctypes.byref(block), ctypes.byref(w), _ptr(x, el, T * d, "x"),
        _ptr(k_cache, el, cache, "k_cache"), _ptr(v_cache, el, cache, "v_cache"), _ptr(pos, torch.int32, T, "pos"),
        _ptr(out, el, T * d, "out"), _ptr(x1_out, el, T * d, "x1_out"), _ptr(moe_in_out, el, T * d, "moe_in_out"),
        _ptr(logits_out, f32, T * E, "logits_out"), wsp, wsn, _stream())
    _check("moe_decode_block_forward", rc)


def moe_profile_enable(max_calls: int) -> None:
    _check("moe_profile_enable", load_library().moe_profile_enable(int(max_calls)))


def moe_profile_select(stage_names=None) -> None:
    """Restrict stage timing to the named stages (None = all)."""
    names = moe_profile_stage_names()
    mask = 0xFFFFFFFF if stage_names is None else sum(1 << names.index(n) for n in stage_names)
    _check("moe_profile_select", load_library().moe_profile_select(mask))


def moe_profile_stride(every_nth_call: int) -> None:
    _check("moe_profile_stride", load_library().moe_profile_stride(int(every_nth_call)))


def moe_profile_calls() -> int:
    return int(load_library().moe_profile_calls())


def moe_profile_stage_names() -> list:
    lib = load_library()
    return [lib.moe_profile_stage_name(i).decode() for i in range(lib.moe_profile_stage_count())]


def moe_profile_elapsed(call: int) -> list:
    lib = load_library()
    n = lib.moe_profile_stage_count()
    buf = (ctypes.c_float * n)()
    _check("moe_profile_elapsed", lib.moe_profile_elapsed(int(call), buf))
    return list(buf)
