"""Thin Python binding of libhexa_moe (argument marshalling only).

Same names as the C ABI in include/hexa_moe.h (and the measurement helpers of
include/hexa_moe_bench.h).  PyTorch supplies device memory
and the current stream; every step of the layer runs in the library's kernels.
Importing this module fails loudly when the library has not been built
(`python -m paper_2411_01288_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# HEXA_MOE_SANITIZE=1 loads the host-sanitizer build instead (build.py --sanitize; CPU-side tests only)
LIB_PATH = os.path.join(_HERE, "libhexa_moe_asan.so" if os.environ.get("HEXA_MOE_SANITIZE") == "1"
                        else "libhexa_moe.so")

HEXA_F32, HEXA_BF16, HEXA_F16 = 0, 1, 2
EXPORTS = ("hexa_moe_index_scratch_bytes", "hexa_moe_workspace_bytes", "hexa_moe_status_string",
           "hexa_moe_index", "hexa_moe_index_static", "hexa_moe_fwd", "hexa_moe_bwd", "hexa_moe_profile_enable",
           "hexa_moe_profile_read", "hexa_moe_mfma_probe", "hexa_moe_route",
           "hexa_moe_allocate", "hexa_moe_padded_capacity", "hexa_moe_padded_index")


class Shape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("activation", ctypes.c_int32)]


class Idx(ctypes.Structure):
    _fields_ = [("counts", ctypes.c_void_p), ("offsets", ctypes.c_void_p),
                ("perm", ctypes.c_void_p), ("inv", ctypes.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2411_01288_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    P, S = ctypes.c_void_p, ctypes.c_size_t
    lib.hexa_moe_index_scratch_bytes.restype = S
    lib.hexa_moe_index_scratch_bytes.argtypes = [ctypes.POINTER(Shape)]
    lib.hexa_moe_workspace_bytes.restype = S
    lib.hexa_moe_workspace_bytes.argtypes = [ctypes.POINTER(Shape)]
    lib.hexa_moe_status_string.restype = ctypes.c_char_p
    lib.hexa_moe_status_string.argtypes = [ctypes.c_int]
    lib.hexa_moe_index.restype = ctypes.c_int
    lib.hexa_moe_index.argtypes = [ctypes.POINTER(Shape), P, Idx, P, S, P]
    lib.hexa_moe_index_static.restype = ctypes.c_int
    lib.hexa_moe_index_static.argtypes = [ctypes.POINTER(Shape), P, Idx, P]
    lib.hexa_moe_fwd.restype = ctypes.c_int
    lib.hexa_moe_fwd.argtypes = [ctypes.POINTER(Shape), P, P, P, P, P, P, P, Idx, P, P, S, P]
    lib.hexa_moe_bwd.restype = ctypes.c_int
    lib.hexa_moe_bwd.argtypes = [ctypes.POINTER(Shape), P, P, P, P, P, P, Idx, P, S, P, P, P, P, P, P, P]
    lib.hexa_moe_mfma_probe.restype = ctypes.c_int
    lib.hexa_moe_mfma_probe.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, P, P,
                                        ctypes.POINTER(ctypes.c_double)]
    lib.hexa_moe_route.restype = ctypes.c_int
    lib.hexa_moe_route.argtypes = [ctypes.POINTER(Shape), P, ctypes.c_int32, P, P, P]
    lib.hexa_moe_padded_capacity.restype = S
    lib.hexa_moe_padded_capacity.argtypes = [ctypes.POINTER(Shape), ctypes.c_int32]
    lib.hexa_moe_padded_index.restype = ctypes.c_int
    lib.hexa_moe_padded_index.argtypes = [ctypes.POINTER(Shape), Idx, ctypes.c_int32, P, S, P, P]
    lib.hexa_moe_allocate.restype = ctypes.c_int
    lib.hexa_moe_allocate.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_double), ctypes.c_int64,
                                      ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    lib.hexa_moe_profile_enable.restype = None
    lib.hexa_moe_profile_enable.argtypes = [ctypes.c_int]
    lib.hexa_moe_profile_read.restype = ctypes.c_int
    lib.hexa_moe_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                          ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int)]
    return lib


lib = _load()


class HexaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"hexa_moe status {code}: {lib.hexa_moe_status_string(code).decode()}")


def _check(code: int):
    if code != 0:
        raise HexaError(code)


ACT_GELU_TANH, ACT_RELU, ACT_SILU = 0, 1, 2


def make_shape(T: int, d_model: int, d_ff: int, E: int, k: int, dtype, activation: int = ACT_GELU_TANH) -> Shape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: HEXA_F32, torch.bfloat16: HEXA_BF16, torch.float16: HEXA_F16}[dtype]
    elif isinstance(dtype, str):
        dtype = {"f32": HEXA_F32, "bf16": HEXA_BF16, "f16": HEXA_F16}[dtype]
    return Shape(T, d_model, d_ff, E, k, dtype, int(activation))


def _tdt(shape: Shape):
    return {HEXA_F32: torch.float32, HEXA_BF16: torch.bfloat16, HEXA_F16: torch.float16}[shape.dtype]


def _ptr(t: Optional[torch.Tensor], dims, dtype, name: str):
    """Device pointer of a dense tensor after checking placement, dtype and size on the host
    (the kernels trust these sizes)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous device tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(dims):
        raise ValueError(f"{name}: expected {tuple(dims)} {dtype}, got {tuple(t.shape)} {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def index_scratch_bytes(shape: Shape) -> int:
    return lib.hexa_moe_index_scratch_bytes(ctypes.byref(shape))


def workspace_bytes(shape: Shape) -> int:
    return lib.hexa_moe_workspace_bytes(ctypes.byref(shape))


def alloc_idx(shape: Shape, device) -> Dict[str, torch.Tensor]:
    A = shape.T * shape.k
    mk = lambda n: torch.empty(n, dtype=torch.int32, device=device)
    return {"counts": mk(shape.E), "offsets": mk(shape.E + 1), "perm": mk(A), "inv": mk(A)}


def _idx_struct(shape: Shape, idx: Dict[str, torch.Tensor]) -> Idx:
    A = shape.T * shape.k
    return Idx(_ptr(idx["counts"], (shape.E,), torch.int32, "counts"),
               _ptr(idx["offsets"], (shape.E + 1,), torch.int32, "offsets"),
               _ptr(idx["perm"], (A,), torch.int32, "perm"),
               _ptr(idx["inv"], (A,), torch.int32, "inv"))


def alloc_workspace(shape: Shape, device) -> torch.Tensor:
    n = workspace_bytes(shape)
    if n == 0:
        _check(lib.hexa_moe_index(ctypes.byref(shape), None, Idx(), None, 0, None))  # raises the reason
    return torch.empty(n, dtype=torch.uint8, device=device)


def hexa_moe_index(shape: Shape, topk_idx: torch.Tensor, idx: Optional[Dict[str, torch.Tensor]] = None,
                   scratch: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    dev = topk_idx.device
    if idx is None:
        idx = alloc_idx(shape, dev)
    if scratch is None:
        scratch = torch.empty(max(index_scratch_bytes(shape), 256), dtype=torch.uint8, device=dev)
    _check(lib.hexa_moe_index(ctypes.byref(shape),
                              _ptr(topk_idx, (shape.T, shape.k), torch.int32, "topk_idx"),
                              _idx_struct(shape, idx), ctypes.c_void_p(scratch.data_ptr()),
                              scratch.numel(), _stream()))
    return idx


INDEX_STATIC_SCRATCH_BYTES = 1 << 20


def hexa_moe_index_static(shape: Shape, topk_idx: torch.Tensor, idx: Dict[str, torch.Tensor]) -> Dict[str, torch.Tensor]:
    """hexa_moe_index without a scratch argument and without any allocation: `idx` must be given."""
    _check(lib.hexa_moe_index_static(ctypes.byref(shape),
                                     _ptr(topk_idx, (shape.T, shape.k), torch.int32, "topk_idx"),
                                     _idx_struct(shape, idx), _stream()))
    return idx


def hexa_moe_fwd(shape: Shape, x, topk_idx, gate, W1, b1, W2, b2, idx, workspace: torch.Tensor,
                 y: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, d, f, E, k = shape.T, shape.d_model, shape.d_ff, shape.E, shape.k
    dt = _tdt(shape)
    if y is None:
        y = torch.empty((T, d), dtype=dt, device=x.device)
    _check(lib.hexa_moe_fwd(ctypes.byref(shape), _ptr(x, (T, d), dt, "x"),
                            _ptr(topk_idx, (T, k), torch.int32, "topk_idx"),
                            _ptr(gate, (T, k), torch.float32, "gate"),
                            _ptr(W1, (E, d, f), dt, "W1"), _ptr(b1, (E, f), dt, "b1"),
                            _ptr(W2, (E, f, d), dt, "W2"), _ptr(b2, (E, d), dt, "b2"),
                            _idx_struct(shape, idx), _ptr(y, (T, d), dt, "y"),
                            ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream()))
    return y


def hexa_moe_bwd(shape: Shape, dY, x, topk_idx, gate, W1, W2, idx, workspace: torch.Tensor,
                 want_dgate: bool = True, out: Optional[Dict[str, torch.Tensor]] = None
                 ) -> Dict[str, torch.Tensor]:
    T, d, f, E, k = shape.T, shape.d_model, shape.d_ff, shape.E, shape.k
    dt = _tdt(shape)
    dev = x.device
    if out is None:
        out = {"dx": torch.empty((T, d), dtype=dt, device=dev),
               "dW1": torch.empty((E, d, f), dtype=torch.float32, device=dev),
               "db1": torch.empty((E, f), dtype=torch.float32, device=dev),
               "dW2": torch.empty((E, f, d), dtype=torch.float32, device=dev),
               "db2": torch.empty((E, d), dtype=torch.float32, device=dev),
               "dgate": torch.empty((T, k), dtype=torch.float32, device=dev) if want_dgate else None}
    _check(lib.hexa_moe_bwd(ctypes.byref(shape), _ptr(dY, (T, d), dt, "dY"), _ptr(x, (T, d), dt, "x"),
                            _ptr(topk_idx, (T, k), torch.int32, "topk_idx"),
                            _ptr(gate, (T, k), torch.float32, "gate"),
                            _ptr(W1, (E, d, f), dt, "W1"), _ptr(W2, (E, f, d), dt, "W2"),
                            _idx_struct(shape, idx), ctypes.c_void_p(workspace.data_ptr()),
                            workspace.numel(), _ptr(out["dx"], (T, d), dt, "dx"),
                            _ptr(out["dW1"], (E, d, f), torch.float32, "dW1"),
                            _ptr(out["db1"], (E, f), torch.float32, "db1"),
                            _ptr(out["dW2"], (E, f, d), torch.float32, "dW2"),
                            _ptr(out["db2"], (E, d), torch.float32, "db2"),
                            _ptr(out.get("dgate"), (T, k), torch.float32, "dgate"), _stream()))
    return out


def profile_enable(on: bool) -> None:
    lib.hexa_moe_profile_enable(1 if on else 0)


def profile_read() -> Dict[str, Tuple[float, int]]:
    """{kernel label: (summed ms, launches)} of the launches recorded since profile_enable(True)."""
    out = {}
    i = 0
    label, ms, n = ctypes.c_char_p(), ctypes.c_float(), ctypes.c_int()
    while lib.hexa_moe_profile_read(i, ctypes.byref(label), ctypes.byref(ms), ctypes.byref(n)):
        out[label.value.decode()] = (ms.value, n.value)
        i += 1
    return out


def mfma_probe(workgroups: int, iters: int, sink: "torch.Tensor", variant: int = 0) -> float:
    """Enqueue the register-only MFMA loop on the current stream; returns its FLOP count.
    variant 0: 16x16x32 on random operands, 1: on zeros, 2: 32x32x16 on random operands."""
    flop = ctypes.c_double()
    _check(lib.hexa_moe_mfma_probe(int(variant), int(workgroups), int(iters),
                                   _ptr(sink, (1,), torch.float32, "sink"), _stream(), ctypes.byref(flop)))
    return flop.value


GATE_SOFTMAX_SELECTED, GATE_SOFTMAX_ALL = 0, 1


def hexa_moe_route(shape: Shape, logits: torch.Tensor, gate_mode: int = GATE_SOFTMAX_SELECTED,
                   topk_idx: Optional[torch.Tensor] = None, gate: Optional[torch.Tensor] = None):
    """Router front-end: (topk_idx [T,k] int32, gate [T,k] float32) from logits [T,E] float32."""
    dev = logits.device
    if topk_idx is None:
        topk_idx = torch.empty((shape.T, shape.k), dtype=torch.int32, device=dev)
    if gate is None:
        gate = torch.empty((shape.T, shape.k), dtype=torch.float32, device=dev)
    _check(lib.hexa_moe_route(ctypes.byref(shape), _ptr(logits, (shape.T, shape.E), torch.float32, "logits"),
                              int(gate_mode), _ptr(topk_idx, (shape.T, shape.k), torch.int32, "topk_idx"),
                              _ptr(gate, (shape.T, shape.k), torch.float32, "gate"), _stream()))
    return topk_idx, gate


def allocate(latency, total: int, granule: int = 1):
    """Shares of `total` proportional to 1 / latency[i] (multiples of granule, exact sum)."""
    n = len(latency)
    lat = (ctypes.c_double * n)(*[float(t) for t in latency])
    out = (ctypes.c_int64 * n)()
    _check(lib.hexa_moe_allocate(n, lat, int(total), int(granule), out))
    return list(out)


def hexa_moe_padded_index(shape: Shape, idx: Dict[str, torch.Tensor], blk: int):
    """(v [A + E*(blk-1)] int32, idx_pad [E+1] int32): the paper's -1-padded form of the index."""
    dev = idx["perm"].device
    cap = lib.hexa_moe_padded_capacity(ctypes.byref(shape), int(blk))
    if cap == 0:
        raise HexaError(2)
    v = torch.empty(cap, dtype=torch.int32, device=dev)
    starts = torch.empty(shape.E + 1, dtype=torch.int32, device=dev)
    _check(lib.hexa_moe_padded_index(ctypes.byref(shape), _idx_struct(shape, idx), int(blk),
                                     _ptr(v, (cap,), torch.int32, "v"), cap,
                                     _ptr(starts, (shape.E + 1,), torch.int32, "idx_pad"), _stream()))
    return v, starts
