"""ctypes front-end for the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays into oracle/hexa_oracle.cpp and nothing else: no
arithmetic of the method lives here.  Allowed callers: tests/, the smoke check
and the benchmark's cpu_baseline leg.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hexa_oracle.cpp")
_LIB = os.path.join(_HERE, "libhexa_oracle.so")

_P = ctypes.c_void_p
_I = ctypes.c_int


# HEXA_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (the process must then run with the ASan runtime preloaded; see
# tests/test_sanitizers.py).
_SAN = os.environ.get("HEXA_ORACLE_SANITIZE") == "1"
if _SAN:
    _LIB = os.path.join(_HERE, "libhexa_oracle_asan.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (-O3, OpenMP over disjoint outputs only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                "-fno-sanitize-recover=undefined"] if _SAN else ["-O3", "-march=native"])
        subprocess.check_call(["g++", *opt, "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.hexa_oracle_gelu.restype = ctypes.c_double
        _lib.hexa_oracle_gelu.argtypes = [ctypes.c_double]
        _lib.hexa_oracle_gelu_grad.restype = ctypes.c_double
        _lib.hexa_oracle_gelu_grad.argtypes = [ctypes.c_double]
        _lib.hexa_oracle_act.restype = ctypes.c_double
        _lib.hexa_oracle_act.argtypes = [ctypes.c_double]
        _lib.hexa_oracle_act_grad.restype = ctypes.c_double
        _lib.hexa_oracle_act_grad.argtypes = [ctypes.c_double]
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_P)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_P)


def _opt_i32(a):
    if a is None:
        return None, None, 0
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_P), int(a.size)


def _dims(x, topk_idx, W1):
    T, d = x.shape
    E, d2, f = W1.shape
    assert d2 == d and topk_idx.shape[0] == T
    return T, d, f, E, topk_idx.shape[1]


def index(topk_idx, E):
    idx, p = _i32(topk_idx)
    T, k = idx.shape
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(T * k, np.int32)
    inv = np.empty(T * k, np.int32)
    rc = lib().hexa_oracle_index(_I(T), _I(k), _I(E), p, counts.ctypes.data_as(_P),
                                 offsets.ctypes.data_as(_P), perm.ctypes.data_as(_P),
                                 inv.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle index: bad shape or expert id out of range")
    return counts, offsets, perm, inv


def fwd(x, topk_idx, gate, W1, b1, W2, b2, tokens=None):
    """y for all tokens, or for `tokens` only (rows in that order), fp64."""
    T, d, f, E, k = _dims(x, topk_idx, W1)
    x, px = _f32(x); idx, pi = _i32(topk_idx); gate, pg = _f32(gate)
    W1, pw1 = _f32(W1); b1, pb1 = _f32(b1); W2, pw2 = _f32(W2); b2, pb2 = _f32(b2)
    tok, pt, nt = _opt_i32(tokens)
    y = np.empty((nt if tok is not None else T, d), np.float64)
    rc = lib().hexa_oracle_fwd(_I(T), _I(d), _I(f), _I(E), _I(k), px, pi, pg, pw1, pb1, pw2, pb2,
                               pt, _I(nt), y.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle fwd: bad arguments")
    return y


def bwd_tokens(x, topk_idx, gate, W1, b1, W2, b2, dY, tokens=None):
    """(dx [n,d], dgate [n,k]) for all tokens or the listed ones, fp64."""
    T, d, f, E, k = _dims(x, topk_idx, W1)
    x, px = _f32(x); idx, pi = _i32(topk_idx); gate, pg = _f32(gate)
    W1, pw1 = _f32(W1); b1, pb1 = _f32(b1); W2, pw2 = _f32(W2); b2, pb2 = _f32(b2)
    dY, pdy = _f32(dY)
    tok, pt, nt = _opt_i32(tokens)
    n = nt if tok is not None else T
    dx = np.empty((n, d), np.float64)
    dgate = np.empty((n, k), np.float64)
    rc = lib().hexa_oracle_bwd_tokens(_I(T), _I(d), _I(f), _I(E), _I(k), px, pi, pg, pw1, pb1,
                                      pw2, pb2, pdy, pt, _I(nt), dx.ctypes.data_as(_P),
                                      dgate.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle bwd_tokens: bad arguments")
    return dx, dgate


def bwd_experts(x, topk_idx, gate, W1, b1, W2, dY, experts=None, cols=None):
    """(dW1 [ne,d,nc], db1 [ne,nc], dW2 [ne,nc,d], db2 [ne,d]) in fp64 for the
    listed experts (default all) and hidden units `cols` (default all f)."""
    T, d, f, E, k = _dims(x, topk_idx, W1)
    x, px = _f32(x); idx, pi = _i32(topk_idx); gate, pg = _f32(gate)
    W1, pw1 = _f32(W1); b1, pb1 = _f32(b1); W2, pw2 = _f32(W2); dY, pdy = _f32(dY)
    if experts is None:
        experts = np.arange(E, dtype=np.int32)
    ex, pe, ne = _opt_i32(experts)
    cl, pc, ncl = _opt_i32(cols)
    nc = ncl if cl is not None else f
    dW1 = np.empty((ne, d, nc), np.float64)
    db1 = np.empty((ne, nc), np.float64)
    dW2 = np.empty((ne, nc, d), np.float64)
    db2 = np.empty((ne, d), np.float64)
    rc = lib().hexa_oracle_bwd_experts(_I(T), _I(d), _I(f), _I(E), _I(k), px, pi, pg, pw1, pb1,
                                       pw2, pdy, pe, _I(ne), pc, _I(ncl),
                                       dW1.ctypes.data_as(_P), db1.ctypes.data_as(_P),
                                       dW2.ctypes.data_as(_P), db2.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle bwd_experts: bad arguments")
    return dW1, db1, dW2, db2


def padded_index(topk_idx, E, blk, cap=None):
    """(v [cap] int32, idx_ [E+1] int32): the paper's -1-padded re-index vector over flat assignment
    ids and the starts of the padded per-expert sub-vectors; cap defaults to A + E*(blk-1)."""
    idx, p = _i32(topk_idx)
    T, k = idx.shape
    if cap is None:
        cap = T * k + E * (blk - 1)
    v = np.empty(cap, np.int32)
    starts = np.empty(E + 1, np.int32)
    rc = lib().hexa_oracle_padded_index(_I(T), _I(k), _I(E), _I(blk), p, ctypes.c_longlong(cap),
                                        v.ctypes.data_as(_P), starts.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle padded_index: bad arguments")
    return v, starts


def route(logits, k, mode=0):
    """(topk_idx [T,k] int32, gate [T,k] fp64): k largest logits per row, ties to the lower
    expert id, slots by descending logit; mode 0 = softmax over the selected logits, mode 1 =
    softmax over all E evaluated at the selected ones."""
    l, pl = _f32(logits)
    T, E = l.shape
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float64)
    rc = lib().hexa_oracle_route(_I(T), _I(E), _I(k), _I(mode), pl, idx.ctypes.data_as(_P),
                                 gate.ctypes.data_as(_P))
    if rc:
        raise ValueError("oracle route: bad arguments (k > E, or non-finite logits)")
    return idx, gate


def gelu(u: float) -> float:
    return lib().hexa_oracle_gelu(float(u))


def gelu_grad(u: float) -> float:
    return lib().hexa_oracle_gelu_grad(float(u))


ACT_GELU_TANH, ACT_RELU, ACT_SILU = 0, 1, 2


def set_activation(kind: int) -> None:
    """Process-wide activation of the oracle (0 GELU-tanh, the default; 1 ReLU; 2 SiLU)."""
    if lib().hexa_oracle_set_activation(int(kind)):
        raise ValueError("oracle: unknown activation")


def act(u: float) -> float:
    return lib().hexa_oracle_act(float(u))


def act_grad(u: float) -> float:
    return lib().hexa_oracle_act_grad(float(u))
