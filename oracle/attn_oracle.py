"""ctypes front end of the fp64 CPU oracle (attn_oracle.c) -- TEST INFRASTRUCTURE ONLY.

The oracle is the plain definition O = softmax(Q K^T * scale) V (paper Sec. 2.2, Eq. 1) with the
score row materialised in fp64.  It shares no code with the GPU library and must never be imported
by it.  Pins: tests/test_oracle_pins.py (closed forms, invariants, brute force, an independent
library routine).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "libattn_oracle.so")

F16, BF16, F64 = 0, 1, 2


def build(force: bool = True) -> str:
    """Compile attn_oracle.c with gcc (strict IEEE arithmetic: no -ffast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        L.attn_oracle_head.restype = ctypes.c_int
        L.attn_oracle_head.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
            ctypes.c_long, ctypes.c_int, ctypes.c_double, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_long,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        L.attn_oracle_decode_f16.restype = ctypes.c_double
        L.attn_oracle_decode_f16.argtypes = [ctypes.c_uint16]
        L.attn_oracle_decode_bf16.restype = ctypes.c_double
        L.attn_oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        L.attn_oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _as_bits(x):
    """Return (contiguous numpy array holding the raw storage, oracle dtype code).

    Accepts numpy float16 / float64 / uint16 (= bfloat16 bit patterns when bf16=True is not
    expressible in numpy) and torch CPU tensors of float16 / bfloat16 / float64.
    """
    try:
        import torch
    except Exception:  # pragma: no cover
        torch = None
    if torch is not None and isinstance(x, torch.Tensor):
        if x.device.type != "cpu":
            raise ValueError("the oracle takes CPU tensors only")
        x = x.contiguous()
        if x.dtype == torch.float16:
            return x.view(torch.int16).numpy().view(np.uint16), F16
        if x.dtype == torch.bfloat16:
            return x.view(torch.int16).numpy().view(np.uint16), BF16
        if x.dtype == torch.float64:
            return x.numpy(), F64
        raise ValueError(f"unsupported tensor dtype {x.dtype}")
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16:
        return x.view(np.uint16), F16
    if x.dtype == np.float64:
        return x, F64
    raise ValueError(f"unsupported array dtype {x.dtype}")


def attention(Q, K, V, scale: float, causal: bool = False, rows=None, return_P: bool = False,
              return_rowsum: bool = False, n_threads: int = 0):
    """fp64 attention of [B, H, N, d] inputs (fp16, bf16 or fp64 storage).

    rows: optional 1-D sequence of query-row indices; the same rows are evaluated for every
    (batch, head).  Returns O as float64 [B, H, R, d] (R = len(rows) or N), followed by P
    [B, H, R, N] and/or the per-row sums of P if requested.
    """
    q, dt = _as_bits(Q)
    k, dtk = _as_bits(K)
    v, dtv = _as_bits(V)
    if not (dt == dtk == dtv):
        raise ValueError("Q, K, V must have the same dtype")
    if q.ndim != 4 or q.shape != k.shape or q.shape != v.shape:
        raise ValueError("Q, K, V must all be [B, H, N, d]")
    B, H, N, d = q.shape
    if rows is None:
        rows_arr, rows_ptr, R = None, None, N
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        rows_ptr, R = rows_arr.ctypes.data, int(rows_arr.shape[0])
    O = np.empty((B, H, R, d), dtype=np.float64)
    P = np.empty((B, H, R, N), dtype=np.float64) if return_P else None
    rs = np.empty((B, H, R), dtype=np.float64) if return_rowsum else None
    L = lib()
    for b in range(B):
        for h in range(H):
            rc = L.attn_oracle_head(
                q[b, h].ctypes.data, k[b, h].ctypes.data, v[b, h].ctypes.data, dt,
                N, d, float(scale), int(bool(causal)), rows_ptr, R,
                O[b, h].ctypes.data,
                rs[b, h].ctypes.data if rs is not None else None,
                P[b, h].ctypes.data if P is not None else None,
                int(n_threads))
            if rc != 0:
                raise RuntimeError("attn_oracle_head failed (bad arguments or out of memory)")
    out = [O]
    if return_P:
        out.append(P)
    if return_rowsum:
        out.append(rs)
    return out[0] if len(out) == 1 else tuple(out)


def num_threads() -> int:
    return int(lib().attn_oracle_num_threads())
