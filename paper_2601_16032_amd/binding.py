"""ctypes binding of libsawattn.so: argument marshalling only, same names as the C ABI.

Every step of the attention forward runs inside the HIP library.  There is no fallback: if the
library has not been built, loading raises.  PyTorch is used for device memory and streams.
"""
from __future__ import annotations

import ctypes
import os

import torch

from .build import LIB_PATH, PROBE_LIB_PATH

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_RUNTIME = 0, 1, 2, 3
SCAN_CYCLIC, SCAN_SAWTOOTH = 0, 1
F16, BF16, F32 = 0, 1, 2

LAUNCH_PERSISTENT, LAUNCH_GRID, LAUNCH_AUTO = 0, 1, 2
DECODE_DOMAIN, DECODE_LINEAR = 0, 1

_DTYPE_CODE = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}
_SCAN_CODE = {"cyclic": SCAN_CYCLIC, "sawtooth": SCAN_SAWTOOTH, SCAN_CYCLIC: SCAN_CYCLIC,
              SCAN_SAWTOOTH: SCAN_SAWTOOTH}


class LaunchInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in (
        "tile_q", "tile_kv", "block_threads", "grid", "lds_bytes", "domains", "slots",
        "parts_per_head", "q_tiles_per_head", "max_local_tiles", "launch", "tiles_per_workgroup",
        "qo_streaming")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Variant(ctypes.Structure):
    """sawattn_variant: which launch / work decode to run (None everywhere = the default)."""
    _fields_ = [("launch", ctypes.c_int), ("decode", ctypes.c_int), ("slots_per_domain", ctypes.c_int),
                ("tiles_per_workgroup", ctypes.c_int), ("rows_per_wavefront", ctypes.c_int),
                ("align_rounds", ctypes.c_int), ("kv_halves", ctypes.c_int), ("qo_streaming", ctypes.c_int)]


_LAUNCH_CODE = {"persistent": LAUNCH_PERSISTENT, "grid": LAUNCH_GRID, "auto": LAUNCH_AUTO}
_DECODE_CODE = {"domain": DECODE_DOMAIN, "linear": DECODE_LINEAR}


def variant(launch="persistent", decode="domain", slots_per_domain=0, tiles_per_workgroup=0,
            rows_per_wavefront=0, align_rounds=0, kv_halves=0, qo_streaming=0) -> Variant:
    return Variant(_LAUNCH_CODE.get(launch, launch), _DECODE_CODE.get(decode, decode),
                   int(slots_per_domain), int(tiles_per_workgroup), int(rows_per_wavefront), int(align_rounds),
                   int(kv_halves), int(qo_streaming))


def _vptr(v):
    return ctypes.byref(v) if v is not None else None


class SawattnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sawattn error {code}: {text}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load libsawattn.so (built by paper_2601_16032_amd.build.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2601_16032_amd.build` "
                "(or __graft_entry__.build()) first -- there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.attn_fwd.restype = ci
        L.attn_fwd.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, ci, ci, ci, ci, vp]
        pv = ctypes.POINTER(Variant)
        L.attn_fwd_variant.restype = ci
        L.attn_fwd_variant.argtypes = L.attn_fwd.argtypes + [pv, vp, vp]
        L.attn_fwd_workspace.restype = ci
        L.attn_fwd_workspace.argtypes = L.attn_fwd_variant.argtypes + [vp, ctypes.c_size_t]
        L.attn_fwd_workspace_bytes.restype = ci
        L.attn_fwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, pv, ctypes.POINTER(ctypes.c_size_t),
                                               ctypes.POINTER(LaunchInfo)]
        L.attn_fwd_static.restype = ci
        L.attn_fwd_static.argtypes = L.attn_fwd.argtypes
        L.attn_fwd_launch_info.restype = ci
        L.attn_fwd_launch_info.argtypes = [ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(LaunchInfo)]
        L.attn_fwd_variant_launch_info.restype = ci
        L.attn_fwd_variant_launch_info.argtypes = [ci, ci, ci, ci, ci, ci, pv, ctypes.POINTER(LaunchInfo)]
        L.attn_fwd_plan.restype = ci
        L.attn_fwd_plan.argtypes = [ci, ci, ci, ci, ci, ci, ci, pv, vp, vp]
        for name in ("attn_last_error", "sawattn_last_error"):
            getattr(L, name).restype = ctypes.c_char_p
            getattr(L, name).argtypes = []
        for name in ("attn_version", "sawattn_version"):
            getattr(L, name).restype = ci
            getattr(L, name).argtypes = []
        _lib = L
    return _lib


_probe_lib = None


def probe_lib() -> ctypes.CDLL:
    """Load libsawattn_probe.so, the benchmark's matrix-rate probe (built with the main library)."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise FileNotFoundError(f"{PROBE_LIB_PATH} is not built; run `python -m paper_2601_16032_amd.build` first")
        L = ctypes.CDLL(PROBE_LIB_PATH)
        L.sawattn_mfma_probe.restype = ctypes.c_int
        L.sawattn_mfma_probe.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.POINTER(ctypes.c_double)]
        L.sawattn_probe_last_error.restype = ctypes.c_char_p
        L.sawattn_probe_last_error.argtypes = []
        _probe_lib = L
    return _probe_lib


def attn_last_error() -> str:
    return lib().attn_last_error().decode()


def attn_version() -> int:
    return int(lib().attn_version())


sawattn_last_error, sawattn_version = attn_last_error, attn_version   # older names


def _check(rc: int):
    if rc != OK:
        raise SawattnError(rc, attn_last_error())


def _in_dtype_code(dtype) -> int:
    return {"f16": F16, "bf16": BF16}.get(dtype, _DTYPE_CODE.get(dtype, dtype))


def attn_fwd_launch_info(B: int, H: int, N: int, d: int, causal: bool = False, scan_order="sawtooth",
                         dtype="f16") -> dict:
    """Launch geometry of attn_fwd."""
    info = LaunchInfo()
    _check(lib().attn_fwd_launch_info(B, H, N, d, int(bool(causal)), _SCAN_CODE[scan_order], _in_dtype_code(dtype),
                                      ctypes.byref(info)))
    return info.as_dict()


def attn_fwd_variant_launch_info(B: int, H: int, N: int, d: int, causal: bool = False, variant: Variant = None,
                                 dtype="f16") -> dict:
    """Launch geometry of attn_fwd_variant (variant None: the default, as attn_fwd_launch_info)."""
    info = LaunchInfo()
    _check(lib().attn_fwd_variant_launch_info(B, H, N, d, int(bool(causal)), _in_dtype_code(dtype), _vptr(variant),
                                              ctypes.byref(info)))
    return info.as_dict()


def attn_fwd_plan(B: int, H: int, N: int, d: int, causal: bool = False, scan_order="sawtooth",
                  variant: Variant = None, dtype="f16"):
    """Host-side schedule: returns (trace[grid, max_local, 4], count[grid]) as CPU int32 tensors."""
    info = attn_fwd_variant_launch_info(B, H, N, d, causal, variant, dtype)
    trace = torch.full((info["grid"], max(info["max_local_tiles"], 1), 4), -1, dtype=torch.int32)
    count = torch.zeros((info["grid"],), dtype=torch.int32)
    _check(lib().attn_fwd_plan(B, H, N, d, int(bool(causal)), _SCAN_CODE[scan_order], _in_dtype_code(dtype),
                               _vptr(variant), trace.data_ptr(), count.data_ptr()))
    return trace, count


def attn_fwd_workspace_bytes(B: int, H: int, N: int, d: int, causal: bool = False, variant: Variant = None,
                             dtype="bf16"):
    """(bytes of workspace attn_fwd_workspace would use -- 0 where it changes nothing --, launch geometry)."""
    n = ctypes.c_size_t(0)
    info = LaunchInfo()
    _check(lib().attn_fwd_workspace_bytes(B, H, N, d, int(bool(causal)), _in_dtype_code(dtype), _vptr(variant),
                                          ctypes.byref(n), ctypes.byref(info)))
    return int(n.value), info.as_dict()


def sawattn_mfma_probe(iters: int, mode: int, stream=None) -> float:
    """Enqueue the matrix-rate probe on the current (or given) stream; returns its flop count."""
    sink = torch.zeros(512, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    st = stream if stream is not None else torch.cuda.current_stream()
    L = probe_lib()
    rc = L.sawattn_mfma_probe(sink.data_ptr(), int(iters), int(mode), st.cuda_stream, ctypes.byref(flops))
    if rc != OK:
        raise SawattnError(rc, L.sawattn_probe_last_error().decode())
    return float(flops.value)


def _marshal(Q, K, V, O, o_dtype):
    for name, t in (("Q", Q), ("K", K), ("V", V)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous [B, H, N, d] device tensor")
    if not (Q.shape == K.shape == V.shape) or not (Q.dtype == K.dtype == V.dtype):
        raise ValueError("Q, K, V must share shape and dtype")
    if Q.dtype not in (torch.float16, torch.bfloat16):
        raise ValueError("inputs must be float16 or bfloat16")
    if O is None:
        O = torch.empty(Q.shape, dtype=o_dtype or Q.dtype, device=Q.device)
    elif not O.is_cuda or not O.is_contiguous() or O.shape != Q.shape or O.dtype not in _DTYPE_CODE:
        raise ValueError("O must be a contiguous device tensor shaped like Q (f16, bf16 or f32)")
    return O


def attn_fwd(Q, K, V, O=None, *, scale: float, causal: bool = False, scan_order="sawtooth",
             o_dtype=None, stream=None):
    """O = softmax(Q K^T * scale) V on the current (or given) stream; returns O without waiting."""
    O = _marshal(Q, K, V, O, o_dtype)
    B, H, N, d = Q.shape
    st = stream if stream is not None else torch.cuda.current_stream(Q.device)
    _check(lib().attn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                          float(scale), int(bool(causal)), _SCAN_CODE[scan_order],
                          _DTYPE_CODE[Q.dtype], _DTYPE_CODE[O.dtype], st.cuda_stream))
    return O


def attn_fwd_variant(Q, K, V, O=None, *, scale: float, causal: bool = False, scan_order="sawtooth",
                     o_dtype=None, stream=None, variant: Variant = None, trace: bool = False):
    """attn_fwd under a launch variant.  Returns O, or with trace=True (O, trace[grid, max_local, 4],
    count[grid]): the schedule the workgroups recorded."""
    O = _marshal(Q, K, V, O, o_dtype)
    B, H, N, d = Q.shape
    tr = cnt = None
    if trace:
        info = attn_fwd_variant_launch_info(B, H, N, d, causal, variant, Q.dtype)
        tr = torch.full((info["grid"], max(info["max_local_tiles"], 1), 4), -1, dtype=torch.int32,
                        device=Q.device)
        cnt = torch.zeros((info["grid"],), dtype=torch.int32, device=Q.device)
    st = stream if stream is not None else torch.cuda.current_stream(Q.device)
    _check(lib().attn_fwd_variant(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                  float(scale), int(bool(causal)), _SCAN_CODE[scan_order],
                                  _DTYPE_CODE[Q.dtype], _DTYPE_CODE[O.dtype], st.cuda_stream, _vptr(variant),
                                  tr.data_ptr() if trace else None, cnt.data_ptr() if trace else None))
    return (O, tr, cnt) if trace else O


def attn_fwd_workspace(Q, K, V, O=None, *, scale: float, causal: bool = False, scan_order="sawtooth",
                       o_dtype=None, stream=None, variant: Variant = None, trace: bool = False, workspace=None):
    """attn_fwd_variant with a workspace (a uint8 CUDA tensor of at least attn_fwd_workspace_bytes bytes; allocated
    here when None and needed).  Returns like attn_fwd_variant."""
    O = _marshal(Q, K, V, O, o_dtype)
    B, H, N, d = Q.shape
    need, info = attn_fwd_workspace_bytes(B, H, N, d, causal, variant, Q.dtype)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    tr = cnt = None
    if trace:
        tr = torch.full((info["grid"], max(info["max_local_tiles"], 1), 4), -1, dtype=torch.int32,
                        device=Q.device)
        cnt = torch.zeros((info["grid"],), dtype=torch.int32, device=Q.device)
    st = stream if stream is not None else torch.cuda.current_stream(Q.device)
    _check(lib().attn_fwd_workspace(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                    float(scale), int(bool(causal)), _SCAN_CODE[scan_order],
                                    _DTYPE_CODE[Q.dtype], _DTYPE_CODE[O.dtype], st.cuda_stream, _vptr(variant),
                                    tr.data_ptr() if trace else None, cnt.data_ptr() if trace else None,
                                    workspace.data_ptr() if workspace is not None else None,
                                    workspace.numel() if workspace is not None else 0))
    return (O, tr, cnt) if trace else O



def attn_fwd_static(Q, K, V, O=None, *, scale: float, causal: bool = False, scan_order="sawtooth", o_dtype=None,
                    stream=None):
    """attn_fwd with the library's fixed scratch array standing in for a workspace (the C call allocates nothing;
    pass O to keep this wrapper from allocating the output)."""
    O = _marshal(Q, K, V, O, o_dtype)
    B, H, N, d = Q.shape
    st = stream if stream is not None else torch.cuda.current_stream(Q.device)
    _check(lib().attn_fwd_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                 float(scale), int(bool(causal)), _SCAN_CODE[scan_order],
                                 _DTYPE_CODE[Q.dtype], _DTYPE_CODE[O.dtype], st.cuda_stream))
    return O
