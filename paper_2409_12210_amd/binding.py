"""ctypes binding of libmodse.so: same names as the C ABI (include/modse.h), argument marshalling only.

PyTorch is used for device memory and streams.  Tensors are passed as raw device pointers together with
the current HIP stream; nothing is computed on this side."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

MODSE_F32, MODSE_BF16 = 0, 1
STAGES = ("route", "permute", "up", "down", "combine", "bwd_prep", "bwd_dgrad", "bwd_wgrad", "bwd_router")


class ModseError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: modse status {code} ({modse_status_string(code)})")
        self.code = code


class _Desc(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_experts", C.c_int32), ("top_k", C.c_int32),
                ("d_ff", C.POINTER(C.c_int32)), ("dtype", C.c_int)]


class _Routing(C.Structure):
    _fields_ = [("topk_idx", C.c_void_p), ("topk_w", C.c_void_p), ("counts", C.c_void_p), ("offsets", C.c_void_p),
                ("row_of", C.c_void_p), ("src_of", C.c_void_p), ("near_tie_count", C.c_void_p)]


class _GateExt(C.Structure):
    _fields_ = [("W_noise", C.c_void_p), ("gamma", C.c_void_p), ("eps", C.c_float), ("noise_pre", C.c_void_p),
                ("aux_alpha", C.c_float), ("probs", C.c_void_p), ("aux_f", C.c_void_p), ("aux_P", C.c_void_p),
                ("aux_loss", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(_HERE, "libmodse.so")


def load_library():
    """Load libmodse.so built in-tree.  Raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2409_12210_amd.build`")
    lib = C.CDLL(path)
    vp, i64, sz = C.c_void_p, C.c_int64, C.c_size_t
    dp, rp = C.POINTER(_Desc), C.POINTER(_Routing)
    lib.modse_status_string.restype = C.c_char_p
    lib.modse_status_string.argtypes = [C.c_int]
    lib.modse_workspace_size.argtypes = [dp, i64, C.c_int, C.POINTER(sz)]
    lib.modse_saved_size.argtypes = [dp, i64, C.POINTER(sz)]
    lib.modse_route.argtypes = [dp, i64, vp, vp, vp, rp, vp, sz, vp]
    lib.modse_route_static.argtypes = [dp, i64, vp, vp, vp, rp, vp]
    lib.modse_layer_fwd.argtypes = [dp, i64, vp, vp, vp, vp, vp, vp, vp, rp, vp, vp, sz, vp]
    lib.modse_layer_bwd.argtypes = [dp, i64, vp, vp, vp, vp, vp, rp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, sz, vp]
    ep = C.POINTER(_GateExt)
    lib.modse_route_ext.argtypes = [dp, i64, vp, vp, vp, ep, rp, vp, sz, vp]
    lib.modse_layer_fwd_ext.argtypes = [dp, i64, vp, vp, vp, ep, vp, vp, vp, vp, rp, vp, vp, sz, vp]
    lib.modse_layer_bwd_ext.argtypes = [dp, i64, vp, vp, ep, C.c_float, vp, vp, vp, rp, vp, vp, vp, vp, vp, vp, vp, vp,
                                        vp, C.c_int, vp, sz, vp]
    lib.modse_routing_stats.argtypes = [dp, i64, rp, vp, vp, vp]
    lib.modse_stage_timing_enable.argtypes = [C.c_int]
    lib.modse_stage_times.argtypes = [C.POINTER(C.c_float)]
    for name in ("modse_workspace_size", "modse_saved_size", "modse_route", "modse_layer_fwd", "modse_layer_bwd",
                 "modse_route_ext", "modse_layer_fwd_ext", "modse_layer_bwd_ext", "modse_routing_stats",
                 "modse_route_static",
                 "modse_stage_timing_enable", "modse_stage_times"):
        getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


def modse_status_string(code: int) -> str:
    return load_library().modse_status_string(int(code)).decode()


def _dtype_code(dtype) -> int:
    if isinstance(dtype, int):
        return dtype
    s = str(dtype)
    if s in ("f32", "torch.float32", "float32"):
        return MODSE_F32
    if s in ("bf16", "torch.bfloat16", "bfloat16"):
        return MODSE_BF16
    return 99   # let the library reject it


def _desc(d_model: int, d_ff: Sequence[int], top_k: int, dtype):
    arr = (C.c_int32 * max(len(d_ff), 1))(*[int(v) for v in d_ff])
    d = _Desc(int(d_model), len(d_ff), int(top_k), C.cast(arr, C.POINTER(C.c_int32)), _dtype_code(dtype))
    d._keepalive = arr
    return d


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(code: int, what: str, raise_on_error: bool) -> int:
    if code != 0 and raise_on_error:
        raise ModseError(code, what)
    return code


@dataclass
class Routing:
    """Device tensors that receive the routing artefacts (see modse_routing in include/modse.h)."""
    topk_idx: object
    topk_w: object
    counts: object
    offsets: object
    row_of: object
    src_of: object
    near_tie_count: object

    @staticmethod
    def empty(T: int, n_experts: int, top_k: int, device="cuda"):
        import torch
        i32 = dict(dtype=torch.int32, device=device)
        return Routing(torch.empty((T, top_k), **i32), torch.empty((T, top_k), dtype=torch.float32, device=device),
                       torch.empty(n_experts, **i32), torch.empty(n_experts + 1, **i32),
                       torch.empty((T, top_k), **i32), torch.empty(T * top_k, **i32), torch.zeros(1, **i32))

    def _c(self):
        return _Routing(*[_ptr(getattr(self, f)) for f in
                          ("topk_idx", "topk_w", "counts", "offsets", "row_of", "src_of", "near_tie_count")])


@dataclass
class GateExt:
    """Optional parts of the gate (see modse_gate_ext in include/modse.h): device tensors or None."""
    W_noise: object = None
    gamma: object = None
    eps: float = 0.0
    noise_pre: object = None
    aux_alpha: float = 0.0
    probs: object = None
    aux_f: object = None
    aux_P: object = None
    aux_loss: object = None

    def _c(self):
        return _GateExt(_ptr(self.W_noise), _ptr(self.gamma), float(self.eps), _ptr(self.noise_pre),
                        float(self.aux_alpha), _ptr(self.probs), _ptr(self.aux_f), _ptr(self.aux_P),
                        _ptr(self.aux_loss))


WS_FWD, WS_BWD, WS_FWD_SAVED = 0, 1, 2   # `which` of modse_workspace_size (MODSE_WS_* in include/modse.h)


def modse_workspace_size(d_model, d_ff, top_k, dtype, T, which=WS_FWD, raise_on_error=True):
    out = C.c_size_t(0)
    d = _desc(d_model, d_ff, top_k, dtype)
    code = load_library().modse_workspace_size(C.byref(d), int(T), int(which), C.byref(out))
    _check(code, "modse_workspace_size", raise_on_error)
    return out.value if code == 0 else code


def modse_saved_size(d_model, d_ff, top_k, dtype, T, raise_on_error=True):
    out = C.c_size_t(0)
    d = _desc(d_model, d_ff, top_k, dtype)
    code = load_library().modse_saved_size(C.byref(d), int(T), C.byref(out))
    _check(code, "modse_saved_size", raise_on_error)
    return out.value if code == 0 else code


def modse_route(d_model, d_ff, top_k, dtype, T, x, W_gate, logit_bias, routing: Routing, ws, ws_bytes=None,
                stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    code = load_library().modse_route(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(logit_bias),
                                      C.byref(r) if r is not None else None, _ptr(ws), nbytes, _stream(stream))
    return _check(code, "modse_route", raise_on_error)


def modse_route_static(d_model, d_ff, top_k, dtype, T, x, W_gate, logit_bias, routing: Routing, stream=None,
                       raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    code = load_library().modse_route_static(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(logit_bias),
                                             C.byref(r) if r is not None else None, _stream(stream))
    return _check(code, "modse_route_static", raise_on_error)


def modse_layer_fwd(d_model, d_ff, top_k, dtype, T, x, W_gate, logit_bias, W1, W3, W2, y,
                    routing: Optional[Routing], saved, ws, ws_bytes=None, stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    code = load_library().modse_layer_fwd(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(logit_bias), _ptr(W1),
                                          _ptr(W3), _ptr(W2), _ptr(y), C.byref(r) if r is not None else None,
                                          _ptr(saved), _ptr(ws), nbytes, _stream(stream))
    return _check(code, "modse_layer_fwd", raise_on_error)


def modse_layer_bwd(d_model, d_ff, top_k, dtype, T, x, W_gate, W1, W3, W2, routing: Routing, saved, dY, dX, dW_gate,
                    dW1, dW3, dW2, accumulate, ws, ws_bytes=None, stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    nbytes = ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)
    code = load_library().modse_layer_bwd(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(W1), _ptr(W3), _ptr(W2),
                                          C.byref(r) if r is not None else None, _ptr(saved), _ptr(dY), _ptr(dX),
                                          _ptr(dW_gate), _ptr(dW1), _ptr(dW3), _ptr(dW2), int(bool(accumulate)),
                                          _ptr(ws), nbytes, _stream(stream))
    return _check(code, "modse_layer_bwd", raise_on_error)


def _nbytes(ws, ws_bytes):
    return ws_bytes if ws_bytes is not None else (ws.numel() * ws.element_size() if ws is not None else 0)


def modse_route_ext(d_model, d_ff, top_k, dtype, T, x, W_gate, logit_bias, ext: Optional[GateExt], routing: Routing,
                    ws, ws_bytes=None, stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    e = ext._c() if ext is not None else None
    code = load_library().modse_route_ext(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(logit_bias),
                                          C.byref(e) if e is not None else None,
                                          C.byref(r) if r is not None else None, _ptr(ws), _nbytes(ws, ws_bytes),
                                          _stream(stream))
    return _check(code, "modse_route_ext", raise_on_error)


def modse_layer_fwd_ext(d_model, d_ff, top_k, dtype, T, x, W_gate, logit_bias, ext: Optional[GateExt], W1, W3, W2, y,
                        routing: Optional[Routing], saved, ws, ws_bytes=None, stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    e = ext._c() if ext is not None else None
    code = load_library().modse_layer_fwd_ext(C.byref(d), int(T), _ptr(x), _ptr(W_gate), _ptr(logit_bias),
                                              C.byref(e) if e is not None else None, _ptr(W1), _ptr(W3), _ptr(W2),
                                              _ptr(y), C.byref(r) if r is not None else None, _ptr(saved), _ptr(ws),
                                              _nbytes(ws, ws_bytes), _stream(stream))
    return _check(code, "modse_layer_fwd_ext", raise_on_error)


def modse_layer_bwd_ext(d_model, d_ff, top_k, dtype, T, x, W_gate, ext: Optional[GateExt], aux_grad, W1, W3, W2,
                        routing: Routing, saved, dY, dX, dW_gate, dW_noise, dgamma, dW1, dW3, dW2, accumulate, ws,
                        ws_bytes=None, stream=None, raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    e = ext._c() if ext is not None else None
    code = load_library().modse_layer_bwd_ext(C.byref(d), int(T), _ptr(x), _ptr(W_gate),
                                              C.byref(e) if e is not None else None, float(aux_grad), _ptr(W1),
                                              _ptr(W3), _ptr(W2), C.byref(r) if r is not None else None, _ptr(saved),
                                              _ptr(dY), _ptr(dX), _ptr(dW_gate), _ptr(dW_noise), _ptr(dgamma),
                                              _ptr(dW1), _ptr(dW3), _ptr(dW2), int(bool(accumulate)), _ptr(ws),
                                              _nbytes(ws, ws_bytes), _stream(stream))
    return _check(code, "modse_layer_bwd_ext", raise_on_error)


def modse_routing_stats(d_model, d_ff, top_k, dtype, T, routing: Routing, slot_counts, summary, stream=None,
                        raise_on_error=True) -> int:
    d = _desc(d_model, d_ff, top_k, dtype)
    r = routing._c() if routing is not None else None
    code = load_library().modse_routing_stats(C.byref(d), int(T), C.byref(r) if r is not None else None,
                                              _ptr(slot_counts), _ptr(summary), _stream(stream))
    return _check(code, "modse_routing_stats", raise_on_error)


def modse_stage_timing_enable(on: bool) -> int:
    return _check(load_library().modse_stage_timing_enable(int(bool(on))), "modse_stage_timing_enable", True)


def modse_stage_times() -> dict:
    buf = (C.c_float * len(STAGES))()
    _check(load_library().modse_stage_times(buf), "modse_stage_times", True)
    return {name: float(buf[i]) for i, name in enumerate(STAGES)}
