"""Thin ctypes binding of libsla_hip.so (the C ABI of include/sla.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory (torch.empty) and the current HIP stream; nothing is
computed with torch ops.  There is no fallback: if the library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsla_hip.so")

SLA_F32, SLA_BF16 = 0, 1
SLA_PHI_SOFTMAX, SLA_PHI_ELU1 = 0, 1
SLA_BHND, SLA_BNHD, SLA_STRIDED = 0, 1, 2
SLA_AGG_GEMM, SLA_AGG_ADD, SLA_AGG_PREAGG, SLA_AGG_FOUR_RUSSIANS = 0, 1, 2, 3
SLA_STATIC_WS_BYTES = 32 << 20
EXPORTS = ("sla_sizes", "sla_build_mask", "sla_build_mask_static", "sla_classify_scores", "sla_forward", "sla_backward",
           "sla_aggregate_ws_bytes", "sla_aggregate_states", "sla_wide_query_tiles",
           "sla_profile_enable", "sla_profile_read", "sla_profile_mfma_peak", "sla_profile_dq_atomics", "sla_strerror")


class sla_params(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32),
                ("d", ctypes.c_int32), ("bq", ctypes.c_int32), ("bkv", ctypes.c_int32),
                ("k_h", ctypes.c_double), ("k_l", ctypes.c_double), ("phi", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("layout", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64)]


class sla_sizes_t(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("n_h", ctypes.c_int32), ("n_l", ctypes.c_int32),
                ("n_0", ctypes.c_int32), ("Tq", ctypes.c_int32), ("reserved", ctypes.c_int32)] + [(n, ctypes.c_uint64) for n in (
                    "mask_bytes", "luts_bytes", "lut_row_idx", "lut_col_ptr", "lut_col_rows", "lut_ind", "lut_ind_t", "lut_col_order",
                    "saved_bytes", "saved_Os", "saved_Ol", "saved_L", "saved_HZ", "saved_Z",
                    "ws_mask_bytes", "ws_mask_qbar", "ws_mask_kbar", "ws_mask_scores",
                    "ws_forward_bytes", "ws_backward_bytes")]


class SLAError(RuntimeError):
    pass


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the HIP library; raises if it has not been built (python -m paper_2509_24006_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SLAError(f"{LIB_PATH} is missing: build it with paper_2509_24006_amd/build.py "
                           "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        pp = ctypes.POINTER(sla_params)
        L.sla_sizes.argtypes = [pp, ctypes.POINTER(sla_sizes_t)]
        L.sla_build_mask.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
        L.sla_build_mask_static.argtypes = [pp, vp, vp, vp, vp, vp]
        L.sla_classify_scores.argtypes = [pp, vp, vp, vp, vp]
        L.sla_forward.argtypes = [pp] + [vp] * 9 + [sz, vp]
        L.sla_backward.argtypes = [pp] + [vp] * 13 + [sz, vp]
        L.sla_aggregate_ws_bytes.argtypes = [pp, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64)]
        L.sla_aggregate_states.argtypes = [pp, ctypes.c_int, vp, vp, vp, vp, vp, sz, vp]
        L.sla_profile_enable.argtypes = [ctypes.c_int]
        L.sla_wide_query_tiles.argtypes = [ctypes.c_int]
        L.sla_profile_read.argtypes = [ctypes.c_char_p, sz]
        L.sla_profile_mfma_peak.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double), vp]
        L.sla_profile_dq_atomics.argtypes = [pp, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.sla_strerror.argtypes = [ctypes.c_int]
        L.sla_strerror.restype = ctypes.c_char_p
        for n in EXPORTS[:-1]:
            getattr(L, n).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise SLAError(f"{what} failed: {lib().sla_strerror(rc).decode()} (code {rc})")


def make_params(B: int, H: int, N: int, d: int, k_h: float, k_l: float, dtype: torch.dtype,
                phi: int = SLA_PHI_SOFTMAX, bq: int = 64, bkv: int = 64,
                layout: int = SLA_BHND, strides: Tuple[int, int, int] = (0, 0, 0)) -> sla_params:
    """layout: SLA_BHND ([B,H,N,d] tensors), SLA_BNHD ([B,N,H,d]) or SLA_STRIDED with
    strides = element strides (batch, head, token) of [B,H,N,d] views, e.g. of the slices of a
    fused projection output.  bq: query block size of the mask, a multiple of 64 up to 256."""
    code = {torch.float32: SLA_F32, torch.bfloat16: SLA_BF16}[dtype]
    return sla_params(B, H, N, d, bq, bkv, k_h, k_l, phi, code, layout, *strides)


def sla_sizes(p: sla_params) -> sla_sizes_t:
    z = sla_sizes_t()
    _check(lib().sla_sizes(ctypes.byref(p), ctypes.byref(z)), "sla_sizes")
    return z


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _buf(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _tdtype(p: sla_params) -> torch.dtype:
    return torch.float32 if p.dtype == SLA_F32 else torch.bfloat16


def _dense(t: torch.Tensor, p: sla_params, what: str) -> torch.Tensor:
    """Q, K, V, O, dO, dQ, dK, dV: the storage type, shape and memory order the params state.  The
    C ABI sees bare pointers, so a tensor of another type or shape would be read out of bounds."""
    if not isinstance(t, torch.Tensor) or t.dtype != _tdtype(p):
        raise SLAError(f"{what}: expected a {_tdtype(p)} tensor, got {getattr(t, 'dtype', type(t))}")
    if p.layout == SLA_STRIDED:
        want, st = (p.B, p.H, p.N, p.d), (p.stride_b, p.stride_h, p.stride_n, 1)
        if tuple(t.shape) != want or tuple(t.stride()) != st or not t.is_cuda:
            raise SLAError(f"{what}: expected a device tensor (view) of shape {want} with strides {st}")
        return t
    want = (p.B, p.N, p.H, p.d) if p.layout == SLA_BNHD else (p.B, p.H, p.N, p.d)
    if tuple(t.shape) != want or not t.is_contiguous() or not t.is_cuda:
        raise SLAError(f"{what}: expected a contiguous device tensor of shape {want}")
    return t


def _packed(t: torch.Tensor, shape, dtype: torch.dtype, what: str) -> torch.Tensor:
    """a contiguous device tensor of exactly this shape and type (W, M_c, dW, block scores)"""
    if (not isinstance(t, torch.Tensor) or t.dtype != dtype or tuple(t.shape) != tuple(shape)
            or not t.is_contiguous() or not t.is_cuda):
        raise SLAError(f"{what}: expected a contiguous {dtype} device tensor of shape {tuple(shape)}, got "
                       f"{getattr(t, 'dtype', type(t))} {tuple(getattr(t, 'shape', ()))}")
    return t


def _bytes(t: torch.Tensor, need: int, what: str) -> torch.Tensor:
    """an opaque byte buffer (tables, saved tensors, workspace) of at least `need` bytes"""
    if (not isinstance(t, torch.Tensor) or t.dtype != torch.uint8 or t.dim() != 1 or not t.is_contiguous()
            or not t.is_cuda or t.numel() < need):
        raise SLAError(f"{what}: expected a contiguous uint8 device buffer of at least {need} bytes")
    return t


def _like(t: torch.Tensor, p: sla_params) -> torch.Tensor:
    """an output tensor laid out as the params say (for strided views: the same strides)"""
    if p.layout == SLA_STRIDED:
        return torch.empty_strided(tuple(t.shape), tuple(t.stride()), dtype=t.dtype, device=t.device)
    return torch.empty_like(t)


def sla_build_mask(p: sla_params, Q: torch.Tensor, K: torch.Tensor,
                   workspace: Optional[torch.Tensor] = None, Mc: Optional[torch.Tensor] = None,
                   luts: Optional[torch.Tensor] = None
                   ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Returns (Mc int8 [B,H,Tq,T], luts, workspace); the workspace keeps pool(Q), pool(K), s."""
    z = sla_sizes(p)
    _dense(Q, p, "Q"); _dense(K, p, "K")
    if Mc is None:
        Mc = torch.empty((p.B, p.H, z.Tq, z.T), dtype=torch.int8, device=Q.device)
    if luts is None:
        luts = _buf(z.luts_bytes, Q.device)
    ws = workspace if workspace is not None else _buf(z.ws_mask_bytes, Q.device)
    _packed(Mc, (p.B, p.H, z.Tq, z.T), torch.int8, "Mc")
    _bytes(luts, z.luts_bytes, "luts"); _bytes(ws, z.ws_mask_bytes, "workspace")
    _check(lib().sla_build_mask(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(Mc), _ptr(luts), _ptr(ws),
                                ws.numel(), _stream()), "sla_build_mask")
    return Mc, luts, ws


def sla_build_mask_static(p: sla_params, Q: torch.Tensor, K: torch.Tensor, Mc: torch.Tensor,
                          luts: torch.Tensor) -> None:
    """sla_build_mask with the workspace inside the library (no allocation in the call): the
    caller passes the outputs Mc int8 [B,H,Tq,T] and luts (luts_bytes)."""
    z = sla_sizes(p)
    _dense(Q, p, "Q"); _dense(K, p, "K")
    _packed(Mc, (p.B, p.H, z.Tq, z.T), torch.int8, "Mc")
    _bytes(luts, z.luts_bytes, "luts")
    _check(lib().sla_build_mask_static(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(Mc), _ptr(luts), _stream()),
           "sla_build_mask_static")


def sla_classify_scores(p: sla_params, s: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    z = sla_sizes(p)
    _packed(s, (p.B, p.H, z.Tq, z.T), torch.float32, "s")
    Mc = torch.empty((p.B, p.H, z.Tq, z.T), dtype=torch.int8, device=s.device)
    luts = _buf(z.luts_bytes, s.device)
    _check(lib().sla_classify_scores(ctypes.byref(p), _ptr(s), _ptr(Mc), _ptr(luts), _stream()),
           "sla_classify_scores")
    return Mc, luts


def sla_forward(p: sla_params, Q, K, V, W, Mc, luts, O: Optional[torch.Tensor] = None,
                saved: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                need_saved: bool = True) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """Returns (O, saved).  saved is None when need_saved is False (inference)."""
    z = sla_sizes(p)
    for n, t in (("Q", Q), ("K", K), ("V", V)):
        _dense(t, p, n)
    if O is None:
        O = _like(Q, p)
    if saved is None and need_saved:
        saved = _buf(z.saved_bytes, Q.device)
    ws = workspace if workspace is not None else _buf(z.ws_forward_bytes, Q.device)
    _dense(O, p, "O")
    _packed(W, (p.d, p.d), _tdtype(p), "W")
    _packed(Mc, (p.B, p.H, z.Tq, z.T), torch.int8, "Mc")
    _bytes(luts, z.luts_bytes, "luts"); _bytes(ws, z.ws_forward_bytes, "workspace")
    if saved is not None:
        _bytes(saved, z.saved_bytes, "saved")
    _check(lib().sla_forward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(W), _ptr(Mc),
                             _ptr(luts), _ptr(O), _ptr(saved), _ptr(ws), ws.numel(), _stream()),
           "sla_forward")
    return O, saved


def sla_backward(p: sla_params, Q, K, V, W, Mc, luts, saved, dO,
                 workspace: Optional[torch.Tensor] = None, out=None):
    """Returns (dQ, dK, dV, dW); dW is float32 [d, d]."""
    z = sla_sizes(p)
    for n, t in (("Q", Q), ("K", K), ("V", V), ("dO", dO)):
        _dense(t, p, n)
    if out is None:
        dQ, dK, dV = _like(Q, p), _like(K, p), _like(V, p)
        dW = torch.empty((p.d, p.d), dtype=torch.float32, device=Q.device)
    else:
        dQ, dK, dV, dW = out
    ws = workspace if workspace is not None else _buf(z.ws_backward_bytes, Q.device)
    for n, t in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        _dense(t, p, n)
    _packed(W, (p.d, p.d), _tdtype(p), "W")
    _packed(dW, (p.d, p.d), torch.float32, "dW")
    _packed(Mc, (p.B, p.H, z.Tq, z.T), torch.int8, "Mc")
    _bytes(luts, z.luts_bytes, "luts"); _bytes(saved, z.saved_bytes, "saved")
    _bytes(ws, z.ws_backward_bytes, "workspace")
    _check(lib().sla_backward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(W), _ptr(Mc),
                              _ptr(luts), _ptr(saved), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV),
                              _ptr(dW), _ptr(ws), ws.numel(), _stream()), "sla_backward")
    return dQ, dK, dV, dW


def sla_aggregate_ws_bytes(p: sla_params, method: int) -> int:
    n = ctypes.c_uint64()
    _check(lib().sla_aggregate_ws_bytes(ctypes.byref(p), method, ctypes.byref(n)), "sla_aggregate_ws_bytes")
    return n.value


def sla_aggregate_states(p: sla_params, method: int, luts: torch.Tensor, h: torch.Tensor,
                         workspace: Optional[torch.Tensor] = None, out=None
                         ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Alg. 1's accumulation line alone.  h: bf16 [B,H,T,d*d+d] state rows; returns
    (H bf16 [B,H,T,d*d], Z float32 [B,H,T,d]).  method: one of SLA_AGG_*."""
    z = sla_sizes(p)
    want = (p.B, p.H, z.T, p.d * p.d + p.d)
    if tuple(h.shape) != want or h.dtype != torch.bfloat16 or not h.is_contiguous() or not h.is_cuda:
        raise SLAError(f"h: expected a contiguous bf16 device tensor of shape {want}")
    if out is None:
        out = (torch.empty((p.B, p.H, z.T, p.d * p.d), dtype=torch.bfloat16, device=h.device),
               torch.empty((p.B, p.H, z.T, p.d), dtype=torch.float32, device=h.device))
    need = sla_aggregate_ws_bytes(p, method)
    ws = workspace if workspace is not None else (_buf(need, h.device) if need else None)
    _bytes(luts, z.luts_bytes, "luts")
    _packed(out[0], (p.B, p.H, z.T, p.d * p.d), torch.bfloat16, "outH")
    _packed(out[1], (p.B, p.H, z.T, p.d), torch.float32, "outZ")
    if need:
        _bytes(ws, need, "workspace")
    _check(lib().sla_aggregate_states(ctypes.byref(p), method, _ptr(luts), _ptr(h), _ptr(out[0]), _ptr(out[1]),
                                      _ptr(ws), ws.numel() if ws is not None else 0, _stream()),
           "sla_aggregate_states")
    return out


def sla_wide_query_tiles(on: bool) -> None:
    """Eight-wave kernels for query blocks of 128 / 256 tokens (off by default: slower)."""
    _check(lib().sla_wide_query_tiles(1 if on else 0), "sla_wide_query_tiles")


def sla_profile_enable(on: bool) -> None:
    _check(lib().sla_profile_enable(1 if on else 0), "sla_profile_enable")


def sla_profile_mfma_peak(iters: int = 4096) -> float:
    """Sustained TFLOP/s of a register-only bf16 MFMA loop on this device (waits for it)."""
    out = ctypes.c_double()
    _check(lib().sla_profile_mfma_peak(iters, ctypes.byref(out), _stream()), "sla_profile_mfma_peak")
    return out.value


def sla_profile_dq_atomics(p: sla_params, luts: torch.Tensor, acc: torch.Tensor) -> float:
    """ms of the float atomics that accumulating dQ inside the column-wise kernel would issue
    (acc: float32 [B,H,N,d], receives one addition of 1 per critical pair and element)."""
    z = sla_sizes(p)
    _bytes(luts, z.luts_bytes, "luts")
    _packed(acc, (p.B, p.H, p.N, p.d), torch.float32, "acc")
    out = ctypes.c_double()
    _check(lib().sla_profile_dq_atomics(ctypes.byref(p), _ptr(luts), _ptr(acc), ctypes.byref(out), _stream()),
           "sla_profile_dq_atomics")
    return out.value


def sla_profile_read() -> Dict[str, Tuple[int, float]]:
    """{kernel name: (launch count, total ms)} of the kernels timed since the last read."""
    buf = ctypes.create_string_buffer(1 << 16)
    _check(lib().sla_profile_read(buf, len(buf)), "sla_profile_read")
    out = {}
    for line in buf.value.decode().splitlines():
        n, c, ms = line.split()
        out[n] = (int(c), float(ms))
    return out


# ---- views into the opaque buffers (layout documented in include/sla.h)

def _view(buf: torch.Tensor, off: int, shape, dtype: torch.dtype) -> torch.Tensor:
    n = 1
    for s in shape:
        n *= s
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    return buf[off:off + nbytes].view(dtype).view(*shape)


def saved_views(p: sla_params, saved: torch.Tensor) -> Dict[str, torch.Tensor]:
    z = sla_sizes(p)
    dt = torch.float32 if p.dtype == SLA_F32 else torch.bfloat16
    d = p.d
    if p.dtype == SLA_F32:
        HZ = _view(saved, z.saved_HZ, (p.B, p.H, z.T, d * d + d), torch.float32)
        Hi = HZ[..., :d * d].view(p.B, p.H, z.T, d, d).transpose(-1, -2)
        Zi = HZ[..., d * d:]
    else:
        Hi = _view(saved, z.saved_HZ, (p.B, p.H, z.T, d, d), torch.bfloat16).transpose(-1, -2)
        Zi = _view(saved, z.saved_Z, (p.B, p.H, z.T, d), torch.float32)
    return {"Os": _view(saved, z.saved_Os, (p.B, p.H, p.N, d), dt),
            "Ol": _view(saved, z.saved_Ol, (p.B, p.H, p.N, d), dt),
            "L": _view(saved, z.saved_L, (p.B, p.H, p.N), torch.float32),
            # H_i[c][e] is stored transposed: element e*d + c
            "Hi": Hi, "Zi": Zi}


def lut_views(p: sla_params, luts: torch.Tensor) -> Dict[str, torch.Tensor]:
    z = sla_sizes(p)
    return {"row_idx": _view(luts, z.lut_row_idx, (p.B, p.H, z.T, z.n_h), torch.int32),
            "col_ptr": _view(luts, z.lut_col_ptr, (p.B, p.H, z.T + 1), torch.int32),
            "col_rows": _view(luts, z.lut_col_rows, (p.B, p.H, z.T * z.n_h), torch.int32),
            "ind": _view(luts, z.lut_ind, (p.B, p.H, z.T, (z.T + 63) // 64), torch.int64),
            "ind_t": _view(luts, z.lut_ind_t, (p.B, p.H, z.T, (z.T + 63) // 64), torch.int64),
            "col_order": _view(luts, z.lut_col_order, (p.B, p.H, z.T), torch.int32)}


def mask_ws_views(p: sla_params, ws: torch.Tensor) -> Dict[str, torch.Tensor]:
    z = sla_sizes(p)
    return {"qbar": _view(ws, z.ws_mask_qbar, (p.B, p.H, z.Tq, p.d), torch.float32),
            "kbar": _view(ws, z.ws_mask_kbar, (p.B, p.H, z.T, p.d), torch.float32),
            "scores": _view(ws, z.ws_mask_scores, (p.B, p.H, z.Tq, z.T), torch.float32)}
