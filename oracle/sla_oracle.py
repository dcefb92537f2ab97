"""ctypes loader for the CPU oracle (oracle/sla_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this module; the
product package never does.  Arrays are numpy, [BH, N, d] (or [B, H, N, d], flattened here).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sla_oracle.cpp")
_LIB = os.path.join(_HERE, "libsla_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fused multiply-add contraction, OpenMP over heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-std=c++17", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _flat(x: np.ndarray, dt) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=dt)
    return x.reshape(-1, x.shape[-2], x.shape[-1])


def counts(Tn: int, k_h: float, k_l: float) -> Tuple[int, int]:
    a, b = ctypes.c_int(), ctypes.c_int()
    lib().sla_oracle_counts(ctypes.c_int(Tn), ctypes.c_double(k_h), ctypes.c_double(k_l),
                            ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


def pool(X: np.ndarray, b: int) -> np.ndarray:
    X = np.ascontiguousarray(X, np.float32)
    N, d = X.shape
    out = np.empty((-(-N // b), d), np.float32)
    lib().sla_oracle_pool(_p(X), N, d, b, _p(out))
    return out


def scores(qbar: np.ndarray, kbar: np.ndarray) -> np.ndarray:
    qbar = np.ascontiguousarray(qbar, np.float32)
    kbar = np.ascontiguousarray(kbar, np.float32)
    s = np.empty((qbar.shape[0], kbar.shape[0]), np.float32)
    lib().sla_oracle_scores(_p(qbar), _p(kbar), qbar.shape[0], kbar.shape[0], qbar.shape[1], _p(s))
    return s


def classify(s: np.ndarray, n_h: int, n_l: int) -> np.ndarray:
    s = np.ascontiguousarray(s, np.float32)
    rows, Tn = s.reshape(-1, s.shape[-1]).shape
    Mc = np.empty(s.shape, np.int8)
    lib().sla_oracle_classify(_p(s), rows, Tn, n_h, n_l, _p(Mc))
    return Mc


def compressed_weights(s: np.ndarray) -> np.ndarray:
    s = np.ascontiguousarray(s, np.float32)
    rows, Tn = s.reshape(-1, s.shape[-1]).shape
    Pc = np.empty(s.shape, np.float32)
    lib().sla_oracle_pc(_p(s), rows, Tn, _p(Pc))
    return Pc


def build_mask(Q: np.ndarray, K: np.ndarray, k_h: float, k_l: float, bq: int = 64, bkv: int = 64,
               return_scores: bool = False):
    shape = Q.shape
    Qf, Kf = _flat(Q, np.float32), _flat(K, np.float32)
    BH, N, d = Qf.shape
    Tm, Tn = -(-N // bq), -(-N // bkv)
    Mc = np.empty((BH, Tm, Tn), np.int8)
    s = np.empty((BH, Tm, Tn), np.float32) if return_scores else None
    rc = lib().sla_oracle_build_mask(BH, N, d, bq, bkv, ctypes.c_double(k_h), ctypes.c_double(k_l),
                                     _p(Qf), _p(Kf), _p(Mc), _p(s))
    assert rc == 0
    Mc = Mc.reshape(shape[:-2] + (Tm, Tn))
    if return_scores:
        return Mc, s.reshape(shape[:-2] + (Tm, Tn))
    return Mc


def accumulate(h: np.ndarray, Mc: np.ndarray) -> np.ndarray:
    """Alg. 1 accumulation line alone: out[..., i, :] = sum of h[..., j, :] over the marginal
    blocks j of row i.  h: [..., Tn, len]; Mc: [..., Tm, Tn]; returns float64 [..., Tm, len]."""
    Tn, ln = h.shape[-2:]
    Tm = Mc.shape[-2]
    hf = np.ascontiguousarray(h, np.float64).reshape(-1, Tn, ln)
    mf = np.ascontiguousarray(Mc, np.int8).reshape(-1, Tm, Tn)
    assert hf.shape[0] == mf.shape[0] and Mc.shape[-1] == Tn
    out = np.empty((hf.shape[0], Tm, ln), np.float64)
    lib().sla_oracle_accumulate(hf.shape[0], Tm, Tn, ln, _p(hf), _p(mf), _p(out))
    return out.reshape(h.shape[:-2] + (Tm, ln))


def forward(Q, K, V, W, Mc, phi: int = 0, bq: int = 64, bkv: int = 64,
            dtype=np.float64) -> Dict[str, np.ndarray]:
    """Algorithm 1 with a given mask.  Returns O, Os, Ol, L, Hi, Zi in `dtype`."""
    shape = Q.shape
    Qf, Kf, Vf = _flat(Q, dtype), _flat(K, dtype), _flat(V, dtype)
    Wf = np.ascontiguousarray(W, dtype)
    BH, N, d = Qf.shape
    Tm, Tn = -(-N // bq), -(-N // bkv)
    Mcf = np.ascontiguousarray(Mc, np.int8).reshape(BH, Tm, Tn)
    O, Os, Ol = (np.empty((BH, N, d), dtype) for _ in range(3))
    L = np.empty((BH, N), dtype)
    Hi = np.empty((BH, Tm, d, d), dtype)
    Zi = np.empty((BH, Tm, d), dtype)
    fn = lib().sla_oracle_forward_f64 if dtype == np.float64 else lib().sla_oracle_forward_f32
    rc = fn(BH, N, d, bq, bkv, phi, _p(Qf), _p(Kf), _p(Vf), _p(Wf), _p(Mcf), _p(O), _p(Os), _p(Ol),
            _p(L), _p(Hi), _p(Zi))
    assert rc == 0
    lead = shape[:-2]
    return {"O": O.reshape(lead + (N, d)), "Os": Os.reshape(lead + (N, d)),
            "Ol": Ol.reshape(lead + (N, d)), "L": L.reshape(lead + (N,)),
            "Hi": Hi.reshape(lead + (Tm, d, d)), "Zi": Zi.reshape(lead + (Tm, d))}


def backward(Q, K, V, W, Mc, fwd: Dict[str, np.ndarray], dO, phi: int = 0, bq: int = 64,
             bkv: int = 64, dtype=np.float64) -> Dict[str, np.ndarray]:
    """Algorithm 2 plus the chain rule through phi and Proj.  Returns dQ, dK, dV, dW, dQphi, dKphi."""
    shape = Q.shape
    Qf, Kf, Vf, dOf = _flat(Q, dtype), _flat(K, dtype), _flat(V, dtype), _flat(dO, dtype)
    Wf = np.ascontiguousarray(W, dtype)
    BH, N, d = Qf.shape
    Tm, Tn = -(-N // bq), -(-N // bkv)
    Mcf = np.ascontiguousarray(Mc, np.int8).reshape(BH, Tm, Tn)
    c = lambda k: np.ascontiguousarray(fwd[k], dtype)
    L, Hi, Zi, Os, Ol = c("L"), c("Hi"), c("Zi"), c("Os"), c("Ol")
    dQ, dK, dV, dQphi, dKphi = (np.empty((BH, N, d), dtype) for _ in range(5))
    dW = np.zeros((d, d), dtype)
    fn = lib().sla_oracle_backward_f64 if dtype == np.float64 else lib().sla_oracle_backward_f32
    rc = fn(BH, N, d, bq, bkv, phi, _p(Qf), _p(Kf), _p(Vf), _p(Wf), _p(Mcf), _p(L), _p(Hi), _p(Zi),
            _p(Os), _p(Ol), _p(dOf), _p(dQ), _p(dK), _p(dV), _p(dW), _p(dQphi), _p(dKphi))
    assert rc == 0
    lead = shape[:-2]
    r = lambda a: a.reshape(lead + (N, d))
    return {"dQ": r(dQ), "dK": r(dK), "dV": r(dV), "dW": dW, "dQphi": r(dQphi), "dKphi": r(dKphi)}
