"""ctypes loader for oracle/libvla_oracle.so (numpy float64 in, float64 out).

Argument marshalling only -- all arithmetic is in vla_oracle.c.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvla_oracle.so")
TRACE_WIDTH = 8

_lib = None


class _Opts(ctypes.Structure):
    _fields_ = [("lambda0", ctypes.c_double), ("eps", ctypes.c_double),
                ("u", ctypes.c_void_p), ("u_scale", ctypes.c_double),
                ("refresh_period", ctypes.c_int), ("refresh_eta", ctypes.c_double),
                ("step_offset", ctypes.c_int), ("normalise_output", ctypes.c_int), ("feature_map", ctypes.c_int),
                ("zkey0", ctypes.c_void_p), ("zkey_T", ctypes.c_void_p)]


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build_oracle
        build_oracle.build()
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.c_void_p
    lib.vla_oracle_forward_f64.restype = ctypes.c_int
    lib.vla_oracle_forward_f64.argtypes = [P] * 9 + [ctypes.c_int] * 5 + [ctypes.POINTER(_Opts)]
    lib.vla_oracle_linear_attention_f64.restype = ctypes.c_int
    lib.vla_oracle_linear_attention_f64.argtypes = [P] * 6 + [ctypes.c_int] * 5
    lib.vla_oracle_trace_width.restype = ctypes.c_int
    lib.vla_oracle_num_threads.restype = ctypes.c_int
    assert lib.vla_oracle_trace_width() == TRACE_WIDTH
    _lib = lib
    return lib


def _f64(x):
    return None if x is None else np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _ptr(x):
    return None if x is None else x.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(load().vla_oracle_num_threads())


def forward(q, k, v, S0=None, A0=None, *, lambda0=0.1, eps=1e-4, u=None, u_scale=1.0,
            refresh_period=0, refresh_eta=1e-3, step_offset=0, normalise_output=False, feature_map=False,
            zkey0=None, trace=False):
    """q,k [B,H,T,d_k], v [B,H,T,d_v] -> dict(o, S_T, A_T[, trace]) in float64."""
    lib = load()
    q, k, v, S0, A0, u, zkey0 = map(_f64, (q, k, v, S0, A0, u, zkey0))
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (B, H, T, dk) and v.shape == (B, H, T, dv)
    if S0 is not None:
        assert S0.shape == (B, H, dv, dk)
    if A0 is not None:
        assert A0.shape == (B, H, dk, dk)
    if u is not None:
        assert u.shape == (B, H, T, dk)
    o = np.empty((B, H, T, dv), dtype=np.float64)
    S_T = np.empty((B, H, dv, dk), dtype=np.float64)
    A_T = np.empty((B, H, dk, dk), dtype=np.float64)
    tr = np.empty((B, H, T, TRACE_WIDTH), dtype=np.float64) if trace else None
    if zkey0 is not None:
        assert zkey0.shape == (B, H, dk)
    zkey_T = np.empty((B, H, dk), dtype=np.float64)
    opts = _Opts(float(lambda0), float(eps), _ptr(u), float(u_scale), int(refresh_period),
                 float(refresh_eta), int(step_offset), int(bool(normalise_output)), int(bool(feature_map)),
                 _ptr(zkey0), _ptr(zkey_T))
    rc = lib.vla_oracle_forward_f64(_ptr(q), _ptr(k), _ptr(v), _ptr(S0), _ptr(A0), _ptr(o),
                                    _ptr(S_T), _ptr(A_T), _ptr(tr), B, H, T, dk, dv,
                                    ctypes.byref(opts))
    if rc != 0:
        raise ValueError(f"vla_oracle_forward_f64 returned {rc}")
    out = {"o": o, "S_T": S_T, "A_T": A_T, "zkey_T": zkey_T}
    if trace:
        out["trace"] = tr
    return out


def linear_attention(q, k, v):
    """Additive baseline S_t = S_{t-1} + v_t k_t^T, o_t = S_t q_t; returns o, S_T, normS."""
    lib = load()
    q, k, v = map(_f64, (q, k, v))
    B, H, T, dk = k.shape
    dv = v.shape[-1]
    o = np.empty((B, H, T, dv), dtype=np.float64)
    S_T = np.empty((B, H, dv, dk), dtype=np.float64)
    normS = np.empty((B, H, T), dtype=np.float64)
    rc = lib.vla_oracle_linear_attention_f64(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(S_T),
                                             _ptr(normS), B, H, T, dk, dv)
    if rc != 0:
        raise ValueError(f"vla_oracle_linear_attention_f64 returned {rc}")
    return {"o": o, "S_T": S_T, "normS": normS}
