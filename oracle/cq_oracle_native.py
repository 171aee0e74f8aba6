"""ctypes front end of the C++ oracle twin (oracle/cq_oracle.cpp): TEST INFRASTRUCTURE ONLY.

Same results as oracle/cq_oracle.py (codes and stored parameters bit for bit, attention to
1e-12, both asserted by tests/test_oracle_native.py), fast enough for whole benchmark-size
calls and spread over all host threads.  Argument marshalling only: the arithmetic is in
the C++ source, which follows the paper step by step.  Independent of the HIP library.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import build as _build

AXIS_CHANNEL, AXIS_TOKEN = 0, 1
CALIB_NONE, CALIB_DYNAMIC, CALIB_FIXED = 0, 1, 2

_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load oracle/libcq_oracle.so, building it first when it is missing or older than its source."""
    global _lib
    if _lib is None:
        path = _build.build_oracle(force=False)
        L = ctypes.CDLL(path)
        V, I, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.cqo_max_threads.restype = I
        L.cqo_max_threads.argtypes = []
        L.cqo_quantize.restype = I
        L.cqo_quantize.argtypes = [V, ctypes.c_int64, I, I, I, I, I, V, V, V]
        L.cqo_decode_attn.restype = I
        L.cqo_decode_attn.argtypes = [V, V, V, V, I, I, V, V, V, I, I, V, V, I, I, I, I, I, I, I, I, I,
                                      D, D, D, D, D, V]
        _lib = L
    return _lib


def max_threads() -> int:
    return int(lib().cqo_max_threads())


def _f16_bits(x) -> np.ndarray:
    x = np.ascontiguousarray(x)
    assert x.dtype == np.float16, x.dtype
    return x.view(np.uint16)


def quantize_tensor(x, bits: int, axis: int, group: int) -> dict:
    """x [..., n, d] float16 -> dict(words uint32, scale float32, min float16, bits, axis, group)
    with the numpy oracle's shapes (codes are not materialised; oracle.cq_oracle.unpack gives them)."""
    xb = _f16_bits(x)
    n, d = xb.shape[-2], xb.shape[-1]
    lead = xb.shape[:-2]
    rows = int(np.prod(lead)) if lead else 1
    meta = (n // group, d) if axis == AXIS_CHANNEL else (n, d // group)
    words = np.empty(lead + (n, d * bits // 32), dtype=np.uint32)
    scale = np.empty(lead + meta, dtype=np.float32)
    minv = np.empty(lead + meta, dtype=np.float16)
    rc = lib().cqo_quantize(xb.ctypes.data, rows, n, d, bits, axis, group, words.ctypes.data,
                            scale.ctypes.data, minv.ctypes.data)
    if rc != 0:
        raise ValueError("cqo_quantize: status %d" % rc)
    return {"words": words, "scale": scale, "min": minv, "bits": bits, "axis": axis, "group": group}


def decode_attn(q, kq: Optional[dict], vq: Optional[dict], k_text=None, v_text=None, n_text: int = 0,
                calib_mode: int = CALIB_DYNAMIC, tau1: float = 0.0, tau2: float = 0.0,
                gamma: float = 0.0, delta: float = 0.0, softmax_scale: float = 0.0) -> np.ndarray:
    """q [B, Hq, d] float16; kq / vq from quantize_tensor for [B, Hkv, n_vis, d] (None when there
    are no quantized tokens); k_text / v_text [B, Hkv, cap, d] float16.  Returns [B, Hq, d] float64."""
    qb = _f16_bits(q)
    B, Hq, d = qb.shape
    if kq is not None and kq["words"].shape[-2] > 0:
        kw, vw = np.ascontiguousarray(kq["words"]), np.ascontiguousarray(vq["words"])
        Hkv, n_vis, bits = kw.shape[1], kw.shape[2], kq["bits"]
        ks, km = np.ascontiguousarray(kq["scale"]), _f16_bits(kq["min"])
        vs, vm = np.ascontiguousarray(vq["scale"]), _f16_bits(vq["min"])
        k_args = (kw.ctypes.data, ks.ctypes.data, km.ctypes.data, kq["axis"], kq["group"])
        v_args = (vw.ctypes.data, vs.ctypes.data, vm.ctypes.data, vq["axis"], vq["group"])
    else:
        n_vis, bits, Hkv = 0, 1, None
        k_args = v_args = (None, None, None, 0, 1)
    kt = vt = None
    cap = 0
    if n_text > 0:
        kt, vt = _f16_bits(k_text), _f16_bits(v_text)
        assert kt.shape == vt.shape and kt.shape[0] == B and kt.shape[3] == d
        cap = kt.shape[2]
        Hkv = kt.shape[1] if Hkv is None else Hkv
        assert kt.shape[1] == Hkv
    out = np.zeros((B, Hq, d), dtype=np.float64)
    rc = lib().cqo_decode_attn(qb.ctypes.data, *k_args, *v_args,
                               kt.ctypes.data if kt is not None else None,
                               vt.ctypes.data if vt is not None else None,
                               B, Hq, Hkv, d, n_vis, bits, n_text, cap, calib_mode,
                               float(tau1), float(tau2), float(gamma), float(delta),
                               float(softmax_scale), out.ctypes.data)
    if rc != 0:
        raise ValueError("cqo_decode_attn: status %d" % rc)
    return out
