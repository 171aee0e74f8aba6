"""C-ABI checks that need no GPU: the library loads, exports what include/cq.h declares, and
rejects bad arguments on the host before any HIP call (fake non-NULL pointers are never
dereferenced because no launch happens)."""
import ctypes
import os
import re

import pytest

from paper_2502_14882_amd import binding as cq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000     # aligned, non-NULL, never touched


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"cq_quantize_kv", "cq_decode_attn", "cq_decode_workspace_bytes", "cq_status_string",
            "cq_last_error", "cq_version", "cq_set_kernel_path"} <= set(names)
    L = cq.lib()
    for n in names:
        assert hasattr(L, n), n
    assert cq.cq_version() >= 100


def test_struct_sizes_match_header():
    assert ctypes.sizeof(cq.CqLayout) == 40
    assert ctypes.sizeof(cq.CqQTensor) == 3 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(cq.CqCalib) == 20


def _quant(layout, k=FAKE, v=FAKE, ko=(FAKE, FAKE, FAKE), vo=(FAKE, FAKE, FAKE)):
    ks = cq.CqQTensor(*ko) if ko is not None else None
    vs = cq.CqQTensor(*vo) if vo is not None else None
    return cq.lib().cq_quantize_kv(ctypes.byref(layout), k, v,
                                   ctypes.byref(ks) if ks else None,
                                   ctypes.byref(vs) if vs else None, None)


def test_quantize_argument_errors():
    ok = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, n_vis=256)
    assert _quant(cq.make_layout(**{**ok, "n_vis": 0})) == cq.CQ_OK          # empty: no-op
    assert _quant(cq.make_layout(**ok), k=None) == cq.CQ_ERR_NULL
    assert _quant(cq.make_layout(**ok), ko=(FAKE, None, FAKE)) == cq.CQ_ERR_NULL
    assert _quant(cq.make_layout(**ok), k=None, ko=None, v=None, vo=None) == cq.CQ_ERR_NULL
    assert _quant(cq.make_layout(**ok), k=FAKE + 2) == cq.CQ_ERR_ALIGN
    assert _quant(cq.make_layout(**{**ok, "head_dim": 100})) == cq.CQ_ERR_SHAPE
    assert _quant(cq.make_layout(**{**ok, "head_dim": 512})) == cq.CQ_ERR_SHAPE
    assert _quant(cq.make_layout(**ok, bits=3)) == cq.CQ_ERR_UNSUPPORTED
    assert _quant(cq.make_layout(**ok, k_group=96)) == cq.CQ_ERR_SHAPE         # 256 % 96
    assert _quant(cq.make_layout(**ok, v_group=48)) == cq.CQ_ERR_SHAPE         # not mult of 32
    assert _quant(cq.make_layout(**ok, k_axis=7)) == cq.CQ_ERR_UNSUPPORTED
    assert _quant(cq.make_layout(**{**ok, "batch": 0})) == cq.CQ_ERR_SHAPE
    _quant(cq.make_layout(**ok, k_group=96))
    assert b"k_group" in cq.lib().cq_last_error()


def _decode(layout, n_text=4, cap=4, calib=None, ws=FAKE, ws_bytes=1 << 40, q=FAKE, out=FAKE,
            kt=FAKE, vt=FAKE, scale=0.0, k=(FAKE, FAKE, FAKE)):
    ks, vs = cq.CqQTensor(*k), cq.CqQTensor(FAKE, FAKE, FAKE)
    return cq.lib().cq_decode_attn(ctypes.byref(layout), q, ctypes.byref(ks), ctypes.byref(vs),
                                   kt, vt, n_text, cap,
                                   ctypes.byref(calib) if calib is not None else None, scale, out,
                                   ws, ws_bytes, None)


def test_decode_argument_errors():
    lay = cq.make_layout(2, 8, 2, 128, 256)
    assert _decode(lay, q=None) == cq.CQ_ERR_NULL
    assert _decode(lay, kt=None) == cq.CQ_ERR_NULL
    assert _decode(lay, k=(None, FAKE, FAKE)) == cq.CQ_ERR_NULL
    assert _decode(lay, n_text=5, cap=4) == cq.CQ_ERR_SHAPE
    assert _decode(lay, n_text=-1) == cq.CQ_ERR_SHAPE
    assert _decode(lay, ws=None) == cq.CQ_ERR_WORKSPACE
    assert _decode(lay, ws=FAKE + 16) == cq.CQ_ERR_WORKSPACE
    assert _decode(lay, ws_bytes=1024) == cq.CQ_ERR_WORKSPACE
    assert _decode(lay, out=FAKE + 8) == cq.CQ_ERR_ALIGN
    assert _decode(lay, calib=cq.make_calib(9)) == cq.CQ_ERR_UNSUPPORTED
    assert _decode(lay, calib=cq.make_calib(cq.CQ_CALIB_FIXED, 1, 2, 3.0, 3.0)) == cq.CQ_ERR_SHAPE
    assert _decode(lay, calib=cq.make_calib(cq.CQ_CALIB_DYNAMIC, float("nan"), 0)) == cq.CQ_ERR_SHAPE
    assert _decode(lay, scale=-1.0) == cq.CQ_ERR_SHAPE
    assert _decode(cq.make_layout(2, 7, 2, 128, 256)) == cq.CQ_ERR_SHAPE       # Hq % Hkv
    assert _decode(cq.make_layout(1, 1, 1, 128, 0), n_text=0, cap=0) == cq.CQ_ERR_SHAPE
    assert cq.lib().cq_status_string(cq.CQ_ERR_WORKSPACE).startswith(b"CQ_ERR_WORKSPACE")


def test_append_argument_errors():
    lay = cq.make_layout(2, 8, 2, 128, 256)
    f = cq.lib().cq_append_text_kv
    assert f(ctypes.byref(lay), None, FAKE, 0, 4, FAKE, FAKE, None) == cq.CQ_ERR_NULL
    assert f(ctypes.byref(lay), FAKE, FAKE, 0, 4, FAKE, None, None) == cq.CQ_ERR_NULL
    assert f(ctypes.byref(lay), FAKE, FAKE + 2, 0, 4, FAKE, FAKE, None) == cq.CQ_ERR_ALIGN
    assert f(ctypes.byref(lay), FAKE, FAKE, 4, 4, FAKE, FAKE, None) == cq.CQ_ERR_SHAPE   # tail full
    assert f(ctypes.byref(lay), FAKE, FAKE, -1, 4, FAKE, FAKE, None) == cq.CQ_ERR_SHAPE
    assert b"full" in cq.lib().cq_last_error()
    assert f(None, FAKE, FAKE, 0, 4, FAKE, FAKE, None) == cq.CQ_ERR_NULL


def test_tau_search_argument_errors():
    lay = cq.make_layout(2, 8, 2, 128, 256)
    L = cq.lib()
    need = cq.cq_tau_search_workspace_bytes(lay, 16, 4, 4)
    assert need > 0 and need % 256 == 0
    assert need >= 2 * 8 * (2 * 256 + 16) * 4        # the logits of both key sets
    assert cq.cq_tau_search_workspace_bytes(lay, 16, 9, 8) == 0      # more than 64 pairs
    assert cq.cq_tau_search_workspace_bytes(lay, 16, 0, 4) == 0
    kq = cq.CqQTensor(FAKE, FAKE, FAKE)
    grid = (ctypes.c_float * 4)(0.0, 1.0, 2.0, 3.0)
    bad = (ctypes.c_float * 4)(0.0, float("nan"), 2.0, 3.0)

    def call(lay=lay, q=FAKE, kx=FAKE, k=kq, kt=FAKE, n_text=16, cap=16, t1=grid, n1=4, t2=grid,
             n2=4, scale=0.0, out=FAKE, ws=FAKE + 0x100, ws_bytes=need):
        return L.cq_tau_search(ctypes.byref(lay), q, kx, ctypes.byref(k), kt, n_text, cap, t1, n1,
                               t2, n2, scale, out, ws, ws_bytes, None)

    assert call(kx=None) == cq.CQ_ERR_NULL
    assert call(out=None) == cq.CQ_ERR_NULL
    assert call(kt=None) == cq.CQ_ERR_NULL
    assert call(q=FAKE + 2) == cq.CQ_ERR_ALIGN
    assert call(out=FAKE + 4) == cq.CQ_ERR_ALIGN
    assert call(n_text=17) == cq.CQ_ERR_SHAPE
    assert call(n1=0) == cq.CQ_ERR_SHAPE
    assert call(t2=bad) == cq.CQ_ERR_SHAPE
    assert b"tau2[1]" in L.cq_last_error()
    assert call(ws=None) == cq.CQ_ERR_WORKSPACE
    assert call(ws_bytes=need - 256) == cq.CQ_ERR_WORKSPACE
    assert call(lay=cq.make_layout(2, 8, 2, 128, 0)) == cq.CQ_ERR_SHAPE    # nothing quantized


def test_measurement_aid_argument_errors():
    """The traffic skeleton of the quantizer rejects what it cannot run before any launch."""
    L = cq.lib()
    f = L.cq_bench_tile_traffic
    assert f(None, FAKE, FAKE, 4, 2048, 768, None) == cq.CQ_ERR_NULL
    assert f(FAKE, None, FAKE, 4, 2048, 768, None) == cq.CQ_ERR_NULL
    assert f(FAKE + 8, FAKE, FAKE, 4, 2048, 768, None) == cq.CQ_ERR_ALIGN
    assert f(FAKE, FAKE, FAKE + 2, 4, 2048, 768, None) == cq.CQ_ERR_ALIGN
    assert f(FAKE, FAKE, FAKE, 4, 2040, 768, None) == cq.CQ_ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, 4, 2048, 770, None) == cq.CQ_ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, 0, 2048, 768, None) == cq.CQ_OK          # nothing to do, no launch


def test_workspace_size_rule():
    lay = cq.make_layout(2, 8, 2, 128, 1024)
    n = cq.cq_decode_workspace_bytes(lay, 32)
    assert n > 0 and n % 256 == 0
    # it at least holds one fp32 logit per (batch, query head, token)
    assert n >= 2 * 8 * (1024 + 32) * 4
    assert cq.cq_decode_workspace_bytes(cq.make_layout(2, 8, 2, 100, 1024), 32) == 0
    bigger = cq.cq_decode_workspace_bytes(cq.make_layout(2, 8, 2, 128, 4096), 32)
    assert bigger > n


def test_kernel_path_switch():
    prev = cq.cq_set_kernel_path(cq.CQ_PATH_GENERIC)
    assert cq.cq_set_kernel_path(prev) == cq.CQ_PATH_GENERIC
    with pytest.raises(cq.CqError):
        cq.cq_set_kernel_path(42)


def test_binding_raises_when_library_is_missing(monkeypatch):
    monkeypatch.setattr(cq, "_lib", None)
    monkeypatch.setattr(cq, "LIB_PATH", "/nonexistent/libcq.so")
    with pytest.raises(RuntimeError, match="not built"):
        cq.lib()
