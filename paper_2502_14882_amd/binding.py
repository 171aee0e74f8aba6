"""ctypes binding of libcq.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module allocates output
tensors with torch (device memory and the current stream are all torch is used for)
and passes raw pointers.  There is no fallback: if libcq.so is missing or a call fails,
an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcq.so")

CQ_AXIS_CHANNEL, CQ_AXIS_TOKEN = 0, 1
CQ_CALIB_NONE, CQ_CALIB_DYNAMIC, CQ_CALIB_FIXED = 0, 1, 2
CQ_PATH_AUTO, CQ_PATH_GENERIC, CQ_PATH_TUNED = 0, 1, 2
CQ_OK, CQ_ERR_NULL, CQ_ERR_SHAPE, CQ_ERR_UNSUPPORTED = 0, -1, -2, -3
CQ_ERR_WORKSPACE, CQ_ERR_HIP, CQ_ERR_ALIGN = -4, -5, -6


class CqLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "n_vis", "bits",
        "k_axis", "v_axis", "k_group", "v_group")]


class CqQTensor(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("min", ctypes.c_void_p)]


class CqCalib(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("tau1", ctypes.c_float), ("tau2", ctypes.c_float),
                ("gamma", ctypes.c_float), ("delta", ctypes.c_float)]


class CqError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("cq status %d: %s" % (status, message))
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load libcq.so (once).  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libcq.so is not built (%s); run `python -m paper_2502_14882_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        P, I, V = ctypes.POINTER, ctypes.c_int32, ctypes.c_void_p
        L.cq_quantize_kv.restype = ctypes.c_int
        L.cq_quantize_kv.argtypes = [P(CqLayout), V, V, P(CqQTensor), P(CqQTensor), V]
        L.cq_decode_workspace_bytes.restype = ctypes.c_size_t
        L.cq_decode_workspace_bytes.argtypes = [P(CqLayout), I, P(CqCalib)]
        L.cq_decode_attn.restype = ctypes.c_int
        L.cq_decode_attn.argtypes = [P(CqLayout), V, P(CqQTensor), P(CqQTensor), V, V, I, I,
                                     P(CqCalib), ctypes.c_float, V, V, ctypes.c_size_t, V]
        L.cq_decode_attn_noalloc.restype = ctypes.c_int
        L.cq_decode_attn_noalloc.argtypes = [P(CqLayout), V, P(CqQTensor), P(CqQTensor), V, V, I, I,
                                             P(CqCalib), ctypes.c_float, V, V]
        L.cq_append_text_kv.restype = ctypes.c_int
        L.cq_append_text_kv.argtypes = [P(CqLayout), V, V, I, I, V, V, V]
        L.cq_append_text_kv_devlen.restype = ctypes.c_int
        L.cq_append_text_kv_devlen.argtypes = [P(CqLayout), V, V, V, I, V, V, V]
        L.cq_decode_attn_devlen.restype = ctypes.c_int
        L.cq_decode_attn_devlen.argtypes = [P(CqLayout), V, P(CqQTensor), P(CqQTensor), V, V, V, I, I,
                                            P(CqCalib), ctypes.c_float, V, V, ctypes.c_size_t, V]
        L.cq_tau_search_workspace_bytes.restype = ctypes.c_size_t
        L.cq_tau_search_workspace_bytes.argtypes = [P(CqLayout), I, I, I]
        L.cq_tau_search.restype = ctypes.c_int
        L.cq_tau_search.argtypes = [P(CqLayout), V, V, P(CqQTensor), V, I, I,
                                    P(ctypes.c_float), I, P(ctypes.c_float), I, ctypes.c_float, V, V,
                                    ctypes.c_size_t, V]
        L.cq_bench_set_kernel_path.restype = ctypes.c_int
        L.cq_bench_set_kernel_path.argtypes = [ctypes.c_int]
        L.cq_bench_set_decode_chunks.restype = ctypes.c_int
        L.cq_bench_set_decode_chunks.argtypes = [ctypes.c_int]
        L.cq_bench_stream_read.restype = ctypes.c_int
        L.cq_bench_stream_read.argtypes = [V, ctypes.c_size_t, V, V]
        L.cq_bench_stream_copy.restype = ctypes.c_int
        L.cq_bench_stream_copy.argtypes = [V, V, ctypes.c_size_t, V]
        L.cq_bench_tile_traffic.restype = ctypes.c_int
        L.cq_bench_tile_traffic.argtypes = [V, V, V, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, V]
        L.cq_status_string.restype = ctypes.c_char_p
        L.cq_status_string.argtypes = [ctypes.c_int]
        L.cq_last_error.restype = ctypes.c_char_p
        L.cq_last_error.argtypes = []
        L.cq_version.restype = ctypes.c_int
        L.cq_version.argtypes = []
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != CQ_OK:
        L = lib()
        msg = L.cq_last_error().decode() or L.cq_status_string(status).decode()
        raise CqError(status, msg)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(t: torch.Tensor) -> Optional[int]:
    if t.is_cuda:
        return torch.cuda.current_stream(t.device).cuda_stream or None
    return None


class QTensor(NamedTuple):
    """Device buffers of one quantized [B, Hkv, n_vis, d] tensor."""
    codes: torch.Tensor   # int32 storage of the uint32 words [B, Hkv, n_vis, d*bits/32]
    scale: torch.Tensor   # float32
    min: torch.Tensor     # float16

    def c_struct(self) -> CqQTensor:
        return CqQTensor(self.codes.data_ptr(), self.scale.data_ptr(), self.min.data_ptr())


def make_layout(batch, n_q_heads, n_kv_heads, head_dim, n_vis, bits=1,
                k_axis=CQ_AXIS_CHANNEL, v_axis=CQ_AXIS_TOKEN, k_group=128, v_group=128) -> CqLayout:
    return CqLayout(batch, n_q_heads, n_kv_heads, head_dim, n_vis, bits, k_axis, v_axis,
                    k_group, v_group)


def _meta_shape(layout: CqLayout, axis: int, group: int):
    B, H, n, d = layout.batch, layout.n_kv_heads, layout.n_vis, layout.head_dim
    if axis == CQ_AXIS_CHANNEL:
        return (B, H, n // max(group, 1), d)
    return (B, H, n, d // max(group, 1))


def alloc_qtensor(layout: CqLayout, axis: int, group: int, device) -> QTensor:
    B, H, n, d = layout.batch, layout.n_kv_heads, layout.n_vis, layout.head_dim
    codes = torch.empty((B, H, n, d * layout.bits // 32), dtype=torch.int32, device=device)
    shape = _meta_shape(layout, axis, group)
    return QTensor(codes, torch.empty(shape, dtype=torch.float32, device=device),
                   torch.empty(shape, dtype=torch.float16, device=device))


def cq_quantize_kv(layout: CqLayout, k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                   k_out: Optional[QTensor] = None, v_out: Optional[QTensor] = None):
    """Quantize fp16 k, v [B, Hkv, n_vis, d]; returns (k_out, v_out) QTensors."""
    ref = k if k is not None else v
    if k is not None and k_out is None:
        k_out = alloc_qtensor(layout, layout.k_axis, layout.k_group, k.device)
    if v is not None and v_out is None:
        v_out = alloc_qtensor(layout, layout.v_axis, layout.v_group, v.device)
    for t in (k, v):
        if t is not None:
            assert t.dtype == torch.float16 and t.is_contiguous()
    ks = k_out.c_struct() if k_out is not None else None
    vs = v_out.c_struct() if v_out is not None else None
    _check(lib().cq_quantize_kv(ctypes.byref(layout), _ptr(k), _ptr(v),
                                ctypes.byref(ks) if ks is not None else None,
                                ctypes.byref(vs) if vs is not None else None,
                                _stream(ref) if ref is not None else None))
    return k_out, v_out


def cq_decode_workspace_bytes(layout: CqLayout, n_text: int, calib: Optional[CqCalib] = None) -> int:
    return int(lib().cq_decode_workspace_bytes(ctypes.byref(layout), int(n_text),
                                               ctypes.byref(calib) if calib is not None else None))


def _check_decode_tensors(layout: CqLayout, q, k_text, v_text, out) -> int:
    """Shapes against the layout (a mismatch would be an out-of-bounds read on the device);
    returns the tail's capacity."""
    assert q.dtype == torch.float16 and q.is_contiguous()
    assert tuple(q.shape) == (layout.batch, layout.n_q_heads, layout.head_dim), \
        "q is %s, the layout says %s" % (tuple(q.shape), (layout.batch, layout.n_q_heads, layout.head_dim))
    assert out.dtype == torch.float16 and out.is_contiguous() and out.shape == q.shape
    if k_text is None:
        assert v_text is None
        return 0
    assert k_text.dtype == torch.float16 and k_text.is_contiguous()
    assert v_text is not None and v_text.dtype == torch.float16 and v_text.is_contiguous()
    assert v_text.shape == k_text.shape and k_text.dim() == 4
    assert tuple(k_text.shape[:2]) == (layout.batch, layout.n_kv_heads) and \
        k_text.shape[3] == layout.head_dim, "text tail is %s" % (tuple(k_text.shape),)
    return int(k_text.shape[2])


def _check_qtensor(layout: CqLayout, t: "QTensor", axis: int, group: int, what: str) -> None:
    want = (layout.batch, layout.n_kv_heads, layout.n_vis, layout.head_dim * layout.bits // 32)
    assert tuple(t.codes.shape) == want and t.codes.is_contiguous(), "%s codes are %s" % (what, tuple(t.codes.shape))
    meta = _meta_shape(layout, axis, group)
    assert tuple(t.scale.shape) == meta and tuple(t.min.shape) == meta, "%s parameters are %s" % (what, tuple(t.scale.shape))
    assert t.scale.dtype == torch.float32 and t.min.dtype == torch.float16
    assert t.scale.is_contiguous() and t.min.is_contiguous()


def make_calib(mode=CQ_CALIB_NONE, tau1=0.0, tau2=0.0, gamma=0.0, delta=0.0) -> CqCalib:
    return CqCalib(mode, tau1, tau2, gamma, delta)


def cq_decode_attn(layout: CqLayout, q: torch.Tensor, k: Optional[QTensor], v: Optional[QTensor],
                   k_text: Optional[torch.Tensor], v_text: Optional[torch.Tensor],
                   n_text: int, calib: Optional[CqCalib] = None, softmax_scale: float = 0.0,
                   out: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decode step; returns out [B, Hq, d] fp16 (allocated here unless given)."""
    if out is None:
        out = torch.empty_like(q)
    n_text_cap = _check_decode_tensors(layout, q, k_text, v_text, out)
    assert 0 <= n_text <= n_text_cap
    if layout.n_vis > 0:
        _check_qtensor(layout, k, layout.k_axis, layout.k_group, "key")
        _check_qtensor(layout, v, layout.v_axis, layout.v_group, "value")
    if workspace is None:
        workspace = torch.empty(cq_decode_workspace_bytes(layout, n_text, calib), dtype=torch.uint8,
                                device=q.device)
    ks = k.c_struct() if k is not None else None
    vs = v.c_struct() if v is not None else None
    _check(lib().cq_decode_attn(
        ctypes.byref(layout), _ptr(q),
        ctypes.byref(ks) if ks is not None else None,
        ctypes.byref(vs) if vs is not None else None,
        _ptr(k_text), _ptr(v_text), int(n_text), int(n_text_cap),
        ctypes.byref(calib) if calib is not None else None, float(softmax_scale),
        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(q)))
    return out


CQ_NOALLOC_SCRATCH_BYTES = 8 << 20


def cq_decode_attn_noalloc(layout: CqLayout, q: torch.Tensor, k: Optional[QTensor],
                           v: Optional[QTensor], k_text: Optional[torch.Tensor],
                           v_text: Optional[torch.Tensor], n_text: int,
                           calib: Optional[CqCalib] = None, softmax_scale: float = 0.0,
                           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """cq_decode_attn without a workspace: the library's own per-GPU scratch array serves.  `out`
    should be given by a caller that must not allocate (it is allocated here otherwise)."""
    if out is None:
        out = torch.empty_like(q)
    n_text_cap = _check_decode_tensors(layout, q, k_text, v_text, out)
    assert 0 <= n_text <= n_text_cap
    if layout.n_vis > 0:
        _check_qtensor(layout, k, layout.k_axis, layout.k_group, "key")
        _check_qtensor(layout, v, layout.v_axis, layout.v_group, "value")
    ks = k.c_struct() if k is not None else None
    vs = v.c_struct() if v is not None else None
    _check(lib().cq_decode_attn_noalloc(
        ctypes.byref(layout), _ptr(q),
        ctypes.byref(ks) if ks is not None else None,
        ctypes.byref(vs) if vs is not None else None,
        _ptr(k_text), _ptr(v_text), int(n_text), int(n_text_cap),
        ctypes.byref(calib) if calib is not None else None, float(softmax_scale),
        _ptr(out), _stream(q)))
    return out


def cq_decode_attn_devlen(layout: CqLayout, q: torch.Tensor, k: Optional[QTensor],
                          v: Optional[QTensor], k_text: torch.Tensor, v_text: torch.Tensor,
                          n_text_dev: torch.Tensor, n_text_max: int,
                          calib: Optional[CqCalib] = None, softmax_scale: float = 0.0,
                          out: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """cq_decode_attn with the tail length read from the device int32 tensor n_text_dev
    (n_text_max is the host's bound of it)."""
    if out is None:
        out = torch.empty_like(q)
    n_text_cap = _check_decode_tensors(layout, q, k_text, v_text, out)
    assert n_text_dev.dtype == torch.int32 and n_text_dev.numel() == 1 and n_text_dev.device == q.device
    assert 0 <= n_text_max <= n_text_cap
    if layout.n_vis > 0:
        _check_qtensor(layout, k, layout.k_axis, layout.k_group, "key")
        _check_qtensor(layout, v, layout.v_axis, layout.v_group, "value")
    if workspace is None:
        workspace = torch.empty(cq_decode_workspace_bytes(layout, n_text_max, calib),
                                dtype=torch.uint8, device=q.device)
    ks = k.c_struct() if k is not None else None
    vs = v.c_struct() if v is not None else None
    _check(lib().cq_decode_attn_devlen(
        ctypes.byref(layout), _ptr(q),
        ctypes.byref(ks) if ks is not None else None,
        ctypes.byref(vs) if vs is not None else None,
        _ptr(k_text), _ptr(v_text), _ptr(n_text_dev), int(n_text_max), int(n_text_cap),
        ctypes.byref(calib) if calib is not None else None, float(softmax_scale),
        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(q)))
    return out


def _check_append_tensors(layout: CqLayout, k_text, v_text, k_new, v_new) -> None:
    for t in (k_text, v_text, k_new, v_new):
        assert t.dtype == torch.float16 and t.is_contiguous()
    assert k_text.shape == v_text.shape and k_new.shape == v_new.shape
    B, H, d = layout.batch, layout.n_kv_heads, layout.head_dim
    assert tuple(k_text.shape[:2]) == (B, H) and k_text.shape[3] == d
    assert tuple(k_new.shape) == (B, H, 1, d), "new token is %s" % (tuple(k_new.shape),)


def cq_append_text_kv(layout: CqLayout, k_text: torch.Tensor, v_text: torch.Tensor, n_text: int,
                      k_new: torch.Tensor, v_new: torch.Tensor) -> int:
    """Write one new token per sequence, k_new / v_new [B, Hkv, 1, d], to slot n_text of the fp16
    tails [B, Hkv, cap, d] (in place); returns the new n_text."""
    _check_append_tensors(layout, k_text, v_text, k_new, v_new)
    _check(lib().cq_append_text_kv(ctypes.byref(layout), _ptr(k_text), _ptr(v_text), int(n_text),
                                   int(k_text.shape[2]), _ptr(k_new), _ptr(v_new), _stream(k_text)))
    return int(n_text) + 1


def cq_append_text_kv_devlen(layout: CqLayout, k_text: torch.Tensor, v_text: torch.Tensor,
                             n_text_dev: torch.Tensor, k_new: torch.Tensor,
                             v_new: torch.Tensor) -> None:
    """The same with the tail length in the device int32 tensor n_text_dev, which the call
    increments on the device (nothing happens when the tail is full)."""
    _check_append_tensors(layout, k_text, v_text, k_new, v_new)
    assert n_text_dev.dtype == torch.int32 and n_text_dev.numel() == 1 and n_text_dev.device == k_text.device
    _check(lib().cq_append_text_kv_devlen(ctypes.byref(layout), _ptr(k_text), _ptr(v_text),
                                          _ptr(n_text_dev), int(k_text.shape[2]), _ptr(k_new),
                                          _ptr(v_new), _stream(k_text)))


def cq_tau_search_workspace_bytes(layout: CqLayout, n_text: int, n_tau1: int, n_tau2: int) -> int:
    return int(lib().cq_tau_search_workspace_bytes(ctypes.byref(layout), int(n_text), int(n_tau1),
                                                   int(n_tau2)))


def cq_tau_search(layout: CqLayout, q: torch.Tensor, k_exact: torch.Tensor, k: QTensor,
                  k_text: Optional[torch.Tensor], n_text: int, tau1=(0.0, 1.0, 2.0, 3.0),
                  tau2=(0.0, 1.0, 2.0, 3.0), softmax_scale: float = 0.0,
                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Mean squared error of the attention weights for every (tau1, tau2) of the grid, as a
    float64 tensor [len(tau1), len(tau2)] on the device; its argmin is the search result."""
    assert q.dtype == torch.float16 and k_exact.dtype == torch.float16
    assert q.is_contiguous() and k_exact.is_contiguous()
    if k_text is not None:
        assert k_text.dtype == torch.float16 and k_text.is_contiguous()
    t1 = (ctypes.c_float * len(tau1))(*[float(t) for t in tau1])
    t2 = (ctypes.c_float * len(tau2))(*[float(t) for t in tau2])
    need = cq_tau_search_workspace_bytes(layout, n_text, len(tau1), len(tau2))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    out = torch.empty((len(tau1), len(tau2)), dtype=torch.float64, device=q.device)
    cap = 0 if k_text is None else int(k_text.shape[2])
    ks = k.c_struct()
    _check(lib().cq_tau_search(ctypes.byref(layout), _ptr(q), _ptr(k_exact), ctypes.byref(ks),
                               _ptr(k_text), int(n_text), cap, t1, len(tau1), t2, len(tau2),
                               float(softmax_scale), _ptr(out), _ptr(workspace),
                               workspace.numel(), _stream(q)))
    return out


def cq_bench_stream_read(buf: torch.Tensor, nbytes: int) -> None:
    """Measurement aid: enqueue a plain streaming read of the first nbytes of buf."""
    assert nbytes <= buf.numel() * buf.element_size()
    _check(lib().cq_bench_stream_read(buf.data_ptr(), int(nbytes), None, _stream(buf)))


def cq_bench_tile_traffic(x: torch.Tensor, codes: torch.Tensor, meta: torch.Tensor, n_tiles: int,
                          code_bytes_per_tile: int, meta_bytes_per_tile: int) -> None:
    """The tuned quantizer's memory traffic without its arithmetic (measurement aid)."""
    assert x.is_cuda and codes.is_cuda and meta.is_cuda
    assert x.numel() * x.element_size() >= n_tiles * 32768
    assert codes.numel() * codes.element_size() >= n_tiles * code_bytes_per_tile
    assert meta.numel() * meta.element_size() >= n_tiles * meta_bytes_per_tile
    _check(lib().cq_bench_tile_traffic(x.data_ptr(), codes.data_ptr(), meta.data_ptr(), int(n_tiles),
                                       int(code_bytes_per_tile), int(meta_bytes_per_tile), _stream(x)))


def cq_bench_stream_copy(dst: torch.Tensor, src: torch.Tensor, nbytes: int) -> None:
    """Measurement aid: enqueue a plain copy of the first nbytes of src to dst."""
    _check(lib().cq_bench_stream_copy(dst.data_ptr(), src.data_ptr(), int(nbytes), _stream(src)))


def cq_bench_set_kernel_path(path: int) -> int:
    """Test / benchmark switch (cq_bench.h), thread-local: returns the previous path."""
    r = lib().cq_bench_set_kernel_path(int(path))
    if r < 0:
        _check(r)
    return r


def cq_bench_set_decode_chunks(n_chunks: int) -> int:
    """Test / benchmark switch (cq_bench.h), thread-local: at least n_chunks chunks per row of the
    tuned decode (0 = automatic); returns the previous value."""
    r = lib().cq_bench_set_decode_chunks(int(n_chunks))
    if r < 0:
        _check(r)
    return r


def cq_version() -> int:
    return int(lib().cq_version())
