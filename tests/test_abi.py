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


def _declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cq_[a-z_0-9]+)\s*\(", text)))


# the product ABI: the two operations of the hot path with their size query, the steps either
# side of them, status reporting, and the entry point for callers that cannot allocate
PRODUCT_ABI = ["cq_append_text_kv", "cq_append_text_kv_devlen", "cq_decode_attn",
               "cq_decode_attn_devlen", "cq_decode_attn_noalloc", "cq_decode_workspace_bytes",
               "cq_last_error", "cq_quantize_kv", "cq_status_string", "cq_tau_search",
               "cq_tau_search_workspace_bytes", "cq_version"]
BENCH_ABI = ["cq_bench_set_decode_chunks", "cq_bench_set_kernel_path", "cq_bench_stream_copy",
             "cq_bench_stream_read", "cq_bench_tile_traffic"]


def test_library_exports_every_declared_symbol():
    assert _declared_functions("cq.h") == sorted(PRODUCT_ABI)
    assert _declared_functions("cq_bench.h") == sorted(BENCH_ABI)
    L = cq.lib()
    for n in PRODUCT_ABI + BENCH_ABI:
        assert hasattr(L, n), n
    assert cq.cq_version() >= 200


def test_library_exports_nothing_else():
    """The dynamic symbol table holds the declared cq_* functions and no other cq_* name (no debug
    hooks, no process-wide switches)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", cq.LIB_PATH], capture_output=True, text=True)
    if out.returncode != 0:
        pytest.skip("nm is not available")
    names = sorted({l.split()[-1] for l in out.stdout.splitlines() if l.split() and l.split()[-1].startswith("cq_")})
    assert names == sorted(PRODUCT_ABI + BENCH_ABI)


def test_library_reads_no_environment_variable():
    """No getenv in the library: a stray variable cannot change what a decode call launches."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--undefined-only", cq.LIB_PATH], capture_output=True, text=True)
    if out.returncode != 0:
        pytest.skip("nm is not available")
    assert not [l for l in out.stdout.splitlines() if "getenv" in l]


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
    assert _decode(lay, ws_bytes=16) == cq.CQ_ERR_WORKSPACE
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
    # the values play no part: an invalid value group is not an error here, an invalid key group is
    assert cq.cq_tau_search_workspace_bytes(cq.make_layout(2, 8, 2, 128, 256, v_group=48), 16, 4, 4) == need
    assert call(lay=cq.make_layout(2, 8, 2, 128, 256, k_group=96)) == cq.CQ_ERR_SHAPE


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


def test_workspace_size_follows_the_kernels_that_will_run():
    dyn = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    # the headline configuration: one workgroup owns a row, one launch, no scratch to speak of
    video = cq.make_layout(64, 32, 8, 128, 8192)
    assert cq.cq_decode_workspace_bytes(video, 512, dyn) == 256
    assert cq.cq_decode_workspace_bytes(video, 512, None) == 256
    # the long-context configuration: rows split into chunks on the streaming kernels -> one 16-bit
    # logit per (batch, query head, visual token), group references, chunk extrema and partials
    long_ctx = cq.make_layout(8, 48, 8, 128, 65536)
    n = cq.cq_decode_workspace_bytes(long_ctx, 1024, dyn)
    logits = 8 * 48 * 65536 * 2
    assert n % 256 == 0 and logits + 8 * 48 * 2 * (128 + 2) * 4 <= n < logits + (4 << 20)
    # a layout the streaming kernels do not take (channel-wise values) splits on the fused kernel:
    # extrema and partials only
    n = cq.cq_decode_workspace_bytes(cq.make_layout(8, 48, 8, 128, 65536, v_axis=0), 1024, dyn)
    assert n % 256 == 0 and 8 * 48 * 2 * (128 + 2) * 4 <= n < logits // 8
    # shape-agnostic kernels (a head dimension the tuned ones do not take): one fp32 logit per
    # (batch, query head, token) and the partials
    lay = cq.make_layout(2, 8, 2, 64, 1024, v_group=64)
    n = cq.cq_decode_workspace_bytes(lay, 32, dyn)
    assert n % 256 == 0 and n >= 2 * 8 * (1024 + 32) * 4
    assert cq.cq_decode_workspace_bytes(cq.make_layout(2, 8, 2, 64, 4096, v_group=64), 32, dyn) > n
    # invalid layout, tail length or calibration mode
    assert cq.cq_decode_workspace_bytes(cq.make_layout(2, 8, 2, 100, 1024), 32, dyn) == 0
    assert cq.cq_decode_workspace_bytes(video, -1, dyn) == 0
    assert cq.cq_decode_workspace_bytes(video, 512, cq.make_calib(9)) == 0


def test_switches_are_per_thread_and_the_size_query_follows_them():
    import threading
    video = cq.make_layout(64, 32, 8, 128, 8192)
    dyn = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    assert cq.cq_bench_set_kernel_path(cq.CQ_PATH_GENERIC) == cq.CQ_PATH_AUTO
    try:
        assert cq.cq_decode_workspace_bytes(video, 512, dyn) >= 64 * 32 * (8192 + 512) * 4
        seen = {}

        def other():        # another thread still sees the defaults, and its changes stay its own
            seen["path"] = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
            seen["chunks"] = cq.cq_bench_set_decode_chunks(5)
            seen["bytes"] = cq.cq_decode_workspace_bytes(video, 512, dyn)

        t = threading.Thread(target=other)
        t.start()
        t.join()
        assert seen["path"] == cq.CQ_PATH_AUTO and seen["chunks"] == 0
        assert seen["bytes"] > 256          # five chunks per row: partials
    finally:
        assert cq.cq_bench_set_kernel_path(cq.CQ_PATH_AUTO) == cq.CQ_PATH_GENERIC
    assert cq.cq_bench_set_decode_chunks(0) == 0
    assert cq.cq_decode_workspace_bytes(video, 512, dyn) == 256
    with pytest.raises(cq.CqError):
        cq.cq_bench_set_kernel_path(42)
    with pytest.raises(cq.CqError):
        cq.cq_bench_set_decode_chunks(-1)
    # TUNED makes a layout without a tuned kernel an error instead of a fallback
    cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        assert cq.cq_decode_workspace_bytes(cq.make_layout(2, 8, 2, 64, 1024, v_group=64), 32, dyn) == 0
        assert _decode(cq.make_layout(2, 8, 2, 64, 256, v_group=64)) == cq.CQ_ERR_UNSUPPORTED
    finally:
        cq.cq_bench_set_kernel_path(cq.CQ_PATH_AUTO)


def test_noalloc_entry_point_rejects_what_its_scratch_cannot_hold():
    """The allocation-free decode checks its arguments like cq_decode_attn and turns a shape whose
    scratch exceeds the library's array into CQ_ERR_WORKSPACE, all before any HIP call."""
    L = cq.lib()
    ks, vs = cq.CqQTensor(FAKE, FAKE, FAKE), cq.CqQTensor(FAKE, FAKE, FAKE)

    def call(lay, q=FAKE, n_text=4, cap=4, calib=None):
        return L.cq_decode_attn_noalloc(ctypes.byref(lay), q, ctypes.byref(ks), ctypes.byref(vs), FAKE,
                                        FAKE, n_text, cap, ctypes.byref(calib) if calib else None,
                                        0.0, FAKE, None)

    dyn = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    # shape-agnostic kernels (head_dim 64) with 16 MB of logits: more than the array holds
    big = cq.make_layout(8, 32, 8, 64, 16384, v_group=64)
    assert cq.cq_decode_workspace_bytes(big, 4, dyn) > cq.CQ_NOALLOC_SCRATCH_BYTES
    assert call(big, calib=dyn) == cq.CQ_ERR_WORKSPACE
    assert b"allocation-free" in L.cq_last_error()
    # (the long-context configuration is not refused although cq_decode_attn would keep 100 MB of
    # logits for it: with the array too small for that, the call takes the kernels that form the
    # logits twice and need extrema and partials only; tests/test_zz_no_alloc.py runs that on a GPU)
    lay = cq.make_layout(2, 8, 2, 128, 256)
    assert call(lay, q=None) == cq.CQ_ERR_NULL
    assert call(lay, q=FAKE + 2) == cq.CQ_ERR_ALIGN
    assert call(lay, n_text=5) == cq.CQ_ERR_SHAPE
    assert call(lay, calib=cq.make_calib(9)) == cq.CQ_ERR_UNSUPPORTED


def test_devlen_argument_errors():
    lay = cq.make_layout(2, 8, 2, 128, 256)
    L = cq.lib()
    ks, vs = cq.CqQTensor(FAKE, FAKE, FAKE), cq.CqQTensor(FAKE, FAKE, FAKE)

    def dec(n_dev=FAKE, n_max=4, cap=4, ws_bytes=1 << 40):
        return L.cq_decode_attn_devlen(ctypes.byref(lay), FAKE, ctypes.byref(ks), ctypes.byref(vs),
                                       FAKE, FAKE, n_dev, n_max, cap, None, 0.0, FAKE, FAKE, ws_bytes, None)

    assert dec(n_dev=None) == cq.CQ_ERR_NULL
    assert dec(n_dev=FAKE + 2) == cq.CQ_ERR_ALIGN
    assert dec(n_max=5) == cq.CQ_ERR_SHAPE
    assert dec(ws_bytes=16) == cq.CQ_ERR_WORKSPACE
    f = L.cq_append_text_kv_devlen
    assert f(ctypes.byref(lay), FAKE, FAKE, None, 4, FAKE, FAKE, None) == cq.CQ_ERR_NULL
    assert f(ctypes.byref(lay), FAKE, FAKE, FAKE + 1, 4, FAKE, FAKE, None) == cq.CQ_ERR_ALIGN
    assert f(ctypes.byref(lay), FAKE, FAKE, FAKE, 0, FAKE, FAKE, None) == cq.CQ_ERR_SHAPE
    assert f(ctypes.byref(lay), None, FAKE, FAKE, 4, FAKE, FAKE, None) == cq.CQ_ERR_NULL


def test_binding_raises_when_library_is_missing(monkeypatch):
    monkeypatch.setattr(cq, "_lib", None)
    monkeypatch.setattr(cq, "LIB_PATH", "/nonexistent/libcq.so")
    with pytest.raises(RuntimeError, match="not built"):
        cq.lib()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it exits with a message before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
