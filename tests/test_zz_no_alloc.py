"""cq_decode_attn_noalloc (the entry point for callers that cannot allocate) against cq_decode_attn:
same kernels, the library's own per-GPU scratch array instead of a caller's workspace, so the
outputs must agree bit for bit - on two calls in a row, the second with a smaller input (the
array keeps the first call's contents), on split rows (which use the scratch), on whole rows (which
do not) and on the shape-agnostic kernels."""
import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from paper_2502_14882_amd import binding as cq
from paper_2502_14882_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu


def _inputs(w, lay):
    x_cpu = synth.make_inputs(w, "cpu")
    x = H.to_device(x_cpu)
    k_dev, v_dev = cq.cq_quantize_kv(lay, x["k"], x["v"])
    return x_cpu, x, k_dev, v_dev


def _both(w, lay, calib):
    x_cpu, x, k_dev, v_dev = _inputs(w, lay)
    kt = x["k_text"] if w.n_text > 0 else None
    vt = x["v_text"] if w.n_text > 0 else None
    want = cq.cq_decode_attn(lay, x["q"], k_dev, v_dev, kt, vt, w.n_text, calib)
    torch.cuda.synchronize()
    out = torch.full_like(x["q"], float("nan"))
    cq.cq_decode_attn_noalloc(lay, x["q"], k_dev, v_dev, kt, vt, w.n_text, calib, 0.0, out)
    torch.cuda.synchronize()
    assert torch.equal(out, want), "allocation-free and workspace entry points differ"
    kq, vq = H.oracle_quantize(x_cpu, lay)
    ref = H.oracle_decode(x_cpu, kq, vq, w.n_text, calib.mode, calib.tau1, calib.tau2)
    err = O.rel_l2(out.cpu().numpy().astype(np.float64), ref)
    assert err <= H.REL_L2_TOL, "rel L2 %.3e" % err


def test_two_calls_in_a_row_the_second_smaller():
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    # g = 6: two blocks of query heads per KV head, rows run as extrema pass + partial pass +
    # combine through the scratch (chunk extrema and online-softmax partials)
    big = synth.WORKLOADS[4].replace(batch=2, n_kv_heads=2, n_q_heads=12, n_vis=2560, n_text=130)
    small = synth.WORKLOADS[4].replace(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=1280, n_text=70,
                                       seed=4321)
    for w in (big, small):
        lay = H.layout_of(w)
        assert cq.cq_decode_workspace_bytes(lay, w.n_text, calib) > 256, "this case must use scratch"
        _both(w, lay, calib)
    _both(small, H.layout_of(small), cq.make_calib(cq.CQ_CALIB_NONE))


def test_forced_chunks_whole_rows_and_generic_kernels(decode_chunks):
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1920, n_text=200)
    lay = H.layout_of(w)
    _both(w, lay, calib)                    # whole rows: the scratch is not touched
    decode_chunks(3)
    _both(w, lay, calib)                    # three chunks per row
    decode_chunks(0)
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_GENERIC)
    try:
        ws = cq.cq_decode_workspace_bytes(lay, w.n_text, calib)
        assert 256 < ws <= cq.CQ_NOALLOC_SCRATCH_BYTES
        _both(w, lay, calib)                # shape-agnostic kernels: logits live in the scratch
    finally:
        cq.cq_bench_set_kernel_path(prev)


def test_a_shape_beyond_the_scratch_is_refused():
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    w = synth.WORKLOADS[1].replace(batch=4, n_kv_heads=8, n_q_heads=32, head_dim=64, n_vis=16384, n_text=8)
    lay = H.layout_of(w, 1, 128, 64)
    x = synth.make_inputs(w, "cuda")
    k_dev, v_dev = cq.cq_quantize_kv(lay, x["k"], x["v"])
    with pytest.raises(cq.CqError) as e:
        cq.cq_decode_attn_noalloc(lay, x["q"], k_dev, v_dev, x["k_text"], x["v_text"], w.n_text, calib)
    assert e.value.status == cq.CQ_ERR_WORKSPACE
