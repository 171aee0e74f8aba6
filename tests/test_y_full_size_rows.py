"""Whole workloads at full size, every (batch, KV head) row, against the C++ oracle twin.

These are the largest cases of the GPU suite (GBs of cache, seconds of CPU oracle each), collected
after the other parity tests; the tuned kernels are forced, so a silent fall-back to the
shape-agnostic kernels would be an error."""
import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from oracle import cq_oracle_native as ON
from paper_2502_14882_amd import binding as cq
from paper_2502_14882_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu


def _all_rows_check(w, bits, what):
    """Whole workload at full size: drawn on the GPU as bench.py does, quantized and decoded by the
    HIP path through the launches bench.py times, and every (batch, head) row - not a sample -
    compared with the C++ oracle twin (itself tied to the numpy oracle by CPU tests): packed
    words, scales and minima bit for bit, attention within the contract, the regression bar and the
    element-wise bound."""
    lay = H.layout_of(w, bits)
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    x = synth.make_inputs(w, "cuda")
    k_dev, v_dev = cq.cq_quantize_kv(lay, x["k"], x["v"])
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        out = cq.cq_decode_attn(lay, x["q"], k_dev, v_dev, x["k_text"], x["v_text"], w.n_text, calib)
        torch.cuda.synchronize()
    finally:
        cq.cq_bench_set_kernel_path(prev)
    host = {n: x[n].cpu().numpy() for n in ("q", "k_text", "v_text")}
    refs = {}
    for name, dev_t, axis, group in (("k", k_dev, O.AXIS_CHANNEL, 128), ("v", v_dev, O.AXIS_TOKEN, 128)):
        ref_t = ON.quantize_tensor(x[name].cpu().numpy(), bits, axis, group)
        del x[name]
        got = H.words_of(dev_t.codes)
        if not np.array_equal(got, ref_t["words"]):
            bad = np.argwhere(got != ref_t["words"])
            first = tuple(int(i) for i in bad[0])
            raise AssertionError("%s %s codes: %d words differ, first at %s (%08x, oracle %08x), last at %s" % (
                what, name, len(bad), first, got[first], ref_t["words"][first], bad[-1].tolist()))
        assert np.array_equal(dev_t.scale.cpu().numpy().view(np.uint32), ref_t["scale"].view(np.uint32))
        assert np.array_equal(dev_t.min.cpu().numpy().view(np.uint16), ref_t["min"].view(np.uint16))
        refs[name] = ref_t
    ref = ON.decode_attn(host["q"], refs["k"], refs["v"], host["k_text"], host["v_text"], w.n_text,
                         O.CALIB_DYNAMIC, 1.0, 2.0)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err, worst = O.rel_l2(got, ref), H.row_rel_l2(got, ref)
    assert err <= H.REGRESSION_TOL, "%s: rel L2 %.3e" % (what, err)
    assert worst <= H.REL_L2_TOL, "%s: worst (batch, head) row rel L2 %.3e" % (what, worst)
    H.assert_elementwise_close(got, ref, what)


@pytest.mark.parametrize("bits", [1, 2])
def test_headline_config_every_row_at_full_size(bits):
    """configs[2] (batch 64, 32 / 8 heads, 8192 + 512 tokens): all 512 (batch, KV head) rows."""
    _all_rows_check(synth.WORKLOADS[2], bits, "configs[2] b=%d" % bits)


@pytest.mark.parametrize("bits", [1, 2])
def test_long_context_config_every_row_at_full_size(bits):
    """configs[4] (batch 8, 48 / 8 heads, 65536 + 1024 tokens, heavy-tailed keys): all 64 rows
    through the split-row launches."""
    _all_rows_check(synth.WORKLOADS[4], bits, "configs[4] b=%d" % bits)


def test_small_layer_config_every_row_at_full_size():
    """configs[1] (batch 16, 32 / 8 heads, 3328 + 128 tokens): all 128 rows."""
    _all_rows_check(synth.WORKLOADS[1], 1, "configs[1]")


def test_full_size_quantizer_config_every_row():
    """configs[3] at full size, b = 1, groups of 128: all 1024 (batch, KV head) rows of both
    tensors (2 x 2.1 G elements) against the C++ oracle twin (tied to the numpy oracle by CPU
    tests), bit for bit, one tensor at a time to bound host memory."""
    w = synth.WORKLOADS[3]
    lay = H.layout_of(w, 1, 128, 128)
    x = synth.make_inputs(w, "cuda", parts=("k", "v"))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        k_out, v_out = cq.cq_quantize_kv(lay, x["k"], x["v"])
        torch.cuda.synchronize()
    finally:
        cq.cq_bench_set_kernel_path(prev)
    for name, out, axis in (("k", k_out, lay.k_axis), ("v", v_out, lay.v_axis)):
        host = x[name].cpu().numpy()
        del x[name]
        ref = ON.quantize_tensor(host, 1, axis, 128)
        del host
        H.assert_qtensor_equal(out, ref, "configs[3] all rows, %s" % name)
        del ref
