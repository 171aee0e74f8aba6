"""GPU parity of cq_decode_attn against the fp64 oracle: relative L2 <= 2e-3 on the fp16 output.

The HIP path consumes the cache written by cq_quantize_kv (asserted bit-identical to the
oracle's), so both sides attend over exactly the same quantized numbers."""
import itertools

import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from oracle import cq_oracle_native as ON
from paper_2502_14882_amd import binding as cq
from paper_2502_14882_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu


def pytest_generate_tests(metafunc):
    """Every case runs on both kernel paths, except the ones marked `tuned_only` (forced tuned
    path, full sizes), which run once."""
    if "kernel_path" in metafunc.fixturenames:
        once = metafunc.definition.get_closest_marker("tuned_only") is not None
        metafunc.parametrize("kernel_path", ["auto"] if once else ["generic", "auto"],
                             indirect=True, scope="module")


@pytest.fixture(autouse=True, scope="module")
def kernel_path(request):
    """Every case runs twice: on the shape-agnostic kernels and on whatever AUTO selects
    (the tuned kernels where the layout allows)."""
    prev = cq.cq_bench_set_kernel_path({"generic": cq.CQ_PATH_GENERIC, "auto": cq.CQ_PATH_AUTO}[request.param])
    yield request.param
    cq.cq_bench_set_kernel_path(prev)


class Case:
    """Inputs on both sides plus the quantized cache, built once per workload/layout."""

    def __init__(self, w, lay, x_cpu=None):
        self.w, self.lay = w, lay
        self.x_cpu = x_cpu or synth.make_inputs(w, "cpu")
        self.kq, self.vq = H.oracle_quantize(self.x_cpu, lay)
        self.x = H.to_device(self.x_cpu)
        if w.n_vis > 0:
            self.k_dev, self.v_dev = cq.cq_quantize_kv(lay, self.x["k"], self.x["v"])
            H.assert_qtensor_equal(self.k_dev, self.kq, "keys")
            H.assert_qtensor_equal(self.v_dev, self.vq, "values")
        else:
            self.k_dev = self.v_dev = None

    def check(self, mode=cq.CQ_CALIB_DYNAMIC, tau1=1.0, tau2=2.0, gamma=0.0, delta=0.0,
              n_text=None, softmax_scale=0.0, tol=H.REL_L2_TOL):
        n_text = self.w.n_text if n_text is None else n_text
        ref = H.oracle_decode(self.x_cpu, self.kq, self.vq, n_text, mode, tau1, tau2, gamma, delta,
                              softmax_scale)
        kt = self.x["k_text"] if self.x["k_text"].shape[2] > 0 else None
        vt = self.x["v_text"] if kt is not None else None
        out = cq.cq_decode_attn(self.lay, self.x["q"], self.k_dev, self.v_dev, kt, vt, n_text,
                                cq.make_calib(mode, tau1, tau2, gamma, delta), softmax_scale)
        torch.cuda.synchronize()
        out = out.cpu().numpy().astype(np.float64)
        assert np.isfinite(out).all()
        err, worst = O.rel_l2(out, ref), H.row_rel_l2(out, ref)
        assert err <= tol, "rel L2 %.3e (worst row %.3e) > %.1e" % (err, worst, tol)
        assert worst <= 4 * tol, "worst row rel L2 %.3e" % worst
        H.assert_elementwise_close(out, ref)
        lay = self.lay
        if (lay.bits <= 2 and lay.k_axis == cq.CQ_AXIS_CHANNEL and lay.v_axis == cq.CQ_AXIS_TOKEN
                and lay.v_group == lay.head_dim and out.size >= 1024):
            assert err <= H.REGRESSION_TOL, "rel L2 %.3e is over the regression bar %.1e" % (
                err, H.REGRESSION_TOL)
        return err


@pytest.fixture(scope="module")
def cfg0(kernel_path):
    w = synth.WORKLOADS[0]
    return Case(w, H.layout_of(w))


@pytest.mark.parametrize("tau1,tau2", list(itertools.product([0, 1, 2, 3], repeat=2)))
def test_config0_every_tau_pair_of_the_papers_grid(cfg0, tau1, tau2):
    cfg0.check(cq.CQ_CALIB_DYNAMIC, float(tau1), float(tau2))


def test_config0_modes(cfg0):
    cfg0.check(cq.CQ_CALIB_NONE)
    cfg0.check(cq.CQ_CALIB_FIXED, 1.0, 2.0, gamma=-20.0, delta=25.0)
    cfg0.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, softmax_scale=0.05)
    cfg0.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, n_text=0)
    cfg0.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, n_text=17)       # capacity 32, 17 used


def test_calibration_with_nonpositive_slope_is_applied_literally(cfg0):
    # delta - gamma + tau1 - tau2 < 0 flips the order of the visual logits; no clamping
    cfg0.check(cq.CQ_CALIB_FIXED, 0.0, 30.0, gamma=-1.0, delta=1.0)


SHRUNK = {
    1: dict(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1280, n_text=128),       # g = 4
    2: dict(batch=3, n_kv_heads=2, n_q_heads=8, n_vis=1536, n_text=600),       # two text chunks
    4: dict(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=4096, n_text=300),      # g = 6, split-K
}


@pytest.mark.parametrize("idx", [1, 2, 4])
@pytest.mark.parametrize("bits", [1, 2])
def test_shrunk_configs(idx, bits):
    w = synth.WORKLOADS[idx].replace(**SHRUNK[idx])
    c = Case(w, H.layout_of(w, bits))
    c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    c.check(cq.CQ_CALIB_NONE)


@pytest.mark.parametrize("kg,vg", [(32, 32), (64, 128), (128, 64)])
def test_group_sizes(kg, vg):
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=640, n_text=40)
    Case(w, H.layout_of(w, 1, kg, vg)).check()


def test_ragged_sizes_and_single_tokens():
    # n_vis not a multiple of the chunk, text tail of 1, then visual-only and text-only
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=1, n_q_heads=4, n_vis=896, n_text=1)
    Case(w, H.layout_of(w)).check()
    w = synth.WORKLOADS[1].replace(batch=1, n_kv_heads=1, n_q_heads=2, n_vis=128, n_text=0)
    Case(w, H.layout_of(w)).check()
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=4, n_vis=0, n_text=77)
    Case(w, H.layout_of(w)).check()


def test_paper_literal_channelwise_values_and_other_layouts():
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=4, n_vis=512, n_text=33)
    Case(w, H.layout_of(w, 1, 128, 128, 0, 0)).check()           # channel-wise K and V
    Case(w, H.layout_of(w, 2, 512, 512, 0, 0)).check()           # whole-sequence statistics
    Case(w, H.layout_of(w, 2, 64, 64, 1, 1)).check()             # token-wise K and V
    Case(w, H.layout_of(w, 4, 64, 64)).check()
    Case(w, H.layout_of(w, 8, 64, 64)).check()


@pytest.mark.parametrize("d", [64, 256])
def test_other_head_dims(d):
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=4, head_dim=d, n_vis=256,
                                   n_text=20)
    Case(w, H.layout_of(w, 1, 64, 32)).check()


def test_many_query_heads_per_kv_head():
    w = synth.WORKLOADS[1].replace(batch=1, n_kv_heads=1, n_q_heads=11, n_vis=256, n_text=9)
    Case(w, H.layout_of(w)).check()


def test_constant_visual_logits_give_slope_one():
    # all keys identical -> every visual logit equal -> delta == gamma
    w = synth.WORKLOADS[0].replace(n_vis=256, n_text=8)
    x = synth.make_inputs(w, "cpu")
    x["k"][:] = x["k"][:, :, :1, :]
    Case(w, H.layout_of(w), x).check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)


def test_output_is_deterministic(cfg0):
    outs = []
    for _ in range(2):
        o = cq.cq_decode_attn(cfg0.lay, cfg0.x["q"], cfg0.k_dev, cfg0.v_dev, cfg0.x["k_text"],
                              cfg0.x["v_text"], 32, cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1, 2))
        torch.cuda.synchronize()
        outs.append(o.cpu())
    assert torch.equal(outs[0], outs[1])


@pytest.mark.tuned_only
def test_tuned_path_takes_the_benchmark_layouts(kernel_path):
    """The layouts of the decode workloads must not fall back silently: forcing the tuned path
    has to succeed (and agree with the oracle) for them."""
    cases = []
    for w in (synth.WORKLOADS[0],
              synth.WORKLOADS[2].replace(batch=2, n_kv_heads=2, n_q_heads=8),   # full-length rows
              synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8)):
        cases.append(Case(w, H.layout_of(w)))
    # 2-bit codes, and the long-context shape (g = 6, rows split into chunks) at both widths
    w2 = synth.WORKLOADS[2].replace(batch=1, n_kv_heads=2, n_q_heads=8)
    cases.append(Case(w2, H.layout_of(w2, 2)))
    w4 = synth.WORKLOADS[4].replace(batch=1, n_kv_heads=1, n_q_heads=6, n_vis=16384, n_text=1024)
    cases.append(Case(w4, H.layout_of(w4, 1)))
    cases.append(Case(w4, H.layout_of(w4, 2)))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check()
    finally:
        cq.cq_bench_set_kernel_path(prev)


# the layouts that bench.py times on configs[2]: (bits, key group, value axis, value group); a group
# of 0 stands for the whole sequence
FULL_SIZE_LAYOUTS = [(1, 128, 1, 128), (2, 128, 1, 128), (4, 128, 1, 128), (8, 128, 1, 128),
                     (1, 32, 1, 128), (2, 32, 1, 128), (1, 64, 1, 128), (1, 128, 0, 128), (2, 128, 0, 128),
                     (1, 0, 1, 128), (1, 0, 0, 0), (2, 0, 0, 0)]


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits,k_group,v_axis,v_group", FULL_SIZE_LAYOUTS)
def test_full_size_benchmark_config_on_sampled_rows(kernel_path, bits, k_group, v_axis, v_group):
    """configs[2] at full size, drawn on the GPU as bench.py does, through the kernels bench.py
    times (every layout of its command line); the oracle checks sampled (batch, KV head) rows,
    each one independently."""
    w = synth.WORKLOADS[2]
    k_group = k_group or w.n_vis
    v_group = v_group or w.n_vis
    lay = H.layout_of(w, bits, k_group, v_group, 0, v_axis)
    x = synth.make_inputs(w, "cuda")
    k_dev, v_dev = cq.cq_quantize_kv(lay, x["k"], x["v"])
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        out = cq.cq_decode_attn(lay, x["q"], k_dev, v_dev, x["k_text"], x["v_text"], w.n_text,
                                cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0))
        torch.cuda.synchronize()
    finally:
        cq.cq_bench_set_kernel_path(prev)
    g = w.n_q_heads // w.n_kv_heads
    rng = np.random.default_rng(5)
    rows = {(0, 0), (w.batch - 1, w.n_kv_heads - 1)}
    while len(rows) < (6 if (bits, k_group, v_axis) == (1, 128, 1) else 3):
        rows.add((int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads))))
    for b, h in sorted(rows):
        k_row = x["k"][b:b + 1, h:h + 1].cpu().numpy()
        v_row = x["v"][b:b + 1, h:h + 1].cpu().numpy()
        kq = O.quantize_tensor(k_row, bits, O.AXIS_CHANNEL, k_group)
        vq = O.quantize_tensor(v_row, bits, v_axis, v_group)
        assert np.array_equal(H.words_of(k_dev.codes[b:b + 1, h:h + 1]), kq["words"])
        assert np.array_equal(H.words_of(v_dev.codes[b:b + 1, h:h + 1]), vq["words"])
        for dev_t, ref_t in ((k_dev, kq), (v_dev, vq)):
            assert np.array_equal(dev_t.scale[b:b + 1, h:h + 1].cpu().numpy().view(np.uint32),
                                  ref_t["scale"].view(np.uint32))
            assert np.array_equal(dev_t.min[b:b + 1, h:h + 1].cpu().numpy().view(np.uint16),
                                  ref_t["min"].view(np.uint16))
        ref = O.decode_attn(x["q"][b:b + 1, h * g:(h + 1) * g].cpu().numpy(), kq, vq,
                            x["k_text"][b:b + 1, h:h + 1].cpu().numpy(),
                            x["v_text"][b:b + 1, h:h + 1].cpu().numpy(), w.n_text,
                            O.CALIB_DYNAMIC, 1.0, 2.0)
        got = out[b:b + 1, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)
        err = O.rel_l2(got, ref)
        assert err <= H.REL_L2_TOL, "row (%d,%d): rel L2 %.3e" % (b, h, err)
        H.assert_elementwise_close(got, ref, "row (%d,%d)" % (b, h))


@pytest.mark.tuned_only
@pytest.mark.parametrize("chunks", [1, 2, 5])
def test_split_rows_agree_with_whole_rows(kernel_path, chunks, decode_chunks):
    """The tuned kernel on whole rows (one launch) and on rows split into chunks (extrema pass,
    partial pass, combine) must both match the oracle; g = 4 and g = 6 (two blocks of heads)."""
    decode_chunks(chunks)
    prev = None
    cases = []
    for w in (synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1920, n_text=200),
              synth.WORKLOADS[4].replace(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=2560, n_text=130)):
        cases.append(Case(w, H.layout_of(w)))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_NONE)
            c.check(cq.CQ_CALIB_FIXED, 1.0, 2.0, gamma=-30.0, delta=30.0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("kg,vg", [(128, 128), (128, 64), (64, 128), (32, 64), (32, 128)])
def test_tuned_channelwise_values(kernel_path, bits, kg, vg):
    """Paper-literal value quantization (channel-wise over groups of tokens, Sec. 3.1) on the
    tuned kernels: whole rows, every calibration mode, g = 4 and g = 6."""
    cases = []
    for w in (synth.WORKLOADS[2].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=2304, n_text=200),
              synth.WORKLOADS[4].replace(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=1280, n_text=70)):
        cases.append(Case(w, H.layout_of(w, bits, kg, vg, 0, 0)))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_NONE)
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, n_text=0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits,v_whole", [(1, False), (2, False), (4, False), (8, False), (1, True), (2, True)])
def test_tuned_whole_sequence_statistics(kernel_path, bits, v_whole, decode_chunks):
    """Sec. 3.1 as printed: one (scale, min) pair per channel over ALL visual tokens, for keys and
    (v_whole) for values too, on the tuned kernels; whole rows and rows split into chunks."""
    cases = []
    for w in (synth.WORKLOADS[2].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=2304, n_text=200),
              synth.WORKLOADS[4].replace(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=1280, n_text=70)):
        lay = H.layout_of(w, bits, w.n_vis, w.n_vis if v_whole else 128, 0, 0 if v_whole else 1)
        cases.append(Case(w, lay))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_NONE, n_text=0)
        decode_chunks(3)
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_FIXED, 1.0, 2.0, gamma=-30.0, delta=30.0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("g", [1, 2, 3, 4, 5, 6, 7, 8])
def test_streaming_kernels_every_head_count(kernel_path, bits, g, decode_chunks):
    """Split rows on the streaming kernels for 1 to 8 query heads per KV head: one or two head sets,
    every count of heads in the last set (the values pass is compiled per count and skips the head
    slots without a head), text tails that leave text waves idle, a ragged last chunk, the
    calibration modes including a falling fixed line (references are then group minima)."""
    decode_chunks(3)
    w = synth.WORKLOADS[4].replace(batch=2, n_kv_heads=2, n_q_heads=2 * g, n_vis=128 * 13,
                                   n_text=(0, 7, 70, 330)[g % 4], seed=8400 + 16 * bits + g)
    c = Case(w, H.layout_of(w, bits))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        dyn = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
        kept_logits = 2 * w.batch * w.n_q_heads * w.n_vis            # 16 bits per visual logit
        assert cq.cq_decode_workspace_bytes(c.lay, w.n_text, dyn) > kept_logits    # the streaming plan
        c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
        c.check(cq.CQ_CALIB_NONE)
        c.check(cq.CQ_CALIB_FIXED, 0.0, 30.0, gamma=-1.0, delta=1.0)
        c.check(cq.CQ_CALIB_DYNAMIC, 2.0, 0.0, softmax_scale=0.05)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("chunks", [2, 3])
def test_tuned_channelwise_values_on_split_rows(kernel_path, chunks, decode_chunks):
    decode_chunks(chunks)
    cases = []
    for kg, vg in ((128, 128), (32, 128), (64, 64)):
        w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1920, n_text=200)
        cases.append(Case(w, H.layout_of(w, 1, kg, vg, 0, 0)))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_FIXED, 1.0, 2.0, gamma=-30.0, delta=30.0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
def test_full_length_row_with_channelwise_values(kernel_path):
    """configs[2]-length rows (8192 + 512 tokens) with channel-wise values, tuned kernels."""
    w = synth.WORKLOADS[2].replace(batch=1, n_kv_heads=2, n_q_heads=8)
    c = Case(w, H.layout_of(w, 1, 128, 128, 0, 0))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("chunks", [1, 3])
def test_decode_replayed_from_a_hip_graph(kernel_path, chunks, decode_chunks):
    """cq_decode_attn allocates nothing and blocks on nothing, so a serving loop can record it
    into a HIP graph: every replay, with eager work and synchronisations in between, must
    reproduce the eager result bit for bit (whole rows and split rows)."""
    decode_chunks(chunks)
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1920, n_text=200)
    c = Case(w, H.layout_of(w))
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    ws = torch.empty(cq.cq_decode_workspace_bytes(c.lay, w.n_text, calib), dtype=torch.uint8, device="cuda")
    qs = [c.x["q"], (c.x["q"] * 0.5).contiguous(), (-c.x["q"]).contiguous()]
    eager = []
    for q in qs:
        out = torch.empty_like(q)
        cq.cq_decode_attn(c.lay, q, c.k_dev, c.v_dev, c.x["k_text"], c.x["v_text"], w.n_text, calib,
                          0.0, out, ws)
        torch.cuda.synchronize()
        eager.append(out.clone())
    outs = [torch.empty_like(q) for q in qs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, as torch asks for
        cq.cq_decode_attn(c.lay, qs[0], c.k_dev, c.v_dev, c.x["k_text"], c.x["v_text"], w.n_text,
                          calib, 0.0, outs[0], ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for q, out in zip(qs, outs):
            cq.cq_decode_attn(c.lay, q, c.k_dev, c.v_dev, c.x["k_text"], c.x["v_text"], w.n_text,
                              calib, 0.0, out, ws)
    for rep in range(3):
        for out in outs:
            out.zero_()
        ws.zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(outs, eager):
            assert torch.equal(got, want), "replay %d differs from the eager result" % rep


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2])
def test_full_size_long_context_config_on_sampled_rows(kernel_path, bits):
    """configs[4] at full size (batch 8, g = 6, 65536 + 1024 tokens) through the launches bench.py
    times (rows split into chunks, two head blocks, extrema + partial + combine); the oracle
    checks sampled (batch, KV head) rows, each one independently."""
    w = synth.WORKLOADS[4]
    lay = H.layout_of(w, bits)
    x = synth.make_inputs(w, "cuda")
    k_dev, v_dev = cq.cq_quantize_kv(lay, x["k"], x["v"])
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        out = cq.cq_decode_attn(lay, x["q"], k_dev, v_dev, x["k_text"], x["v_text"], w.n_text,
                                cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0))
        torch.cuda.synchronize()
    finally:
        cq.cq_bench_set_kernel_path(prev)
    g = w.n_q_heads // w.n_kv_heads
    for b, h in ((0, 0), (w.batch - 1, w.n_kv_heads - 1), (3, 5)):
        kq = O.quantize_tensor(x["k"][b:b + 1, h:h + 1].cpu().numpy(), bits, O.AXIS_CHANNEL, 128)
        vq = O.quantize_tensor(x["v"][b:b + 1, h:h + 1].cpu().numpy(), bits, O.AXIS_TOKEN, 128)
        assert np.array_equal(H.words_of(k_dev.codes[b:b + 1, h:h + 1]), kq["words"])
        assert np.array_equal(H.words_of(v_dev.codes[b:b + 1, h:h + 1]), vq["words"])
        ref = O.decode_attn(x["q"][b:b + 1, h * g:(h + 1) * g].cpu().numpy(), kq, vq,
                            x["k_text"][b:b + 1, h:h + 1].cpu().numpy(),
                            x["v_text"][b:b + 1, h:h + 1].cpu().numpy(), w.n_text,
                            O.CALIB_DYNAMIC, 1.0, 2.0)
        got = out[b:b + 1, h * g:(h + 1) * g].cpu().numpy().astype(np.float64)
        err = O.rel_l2(got, ref)
        assert err <= H.REL_L2_TOL, "row (%d,%d): rel L2 %.3e" % (b, h, err)
        H.assert_elementwise_close(got, ref, "row (%d,%d)" % (b, h))


def test_decoding_several_steps_with_a_growing_text_tail(kernel_path):
    """Sec. 3: the quantized visual cache is fixed after the prefill while the fp16 tail grows by
    one token per decode step.  cq_append_text_kv + cq_decode_attn over four steps against the
    oracle on the same growing tail."""
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1280, n_text=61)
    c = Case(w, H.layout_of(w))
    cap = 64
    B, Hkv, d = w.batch, w.n_kv_heads, w.head_dim
    gen = torch.Generator().manual_seed(77)
    k_tail = torch.zeros(B, Hkv, cap, d, dtype=torch.float16)
    v_tail = torch.zeros(B, Hkv, cap, d, dtype=torch.float16)
    k_tail[:, :, :w.n_text] = c.x_cpu["k_text"]
    v_tail[:, :, :w.n_text] = c.x_cpu["v_text"]
    k_dev, v_dev = k_tail.cuda(), v_tail.cuda()
    n_text = w.n_text
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    for step in range(4):
        q = torch.randn(B, w.n_q_heads, d, generator=gen).to(torch.float16)
        out = cq.cq_decode_attn(c.lay, q.cuda(), c.k_dev, c.v_dev, k_dev, v_dev, n_text, calib)
        torch.cuda.synchronize()
        ref = O.decode_attn(q.numpy(), c.kq, c.vq, k_tail.numpy(), v_tail.numpy(), n_text,
                            O.CALIB_DYNAMIC, 1.0, 2.0)
        err = O.rel_l2(out.cpu().numpy().astype(np.float64), ref)
        assert err <= H.REL_L2_TOL, "step %d: rel L2 %.3e" % (step, err)
        if n_text == cap:
            with pytest.raises(cq.CqError):
                cq.cq_append_text_kv(c.lay, k_dev, v_dev, n_text, k_dev[:, :, :1].contiguous(),
                                     v_dev[:, :, :1].contiguous())
            break
        k_new = torch.randn(B, Hkv, 1, d, generator=gen).to(torch.float16)
        v_new = torch.randn(B, Hkv, 1, d, generator=gen).to(torch.float16)
        k_tail[:, :, n_text] = k_new[:, :, 0]
        v_tail[:, :, n_text] = v_new[:, :, 0]
        n_text = cq.cq_append_text_kv(c.lay, k_dev, v_dev, n_text, k_new.cuda(), v_new.cuda())
        torch.cuda.synchronize()
        assert torch.equal(k_dev.cpu(), k_tail) and torch.equal(v_dev.cpu(), v_tail)


@pytest.mark.parametrize("chunks", [0, 3])
def test_growing_step_recorded_once_and_replayed(kernel_path, chunks, decode_chunks):
    """Sec. 2.1: every decode step appends the new token's key and value to the cache and attends
    to all of it.  With the tail length in device memory the step (cq_append_text_kv_devlen, then
    cq_decode_attn_devlen) is recorded ONCE into a HIP graph and replayed eight times while the
    tail grows, with eager work and synchronisations between the replays; every replay is checked
    against the oracle on the tail as it then stands.  Whole rows and rows split into chunks."""
    if chunks and kernel_path == "generic":
        pytest.skip("the chunk override only concerns the tuned kernels")
    decode_chunks(chunks)
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1280, n_text=59)
    c = Case(w, H.layout_of(w))
    cap, steps = 70, 8
    B, Hkv, d = w.batch, w.n_kv_heads, w.head_dim
    gen = torch.Generator().manual_seed(91)
    k_tail = torch.zeros(B, Hkv, cap, d, dtype=torch.float16)
    v_tail = torch.zeros(B, Hkv, cap, d, dtype=torch.float16)
    k_tail[:, :, :w.n_text] = c.x_cpu["k_text"]
    v_tail[:, :, :w.n_text] = c.x_cpu["v_text"]
    k_dev, v_dev = k_tail.cuda(), v_tail.cuda()
    calib = cq.make_calib(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
    n_max = w.n_text + steps
    ws = torch.empty(cq.cq_decode_workspace_bytes(c.lay, n_max, calib), dtype=torch.uint8, device="cuda")
    n_dev = torch.tensor([w.n_text], dtype=torch.int32, device="cuda")
    q_buf = torch.zeros(B, w.n_q_heads, d, dtype=torch.float16, device="cuda")
    k_new = torch.zeros(B, Hkv, 1, d, dtype=torch.float16, device="cuda")
    v_new = torch.zeros(B, Hkv, 1, d, dtype=torch.float16, device="cuda")
    out = torch.zeros_like(q_buf)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream (decode only: the tail stays)
        cq.cq_decode_attn_devlen(c.lay, q_buf, c.k_dev, c.v_dev, k_dev, v_dev, n_dev, n_max, calib,
                                 0.0, out, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cq.cq_append_text_kv_devlen(c.lay, k_dev, v_dev, n_dev, k_new, v_new)
        cq.cq_decode_attn_devlen(c.lay, q_buf, c.k_dev, c.v_dev, k_dev, v_dev, n_dev, n_max, calib,
                                 0.0, out, ws)
    torch.cuda.synchronize()
    assert int(n_dev.item()) == w.n_text, "recording a graph must not run it"
    n_text = w.n_text
    for step in range(steps):
        q = torch.randn(B, w.n_q_heads, d, generator=gen).to(torch.float16)
        kn = torch.randn(B, Hkv, 1, d, generator=gen).to(torch.float16)
        vn = torch.randn(B, Hkv, 1, d, generator=gen).to(torch.float16)
        q_buf.copy_(q)                  # eager work between the replays
        k_new.copy_(kn)
        v_new.copy_(vn)
        out.zero_()
        ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        k_tail[:, :, n_text] = kn[:, :, 0]
        v_tail[:, :, n_text] = vn[:, :, 0]
        n_text += 1
        assert int(n_dev.item()) == n_text
        assert torch.equal(k_dev.cpu(), k_tail) and torch.equal(v_dev.cpu(), v_tail)
        ref = O.decode_attn(q.numpy(), c.kq, c.vq, k_tail.numpy(), v_tail.numpy(), n_text,
                            O.CALIB_DYNAMIC, 1.0, 2.0)
        got = out.cpu().numpy().astype(np.float64)
        err = O.rel_l2(got, ref)
        assert err <= H.REL_L2_TOL, "replay %d (tail of %d): rel L2 %.3e" % (step, n_text, err)
    # a full tail: the append leaves tails and counter alone, and the decode still attends to cap tokens
    n_dev.fill_(cap)
    before = (k_dev.clone(), v_dev.clone())
    cq.cq_append_text_kv_devlen(c.lay, k_dev, v_dev, n_dev, k_new, v_new)
    torch.cuda.synchronize()
    assert int(n_dev.item()) == cap
    assert torch.equal(k_dev, before[0]) and torch.equal(v_dev, before[1])


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("kg", [32, 64, 128])
def test_tuned_wide_codes(kernel_path, bits, kg):
    """4- and 8-bit codes on the tuned kernels (nibbles and bytes as matrix operands, the
    offset of the 8-bit operand carried by the additive terms): g = 4 and g = 6, every mode."""
    cases = []
    for w in (synth.WORKLOADS[2].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1536, n_text=200),
              synth.WORKLOADS[4].replace(batch=1, n_kv_heads=2, n_q_heads=12, n_vis=1280, n_text=70)):
        cases.append(Case(w, H.layout_of(w, bits, kg, 128)))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for c in cases:
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
            c.check(cq.CQ_CALIB_NONE)
            c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, n_text=0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [4, 8])
def test_tuned_wide_codes_on_split_and_full_length_rows(kernel_path, bits, decode_chunks):
    w_full = synth.WORKLOADS[2].replace(batch=1, n_kv_heads=2, n_q_heads=8)
    full = Case(w_full, H.layout_of(w_full, bits))
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=8, n_vis=1920, n_text=200)
    split = Case(w, H.layout_of(w, bits))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        full.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
        decode_chunks(3)
        split.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
        split.check(cq.CQ_CALIB_FIXED, 1.0, 2.0, gamma=-30.0, delta=30.0)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("n_q_heads", [4, 3])
@pytest.mark.parametrize("n_text", [5, 64, 130, 1100, 8704])
def test_text_only_rows_on_the_tuned_kernel(kernel_path, n_text, n_q_heads):
    """A cache left entirely in fp16 (the 16-bit baseline of the benchmark): the text waves alone,
    with shares of 64 and of 16 tokens, ragged ends and a padded head.  The weights reach the value
    contraction as fp16 pairs hi + lo: the error stays the fp16 rounding of the output (2.0e-4 to
    2.2e-4 measured), where one fp16 number per weight would add 2^-11 / sqrt(3) = 2.8e-4 in
    quadrature (3.5e-4), hence the bar of 3e-4 here."""
    w = synth.WORKLOADS[2].replace(batch=2, n_kv_heads=1, n_q_heads=n_q_heads, n_vis=0,
                                   n_text=n_text, seed=7300 + n_text)
    c = Case(w, H.layout_of(w))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        c.check(cq.CQ_CALIB_NONE, tol=3e-4)
        c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0, tol=3e-4)      # no visual tokens: nothing to calibrate
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("n_vis,n_text", [(6144, 100), (8192, 512), (10240, 0)])
def test_long_whole_rows(kernel_path, bits, n_vis, n_text):
    """Whole rows of 48 and more key groups run the kernel variant with three key groups in
    flight per wave; short text tails take the 16-token value shares."""
    w = synth.WORKLOADS[2].replace(batch=1, n_kv_heads=2, n_q_heads=8, n_vis=n_vis, n_text=n_text,
                                   seed=7100 + bits)
    c = Case(w, H.layout_of(w, bits))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        c.check(cq.CQ_CALIB_DYNAMIC, 1.0, 2.0)
        c.check(cq.CQ_CALIB_NONE)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
def test_random_layouts_on_the_tuned_kernels(kernel_path, decode_chunks):
    """Seeded sweep over the layouts the tuned kernels accept: code width, group sizes, value
    axis, heads per KV head (1..8), ragged text tails, forced row splits, calibration modes."""
    rng = np.random.default_rng(2024)
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for trial in range(24):
            bits = int(rng.choice([1, 2, 4, 8]))
            kg = int(rng.choice([32, 64, 128]))
            vch = bits <= 2 and rng.random() < 0.4
            vg = int(rng.choice([64, 128])) if vch else 128
            g = int(rng.integers(1, 9))
            hkv = int(rng.integers(1, 3))
            n_vis = 128 * int(rng.integers(1, 13))
            if n_vis > 128 and trial % 4 == 3:          # statistics over the whole sequence
                kg = n_vis
                if vch:
                    vg = n_vis
            n_text = int(rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 130, 257]))
            chunks = int(rng.choice([1, 1, 2, 3]))
            unit = max(128, min(vg, 128) if vch else 64, min(kg, 128))
            if n_vis // unit < chunks:
                chunks = 1
            decode_chunks(chunks)
            w = synth.WORKLOADS[int(rng.choice([1, 4]))].replace(
                batch=int(rng.integers(1, 3)), n_kv_heads=hkv, n_q_heads=hkv * g, n_vis=n_vis,
                n_text=n_text, seed=5000 + trial)
            c = Case(w, H.layout_of(w, bits, kg, vg, 0, 0 if vch else 1))
            mode = int(rng.choice([cq.CQ_CALIB_NONE, cq.CQ_CALIB_DYNAMIC, cq.CQ_CALIB_FIXED]))
            try:
                c.check(mode, float(rng.integers(0, 4)), float(rng.integers(0, 4)), gamma=-25.0, delta=25.0)
            except AssertionError as e:
                raise AssertionError("trial %d (bits %d kg %d vg %d vch %s g %d hkv %d n_vis %d n_text %d "
                                     "chunks %d mode %d): %s" % (trial, bits, kg, vg, vch, g, hkv, n_vis,
                                                                 n_text, chunks, mode, e))
    finally:
        cq.cq_bench_set_kernel_path(prev)
