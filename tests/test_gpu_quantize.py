"""GPU parity of cq_quantize_kv against the oracle: packed codes, scale and min bit-exact."""
import numpy as np
import pytest
import torch

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
    """Every case runs on the shape-agnostic kernels and on whatever AUTO selects."""
    prev = cq.cq_bench_set_kernel_path({"generic": cq.CQ_PATH_GENERIC, "auto": cq.CQ_PATH_AUTO}[request.param])
    yield request.param
    cq.cq_bench_set_kernel_path(prev)


def _run(w, lay, x_cpu=None, what=""):
    x_cpu = x_cpu or synth.make_inputs(w, "cpu", parts=("k", "v"))
    kq, vq = H.oracle_quantize(x_cpu, lay)
    x = H.to_device(x_cpu)
    k_out, v_out = cq.cq_quantize_kv(lay, x["k"], x["v"])
    torch.cuda.synchronize()
    H.assert_qtensor_equal(k_out, kq, what + " keys")
    H.assert_qtensor_equal(v_out, vq, what + " values")


def test_config0_full_size():
    w = synth.WORKLOADS[0]
    _run(w, H.layout_of(w), what="config0")


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_config3_shrunk_sweep(bits, group):
    # same law as the quantizer-only workload (outliers in keys and values), fewer rows/tokens,
    # several 128-token tiles per row
    w = synth.WORKLOADS[3].replace(batch=3, n_kv_heads=2, n_q_heads=2, n_vis=640)
    _run(w, H.layout_of(w, bits, group, group), what="cfg3 b=%d G=%d" % (bits, group))


@pytest.mark.parametrize("idx", [1, 2, 4])
def test_decode_configs_shrunk(idx):
    w = synth.WORKLOADS[idx].replace(batch=2, n_kv_heads=2, n_q_heads=2, n_vis=768)
    _run(w, H.layout_of(w), what="cfg%d" % idx)


@pytest.mark.parametrize("bits", [4, 8])
def test_wider_codes(bits):
    w = synth.WORKLOADS[1].replace(batch=1, n_kv_heads=2, n_q_heads=2, n_vis=256)
    _run(w, H.layout_of(w, bits, 64, 32), what="b=%d" % bits)


@pytest.mark.parametrize("d", [32, 64, 256])
def test_other_head_dims(d):
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=1, n_q_heads=1, head_dim=d, n_vis=192)
    _run(w, H.layout_of(w, 2, 64, 32), what="d=%d" % d)


def test_swapped_axes_and_whole_sequence_group():
    w = synth.WORKLOADS[1].replace(batch=2, n_kv_heads=2, n_q_heads=2, n_vis=384)
    # paper-literal: channel-wise keys AND values over the whole sequence
    _run(w, H.layout_of(w, 1, 384, 384, 0, 0), what="G=n")
    _run(w, H.layout_of(w, 2, 64, 128, 1, 0), what="token-wise keys, channel-wise values")


def test_ties_constants_zeros_and_extremes():
    w = synth.WORKLOADS[0].replace(n_vis=256)
    x = synth.make_inputs(w, "cpu", parts=("k", "v"))
    k, v = x["k"], x["v"]
    k[0, 0, :128, 0] = 1.5                       # constant group
    k[0, 0, :128, 1] = 0.0
    k[0, 0, 5, 1] = -0.0                         # zeros of both signs only
    k[0, 0, :128, 2] = torch.tensor([0.0, 1.0, 0.5, 0.25] * 32)      # exact midpoint ties (b=1)
    k[0, 0, :128, 3] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * 16)  # b=2 ties
    k[0, 0, :128, 4] = torch.tensor([-65504.0, 65504.0, 6e-8, -6e-8] * 32)  # 41-bit differences
    k[0, 0, 128:, 6] = -0.0                      # constant negative zero
    v[0, 0, 0, :] = 2.0                          # constant token
    v[0, 0, 1, :] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * 16)
    v[0, 0, 2, :] = torch.tensor([-0.0, 0.0] * 64)
    v[0, 0, 3, :] = torch.tensor([60000.0, 1e-4, -1e-4, 0.33] * 32)
    for bits in (1, 2):
        _run(w, H.layout_of(w, bits, 128, 128), x, what="edge b=%d" % bits)
        _run(w, H.layout_of(w, bits, 32, 32), x, what="edge G=32 b=%d" % bits)


def test_keys_only_and_values_only():
    w = synth.WORKLOADS[0].replace(n_vis=256)
    lay = H.layout_of(w)
    x_cpu = synth.make_inputs(w, "cpu", parts=("k", "v"))
    kq, vq = H.oracle_quantize(x_cpu, lay)
    x = H.to_device(x_cpu)
    k_out, none = cq.cq_quantize_kv(lay, x["k"], None)
    assert none is None
    H.assert_qtensor_equal(k_out, kq, "keys only")
    none, v_out = cq.cq_quantize_kv(lay, None, x["v"])
    assert none is None
    H.assert_qtensor_equal(v_out, vq, "values only")


def test_runs_on_a_side_stream():
    w = synth.WORKLOADS[0].replace(n_vis=512)
    lay = H.layout_of(w)
    x_cpu = synth.make_inputs(w, "cpu", parts=("k", "v"))
    kq, vq = H.oracle_quantize(x_cpu, lay)
    x = H.to_device(x_cpu)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        k_out, v_out = cq.cq_quantize_kv(lay, x["k"], x["v"])
    st.synchronize()
    H.assert_qtensor_equal(k_out, kq, "side stream keys")
    H.assert_qtensor_equal(v_out, vq, "side stream values")


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_tuned_path_takes_the_benchmark_layouts(kernel_path, bits, group):
    """head_dim 128, b in {1,2}, groups 32/64/128 must run on the tuned kernels (no silent
    fallback) and stay bit-exact, including exact ties and heavy-tailed outliers."""
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        w = synth.WORKLOADS[4].replace(batch=2, n_kv_heads=2, n_q_heads=2, n_vis=1024)
        x = synth.make_inputs(w, "cpu", parts=("k", "v"))
        x["k"][0, 0, :128, 2] = torch.tensor([0.0, 1.0, 0.5, 0.25] * 32)
        x["k"][0, 0, :128, 3] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * 16)
        x["k"][0, 1, :256, 9] = 0.75
        x["v"][1, 0, 7, :] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * 16)
        x["v"][1, 1, 9, :] = -2.5
        x["v"][1, 1, 10, :] = torch.tensor([-0.0, 0.0] * 64)
        _run(w, H.layout_of(w, bits, group, group), x, what="tuned b=%d G=%d" % (bits, group))
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("n_vis", [256, 640, 2304])
def test_tuned_whole_sequence_statistics(kernel_path, bits, n_vis):
    """Sec. 3.1 as printed (one pair per channel over all tokens, keys and values) on the tuned
    kernels: extrema pass + tile pass, with exact ties, a constant channel, signed zeros and rows
    whose extreme elements sit in the first and in the last tile."""
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        w = synth.WORKLOADS[4].replace(batch=2, n_kv_heads=2, n_q_heads=2, n_vis=n_vis)
        x = synth.make_inputs(w, "cpu", parts=("k", "v"))
        x["k"][0, 0, :, 2] = torch.tensor([0.0, 1.0, 0.5, 0.25] * (n_vis // 4))
        x["k"][0, 0, :, 3] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * (n_vis // 8))
        x["k"][0, 1, :, 9] = 0.75
        x["k"][1, 0, :, 11] = torch.tensor([-0.0, 0.0] * (n_vis // 2))
        x["k"][1, 1, 0, 5] = 900.0            # the row's maximum in its first tile
        x["k"][1, 1, n_vis - 1, 6] = -900.0   # the row's minimum in its last token
        x["v"][1, 0, :, 7] = torch.tensor([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 3.0] * (n_vis // 8))
        x["v"][1, 1, :, 9] = -2.5
        x["v"][0, 0, n_vis // 2, 64] = 60000.0
        _run(w, H.layout_of(w, bits, n_vis, n_vis, 0, 0), x, what="whole sequence b=%d" % bits)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits,group", [(1, 128), (2, 32), (4, 64), (8, 128)])
def test_full_size_quantizer_config_on_sampled_rows(kernel_path, bits, group):
    """configs[3] at full size (batch 128, 8 KV heads, 16384 tokens), drawn on the GPU as
    bench.py does and quantized by the launch bench.py times; the oracle checks sampled
    (batch, KV head) rows bit for bit, each one independently (rows do not interact)."""
    from oracle import cq_oracle as O
    w = synth.WORKLOADS[3]
    lay = H.layout_of(w, bits, group, group)
    x = synth.make_inputs(w, "cuda", parts=("k", "v"))
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        k_out, v_out = cq.cq_quantize_kv(lay, x["k"], x["v"])
        torch.cuda.synchronize()
    finally:
        cq.cq_bench_set_kernel_path(prev)
    rng = np.random.default_rng(11)
    rows = {(0, 0), (w.batch - 1, w.n_kv_heads - 1)}
    while len(rows) < 5:
        rows.add((int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads))))
    for b, h in sorted(rows):
        for name, out, axis in (("k", k_out, lay.k_axis), ("v", v_out, lay.v_axis)):
            ref = O.quantize_tensor(x[name][b:b + 1, h:h + 1].cpu().numpy(), bits, axis, group)
            got = cq.QTensor(out.codes[b:b + 1, h:h + 1], out.scale[b:b + 1, h:h + 1],
                             out.min[b:b + 1, h:h + 1])
            H.assert_qtensor_equal(got, ref, "configs[3] %s row (%d,%d)" % (name, b, h))


@pytest.mark.tuned_only
@pytest.mark.parametrize("bits", [4, 8])
def test_wide_codes_round_exact_ties_to_even_on_the_tuned_path(kernel_path, bits):
    """Every code boundary of a 4- or 8-bit grid hit exactly: values k + 1/2 steps of a group
    whose range makes the step a power of two, on both axes."""
    L = (1 << bits) - 1
    w = synth.WORKLOADS[1].replace(batch=1, n_kv_heads=1, n_q_heads=1, n_vis=512)
    x = synth.make_inputs(w, "cpu", parts=("k", "v"))
    # group range [0, L/8] -> step 1/8: multiples of 1/16 are representable and odd ones are ties
    grid = (torch.arange(0, 2 * L + 1, dtype=torch.float32) / 16.0).to(torch.float16)
    ties = grid.repeat((512 + grid.numel() - 1) // grid.numel())[:512]
    x["k"][0, 0, :, 7] = ties                       # channel 7 over the tokens
    x["k"][0, 0, :, 8] = -ties
    for t in range(0, 512, 37):
        x["v"][0, 0, t, :] = ties[:128] if bits == 4 else ties[t % 64:t % 64 + 128]
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for group in (32, 128):
            _run(w, H.layout_of(w, bits, group, group), x, what="ties b=%d G=%d" % (bits, group))
            _run(w, H.layout_of(w, bits, group, group, 1, 0), x, what="ties swapped b=%d" % bits)
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
def test_random_layouts_on_the_tuned_quantizer(kernel_path):
    """Seeded sweep over what the tuned quantizer accepts: code width, group size, either axis for
    keys and values, row counts and lengths; heavy-tailed and outlier inputs; bit-exact."""
    rng = np.random.default_rng(99)
    prev = cq.cq_bench_set_kernel_path(cq.CQ_PATH_TUNED)
    try:
        for trial in range(20):
            bits = int(rng.choice([1, 2, 4, 8]))
            kg, vg = int(rng.choice([32, 64, 128])), int(rng.choice([32, 64, 128]))
            ka, va = int(rng.integers(0, 2)), int(rng.integers(0, 2))
            w = synth.WORKLOADS[int(rng.choice([1, 3, 4]))].replace(
                batch=int(rng.integers(1, 4)), n_kv_heads=int(rng.integers(1, 4)), n_q_heads=1,
                n_vis=128 * int(rng.integers(1, 9)), seed=7000 + trial)
            w = w.replace(n_q_heads=w.n_kv_heads)
            _run(w, H.layout_of(w, bits, kg, vg, ka, va),
                 what="trial %d b=%d kg=%d vg=%d axes=%d%d" % (trial, bits, kg, vg, ka, va))
    finally:
        cq.cq_bench_set_kernel_path(prev)


@pytest.mark.tuned_only
def test_traffic_measurement_aid_runs(kernel_path):
    """The quantizer's traffic skeleton (measurement aid) reads its tiles and writes the byte counts
    it is asked for, and nothing beyond them."""
    n_tiles, cb, mb = 37, 2048, 768
    x = torch.randn(n_tiles * 128, 128, device="cuda").half()
    codes = torch.full((n_tiles * cb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    meta = torch.full((n_tiles * mb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    cq.cq_bench_tile_traffic(x, codes, meta, n_tiles, cb, mb)
    torch.cuda.synchronize()
    assert bool((codes[n_tiles * cb:] == 0xA5).all()) and bool((meta[n_tiles * mb:] == 0xA5).all())
    # every tile wrote something (the fold of a random tile is not the fill pattern throughout)
    assert not bool((codes[:n_tiles * cb].view(n_tiles, cb) == 0xA5).all(dim=1).any())
