"""Pins of the oracle's attention half: identities, closed forms, a library routine
(CPU scaled_dot_product_attention) and a pure-Python brute force."""
import math

import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from paper_2502_14882_amd import synth


def _small(seed=3, B=2, Hq=4, Hkv=2, d=64, nv=96, nt=7, kind="uniform"):
    w = synth.Workload("t", seed, B, Hq, Hkv, d, nv, nt, kind)
    t = synth.make_inputs(w, "cpu")
    return w, {k: v.numpy() for k, v in t.items()}


def _quant(x, bits=1, kg=32, vg=None, v_axis=O.AXIS_TOKEN):
    k = O.quantize_tensor(x["k"], bits, O.AXIS_CHANNEL, kg)
    v = O.quantize_tensor(x["v"], bits, v_axis, vg or x["v"].shape[-1])
    return k, v


# --------------------------------------------------------------------------- post-scaling (Sec. 3.1)
@pytest.mark.parametrize("bits", [1, 2, 4])
def test_postscale_identity(bits):
    w, x = _small()
    kq, _ = _quant(x, bits)
    k_deq = O.dequantize(kq["codes"], kq["scale"], kq["min"], 0, 32)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            q = x["q"][b, 2 * h].astype(np.float64)
            lhs = O.logits_postscale(q, kq["codes"][b, h], kq["scale"][b, h], kq["min"][b, h],
                                     32, 0.125)
            rhs = O.logits_dequant(q, k_deq[b, h], 0.125)
            np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------- calibration (Sec. 3.2)
@pytest.mark.parametrize("t1,t2", [(0, 0), (1, 2), (3, 0), (0, 3), (2.5, 0.5)])
def test_calibration_maps_interval_ends_and_is_affine(t1, t2):
    rng = np.random.default_rng(5)
    s = rng.standard_normal(200) * 7
    g = O.calibrate(s, t1, t2, O.CALIB_DYNAMIC)
    lo, hi = s.argmin(), s.argmax()
    assert g[lo] == pytest.approx(s[lo] - t1, abs=1e-12)
    assert g[hi] == pytest.approx(s[hi] - t2, abs=1e-12)
    # affine: every point lies on the chord between the mapped ends
    lam = (s - s[lo]) / (s[hi] - s[lo])
    np.testing.assert_allclose(g, (1 - lam) * (s[lo] - t1) + lam * (s[hi] - t2), atol=1e-10)
    if t1 == t2 == 0:
        np.testing.assert_allclose(g, s, atol=1e-12)


def test_calibration_fixed_none_and_degenerate():
    s = np.array([-2.0, 0.5, 4.0])
    np.testing.assert_array_equal(O.calibrate(s, 1, 2, O.CALIB_NONE), s)
    g = O.calibrate(s, 1.0, 2.0, O.CALIB_FIXED, gamma=-4.0, delta=6.0)
    # [-4, 6] -> [-5, 4]: slope 0.9; g(-4) = -5
    np.testing.assert_allclose(g, 0.9 * (s + 4.0) - 5.0, atol=1e-12)
    # a single-valued row: slope 1, shifted by tau1
    np.testing.assert_allclose(O.calibrate(np.full(4, 3.0), 1.0, 2.0), np.full(4, 2.0))


def test_equal_taus_without_text_leave_attention_unchanged():
    w, x = _small(nt=0)
    kq, vq = _quant(x)
    a = O.decode_attn(x["q"], kq, vq, calib_mode=O.CALIB_NONE)
    b = O.decode_attn(x["q"], kq, vq, calib_mode=O.CALIB_DYNAMIC, tau1=2.0, tau2=2.0)
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)
    c = O.decode_attn(x["q"], kq, vq, calib_mode=O.CALIB_DYNAMIC, tau1=1.0, tau2=2.0)
    assert O.rel_l2(c, a) > 1e-4       # unequal taus do change it


def test_calibration_touches_visual_logits_only_and_softmax_is_joint():
    w, x = _small(nt=9)
    kq, vq = _quant(x)
    t1, t2 = 1.0, 3.0
    _, p0 = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], 9, O.CALIB_NONE,
                          return_parts=True)
    _, p1 = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], 9, O.CALIB_DYNAMIC, t1, t2,
                          return_parts=True)
    for (s_vis, s_txt, w0), (c_vis, c_txt, w1) in zip(p0, p1):
        nv = s_vis.size
        np.testing.assert_array_equal(s_txt, c_txt)
        hi, lo = s_vis.argmax(), s_vis.argmin()
        assert w1.sum() == pytest.approx(1.0, abs=1e-12)
        for k in range(9):
            # log-odds against an untouched text token move by exactly -tau at the ends
            assert math.log(w1[hi] / w1[nv + k]) == pytest.approx(
                math.log(w0[hi] / w0[nv + k]) - t2, abs=1e-9)
            assert math.log(w1[lo] / w1[nv + k]) == pytest.approx(
                math.log(w0[lo] / w0[nv + k]) - t1, abs=1e-9)


# --------------------------------------------------------------------------- textbook attention
@pytest.mark.parametrize("bits,v_axis,nt", [(1, O.AXIS_TOKEN, 7), (2, O.AXIS_TOKEN, 0),
                                            (1, O.AXIS_CHANNEL, 5)])
def test_reduces_to_library_attention_on_dequantized_cache(bits, v_axis, nt):
    w, x = _small(seed=9, nt=nt)
    kq, vq = _quant(x, bits, 32, 32, v_axis)
    out = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], nt, O.CALIB_NONE)
    k_deq = O.dequantize(kq["codes"], kq["scale"], kq["min"], 0, 32)
    v_deq = O.dequantize(vq["codes"], vq["scale"], vq["min"], v_axis, 32)
    kk = np.concatenate([k_deq, x["k_text"][:, :, :nt].astype(np.float64)], axis=2)
    vv = np.concatenate([v_deq, x["v_text"][:, :, :nt].astype(np.float64)], axis=2)
    g = w.n_q_heads // w.n_kv_heads
    kk = torch.from_numpy(kk).repeat_interleave(g, dim=1)
    vv = torch.from_numpy(vv).repeat_interleave(g, dim=1)
    qq = torch.from_numpy(x["q"].astype(np.float64))[:, :, None, :]
    ref = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv)[:, :, 0, :].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)


def test_brute_force_python_loops_tiny():
    w, x = _small(seed=4, B=1, Hq=2, Hkv=1, d=32, nv=8, nt=3, kind="none")
    kq, vq = _quant(x, 1, 4, 32)
    out = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], 3, O.CALIB_NONE)
    # bits -> {min, max}: rebuild the dequantized cache from the packed words by hand
    for hq in range(2):
        logits, vals = [], []
        for j in range(8):
            word = int(kq["words"][0, 0, j, 0])
            vword = int(vq["words"][0, 0, j, 0])
            acc, vrow = 0.0, []
            for c in range(32):
                kbit = (word >> (31 - c)) & 1
                kval = float(kq["min"][0, 0, j // 4, c]) + kbit * float(kq["scale"][0, 0, j // 4, c])
                acc += float(x["q"][0, hq, c]) * kval
                vbit = (vword >> (31 - c)) & 1
                vrow.append(float(vq["min"][0, 0, j, 0]) + vbit * float(vq["scale"][0, 0, j, 0]))
            logits.append(acc / math.sqrt(32.0))
            vals.append(vrow)
        for t in range(3):
            logits.append(sum(float(x["q"][0, hq, c]) * float(x["k_text"][0, 0, t, c])
                              for c in range(32)) / math.sqrt(32.0))
            vals.append([float(v) for v in x["v_text"][0, 0, t]])
        m = max(logits)
        e = [math.exp(s - m) for s in logits]
        z = sum(e)
        for c in range(32):
            want = sum(e[j] * vals[j][c] for j in range(11)) / z
            assert out[0, hq, c] == pytest.approx(want, rel=1e-10, abs=1e-12)


def test_eight_bits_is_close_to_exact_attention_and_one_bit_is_not():
    w, x = _small(seed=21, nv=128, nt=4)
    g = w.n_q_heads // w.n_kv_heads
    kk = torch.from_numpy(np.concatenate([x["k"], x["k_text"]], 2).astype(np.float64))
    vv = torch.from_numpy(np.concatenate([x["v"], x["v_text"]], 2).astype(np.float64))
    qq = torch.from_numpy(x["q"].astype(np.float64))[:, :, None, :]
    exact = torch.nn.functional.scaled_dot_product_attention(
        qq, kk.repeat_interleave(g, 1), vv.repeat_interleave(g, 1))[:, :, 0].numpy()
    errs = {}
    for bits in (1, 2, 4, 8):
        kq, vq = _quant(x, bits, 32, 64)
        out = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], 4, O.CALIB_NONE)
        errs[bits] = O.rel_l2(out, exact)
    assert errs[8] < 0.02 and errs[8] < errs[4] < errs[2] < errs[1]


def test_text_capacity_larger_than_n_text_is_ignored():
    w, x = _small(nt=6)
    kq, vq = _quant(x)
    a = O.decode_attn(x["q"], kq, vq, x["k_text"], x["v_text"], 4, O.CALIB_DYNAMIC, 1, 2)
    kt, vt = x["k_text"].copy(), x["v_text"].copy()
    kt[:, :, 4:] = 99.0
    vt[:, :, 4:] = -99.0
    b = O.decode_attn(x["q"], kq, vq, kt, vt, 4, O.CALIB_DYNAMIC, 1, 2)
    np.testing.assert_array_equal(a, b)


# --------------------------------------------------------------------------- the generators
def test_synth_shapes_determinism_and_outliers():
    w = synth.WORKLOADS[0]
    a = synth.make_inputs(w, "cpu")
    b = synth.make_inputs(w, "cpu")
    assert a["k"].shape == (1, 1, 1024, 128) and a["k_text"].shape == (1, 1, 32, 128)
    assert a["q"].shape == (1, 1, 128) and a["k"].dtype == torch.float16
    for name in a:
        assert torch.equal(a[name], b[name])
    std = a["k"].float().std(dim=2)[0, 0]
    assert std[5] > 6 and std[77] > 6 and std[6] < 1.5
    w1 = synth.WORKLOADS[1].replace(batch=1, n_vis=256, n_text=8)
    k = synth.make_inputs(w1, "cpu", parts=("k",))["k"]
    big = (k.float().std(dim=2)[0] > 4).sum(dim=1)
    assert big.tolist() == [5] * 8
    w4 = synth.WORKLOADS[4].replace(batch=1, n_vis=512, n_text=8)
    k4 = synth.make_inputs(w4, "cpu", parts=("k",))["k"]
    assert torch.isfinite(k4).all() and k4.abs().max() > 20


def test_rel_l2_by_hand():
    """The parity metric itself, on numbers worked by hand: a = (3, 4, 0), b = (0, 0, 5) ->
    ||a - b|| = sqrt(9 + 16 + 25) = sqrt(50), ||b|| = 5 -> sqrt(2); the order of the arguments
    matters (the second one is the reference); identical tensors give 0; a zero reference does not
    divide by zero; the shape is ignored (norm over the whole tensor)."""
    a, b = np.array([3.0, 4.0, 0.0]), np.array([0.0, 0.0, 5.0])
    assert abs(O.rel_l2(a, b) - 2.0 ** 0.5) < 1e-15
    assert abs(O.rel_l2(b, np.array([3.0, 4.0, 12.0])) - (9 + 16 + 49) ** 0.5 / 13.0) < 1e-15
    assert O.rel_l2(b, b) == 0.0
    assert O.rel_l2(a, np.zeros(3)) == 5.0
    assert abs(O.rel_l2(a.reshape(3, 1), b.reshape(1, 3).T) - 2.0 ** 0.5) < 1e-15
    # one element off by 1 % in a tensor of 100 equal elements: 0.01 / sqrt(100)
    x = np.ones(100)
    y = x.copy()
    y[7] = 1.01
    assert abs(O.rel_l2(y, x) - 1e-3) < 1e-12
