"""The C++ oracle twin (oracle/cq_oracle.cpp) against what pins the numpy oracle, and against the
numpy oracle itself: packed words, scales and minima bit for bit, attention outputs to 1e-12.

The twin exists so that whole benchmark-size calls can be checked row by row and timed on all host
cores; these CPU-only tests make sure it states the same method: hand-worked examples of the
quantize equation and of the packing formula (tests/golden), exact rational rounding, and a sweep
of layouts, calibration modes and shapes against the numpy oracle."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import cq_oracle as O
from oracle import cq_oracle_native as N

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [part.split() for part in line.split("|")]


def test_builds_loads_and_reports_its_threads():
    assert N.max_threads() >= 1


def test_hand_worked_quantize_examples():
    """tests/golden/quantize_equation_examples.txt: one group of tokens of one channel per line."""
    for (b,), values, codes in _lines("quantize_equation_examples.txt"):
        bits = int(b)
        x = np.array([float(v) for v in values], dtype=np.float16)
        n = len(x)
        pad = 32 // bits                       # d must fill whole words: repeat the channel
        qt = N.quantize_tensor(np.repeat(x.reshape(1, n, 1), pad, axis=2), bits, N.AXIS_CHANNEL, n)
        got = O.unpack(qt["words"], bits, 32)[0, :, 0]
        assert got.tolist() == [int(c) for c in codes], (values, got.tolist())
        assert float(qt["min"][0, 0, 0]) == float(x.astype(np.float64).min())


def test_hand_worked_packing_examples():
    """tests/golden/packing_appendix_examples.txt, the 32-bit containers: codes chosen so that
    quantization returns them unchanged (min 0, max 2^b - 1 present in every group) and the
    packed word must be the hand-computed one."""
    n_checked = 0
    for (nb, m), codes, (word,) in _lines("packing_appendix_examples.txt"):
        bits, M = int(nb), int(m)
        codes = [int(c) for c in codes]
        if M != 32:
            continue
        L = (1 << bits) - 1
        # token-wise group over the 32/bits channels of the word plus a second word holding 0 and L,
        # so the group's statistics are (0, L) whatever the codes are
        per = 32 // bits
        row = np.array(codes + [0, L] + [0] * (per - 2), dtype=np.float16).reshape(1, 1, 2 * per)
        qt = N.quantize_tensor(row, bits, N.AXIS_TOKEN, 2 * per)
        assert int(qt["words"][0, 0, 0]) == int(word), (codes, hex(int(qt["words"][0, 0, 0])))
        assert float(qt["scale"][0, 0, 0]) == 1.0 and float(qt["min"][0, 0, 0]) == 0.0
        n_checked += 1
    assert n_checked >= 4


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_codes_equal_exact_rational_rounding(bits):
    rng = np.random.default_rng(300 + bits)
    L = (1 << bits) - 1
    for trial in range(30):
        n = int(rng.integers(2, 65))
        kind = trial % 4
        if kind == 0:
            x = rng.standard_normal(n)
        elif kind == 1:          # differences that need more than 24 bits
            x = rng.standard_normal(n) * 10.0 ** rng.integers(-6, 5, size=n)
        elif kind == 2:          # few distinct values: many exact ties
            x = rng.integers(-3, 4, size=n) * 0.25
        else:                    # extremes and a subnormal
            x = np.concatenate([[-60000.0, 6e-8], rng.standard_normal(n - 2)])
        x = x.astype(np.float16)
        qt = N.quantize_tensor(np.repeat(x.reshape(1, n, 1), 32, axis=2), bits, N.AXIS_CHANNEL, n)
        got = O.unpack(qt["words"], bits, 32)[0, :, 0]
        A, B = Fraction(float(x.min())), Fraction(float(x.max()))
        want = [0 if A == B else int(round((Fraction(float(v)) - A) * L / (B - A))) for v in x]
        assert got.tolist() == want
        # the stored scale is the float32 nearest to the exact rational
        exact = (B - A) / L
        s = Fraction(float(qt["scale"][0, 0, 0]))
        for nb in (np.nextafter(qt["scale"][0, 0, 0], np.float32(np.inf)),
                   np.nextafter(qt["scale"][0, 0, 0], np.float32(-np.inf))):
            assert abs(s - exact) <= abs(Fraction(float(nb)) - exact)


def _random_cache(rng, B, H, n, d, outliers=True):
    k = rng.standard_normal((B, H, n, d))
    if outliers:
        k[..., rng.integers(0, d, size=3)] *= 8.0
    k[0, 0, : min(n, 16), 0] = 1.5           # a constant stretch: groups with max == min
    k[0, 0, :, 1] = np.where(np.arange(n) % 2 == 0, -0.0, 0.0)   # zeros of both signs
    return k.astype(np.float16)


LAYOUTS = [(1, 0, 128), (1, 0, 32), (2, 0, 64), (1, 1, 128), (2, 1, 32), (4, 0, 128), (8, 1, 64),
           (1, 0, 256), (2, 0, 256), (4, 1, 128)]


@pytest.mark.parametrize("bits,axis,group", LAYOUTS)
def test_quantizer_matches_the_numpy_oracle_bit_for_bit(bits, axis, group):
    rng = np.random.default_rng(11 * bits + axis + group)
    x = _random_cache(rng, 2, 3, 256, 128)
    a = O.quantize_tensor(x, bits, axis, group)
    b = N.quantize_tensor(x, bits, axis, group)
    assert np.array_equal(a["words"], b["words"])
    assert np.array_equal(a["scale"].view(np.uint32), b["scale"].view(np.uint32))
    assert np.array_equal(a["min"].view(np.uint16), b["min"].view(np.uint16))


CASES = [
    # B, Hq, Hkv, n_vis, n_text, cap, bits, (k_axis, k_group), (v_axis, v_group)
    (1, 1, 1, 1024, 32, 32, 1, (0, 128), (1, 128)),
    (2, 8, 2, 384, 40, 64, 1, (0, 128), (1, 128)),
    (1, 12, 2, 256, 7, 7, 2, (0, 64), (1, 128)),
    (2, 4, 4, 256, 0, 0, 1, (0, 256), (0, 256)),
    (1, 6, 3, 128, 19, 32, 4, (0, 32), (0, 64)),
    (2, 4, 2, 128, 5, 8, 8, (1, 64), (1, 32)),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("mode", [O.CALIB_NONE, O.CALIB_DYNAMIC, O.CALIB_FIXED])
def test_decode_matches_the_numpy_oracle(case, mode):
    B, Hq, Hkv, n_vis, n_text, cap, bits, (ka, kg), (va, vg) = case
    rng = np.random.default_rng(sum(case[:6]) + mode)
    d = 128
    k, v = _random_cache(rng, B, Hkv, n_vis, d), _random_cache(rng, B, Hkv, n_vis, d, False)
    q = rng.standard_normal((B, Hq, d)).astype(np.float16)
    kt = rng.standard_normal((B, Hkv, cap, d)).astype(np.float16)
    vt = rng.standard_normal((B, Hkv, cap, d)).astype(np.float16)
    kq_a, vq_a = O.quantize_tensor(k, bits, ka, kg), O.quantize_tensor(v, bits, va, vg)
    kq_b, vq_b = N.quantize_tensor(k, bits, ka, kg), N.quantize_tensor(v, bits, va, vg)
    args = dict(n_text=n_text, calib_mode=mode, tau1=1.0, tau2=2.0, gamma=-20.0, delta=25.0)
    ref = O.decode_attn(q, kq_a, vq_a, kt, vt, **args)
    got = N.decode_attn(q, kq_b, vq_b, kt, vt, **args)
    assert O.rel_l2(got, ref) <= 1e-12
    assert np.abs(got - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
    # other softmax scale, and a shorter tail than the capacity
    if n_text > 1:
        args2 = dict(args, n_text=n_text - 1, softmax_scale=0.05)
        assert O.rel_l2(N.decode_attn(q, kq_b, vq_b, kt, vt, **args2),
                        O.decode_attn(q, kq_a, vq_a, kt, vt, **args2)) <= 1e-12


def test_text_only_and_visual_only_rows():
    rng = np.random.default_rng(5)
    d = 128
    q = rng.standard_normal((2, 4, d)).astype(np.float16)
    kt = rng.standard_normal((2, 2, 33, d)).astype(np.float16)
    vt = rng.standard_normal((2, 2, 33, d)).astype(np.float16)
    got = N.decode_attn(q, None, None, kt, vt, n_text=33, calib_mode=O.CALIB_DYNAMIC, tau1=1, tau2=2)
    # no quantized tokens: textbook attention over the tail
    for b in range(2):
        for hq in range(4):
            h = hq // 2
            s = kt[b, h].astype(np.float64) @ q[b, hq].astype(np.float64) / np.sqrt(d)
            w = np.exp(s - s.max())
            want = (w / w.sum()) @ vt[b, h].astype(np.float64)
            assert np.abs(got[b, hq] - want).max() <= 1e-12
    # equal taus without text leave the output unchanged (softmax shift invariance, Sec. 3.2)
    k = _random_cache(rng, 1, 2, 256, d)
    kq, vq = N.quantize_tensor(k, 1, 0, 128), N.quantize_tensor(k[::-1].copy(), 1, 1, 128)
    q1 = q[:1]
    a = N.decode_attn(q1, kq, vq, None, None, 0, O.CALIB_NONE)
    b_ = N.decode_attn(q1, kq, vq, None, None, 0, O.CALIB_DYNAMIC, 2.0, 2.0)
    assert O.rel_l2(b_, a) <= 1e-12
