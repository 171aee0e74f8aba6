"""Pins of the oracle's quantizer half against what the paper and arithmetic fix.

None of these tests re-types the oracle's formulas: they use exact rational
arithmetic (fractions.Fraction), closed forms from the paper's appendix,
invariants stated in the paper's text, and hand-computed examples.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import cq_oracle as O


# --------------------------------------------------------------------------- packing
def test_pack_hand_examples():
    # Appendix formula by hand: 1-bit codes into a byte, MSB first.
    assert int(O.pack([1, 0, 1, 1, 0, 0, 0, 1], 1, 8)[0]) == 0b10110001
    # 2-bit codes (3,0,2,1) -> 3*64 + 0*16 + 2*4 + 1
    assert int(O.pack([3, 0, 2, 1], 2, 8)[0]) == 201
    # 32-bit container, first element lands in the top bit
    v = np.zeros(32, dtype=np.uint8)
    v[0] = 1
    assert int(O.pack(v, 1, 32)[0]) == 1 << 31


@pytest.mark.parametrize("N", [1, 2, 4, 8])
@pytest.mark.parametrize("M", [8, 32])
def test_pack_unit_vectors_are_powers_of_two(N, M):
    per = M // N
    for i in range(per):
        for val in (1, (1 << N) - 1):
            e = np.zeros(per, dtype=np.uint8)
            e[i] = val
            assert int(O.pack(e, N, M)[0]) == val * 2 ** (M - N * (1 + i))


@pytest.mark.parametrize("N", [1, 2, 4, 8])
def test_unpack_matches_integer_arithmetic_and_round_trips(N):
    rng = np.random.default_rng(7 + N)
    codes = rng.integers(0, 1 << N, size=(3, 5, 128), dtype=np.uint8)
    words = O.pack(codes, N, 32)
    assert words.dtype == np.uint32 and words.shape == (3, 5, 128 * N // 32)
    back = O.unpack(words, N, 32)
    assert np.array_equal(back, codes)
    # element i by plain Python integers: floor(u / 2^(M-N(1+i))) mod 2^N
    per = 32 // N
    u = int(words[1, 2, 3])
    for i in range(per):
        assert (u // 2 ** (32 - N * (1 + i))) % (1 << N) == int(codes[1, 2, 3 * per + i])


# --------------------------------------------------------------------------- rounding rule
def _exact_code(x, alpha, beta, bits):
    """Quantize equation in exact rationals; Python rounds Fractions half-to-even."""
    X, A, B = Fraction(float(x)), Fraction(float(alpha)), Fraction(float(beta))
    if B == A:
        return 0
    return int(round((X - A) * ((1 << bits) - 1) / (B - A)))


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
def test_codes_equal_exact_rational_rounding(bits):
    rng = np.random.default_rng(100 + bits)
    for trial in range(40):
        n = int(rng.integers(2, 65))
        kind = trial % 4
        if kind == 0:
            x = rng.standard_normal(n)
        elif kind == 1:   # huge dynamic range: differences need > 24 bits
            x = rng.standard_normal(n) * 10.0 ** rng.integers(-6, 5, size=n)
        elif kind == 2:   # few distinct values -> many exact ties
            x = rng.integers(-3, 4, size=n) * 0.25
        else:
            x = np.concatenate([[-60000.0, 6e-8], rng.standard_normal(n - 2)])
        x = x.astype(np.float16)
        xs = x.reshape(1, n, 1)                    # one channel, n tokens, one group
        qt = O.quantize_tensor(np.repeat(xs, 32, axis=2), bits, O.AXIS_CHANNEL, n)
        a, b = float(x.astype(np.float64).min()), float(x.astype(np.float64).max())
        want = [_exact_code(v, a, b, bits) for v in x]
        assert qt["codes"][0, :, 0].tolist() == want


def test_constructed_ties_and_degenerate_group():
    # b=1: the exact midpoint rounds to 0 (0.5 -> even)
    x = np.array([0.0, 1.0, 0.5, 0.50048828125, 0.499755859375], dtype=np.float16)
    c = O.discretize(x.astype(np.float64), 0.0, 1.0, 1)
    assert c.tolist() == [0, 1, 0, 1, 0]
    # b=2, alpha=0, beta=3: quotient = x; 0.5->0, 1.5->2, 2.5->2 (ties to even)
    x = np.array([0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0], dtype=np.float16)
    c = O.discretize(x.astype(np.float64), 0.0, 3.0, 2)
    assert c.tolist() == [0, 3, 0, 2, 2, 1, 2]
    # constant group: codes 0, scale 0, dequantized value is the constant itself
    k = np.full((1, 4, 32), -1.25, dtype=np.float16)
    qt = O.quantize_tensor(k, 1, O.AXIS_CHANNEL, 4)
    assert not qt["codes"].any() and not qt["scale"].any()
    assert np.all(O.dequantize(qt["codes"], qt["scale"], qt["min"], 0, 4) == -1.25)


def test_negative_zero_minimum_is_stored_as_plus_zero():
    k = np.zeros((1, 2, 32), dtype=np.float16)
    k[0, 0, :] = -0.0
    k[0, 1, :] = 1.0
    qt = O.quantize_tensor(k, 1, O.AXIS_CHANNEL, 2)
    assert np.all(qt["min"].view(np.uint16) == 0)


# --------------------------------------------------------------------------- invariants of Sec. 2.2 / 3.2
def _rand_cache(seed, shape, outliers=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape)
    if outliers:
        x[..., 5] *= 8.0
    return x.astype(np.float16)


@pytest.mark.parametrize("axis,group", [(O.AXIS_CHANNEL, 32), (O.AXIS_CHANNEL, 128),
                                        (O.AXIS_TOKEN, 32), (O.AXIS_TOKEN, 128)])
def test_one_bit_dequantizes_onto_group_min_and_max(axis, group):
    x = _rand_cache(1, (2, 3, 256, 128))
    qt = O.quantize_tensor(x, 1, axis, group)
    deq = O.dequantize(qt["codes"], qt["scale"], qt["min"], axis, group)
    alpha, beta = O.group_min_max(x, axis, group)
    lo = O._ungrouped(np.broadcast_to(alpha[..., None], alpha.shape + (group,)), axis, 256, 128)
    hi = O._ungrouped(np.broadcast_to(beta[..., None], beta.shape + (group,)), axis, 256, 128)
    is_lo = deq == lo
    # the upper level is min + float32(beta - alpha): equal to beta whenever that
    # difference fits float32, never further than one float32 ulp of it
    ulp = np.spacing((hi - lo).astype(np.float32)).astype(np.float64)
    is_hi = np.abs(deq - hi) <= ulp
    assert np.all(is_lo | is_hi)
    exact = (hi - lo) == (hi - lo).astype(np.float32)
    assert np.all((deq == hi)[~is_lo & exact])
    # every group attains both levels, and its extreme elements map to them
    x64 = x.astype(np.float64)
    assert np.all(qt["codes"][x64 == lo] == 0)
    assert np.all(qt["codes"][(x64 == hi) & (hi > lo)] == 1)


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("axis", [O.AXIS_CHANNEL, O.AXIS_TOKEN])
def test_codes_in_range_endpoints_and_error_bound(bits, axis):
    group = 64
    x = _rand_cache(2 + bits, (1, 2, 128, 128))
    L = (1 << bits) - 1
    qt = O.quantize_tensor(x, bits, axis, group)
    assert qt["codes"].max() <= L
    alpha, beta = O.group_min_max(x, axis, group)
    lo = O._ungrouped(np.broadcast_to(alpha[..., None], alpha.shape + (group,)), axis, 128, 128)
    hi = O._ungrouped(np.broadcast_to(beta[..., None], beta.shape + (group,)), axis, 128, 128)
    x64 = x.astype(np.float64)
    assert np.all(qt["codes"][x64 == lo] == 0) and np.all(qt["codes"][x64 == hi] == L)
    deq = O.dequantize(qt["codes"], qt["scale"], qt["min"], axis, group)
    # |x - x_deq| <= (beta-alpha)/(2L), plus the float32 rounding of the stored scale
    bound = (hi - lo) / (2.0 * L) + L * np.spacing(((hi - lo) / L).astype(np.float32))
    assert np.all(np.abs(x64 - deq) <= bound)
    # more bits, smaller error
    if bits > 1:
        q1 = O.quantize_tensor(x, bits - 1 if bits == 2 else bits // 2, axis, group)
        d1 = O.dequantize(q1["codes"], q1["scale"], q1["min"], axis, group)
        assert np.abs(x64 - deq).mean() < np.abs(x64 - d1).mean()


@pytest.mark.parametrize("bits", [1, 2])
def test_scale_is_nearest_float32_and_min_is_a_copy(bits):
    x = _rand_cache(11, (1, 1, 256, 128))
    x[0, 0, 3, 7] = 60000.0          # a difference that does not fit float32
    x[0, 0, 4, 7] = 3e-7
    L = (1 << bits) - 1
    qt = O.quantize_tensor(x, bits, O.AXIS_CHANNEL, 128)
    for t in range(2):
        for c in (0, 5, 7, 100):
            col = [Fraction(float(v)) for v in x[0, 0, t * 128:(t + 1) * 128, c]]
            exact = (max(col) - min(col)) / L
            s = np.float32(qt["scale"][0, 0, t, c])
            err = abs(Fraction(float(s)) - exact)
            for nb in (np.nextafter(s, np.float32(np.inf)), np.nextafter(s, np.float32(-np.inf))):
                assert err <= abs(Fraction(float(nb)) - exact)
            assert Fraction(float(qt["min"][0, 0, t, c])) == min(col)
    assert qt["scale"].dtype == np.float32 and qt["min"].dtype == np.float16


@pytest.mark.parametrize("bits", [1, 2])
def test_scale_single_rounding_on_wide_differences(bits):
    # two-token groups whose difference needs far more than 24 bits: rounding the
    # difference to float32 first and dividing afterwards would be caught here
    rng = np.random.default_rng(77)
    d = 2048
    x = np.empty((1, 1, 2, d), dtype=np.float16)
    x[0, 0, 0] = (rng.uniform(1.0, 2.0, d) * 2.0 ** rng.integers(-20, -8, d)).astype(np.float16)
    x[0, 0, 1] = (rng.uniform(1.0, 2.0, d) * 2.0 ** rng.integers(4, 15, d)).astype(np.float16)
    L = (1 << bits) - 1
    qt = O.quantize_tensor(x, bits, O.AXIS_CHANNEL, 2)
    for c in range(d):
        exact = (Fraction(float(x[0, 0, 1, c])) - Fraction(float(x[0, 0, 0, c]))) / L
        s = np.float32(qt["scale"][0, 0, 0, c])
        err = abs(Fraction(float(s)) - exact)
        up, dn = np.nextafter(s, np.float32(np.inf)), np.nextafter(s, np.float32(-np.inf))
        assert err <= abs(Fraction(float(up)) - exact) and err <= abs(Fraction(float(dn)) - exact)


def test_group_equal_to_sequence_is_the_papers_channelwise_definition():
    x = _rand_cache(12, (1, 2, 96, 64))
    qt = O.quantize_tensor(x, 2, O.AXIS_CHANNEL, 96)
    assert qt["min"].shape == (1, 2, 1, 64)
    assert np.array_equal(qt["min"][:, :, 0, :], x.min(axis=2))
    want = ((x.astype(np.float64).max(axis=2) - x.astype(np.float64).min(axis=2)) / 3.0)
    assert np.array_equal(qt["scale"][:, :, 0, :], want.astype(np.float32))


def test_axis_semantics_by_hand():
    # 2 tokens x 64 channels; token axis with channel groups of 32
    x = np.zeros((1, 1, 2, 64), dtype=np.float16)
    x[0, 0, 0, :32] = np.linspace(-1, 1, 32)
    x[0, 0, 0, 32:] = 5.0
    x[0, 0, 1, :] = np.linspace(0, 2, 64)
    qt = O.quantize_tensor(x, 1, O.AXIS_TOKEN, 32)
    assert qt["min"].shape == (1, 1, 2, 2) and qt["words"].shape == (1, 1, 2, 2)
    assert float(qt["min"][0, 0, 0, 0]) == -1.0 and float(qt["scale"][0, 0, 0, 0]) == 2.0
    assert float(qt["min"][0, 0, 0, 1]) == 5.0 and float(qt["scale"][0, 0, 0, 1]) == 0.0
    # first token, first group: negative half -> 0, positive half -> 1, MSB first
    assert int(qt["words"][0, 0, 0, 0]) == 0x0000FFFF
    assert int(qt["words"][0, 0, 0, 1]) == 0
    # channel axis with token groups of 2: channel c has values {x0c, x1c}
    qc = O.quantize_tensor(x, 1, O.AXIS_CHANNEL, 2)
    assert qc["min"].shape == (1, 1, 1, 64)
    assert np.array_equal(qc["min"][0, 0, 0], np.minimum(x[0, 0, 0], x[0, 0, 1]))
    # the larger of the two tokens gets code 1 (when they differ)
    bigger0 = x[0, 0, 0] > x[0, 0, 1]
    assert np.array_equal(qc["codes"][0, 0, 0].astype(bool), bigger0)


# --------------------------------------------------------------------------- golden fixtures
def _golden_lines(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            yield [part.split() for part in line.split("|")]


def test_golden_packing_examples_worked_by_hand():
    n = 0
    for (N, M), codes, (word,) in _golden_lines("packing_appendix_examples.txt"):
        N, M, codes, word = int(N), int(M), [int(c) for c in codes], int(word)
        assert len(codes) == M // N
        assert int(O.pack(codes, N, M)[0]) == word
        assert [int(c) for c in O.unpack(np.array([word], dtype=np.uint64), N, M)[:len(codes)]] == codes
        n += 1
    assert n >= 10


def test_golden_quantize_examples_worked_by_hand():
    n = 0
    for (b,), values, codes in _golden_lines("quantize_equation_examples.txt"):
        x = np.array([float(v) for v in values], dtype=np.float64)
        got = O.discretize(x, x.min(), x.max(), int(b))
        assert [int(c) for c in np.asarray(got).ravel()] == [int(c) for c in codes], (b, values)
        n += 1
    assert n >= 6
