"""Pins of the oracle's tau grid search (Sec. 3.2): a closed form with a known winner, a library
softmax, shift invariance and a pure-Python brute force."""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from paper_2502_14882_amd import synth

GRID = (0.0, 1.0, 2.0, 3.0)


def _small(seed=5, B=2, Hq=4, Hkv=2, d=64, nv=96, nt=7, kind="uniform"):
    w = synth.Workload("t", seed, B, Hq, Hkv, d, nv, nt, kind)
    t = synth.make_inputs(w, "cpu")
    return w, {k: v.numpy() for k, v in t.items()}


@pytest.mark.parametrize("t1,t2", [(1.0, 2.0), (3.0, 0.0), (2.0, 2.0)])
def test_logits_distorted_by_the_inverse_map_are_repaired_exactly_by_their_taus(t1, t2):
    """g maps [gamma, delta] onto [gamma - tau1, delta - tau2].  Stretch exact logits so that
    their range becomes [min + tau1, max + tau2]: calibration with (tau1, tau2) restores them,
    the error is zero there and positive at every other grid point."""
    rng = np.random.default_rng(7)
    s_exact = rng.normal(0.0, 1.5, 200)
    s_text = rng.normal(0.0, 1.0, 9)
    lo, hi = s_exact.min(), s_exact.max()
    gamma, delta = lo + t1, hi + t2
    s_quant = (s_exact - lo) * (delta - gamma) / (hi - lo) + gamma
    errs = {(a, b): O.softmax_mse(s_exact, s_quant, s_text, a, b)
            for a, b in itertools.product(GRID, GRID)}
    assert errs[(t1, t2)] < 1e-30
    assert all(e > 1e-12 for tt, e in errs.items() if tt != (t1, t2))


def test_zero_taus_compare_two_plain_softmaxes_library():
    rng = np.random.default_rng(8)
    s_exact, s_quant, s_text = rng.normal(size=50), rng.normal(size=50) * 2.0, rng.normal(size=6)
    p_ref = torch.softmax(torch.from_numpy(np.concatenate([s_exact, s_text])), 0).numpy()
    p_q = torch.softmax(torch.from_numpy(np.concatenate([s_quant, s_text])), 0).numpy()
    want = float(((p_q - p_ref) ** 2).sum() / 56.0)
    assert O.softmax_mse(s_exact, s_quant, s_text, 0.0, 0.0) == pytest.approx(want, rel=1e-12)


def test_equal_taus_without_text_only_shift_the_logits():
    rng = np.random.default_rng(9)
    s_exact, s_quant = rng.normal(size=40), rng.normal(size=40) * 3.0
    none = np.zeros((0,))
    base = O.softmax_mse(s_exact, s_quant, none, 0.0, 0.0)
    assert O.softmax_mse(s_exact, s_quant, none, 2.0, 2.0) == pytest.approx(base, rel=1e-10)
    # with text the shift matters: the visual block loses weight against the text block
    s_text = rng.normal(size=5)
    assert O.softmax_mse(s_exact, s_quant, s_text, 2.0, 2.0) != pytest.approx(
        O.softmax_mse(s_exact, s_quant, s_text, 0.0, 0.0), rel=1e-3)


def test_grid_on_a_cache_brute_force_python_loops_tiny():
    """tau_grid_mse end to end (GQA head mapping, stored parameters, text tail, averaging) against
    plain Python arithmetic on a tiny cache."""
    w, x = _small(seed=12, B=1, Hq=2, Hkv=1, d=32, nv=8, nt=3, kind="none")
    kq = O.quantize_tensor(x["k"], 1, O.AXIS_CHANNEL, 4)
    grid1, grid2 = (0.0, 1.5), (0.5, 3.0)
    got = O.tau_grid_mse(x["q"], x["k"], kq, x["k_text"], 3, grid1, grid2)
    want = [[0.0, 0.0], [0.0, 0.0]]
    for hq in range(2):
        qv = [float(v) for v in x["q"][0, hq]]
        s_exact, s_quant, s_text = [], [], []
        for j in range(8):
            word = int(kq["words"][0, 0, j, 0])
            a = e = 0.0
            for c in range(32):
                bit = (word >> (31 - c)) & 1
                a += qv[c] * (float(kq["min"][0, 0, j // 4, c]) + bit * float(kq["scale"][0, 0, j // 4, c]))
                e += qv[c] * float(x["k"][0, 0, j, c])
            s_quant.append(a / math.sqrt(32.0))
            s_exact.append(e / math.sqrt(32.0))
        for t in range(3):
            s_text.append(sum(qv[c] * float(x["k_text"][0, 0, t, c]) for c in range(32)) / math.sqrt(32.0))

        def weights(vis):
            s = vis + s_text
            m = max(s)
            ex = [math.exp(v - m) for v in s]
            z = sum(ex)
            return [v / z for v in ex]

        p_ref = weights(s_exact)
        gam, dlt = min(s_quant), max(s_quant)
        for i, t1 in enumerate(grid1):
            for j, t2 in enumerate(grid2):
                slope = (dlt - gam + t1 - t2) / (dlt - gam)
                p = weights([slope * (v - gam) + gam - t1 for v in s_quant])
                want[i][j] += sum((a - b) ** 2 for a, b in zip(p, p_ref)) / 11.0 / 2.0
    assert got == pytest.approx(np.array(want), rel=1e-9, abs=1e-15)


def test_finer_codes_have_smaller_error_and_one_bit_gains_from_calibration():
    """On keys with outlier channels the 1-bit attention weights are far from the exact ones,
    8-bit ones are close (Sec. 3.2's motivation), and some grid point beats tau = (0, 0) at 1 bit
    (the section's claim for its calibration; the winner itself is data dependent)."""
    w, x = _small(seed=31, B=2, Hq=8, Hkv=2, d=128, nv=512, nt=16)
    err = {}
    for bits in (1, 2, 4, 8):
        kq = O.quantize_tensor(x["k"], bits, O.AXIS_CHANNEL, 128)
        err[bits] = O.tau_grid_mse(x["q"], x["k"], kq, x["k_text"], 16, GRID, GRID)
    assert err[8][0, 0] < err[4][0, 0] < err[2][0, 0] < err[1][0, 0]
    assert err[8][0, 0] < 1e-3 * err[1][0, 0]
    assert err[1].min() < err[1][0, 0]
