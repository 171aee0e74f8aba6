"""GPU parity of cq_tau_search against the oracle's grid search (Sec. 3.2): every grid entry
within 1e-4 relative (fp32 logits, fp64 weights), and the same winner."""
import numpy as np
import pytest
import torch

from oracle import cq_oracle as O
from paper_2502_14882_amd import binding as cq
from paper_2502_14882_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu

GRID = (0.0, 1.0, 2.0, 3.0)
REL_TOL = 1e-4     # logits are fp32 dot products of 128 terms (~1e-6 relative each); the weights and
                   # every sum are formed in fp64 on both sides


def _check(w, lay, n_text=None, grid1=GRID, grid2=GRID, softmax_scale=0.0):
    n_text = w.n_text if n_text is None else n_text
    x_cpu = synth.make_inputs(w, "cpu")
    kq = O.quantize_tensor(x_cpu["k"].numpy(), lay.bits, lay.k_axis, lay.k_group)
    want = O.tau_grid_mse(x_cpu["q"].numpy(), x_cpu["k"].numpy(), kq,
                          x_cpu["k_text"].numpy() if n_text > 0 else None, n_text, grid1, grid2,
                          softmax_scale)
    x = H.to_device(x_cpu)
    k_dev, _ = cq.cq_quantize_kv(lay, x["k"], x["v"])
    H.assert_qtensor_equal(k_dev, kq, "keys")
    kt = x["k_text"] if x["k_text"].shape[2] > 0 else None
    got = cq.cq_tau_search(lay, x["q"], x["k"], k_dev, kt, n_text, grid1, grid2, softmax_scale)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got.shape == want.shape and np.isfinite(got).all()
    rel = np.abs(got - want) / np.maximum(np.abs(want), 1e-300)
    assert rel.max() <= REL_TOL, "largest relative deviation %.3e\n%s\n%s" % (rel.max(), got, want)
    assert np.unravel_index(got.argmin(), got.shape) == np.unravel_index(want.argmin(), want.shape)
    return got


def test_config0_grid_of_the_paper():
    w = synth.WORKLOADS[0]
    _check(w, H.layout_of(w))


@pytest.mark.parametrize("idx", [1, 2, 4])
@pytest.mark.parametrize("bits", [1, 2])
def test_shrunk_configs(idx, bits):
    # several 512-token chunks and a ragged last one, GQA 4:1 and 6:1, outlier channels
    w = synth.WORKLOADS[idx].replace(batch=2, n_kv_heads=2, n_q_heads=2 * (6 if idx == 4 else 4),
                                     n_vis=1408, n_text=77)
    _check(w, H.layout_of(w, bits))


def test_other_layouts_and_grids():
    w = synth.WORKLOADS[1].replace(batch=1, n_kv_heads=2, n_q_heads=4, n_vis=384, n_text=5)
    _check(w, H.layout_of(w, 1, 384, 384, 0, 0))                     # whole-sequence statistics
    _check(w, H.layout_of(w, 4, 32, 128, 0, 1), grid1=(0.5,), grid2=(0.0, 0.25, 4.0))
    _check(w, H.layout_of(w, 2, 64, 128, 1, 0), n_text=0)            # token-wise keys, no text
    w = w.replace(head_dim=64, n_vis=192)
    _check(w, H.layout_of(w, 1, 64, 64), softmax_scale=0.2)


def test_grid_with_a_decreasing_map():
    """tau2 - tau1 larger than the logit range turns g's slope negative; the formula is applied
    literally on both sides."""
    w = synth.WORKLOADS[0]
    _check(w, H.layout_of(w), grid1=(0.0,), grid2=(0.0, 200.0))


def test_full_length_rows():
    """Rows of configs[2]'s length (8192 + 512 tokens) on a few heads."""
    w = synth.WORKLOADS[2].replace(batch=1, n_kv_heads=1, n_q_heads=4)
    _check(w, H.layout_of(w))
