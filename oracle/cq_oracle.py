"""CPU oracle for CalibQuant's hot path (arxiv 2502.14882): TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the path computes, written from the
paper and independent of the HIP kernels (it shares no code, tables or helpers
with them and never imports them).  Only tests, the smoke check and the
benchmark's `cpu_baseline` leg may call it; the product path never does.

What each function follows
  pack / unpack                Appendix "Details for Low-bit Quantization with Packing"
  group_min_max                Sec. 3.1, the channel-wise alpha/beta definition,
                               restricted to a group (see reading R2 below)
  discretize / dequantize      Sec. 2.2, the quantize and dequantize equations
  quantize_tensor              the two above + the stored "scale factor and bias term"
                               of Sec. 3.1 (post-scale paragraph)
  logits_dequant               Sec. 2.1 attention logits on the dequantized keys (Sec. 3.2)
  logits_postscale             Sec. 3.1 post-scaling rearrangement of the same number
  calibrate                    Sec. 3.2, the linear map g
  decode_attn                  Sec. 2.1 softmax(.)V with Sec. 3.2's g on the visual
                               logits and the 16-bit text tail of Sec. 3 / Sec. 3.3
  softmax_mse / tau_grid_mse   Sec. 3.2, the grid search over tau1, tau2, scored by the
                               error measure of the section's second figure (reading R7)

Readings taken where the paper is silent (every one is repeated in the design notes)
  R1  Rounding operator of the quantize equation: exact real arithmetic, ties to even.
      All inputs are fp16, so x-alpha, beta-alpha and their small multiples are exact
      in fp64 and numpy's rint of the fp64 quotient equals the exact rule.
  R2  Statistics are taken per group: keys over `group` consecutive tokens of one
      channel (group = n reproduces the paper's whole-sequence alpha/beta), per-token
      tensors over `group` consecutive channels of one token.
  R3  Stored parameters: min = alpha as fp16 (a zero is stored as +0), scale =
      float32((beta-alpha)/(2^b-1)) with one rounding.  Dequantization uses the
      stored parameters.  A constant group (beta == alpha) gives codes 0, scale 0.
  R4  Container: M = 32 bits, packed along the head dimension, element i of a word
      at bits [32-b(1+i), 32-b i) as in the appendix formula.
  R5  gamma, delta of the calibration are the min and max of the *visual* logits of
      one query row (after the 1/sqrt(d) scaling); text logits are neither included
      nor transformed; the softmax is joint.  delta == gamma gives slope 1.
  R6  Query head hq reads KV head hq // (Hq / Hkv).
  R7  The paper searches tau1, tau2 on a grid but does not print the criterion; the
      section's figure scores calibration by the mean squared error of the attention
      weights against those of the exact keys, so the search takes that: per query row
      the mean over all attended tokens (visual and text, joint softmax on both sides)
      of the squared difference of the weights, averaged over the rows.

parity unpinned: the values of tau1, tau2 (the paper searches {0,1,2,3}^2 but does
not print the winners), the per-token value axis, the group sizes and the fp32
scale are this build's choices, not facts of the paper; no test can pin them.
"""
from __future__ import annotations

import numpy as np

AXIS_CHANNEL = 0   # statistics over a group of tokens, one (alpha, beta) per channel
AXIS_TOKEN = 1     # statistics over a group of channels, one (alpha, beta) per token

CALIB_NONE = 0
CALIB_DYNAMIC = 1
CALIB_FIXED = 2

WORD_BITS = 32


# ----------------------------------------------------------------------------- packing
def pack(v, N: int, M: int = WORD_BITS) -> np.ndarray:
    """pack(v, N, M) of the appendix along the last axis.

    v[..., n] holds N-bit codes; every M/N consecutive codes form one M-bit word,
    code i of a word shifted left by M - N(1+i); the shifted codes are summed.
    """
    v = np.asarray(v)
    per = M // N
    assert M % N == 0 and v.shape[-1] % per == 0
    g = v.reshape(v.shape[:-1] + (v.shape[-1] // per, per)).astype(np.uint64)
    shifts = np.array([M - N * (1 + i) for i in range(per)], dtype=np.uint64)
    words = (g << shifts).sum(axis=-1)
    return words.astype(np.uint32 if M == 32 else np.uint64)


def unpack(u, N: int, M: int = WORD_BITS) -> np.ndarray:
    """unpack(u, N, M) of the appendix: element i = (u >> (M - N(1+i))) mod 2^N."""
    u = np.asarray(u).astype(np.uint64)
    per = M // N
    shifts = np.array([M - N * (1 + i) for i in range(per)], dtype=np.uint64)
    codes = (u[..., None] >> shifts) & np.uint64((1 << N) - 1)
    return codes.reshape(u.shape[:-1] + (u.shape[-1] * per,)).astype(np.uint8)


# ----------------------------------------------------------------------------- quantizer
def _grouped(x: np.ndarray, axis: int, group: int) -> np.ndarray:
    """View x [..., n, d] so that the statistics axis is the last one.

    AXIS_CHANNEL -> [..., n/group, d, group]; AXIS_TOKEN -> [..., n, d/group, group].
    """
    n, d = x.shape[-2], x.shape[-1]
    lead = x.shape[:-2]
    if axis == AXIS_CHANNEL:
        assert n % group == 0
        return np.swapaxes(x.reshape(lead + (n // group, group, d)), -1, -2)
    assert d % group == 0
    return x.reshape(lead + (n, d // group, group))


def _ungrouped(xg: np.ndarray, axis: int, n: int, d: int) -> np.ndarray:
    lead = xg.shape[:-3]
    if axis == AXIS_CHANNEL:
        return np.swapaxes(xg, -1, -2).reshape(lead + (n, d))
    return xg.reshape(lead + (n, d))


def group_min_max(x, axis: int, group: int):
    """alpha = min, beta = max over each group (Sec. 3.1, reading R2), in fp64."""
    xg = _grouped(np.asarray(x, dtype=np.float64), axis, group)
    alpha = xg.min(axis=-1) + 0.0     # "+ 0.0" turns a negative zero into +0 (R3)
    beta = xg.max(axis=-1) + 0.0
    return alpha, beta


def discretize(x, alpha, beta, bits: int) -> np.ndarray:
    """x_dis = round((x - alpha) (2^b - 1) / (beta - alpha)), ties to even (R1)."""
    L = float((1 << bits) - 1)
    x = np.asarray(x, dtype=np.float64)
    D = np.asarray(beta, dtype=np.float64) - np.asarray(alpha, dtype=np.float64)
    safe = np.where(D > 0.0, D, 1.0)
    code = np.rint((x - alpha) * L / safe)
    return np.where(D > 0.0, code, 0.0).astype(np.uint8)


def dequantize(codes, scale, minv, axis: int, group: int) -> np.ndarray:
    """x_deq = x_dis * scale + min with the stored parameters, fp64."""
    codes = np.asarray(codes)
    n, d = codes.shape[-2], codes.shape[-1]
    cg = _grouped(codes.astype(np.float64), axis, group)
    s = np.asarray(scale, dtype=np.float64)[..., None]
    m = np.asarray(minv, dtype=np.float64)[..., None]
    return _ungrouped(cg * s + m, axis, n, d)


def quantize_tensor(x, bits: int, axis: int, group: int) -> dict:
    """Quantize one cache tensor x [..., n, d] (fp16 values).

    Returns codes (uint8, unpacked), words (uint32, packed along d), scale (float32)
    and min (float16); meta shape is [..., n/group, d] (AXIS_CHANNEL) or
    [..., n, d/group] (AXIS_TOKEN).
    """
    x = np.asarray(x)
    n, d = x.shape[-2], x.shape[-1]
    L = (1 << bits) - 1
    alpha, beta = group_min_max(x, axis, group)
    xg = _grouped(x.astype(np.float64), axis, group)
    cg = discretize(xg, alpha[..., None], beta[..., None], bits)
    codes = _ungrouped(cg, axis, n, d)
    scale = ((beta - alpha) / float(L)).astype(np.float32)
    minv = alpha.astype(np.float16)
    return {"codes": codes, "words": pack(codes, bits, WORD_BITS), "scale": scale,
            "min": minv, "bits": bits, "axis": axis, "group": group}


# ----------------------------------------------------------------------------- logits
def logits_dequant(q, k_deq, softmax_scale: float) -> np.ndarray:
    """q k_deq^T * softmax_scale for one head: q [d], k_deq [n, d] -> [n]."""
    return (np.asarray(k_deq, np.float64) @ np.asarray(q, np.float64)) * softmax_scale


def logits_postscale(q, codes, scale, minv, group: int, softmax_scale: float) -> np.ndarray:
    """The same logits by Sec. 3.1's rearrangement, channel-wise keys:
    (q * scale_t) . k_dis + q . alpha_t for the token's group t."""
    q = np.asarray(q, np.float64)
    codes = np.asarray(codes, np.float64)
    n = codes.shape[0]
    out = np.empty(n, dtype=np.float64)
    for j in range(n):
        t = j // group
        qs = q * np.asarray(scale[t], np.float64)
        out[j] = (qs @ codes[j] + q @ np.asarray(minv[t], np.float64)) * softmax_scale
    return out


def calibrate(s, tau1: float, tau2: float, mode: int = CALIB_DYNAMIC,
              gamma: float = 0.0, delta: float = 0.0) -> np.ndarray:
    """g(x) = (delta-gamma+tau1-tau2)/(delta-gamma) (x-gamma) + gamma - tau1  (Sec. 3.2)."""
    s = np.asarray(s, np.float64)
    if mode == CALIB_NONE or s.size == 0:
        return s.copy()
    if mode == CALIB_DYNAMIC:
        gamma, delta = float(s.min()), float(s.max())
    width = float(delta) - float(gamma)
    slope = 1.0 if width == 0.0 else (width + tau1 - tau2) / width
    return slope * (s - gamma) + gamma - tau1


# ----------------------------------------------------------------------------- attention
def decode_attn(q, kq: dict, vq: dict, k_text=None, v_text=None, n_text: int = 0,
                calib_mode: int = CALIB_DYNAMIC, tau1: float = 0.0, tau2: float = 0.0,
                gamma: float = 0.0, delta: float = 0.0, softmax_scale: float = 0.0,
                return_parts: bool = False):
    """One decode step over a quantized visual cache plus a 16-bit text tail.

    q [B, Hq, d]; kq / vq as returned by quantize_tensor for [B, Hkv, n_vis, d];
    k_text / v_text [B, Hkv, >= n_text, d].  Returns out [B, Hq, d] in fp64.
    """
    q = np.asarray(q, np.float64)
    B, Hq, d = q.shape
    k_deq = dequantize(kq["codes"], kq["scale"], kq["min"], kq["axis"], kq["group"])
    v_deq = dequantize(vq["codes"], vq["scale"], vq["min"], vq["axis"], vq["group"])
    Hkv = k_deq.shape[1]
    g = Hq // Hkv
    if softmax_scale == 0.0:
        softmax_scale = 1.0 / np.sqrt(float(d))
    out = np.zeros((B, Hq, d), dtype=np.float64)
    parts = []
    for b in range(B):
        for hq in range(Hq):
            h = hq // g
            s_vis = logits_dequant(q[b, hq], k_deq[b, h], softmax_scale)
            s_vis = calibrate(s_vis, tau1, tau2, calib_mode, gamma, delta)
            if n_text > 0:
                kt = np.asarray(k_text[b, h, :n_text], np.float64)
                vt = np.asarray(v_text[b, h, :n_text], np.float64)
                s_txt = (kt @ q[b, hq]) * softmax_scale
            else:
                vt = np.zeros((0, d))
                s_txt = np.zeros((0,))
            s = np.concatenate([s_vis, s_txt])
            if s.size == 0:
                continue
            e = np.exp(s - s.max())
            w = e / e.sum()
            out[b, hq] = w[: s_vis.size] @ v_deq[b, h] + w[s_vis.size:] @ vt
            if return_parts:
                parts.append((s_vis, s_txt, w))
    return (out, parts) if return_parts else out


# ----------------------------------------------------------------------------- tau search
def _softmax(s):
    s = np.asarray(s, np.float64)
    e = np.exp(s - s.max())
    return e / e.sum()


def softmax_mse(s_exact, s_quant, s_text, tau1: float, tau2: float) -> float:
    """Mean squared difference between the attention weights of one query row with the
    calibrated quantized visual logits, softmax([g(s_quant), s_text]), and those with the
    exact visual logits, softmax([s_exact, s_text])  (Sec. 3.2; gamma, delta as in R5)."""
    s_text = np.asarray(s_text, np.float64)
    p_ref = _softmax(np.concatenate([np.asarray(s_exact, np.float64), s_text]))
    p_cal = _softmax(np.concatenate([calibrate(s_quant, tau1, tau2, CALIB_DYNAMIC), s_text]))
    return float(np.mean((p_cal - p_ref) ** 2))


def tau_grid_mse(q, k_exact, kq: dict, k_text=None, n_text: int = 0, tau1_grid=(0, 1, 2, 3),
                 tau2_grid=(0, 1, 2, 3), softmax_scale: float = 0.0) -> np.ndarray:
    """The grid search of Sec. 3.2: for every (tau1, tau2) of the grid, softmax_mse averaged
    over all (batch, query head) rows.  q [B, Hq, d]; k_exact [B, Hkv, n_vis, d] the 16-bit
    keys that kq quantizes; k_text [B, Hkv, >= n_text, d].  Returns [len(tau1_grid),
    len(tau2_grid)] in fp64; the search result is its argmin."""
    q = np.asarray(q, np.float64)
    B, Hq, d = q.shape
    k_deq = dequantize(kq["codes"], kq["scale"], kq["min"], kq["axis"], kq["group"])
    Hkv = k_deq.shape[1]
    g = Hq // Hkv
    if softmax_scale == 0.0:
        softmax_scale = 1.0 / np.sqrt(float(d))
    out = np.zeros((len(tau1_grid), len(tau2_grid)), dtype=np.float64)
    for b in range(B):
        for hq in range(Hq):
            h = hq // g
            s_exact = logits_dequant(q[b, hq], np.asarray(k_exact[b, h], np.float64), softmax_scale)
            s_quant = logits_dequant(q[b, hq], k_deq[b, h], softmax_scale)
            if n_text > 0:
                s_text = (np.asarray(k_text[b, h, :n_text], np.float64) @ q[b, hq]) * softmax_scale
            else:
                s_text = np.zeros((0,))
            for i, t1 in enumerate(tau1_grid):
                for j, t2 in enumerate(tau2_grid):
                    out[i, j] += softmax_mse(s_exact, s_quant, s_text, float(t1), float(t2))
    return out / float(B * Hq)


def rel_l2(a, b) -> float:
    """|| a - b ||_2 / || b ||_2 over the whole tensor (the parity metric for floats)."""
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (den if den > 0 else 1.0)
