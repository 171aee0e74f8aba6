"""Seeded synthetic inputs shaped like the visual/text KV caches the paper decodes over.

This module only draws random tensors.  It contains none of the method's
arithmetic (no min/max statistics, no rounding, no packing, no attention) and
imports neither the HIP binding nor the CPU oracle, so both sides of a parity
test can be fed from it.

The workloads stand in for InternVL-2.5 caches (Sec. 4.4 of the paper decodes
over n = 3328 and n = 8192 visual tokens): keys are standard normal with a few
large-magnitude "outlier" channels, which is the structure that motivates
channel-wise key statistics (Sec. 3.1); values, queries and the 16-bit text
tail are standard normal.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and distribution recipe of one decode-attention / quantizer workload."""

    name: str
    seed: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_vis: int          # quantized (visual) tokens
    n_text: int         # 16-bit (text) tokens
    k_outliers: str     # "fixed" | "uniform" | "student_t" | "none"
    v_outliers: bool = False   # values get the same outlier law as keys

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# Index = position in the benchmark's list of configurations.
WORKLOADS: Dict[int, Workload] = {
    0: Workload("tiny_decode", 1000, 1, 1, 1, 128, 1024, 32, "fixed"),
    1: Workload("internvl8b_layer", 1001, 16, 32, 8, 128, 3328, 128, "uniform"),
    2: Workload("video_layer", 1002, 64, 32, 8, 128, 8192, 512, "uniform"),
    3: Workload("quantizer_prefill", 1003, 128, 8, 8, 128, 16384, 0, "uniform", True),
    4: Workload("long_context_layer", 1004, 8, 48, 8, 128, 65536, 1024, "student_t"),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _outlier_plan(w: Workload, gen: torch.Generator, device):
    """Per KV head: which channels are outliers and by how much they are scaled.

    Returns (mask [Hkv, d] bool, factor [Hkv, d] float32).  The plan is a property
    of the head (of the model's weights), so it is shared by every batch item.
    """
    H, d = w.n_kv_heads, w.head_dim
    mask = torch.zeros(H, d, dtype=torch.bool, device=device)
    factor = torch.ones(H, d, dtype=torch.float32, device=device)
    kind = w.k_outliers
    if kind == "none":
        return mask, factor
    if kind == "fixed":
        for c in (5, 77):
            if c < d:
                mask[:, c] = True
                factor[:, c] = 8.0
        return mask, factor
    n_out = max(1, round((0.04 if kind == "uniform" else 0.03) * d))
    for h in range(H):
        perm = torch.randperm(d, generator=gen, device=device)[:n_out]
        mask[h, perm] = True
        if kind == "uniform":
            u = torch.rand(n_out, generator=gen, device=device)
            factor[h, perm] = 6.0 + 4.0 * u
    return mask, factor


def _student_t3(shape, gen, device):
    z = torch.randn(shape, generator=gen, device=device)
    c = torch.randn(shape + (3,), generator=gen, device=device)
    return z / torch.sqrt((c * c).sum(-1) / 3.0)


def _draw_cache(w: Workload, gen, device, mask, factor, with_outliers: bool):
    """One [B, Hkv, n_vis, d] fp16 tensor, drawn batch item by batch item."""
    B, H, N, d = w.batch, w.n_kv_heads, w.n_vis, w.head_dim
    out = torch.empty(B, H, N, d, dtype=torch.float16, device=device)
    for b in range(B):
        x = torch.randn(H, N, d, generator=gen, device=device)
        if with_outliers and w.k_outliers in ("fixed", "uniform"):
            x = x * factor[:, None, :]
        elif with_outliers and w.k_outliers == "student_t":
            t = 6.0 * _student_t3((H, N, d), gen, device)
            x = torch.where(mask[:, None, :], t, x)
            x = x.clamp_(-60000.0, 60000.0)
        out[b] = x.to(torch.float16)
    return out


def make_inputs(w: Workload, device="cpu", seed: Optional[int] = None,
                parts=("k", "v", "q", "k_text", "v_text")) -> Dict[str, torch.Tensor]:
    """Draw the tensors of one workload on `device` (fp16, contiguous).

    k, v        [B, Hkv, n_vis, d]   visual-token cache, to be quantized
    q           [B, Hq, d]           one decode query per sequence
    k_text/v_text [B, Hkv, n_text, d] text-token tail, kept in 16 bits
    The stream of random numbers depends on the device type, so a parity test
    draws once and hands the same tensors to both implementations.
    """
    device = torch.device(device)
    gen = _gen(w.seed if seed is None else seed, device)
    mask, factor = _outlier_plan(w, gen, device)
    res: Dict[str, torch.Tensor] = {}
    if "k" in parts:
        res["k"] = _draw_cache(w, gen, device, mask, factor, True)
    if "v" in parts:
        res["v"] = _draw_cache(w, gen, device, mask, factor, w.v_outliers)
    if "q" in parts:
        res["q"] = torch.randn(w.batch, w.n_q_heads, w.head_dim, generator=gen,
                               device=device).to(torch.float16)
    for name in ("k_text", "v_text"):
        if name in parts:
            res[name] = torch.randn(w.batch, w.n_kv_heads, max(w.n_text, 0), w.head_dim,
                                    generator=gen, device=device).to(torch.float16)
    return res
