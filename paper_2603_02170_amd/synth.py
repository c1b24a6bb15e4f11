"""Seeded synthetic attention inputs shaped like the paper's workloads.

Holds no arithmetic of the method: only random tensors and the upstream model
transforms that produce them (QK-norm is a model-side RMS normalisation in the
paper's Sec. 4, applied here with a unit gain and epsilon 1e-6 as in its
Sec. 5.1 setup).  Both the GPU tests / benchmark and the CPU oracle tests draw
their inputs from here so that they see identical bf16 values.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

BASE_SEED = 20260302


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    H: int
    N: int
    d: int
    causal: bool
    qk_norm: bool = True
    k_smooth: bool = True
    q_smooth: bool = False
    do_std: float = 1.0
    outliers: bool = False


WORKLOADS = {
    # Tiny causal case the CPU oracle finishes in well under a second.
    "tiny": Workload("tiny", 0, 1, 2, 128, 64, True),
    # Pre-training shape (context 2048, head dim 128), K-smoothing on, Q-smoothing off.
    "pretrain": Workload("pretrain", 1, 4, 16, 2048, 128, True),
    # Outlier stress: per-channel K bias, a few amplified Q channels, no QK-norm.
    "outlier": Workload("outlier", 2, 2, 16, 4096, 128, True, qk_norm=False, outliers=True),
    # Headline: the shape the throughput metric is quoted on.
    "headline": Workload("headline", 3, 2, 32, 8192, 128, True),
    # Long context, non-causal, small-magnitude upstream gradient (variance 1e-2).
    "long": Workload("long", 4, 1, 32, 32768, 128, False, do_std=0.1),
    # The headline shape with Q-smoothing on (the paper's Sec. 5.4 ablation), and at the paper's
    # other benchmarked head dimension (Sec. 5.5).
    "headline_qsmooth": Workload("headline_qsmooth", 5, 2, 32, 8192, 128, True, q_smooth=True),
    "headline_d64": Workload("headline_d64", 6, 2, 32, 8192, 64, True),
    # One token short of the headline length: the last block is partial.
    "headline_n8191": Workload("headline_n8191", 8, 2, 32, 8191, 128, True),
}


def _rms_norm(x: torch.Tensor, eps: float = 1e-6) -> torch.Tensor:
    return x / torch.sqrt((x * x).mean(dim=-1, keepdim=True) + eps)


def make_inputs(w: Workload, heads=None):
    """Return bf16 CPU tensors (Q, K, V, dO), each [B, H, N, d].

    `heads`: optional list of flat (b*H + h) indices; when given only those
    heads are kept (result [len(heads), 1, N, d]) -- the values are the same as
    in the full tensors because generation is per head.
    """
    flat = list(range(w.B * w.H)) if heads is None else list(heads)
    outs = [[], [], [], []]
    # outlier recipe: per batch element, 1% of the H*d (head, channel) pairs of Q are x20
    amp = {}
    if w.outliers:
        for b in range(w.B):
            g = torch.Generator().manual_seed(BASE_SEED + 7919 * (w.index + 1) + b)
            perm = torch.randperm(w.H * w.d, generator=g)[: max(1, round(0.01 * w.H * w.d))]
            mask = torch.zeros(w.H * w.d, dtype=torch.bool)
            mask[perm] = True
            amp[b] = mask.view(w.H, w.d)
    for f in flat:
        b, h = divmod(f, w.H)
        g = torch.Generator().manual_seed(BASE_SEED + 1000003 * (w.index + 1) + f)
        q = torch.randn(w.N, w.d, generator=g, dtype=torch.float32)
        k = torch.randn(w.N, w.d, generator=g, dtype=torch.float32)
        v = torch.randn(w.N, w.d, generator=g, dtype=torch.float32)
        do = torch.randn(w.N, w.d, generator=g, dtype=torch.float32) * w.do_std
        if w.outliers:
            kbias = torch.randn(w.d, generator=g, dtype=torch.float32) * 5.0
            k = k + kbias[None, :]
            q = torch.where(amp[b][h][None, :], q * 20.0, q)
        if w.qk_norm:
            q = _rms_norm(q)
            k = _rms_norm(k)
        for lst, t in zip(outs, (q, k, v, do)):
            lst.append(t.to(torch.bfloat16))
    if heads is None:
        return tuple(torch.stack(l).view(w.B, w.H, w.N, w.d) for l in outs)
    return tuple(torch.stack(l).view(len(flat), 1, w.N, w.d) for l in outs)


def gaussian_inputs(N, d, sigma_qk=1.0, seed=0, heads=1):
    """Gaussian Q, K with a controlled standard deviation and unit-variance V, dO
    (the synthetic recipe of the paper's QK-standard-deviation study)."""
    g = torch.Generator().manual_seed(BASE_SEED + 31 * seed + 17)
    q = torch.randn(1, heads, N, d, generator=g) * sigma_qk
    k = torch.randn(1, heads, N, d, generator=g) * sigma_qk
    v = torch.randn(1, heads, N, d, generator=g)
    do = torch.randn(1, heads, N, d, generator=g)
    return tuple(t.to(torch.bfloat16) for t in (q, k, v, do))
