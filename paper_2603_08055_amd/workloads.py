"""Seeded synthetic inputs shaped like the paper's multi-view workloads.

This module only draws random tensors.  It holds none of the attention method's
arithmetic, so both the tests' oracle side and the device side may be fed from
it.  The token counts follow Sec. 3.1 / Sec. 4 of the paper's setting: a
518x518 image at patch size 14 gives 37x37 = 1369 patch tokens per view, plus
1 camera and 4 register tokens for the VGGT-shaped cases (1374 per view); the
pi3-shaped case has patch tokens only (Sec. 3.4).  The paper's datasets are
not available; these tensors stand in for Q/K/V activations of such scenes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    views: int
    tokens_per_view: int
    heads: int
    head_dim: int
    dtype: str          # "f32" | "bf16"  (the I/O type of q, k, v, out)
    block: int          # tokens per pooling block
    topk: int           # key blocks selected per query block
    seed: int
    kind: str           # "normal" | "clustered" | "outliers"
    q_prescale: float = 1.0   # factor applied to the drawn Q (data property, not the softmax scale)

    @property
    def n_tok(self) -> int:
        return self.views * self.tokens_per_view

    @property
    def n_blk(self) -> int:
        return (self.n_tok + self.block - 1) // self.block

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five benchmark configurations (index i-1 here = "config i").
CONFIGS = (
    Workload("tiny_4x256_f32", 4, 256, 2, 64, "f32", 64, 4, 0, "normal", q_prescale=0.125),
    Workload("vggt_8x1374_bf16", 8, 1374, 16, 64, "bf16", 64, 16, 1, "normal"),
    Workload("vggt_100x1374_bf16_clustered", 100, 1374, 16, 64, "bf16", 64, 32, 2, "clustered"),
    Workload("vggt_1000x1374_bf16_clustered", 1000, 1374, 16, 64, "bf16", 64, 64, 3, "clustered"),
    Workload("pi3_300x1369_bf16_outliers", 300, 1369, 16, 64, "bf16", 128, 64, 4, "outliers"),
)


def config(i: int, **overrides) -> Workload:
    """Config i (1-based), optionally with fields replaced (e.g. topk=16, views=3)."""
    return replace(CONFIGS[i - 1], **overrides)


N_CENTROIDS = 8       # Gaussian centroids per (view, head) of the clustered generator
CLUSTER_SIGMA = 0.3   # noise around the unit-norm centroids
OUTLIER_FRACTION = 0.05
OUTLIER_GAIN = 4.0


def _randn(shape, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def make_inputs(wl: Workload, device="cpu", q_like_k: bool = True):
    """Draw (q, k, v), each [n_tok, heads, head_dim] in wl's dtype, on `device`.

    Values are drawn in float32 from a generator seeded with wl.seed (one view
    at a time, so memory stays bounded) and rounded once to the I/O dtype.

    kind "normal":    q, k, v ~ N(0, 1) i.i.d.
    kind "clustered": per (view, head) 8 centroids uniform on the unit sphere;
                      token p of a view belongs to centroid floor(8 p / tokens_per_view)
                      (contiguous runs); k = centroid + 0.3 N(0, I); q is drawn the same
                      way around the same centroids with its own noise (q_like_k) or
                      ~ N(0, 1); v ~ N(0, 1).
    kind "outliers":  N(0, 1) with a Bernoulli(5 %) subset of token positions (shared by
                      all heads and by q, k, v) multiplied by 4.
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed)
    T, H, D = wl.tokens_per_view, wl.heads, wl.head_dim
    dt = wl.torch_dtype
    q = torch.empty((wl.n_tok, H, D), dtype=dt, device=device)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    if wl.kind == "clustered":
        assign = (torch.arange(T, device=device) * N_CENTROIDS) // T       # [T] -> centroid id
    for vw in range(wl.views):
        sl = slice(vw * T, (vw + 1) * T)
        if wl.kind == "normal":
            qv, kv, vv = (_randn((T, H, D), gen, device) for _ in range(3))
        elif wl.kind == "clustered":
            cen = _randn((N_CENTROIDS, H, D), gen, device)
            cen = cen / cen.norm(dim=-1, keepdim=True)
            base = cen[assign]                                              # [T, H, D]
            kv = base + CLUSTER_SIGMA * _randn((T, H, D), gen, device)
            if q_like_k:
                qv = base + CLUSTER_SIGMA * _randn((T, H, D), gen, device)
            else:
                qv = _randn((T, H, D), gen, device)
            vv = _randn((T, H, D), gen, device)
        elif wl.kind == "outliers":
            qv, kv, vv = (_randn((T, H, D), gen, device) for _ in range(3))
            hot = torch.rand((T,), generator=gen, device=device) < OUTLIER_FRACTION
            gain = torch.where(hot, OUTLIER_GAIN, 1.0).to(torch.float32)[:, None, None]
            qv, kv, vv = qv * gain, kv * gain, vv * gain
        else:
            raise ValueError(f"unknown workload kind {wl.kind!r}")
        q[sl] = (qv * wl.q_prescale).to(dt)
        k[sl] = kv.to(dt)
        v[sl] = vv.to(dt)
    return q, k, v


def make_gate_logits(wl: Workload, device="cpu"):
    """N(0, 1) gate logits [n_tok, heads, head_dim] in wl's dtype (seed wl.seed + 1000)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed + 1000)
    g = torch.randn((wl.n_tok, wl.heads, wl.head_dim), generator=gen, device=device,
                    dtype=torch.float32)
    return g.to(wl.torch_dtype)


def vggt_forced_blocks(wl: Workload, view_stride: int = 100):
    """Block indices of the fixed global context of the VGGT variant (Sec. 3.3): every block that
    holds a token of the reference view (view 0) or of a view at a multiple of `view_stride`.
    Ascending, distinct, int32 numpy array."""
    import numpy as np
    blocks = []
    for view in range(0, wl.views, view_stride):
        first = view * wl.tokens_per_view // wl.block
        last = ((view + 1) * wl.tokens_per_view - 1) // wl.block
        blocks.extend(range(first, last + 1))
    return np.unique(np.asarray(blocks, dtype=np.int32))
