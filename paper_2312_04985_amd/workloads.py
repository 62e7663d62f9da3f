"""Seeded synthetic inputs for the SparQ decode step.

This module only draws inputs.  It holds none of the method's arithmetic and is the one
piece of code that both the HIP path's callers and the CPU oracle's callers use, so that
both sides see bit-identical 16-bit tensors.

Recipe (stands in for the model-shaped caches of the paper's evaluation, whose real
activations are not available): keys are N(0,1) scaled per channel by exp(N(0,1)) so a few
channels dominate (the heavy-tailed query components of Section 3 then appear in q), values
are N(0,1) (optionally shifted per channel so the mean value vector is O(1)), and each query
is the sum of a few "planted" cached key rows plus N(0, 0.5^2) noise, so a few positions
carry most of the attention mass (the score sparsity of Section 3).  The plain N(0,1)
keys/values/queries of the paper's microbenchmark (Appendix F) are the `gaussian` recipe.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    H_kv: int
    d_h: int
    S: int                         # sequence length (upper bound when ragged)
    r: int
    k: int                         # fixed k; ignored when k_div is set
    dtype: str                     # "f16" | "bf16"
    planted: Tuple[int, int] = (8, 8)        # planted key rows per query head, uniform in [lo, hi]
    ragged: Optional[Tuple[int, int]] = None  # per-sequence S drawn uniform in [lo, hi]
    k_div: Optional[int] = None    # k_b = ceil(S_b / k_div)
    recipe: str = "planted"        # "planted" | "gaussian"
    seed: int = 0

    @property
    def g(self) -> int:
        return self.H // self.H_kv

    @property
    def torch_dtype(self):
        return torch.float16 if self.dtype == "f16" else torch.bfloat16

    @property
    def dtype_code(self) -> int:
        return 0 if self.dtype == "f16" else 1


# The five workloads the benchmark contract names, the paper's own microbenchmark shape
# (Table 2: batch 64, 32 heads, d_h = 128, S = 4096, r = 32, k = 128, N(0,1) tensors), and one long-cache shape.
CONFIGS = {
    "c1_single_head": Workload("c1_single_head", 1, 1, 1, 128, 1024, 16, 128, "f16", planted=(4, 4), seed=1),
    "c2_llama2_7b": Workload("c2_llama2_7b", 16, 32, 32, 128, 4096, 32, 512, "f16", planted=(8, 8), seed=2),
    "c3_llama3_8b_gqa": Workload("c3_llama3_8b_gqa", 1, 32, 8, 128, 32768, 32, 2048, "bf16", planted=(8, 8), seed=3),
    "c4_large_batch": Workload("c4_large_batch", 64, 32, 32, 128, 8192, 16, 256, "f16", planted=(8, 8), seed=4),
    "c5_gemma_7b_ragged": Workload("c5_gemma_7b_ragged", 32, 16, 16, 256, 16384, 64, 2048, "bf16",
                                   planted=(1, 16), ragged=(1024, 16384), k_div=8, seed=5),
    "paper_table2": Workload("paper_table2", 64, 32, 32, 128, 4096, 32, 128, "f16", recipe="gaussian", seed=6),
    # beyond the contract: many heads with caches longer than one workgroup's LDS holds (the two-level selection
    # plan, whose launches give Step 1 and Step 2 separately to the profiler's counters)
    "long_many_heads": Workload("long_many_heads", 16, 32, 32, 128, 40960, 32, 1024, "bf16", planted=(8, 8), seed=7),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    return replace(w, **kw)


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def draw_seq_lens(w: Workload) -> torch.Tensor:
    """Per-sequence lengths (CPU int32): uniform S, or drawn uniform in w.ragged."""
    if w.ragged is None:
        return torch.full((w.B,), w.S, dtype=torch.int32)
    lo, hi = w.ragged
    g = _gen(w.seed * 1000 + 7, "cpu")
    return torch.randint(lo, hi + 1, (w.B,), generator=g, dtype=torch.int32)


def k_per_seq(w: Workload, seq_lens: torch.Tensor) -> Optional[torch.Tensor]:
    """k_b = ceil(S_b / k_div) when the workload asks for a per-sequence k, else None."""
    if w.k_div is None:
        return None
    return ((seq_lens.to(torch.int64) + w.k_div - 1) // w.k_div).to(torch.int32)


def draw_kv(w: Workload, device, *, n_rows: Optional[int] = None, v_offset: bool = False,
            dup_rows: int = 0):
    """Key and value rows to be appended: K_src, V_src of shape [B, H_kv, n_rows, d_h] in the
    cache dtype.  `v_offset` adds a per-channel N(0,1) shift to the values; `dup_rows` copies
    that many random key rows over other random rows of the same head (forces exact score ties)."""
    n_rows = w.S if n_rows is None else n_rows
    dt = w.torch_dtype
    K = torch.empty((w.B, w.H_kv, n_rows, w.d_h), dtype=dt, device=device)
    V = torch.empty_like(K)
    for b in range(w.B):                       # per sequence: bounds the fp32 temporaries
        g = _gen(w.seed * 100003 + b, device)
        kn = torch.randn((w.H_kv, n_rows, w.d_h), generator=g, device=device, dtype=torch.float32)
        if w.recipe == "planted":
            scale = torch.exp(torch.randn((w.H_kv, 1, w.d_h), generator=g, device=device, dtype=torch.float32))
            kn = kn * scale
        K[b] = kn.to(dt)
        vn = torch.randn((w.H_kv, n_rows, w.d_h), generator=g, device=device, dtype=torch.float32)
        if v_offset:
            vn = vn + torch.randn((w.H_kv, 1, w.d_h), generator=g, device=device, dtype=torch.float32)
        V[b] = vn.to(dt)
        if dup_rows:
            gc = _gen(w.seed * 7919 + b, "cpu")
            for h in range(w.H_kv):
                src = torch.randint(0, n_rows, (dup_rows,), generator=gc)
                dst = torch.randint(0, n_rows, (dup_rows,), generator=gc)
                K[b, h, dst] = K[b, h, src]
    return K, V


def draw_queries(w: Workload, K_src: torch.Tensor, seq_lens: torch.Tensor, *, n: int = 1,
                 q_scale: float = 1.0, tie_channels: int = 0, stream: int = 0) -> torch.Tensor:
    """n query tensors [n, B, H, d_h] in the cache dtype.  Planted recipe: each query head is the
    sum of P distinct cached key rows of its KV head (P uniform in w.planted, rows uniform in
    [0, S_b)) plus N(0, 0.25) noise, times q_scale.  Gaussian recipe: N(0,1).  `tie_channels` > 0
    overwrites that many random channels of every query with +-(the magnitude of another
    channel), which puts equal magnitudes around the top-r boundary."""
    device = K_src.device
    dt = w.torch_dtype
    q = torch.empty((n, w.B, w.H, w.d_h), dtype=dt, device=device)
    gc = _gen(w.seed * 31337 + 11 + stream, "cpu")
    gd = _gen(w.seed * 31337 + 13 + stream, device)
    lo, hi = w.planted
    for i in range(n):
        noise = torch.randn((w.B, w.H, w.d_h), generator=gd, device=device, dtype=torch.float32)
        if w.recipe == "gaussian":
            acc = noise
        else:
            acc = 0.5 * noise
            for b in range(w.B):
                S_b = int(seq_lens[b])
                if S_b <= 0:
                    continue
                counts = torch.randint(lo, hi + 1, (w.H,), generator=gc)
                pmax = int(counts.max())
                # distinct rows per head (sampling without replacement); with fewer rows than
                # planted keys, rows may repeat
                if S_b >= pmax:
                    rows = torch.multinomial(torch.ones((w.H, S_b)), pmax, replacement=False, generator=gc)
                else:
                    rows = torch.randint(0, S_b, (w.H, pmax), generator=gc)
                keep = (torch.arange(pmax)[None, :] < counts[:, None]).to(torch.float32)
                kv_head = torch.arange(w.H) // w.g
                picked = K_src[b][kv_head.to(device)[:, None], rows.to(device)]       # [H, pmax, d_h]
                acc[b] += (picked.to(torch.float32) * keep.to(device)[:, :, None]).sum(dim=1)
        qi = (acc * q_scale).to(dt)
        if tie_channels:
            for _ in range(tie_channels):
                a = torch.randint(0, w.d_h, (w.B, w.H, 1), generator=gc).to(device)
                c = torch.randint(0, w.d_h, (w.B, w.H, 1), generator=gc).to(device)
                sign = (torch.randint(0, 2, (w.B, w.H, 1), generator=gc).to(device) * 2 - 1).to(dt)
                qi.scatter_(2, c, qi.gather(2, a).abs() * sign)
        q[i] = qi
    return q


def to_codes(t: torch.Tensor):
    """Raw 16-bit codes of an fp16/bf16 tensor as a numpy uint16 array on the host."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
