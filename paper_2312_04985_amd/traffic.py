"""Transfer model of the decode step: what the method must move, per head and per step.

Element counts follow the paper's two transfer equations (Section 3, Eq. 3 for dense
attention; Section 4 for SparQ); the byte figures used for the roofline split the SparQ
count into its stages.  Nothing here touches a GPU.
"""
from __future__ import annotations

from typing import Iterable, Optional


def dense_elements(S: int, d_h: int) -> int:
    """M_dense = 2 S d_h + 2 d_h : read K and V, write the new k and v (Section 3, Eq. 3)."""
    return 2 * S * d_h + 2 * d_h


def sparq_elements(S: int, d_h: int, r: int, k: int) -> int:
    """M_SparQ = S r + 2 k d_h + 4 d_h : r channel rows of K, k rows of K and V, write k and v,
    read and write the mean value vector (Section 4)."""
    return S * r + 2 * min(k, S) * d_h + 4 * d_h


def sparq_decode_bytes(seq_lens: Iterable[int], H: int, d_h: int, r: int, k: int, e: int = 2,
                       k_per_seq: Optional[Iterable[int]] = None, group_kv_heads: Optional[int] = None) -> dict:
    """Algorithmic HBM bytes of ONE sparq_decode launch, per stage, counted per query head:
    stage 1 reads r channel rows of S_b elements plus q; stage 3 reads k_b rows of K and of V;
    the blend reads the fp32 mean value vector and writes the output row.  Under the paper's grouped-query
    rule (group_kv_heads = H_kv) the channel rows and the selected rows are read once per KV head."""
    seq = list(seq_lens)
    ks = list(k_per_seq) if k_per_seq is not None else [k] * len(seq)
    Hr = H if group_kv_heads is None else group_kv_heads
    s1 = sum(Hr * r * S * e + H * d_h * e for S in seq)
    s3 = sum(Hr * (2 * min(kb, S) * d_h * e) for S, kb in zip(seq, ks))
    blend = len(seq) * H * (4 * d_h + d_h * e)
    return {"stage1": s1, "stage3": s3, "blend": blend, "total": s1 + s3 + blend}


def kv_append_bytes(B: int, H_kv: int, d_h: int, e: int = 2, n_new: int = 1) -> int:
    """Algorithmic bytes of one sparq_kv_append call: read k and v, write K, Kt and V rows,
    read-modify-write the fp32 mean value vector."""
    return B * H_kv * (n_new * (2 * d_h * e + 3 * d_h * e) + 8 * d_h)


def dense_decode_bytes(seq_lens: Iterable[int], H: int, H_kv: int, d_h: int, e: int = 2) -> int:
    """Algorithmic bytes of one dense_decode launch: every KV head's K and V rows are read once
    (shared by the query heads of its group), plus q in and the output row out."""
    seq = list(seq_lens)
    return sum(H_kv * 2 * S * d_h * e for S in seq) + len(seq) * H * 2 * d_h * e
