"""Synthetic approximation study (the ablations of Section 5.3 on generated caches, GPU only).

For a cache drawn by workloads.py it runs sparq_decode over a grid of (r, k) and the method switches
(fixed temperatures, no mean-value blend, local window) and reports, against dense_decode on the same cache:
  - top-k correspondence: the share of SparQ's k positions that are among the k positions of largest exact
    score (the exact set comes from the same kernel run with r = d_h, where the approximate scores are exact);
  - the relative L2 error of the output, ||y - y_dense|| / ||y_dense||, averaged over heads.
There are no model weights here: the numbers describe the generators, not a language model.

    python -m paper_2312_04985_amd.approx_study [--S 4096] [--q-scale 0.05]
"""
import argparse

import torch

from . import binding as B
from . import workloads as W
from .cache import DecodeCache


def run(S: int, q_scale: float, seed: int):
    w = W.Workload("study", 4, 8, 8, 128, S, 32, 512, "f16", planted=(8, 8), seed=seed)
    dev = torch.device("cuda:0")
    seq = W.draw_seq_lens(w)
    K_src, V_src = W.draw_kv(w, dev, n_rows=S, v_offset=True)
    c = DecodeCache(w.B, w.H, w.H_kv, W.round_up(S, 64), w.d_h, w.r, w.k, w.torch_dtype, device=dev)
    c.append(K_src, V_src, seq.to(dev))
    q = W.draw_queries(w, K_src, seq, n=1, q_scale=q_scale)[0]
    y_dense = c.dense(q).float()

    def measure(r, k, flags=0, window=0):
        c.with_params(r, k, flags, window)
        y, alpha, idx, _ = c.decode(q, aux=True, idx_stride=k)
        c.with_params(w.d_h, k, 0, 0)                       # exact scores: the k largest of s
        _, _, exact, _ = c.decode(q, aux=True, idx_stride=k)
        hit = 0
        for b in range(w.B):
            for h in range(w.H):
                hit += len(set(idx[b, h].tolist()) & set(exact[b, h].tolist()))
        err = ((y.float() - y_dense).norm(dim=-1) / y_dense.norm(dim=-1)).mean().item()
        return hit / (w.B * w.H * k), err, alpha.mean().item()

    print(f"S = {S}, d_h = 128, 4 x 8 heads, q_scale = {q_scale} (mean alpha tells how peaked the scores are)")
    print("| r | k | top-k correspondence | rel. error | mean alpha |")
    print("|---|---|---|---|---|")
    for r in (8, 16, 32, 64, 128):
        for k in (64, 256, 512):
            corr, err, al = measure(r, k)
            print(f"| {r} | {k} | {corr:.3f} | {err:.4f} | {al:.3f} |")
    print()
    print("| r = 32, k = 256, variant | top-k correspondence | rel. error | mean alpha |")
    print("|---|---|---|---|")
    for name, flags, window in (("Eq. (9) temperature", 0, 0), ("tau = sqrt(d_h)", B.SPARQ_FLAG_TAU_SQRT_DH, 0),
                                ("tau = sqrt(r)", B.SPARQ_FLAG_TAU_SQRT_R, 0), ("no mean-value blend", B.SPARQ_FLAG_NO_REALLOC, 0),
                                ("local window 64", 0, 64)):
        corr, err, al = measure(32, 256, flags, window)
        print(f"| {name} | {corr:.3f} | {err:.4f} | {al:.3f} |")
    torch.cuda.synchronize()
    assert c.error_flags() == 0


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--S", type=int, default=4096)
    ap.add_argument("--q-scale", type=float, default=0.05)
    ap.add_argument("--seed", type=int, default=11)
    a = ap.parse_args()
    run(a.S, a.q_scale, a.seed)
