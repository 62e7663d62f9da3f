"""Host-side checks (no GPU): the paper's transfer model and the seeded input generators."""
import os

import numpy as np
import torch

from paper_2312_04985_amd import traffic as T
from paper_2312_04985_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_printed_theoretical_speedups():
    """M_dense / M_SparQ reproduces the two theoretical speed-ups printed in Section 6.1."""
    for line in open(os.path.join(GOLDEN, "transfer_speedups.txt")):
        if line.startswith("#") or not line.strip():
            continue
        S, d_h, r, k, printed, dec = line.split()
        S, d_h, r, k, dec = int(S), int(d_h), int(r), int(k), int(dec)
        ratio = T.dense_elements(S, d_h) / T.sparq_elements(S, d_h, r, k)
        assert abs(ratio - float(printed)) <= 10.0 ** (-dec), (ratio, printed)


def test_element_counts_term_by_term():
    # Section 3 Eq. (3) and the transfer equation of Section 4, on a shape small enough to count by hand
    assert T.dense_elements(10, 4) == 2 * 10 * 4 + 2 * 4
    assert T.sparq_elements(10, 4, 2, 3) == 10 * 2 + 2 * 3 * 4 + 4 * 4
    b = T.sparq_decode_bytes([4096] * 16, H=32, d_h=128, r=32, k=512)
    assert b["stage1"] == 16 * 32 * (32 * 4096 * 2 + 256) and b["stage3"] == 16 * 32 * 2 * 512 * 128 * 2
    assert abs(b["total"] / 1e6 - 269) < 1.0          # the ~269 MB per step of the Llama-2-7B-shaped config
    assert T.dense_decode_bytes([4096] * 16, 32, 32, 128) // 10**6 == 1074


def test_workloads_are_seeded_and_shaped():
    w = W.scaled(W.CONFIGS["c5_gemma_7b_ragged"], B=3, H=4, H_kv=2, S=96, ragged=(10, 96), d_h=32, r=8)
    seq = W.draw_seq_lens(w)
    assert seq.dtype == torch.int32 and int(seq.min()) >= 10 and int(seq.max()) <= 96
    assert torch.equal(seq, W.draw_seq_lens(w))
    kk = W.k_per_seq(w, seq)
    assert kk.tolist() == [-(-int(s) // 8) for s in seq]
    K, V = W.draw_kv(w, "cpu", v_offset=True, dup_rows=2)
    K2, V2 = W.draw_kv(w, "cpu", v_offset=True, dup_rows=2)
    assert K.shape == (3, 2, 96, 32) and K.dtype == torch.bfloat16
    assert torch.equal(K.view(torch.int16), K2.view(torch.int16)) and torch.equal(V.view(torch.int16), V2.view(torch.int16))
    q = W.draw_queries(w, K, seq, n=2, tie_channels=2)
    assert q.shape == (2, 3, 4, 32) and torch.isfinite(q.float()).all()
    assert torch.equal(q.view(torch.int16), W.draw_queries(w, K, seq, n=2, tie_channels=2).view(torch.int16))
    assert not torch.equal(q[0], q[1])
    assert W.to_codes(q).dtype == np.uint16
    # a few channels dominate the keys (lognormal channel scales)
    scale = K.float().abs().mean(dim=2)
    assert float(scale.max() / scale.median()) > 3.0


def test_named_configs_match_the_contract():
    c = W.CONFIGS
    assert (c["c2_llama2_7b"].B, c["c2_llama2_7b"].H, c["c2_llama2_7b"].S, c["c2_llama2_7b"].r, c["c2_llama2_7b"].k) == (16, 32, 4096, 32, 512)
    assert c["c3_llama3_8b_gqa"].g == 4 and c["c3_llama3_8b_gqa"].dtype == "bf16"
    assert c["c4_large_batch"].B == 64 and c["c4_large_batch"].S == 8192
    assert c["c5_gemma_7b_ragged"].d_h == 256 and c["c5_gemma_7b_ragged"].k_div == 8
