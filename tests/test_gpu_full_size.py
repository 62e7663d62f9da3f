"""GPU parity at the full sizes of the five named workloads, in the launch configuration the
benchmark uses.  The whole batch runs on the GPU; the oracle checks a seeded sample of
(sequence, KV head) units (all query heads of each), whose rows alone are copied to the host."""
import sys

import pytest
import torch

from paper_2312_04985_amd import binding as B
from paper_2312_04985_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu
C = W.CONFIGS


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("name,n_units,singles", [
    ("c1_single_head", 1, 2), ("c2_llama2_7b", 48, 2), ("c3_llama3_8b_gqa", 8, 1),
    ("c4_large_batch", 40, 1), ("c5_gemma_7b_ragged", 24, 1), ("paper_table2", 32, 1)])
def test_full_size_sampled(name, n_units, singles):
    w = C[name]
    say(f"[full-size] {name}: B={w.B} H={w.H}/{w.H_kv} d_h={w.d_h} S={w.S} r={w.r} k={w.k} {w.dtype} ragged={w.ragged}")
    b = Hn.build_cache(w, single_appends=singles, poison=None)
    say("   cache built:", tuple(b.cache.K.shape), "seq_lens", b.seq_lens[:8].tolist())
    q = W.draw_queries(w, b.K_src, b.seq_lens, n=1)[0]
    flags = B.SPARQ_FLAG_RAGGED_BATCH if w.ragged else 0           # as bench.py launches it
    stats = Hn.compare_sampled(b, q, n_units=n_units, seed=w.seed, flags=flags)
    say("   ", stats)
    del b
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,n_units", [("c2_llama2_7b", 48), ("c4_large_batch", 24), ("c5_gemma_7b_ragged", 16)])
def test_full_size_one_launch_step(name, n_units):
    """The launch the benchmark times: sparq_decode_step on the full batch, the new row landing at S_b - 1
    of every sequence; sampled units against the oracle on the grown cache, cache state included."""
    w = C[name]
    seq = W.draw_seq_lens(w)                       # lengths AFTER the step
    K_src, V_src = W.draw_kv(w, "cuda", n_rows=int(seq.max()))
    S_max = W.round_up(int(seq.max()), 64)
    from paper_2312_04985_amd.cache import DecodeCache
    flags = B.SPARQ_FLAG_RAGGED_BATCH if w.ragged else 0
    c = DecodeCache(w.B, w.H, w.H_kv, S_max, w.d_h, w.r, w.k, w.torch_dtype, flags=flags)
    c.append(K_src, V_src, (seq - 1).cuda())       # all but the last row of every sequence
    last = (seq - 1).to(torch.int64).cuda().view(w.B, 1, 1, 1).expand(w.B, w.H_kv, 1, w.d_h)
    k_new = K_src.gather(2, last).squeeze(2).contiguous(); v_new = V_src.gather(2, last).squeeze(2).contiguous()
    b = Hn.Built(w, c, K_src, V_src, seq, W.k_per_seq(w, seq))
    q = W.draw_queries(w, K_src, seq, n=1)[0]
    say(f"[full-size step] {name}: seq_lens {seq[:6].tolist()}")
    stats = Hn.compare_sampled(b, q, n_units=n_units, seed=w.seed + 1, flags=flags, with_dense=False,
                               step_rows=(k_new, v_new))
    say("   ", stats)
    del b, c
    torch.cuda.empty_cache()
