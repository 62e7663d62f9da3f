#!/usr/bin/env python3
"""Benchmark of the SparQ decode step on one MI355X.

A "step" is one pass of the whole hot path for one new token of every sequence in the batch:
sparq_kv_append (write k, v, the second key layout, update the mean value vector) followed by
sparq_decode (Steps 1-3 of Section 4 for all B x H heads).  Inputs are synthetic, seeded, shaped
like the named workload and resident in HBM before the timed region.  To keep the timed steps
out of the 256 MB last-level cache, the run rotates over several identical cache copies and a
pool of queries.

Prints ONE JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
CLOCK_WARMUP_STEPS = 300       # untimed steps before the W warm-up steps: the first ~10 ms after idle run at lower clocks


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_llama2_7b")
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = enough for > 1 GB touched)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


def traffic_from_profile(workload: str):
    """HBM bytes per sparq_decode launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
    read from the committed summary if there is one for this workload."""
    path = os.path.join(ROOT, "profiles", f"sparq_decode_{workload}_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(units shard over batch and KV heads with no exchange; see DESIGN.md)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU: libsparq has no CPU path", file=sys.stderr)
        sys.exit(1)
    from paper_2312_04985_amd import binding as B
    from paper_2312_04985_amd import traffic as T
    from paper_2312_04985_amd import workloads as W
    from paper_2312_04985_amd.cache import DecodeCache

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    w = W.CONFIGS[args.workload]
    K, Wm = args.steps, args.warmup
    seq0 = W.draw_seq_lens(w)                       # lengths seen by the first timed decode
    kps = W.k_per_seq(w, seq0)
    e = 2
    step_bytes0 = T.sparq_decode_bytes(seq0.tolist(), w.H, w.d_h, w.r, w.k, e, None if kps is None else kps.tolist())
    copies = args.copies or max(2, -(-(1 << 30) // step_bytes0["total"]))
    pre = max(0, CLOCK_WARMUP_STEPS - Wm)           # untimed extra steps so that the clocks have ramped up
    per_copy = -(-max(K, Wm, pre) // copies) + 1     # appends one copy receives in one pass
    S_max = W.round_up(int(seq0.max()) + per_copy, 64)

    # ---- build the caches through the library (bulk append of S_b - 1 rows) ----
    K_src, V_src = W.draw_kv(w, dev, n_rows=int(seq0.max()))
    caches = []
    for _ in range(copies):
        c = DecodeCache(w.B, w.H, w.H_kv, S_max, w.d_h, w.r, w.k, w.torch_dtype, device=dev,
                        flags=B.SPARQ_FLAG_RAGGED_BATCH if w.ragged else 0)
        c.append(K_src, V_src, (seq0 - 1).to(dev))
        caches.append(c)
    torch.cuda.synchronize()
    snap = [(c.v_mean.clone(), c.seq_lens.clone()) for c in caches]
    n_pool = 16
    q_pool = W.draw_queries(w, K_src, seq0, n=n_pool)
    kn_pool, vn_pool = W.draw_kv(W.scaled(w, seed=w.seed + 1000), dev, n_rows=n_pool)
    kn_pool = kn_pool.transpose(0, 2).transpose(1, 2).contiguous()     # [n_pool, B, H_kv, d_h]
    vn_pool = vn_pool.transpose(0, 2).transpose(1, 2).contiguous()
    kps_dev = None if kps is None else kps.to(dev)
    outs = [torch.empty((w.B, w.H, w.d_h), dtype=w.torch_dtype, device=dev) for _ in range(2)]

    lib = B.load()
    stream = torch.cuda.current_stream().cuda_stream
    vp = ctypes.c_void_p

    def ptr(t):
        return None if t is None else vp(t.data_ptr())

    # Every cache copy has two (v_mean, seq_lens) pairs: the one-launch step reads one pair and
    # writes the other, and the roles swap on the next visit of that copy.
    vm = [[c.v_mean, torch.empty_like(c.v_mean)] for c in caches]
    sl = [[c.seq_lens, torch.empty_like(c.seq_lens)] for c in caches]
    cs = [[B.make_cache(c.K, c.Kt, c.V, vm[i][p], sl[i][p]) for p in (0, 1)] for i, c in enumerate(caches)]
    par = [0] * copies

    # pre-marshalled argument tuples: the timed loops only call into the C ABI
    def args_for(ci, p, j, o):
        c = caches[ci]
        sh, cc, ws, wsb = ctypes.byref(c.shape), ctypes.byref(cs[ci][p]), ptr(c.workspace), c.workspace.numel()
        return {
            "step": (sh, cc, ptr(kn_pool[j]), ptr(vn_pool[j]), ptr(vm[ci][1 - p]), ptr(sl[ci][1 - p]), ptr(q_pool[j]),
                     ptr(kps_dev), ptr(outs[o]), None, None, 0, None, ws, wsb, stream),
            "append": (sh, cc, ptr(kn_pool[j]), ptr(vn_pool[j]), 1, None, ws, wsb, stream),
            "decode": (sh, cc, ptr(q_pool[j]), ptr(kps_dev), ptr(outs[o]), None, None, 0, None, ws, wsb, stream),
            "dense": (sh, cc, ptr(q_pool[j]), ptr(outs[o]), ws, wsb, stream),
        }
    table = [[[args_for(ci, p, j, (ci + j) % 2) for j in range(n_pool)] for p in (0, 1)] for ci in range(copies)]

    def restore():
        for ci, (v0, s0) in enumerate(snap):
            vm[ci][0].copy_(v0); sl[ci][0].copy_(s0); par[ci] = 0
        torch.cuda.synchronize()

    def check(rc):
        if rc:
            raise RuntimeError(f"libsparq call failed: {B.status_string(rc)}")

    def fused_step(i):            # the step: append + decode in one launch
        ci = i % copies
        check(lib.sparq_decode_step(*table[ci][par[ci]][i % n_pool]["step"]))
        par[ci] ^= 1

    def two_call_step(i):         # the same step as two launches (state updated in place)
        a = table[i % copies][par[i % copies]][i % n_pool]
        check(lib.sparq_kv_append(*a["append"]) or lib.sparq_decode(*a["decode"]))

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def timed_events(fn, n):      # HIP events on the stream the kernels are launched on
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # ---- warm-up, then the timed region: exactly K steps between two device syncs ----
    for i in range(pre):
        fused_step(i)
    restore()
    for i in range(Wm):
        fused_step(i)
    restore()
    ms_per_step = timed(fused_step, K)
    flags = sum(B.sparq_async_error(c.workspace) for c in caches)
    if flags:
        raise RuntimeError(f"device error word set during the timed region: {flags}")

    # ---- average launch duration of the dominant kernel (the one-launch step) over the same K steps,
    # HIP events on its stream; K back-to-back launches, launch gaps included ----
    restore()
    step_avg_ms = timed_events(fused_step, K)

    # for the record: the step as two launches, the decode launch alone, the append launch alone
    restore()
    two_call_ms = timed(two_call_step, K)
    restore()
    for ci in range(copies):
        check(lib.sparq_kv_append(*table[ci][0][0]["append"]))           # lengths S_b, as in the first timed step
    dec_avg_ms = timed_events(lambda i: check(lib.sparq_decode(*table[i % copies][0][i % n_pool]["decode"])), K)
    restore()
    append_ms = timed(lambda i: check(lib.sparq_kv_append(*table[i % copies][0][i % n_pool]["append"])), K)
    restore()

    # algorithmic bytes of the K timed launches: copy c is visited at steps c, c + copies, ... and holds
    # S_b + (visit number) rows when it is decoded
    tot = {"stage1": 0, "stage3": 0, "blend": 0, "total": 0}
    kk = None if kps is None else kps.tolist()
    for i in range(K):
        bts = T.sparq_decode_bytes((seq0 + (i // copies)).tolist(), w.H, w.d_h, w.r, w.k, e, kk)
        for key in tot:
            tot[key] += bts[key]
    dec_bytes = tot["total"] / K
    app_bytes = T.kv_append_bytes(w.B, w.H_kv, w.d_h, e)
    dec_bytes0 = T.sparq_decode_bytes(seq0.tolist(), w.H, w.d_h, w.r, w.k, e, kk)["total"]
    achieved = (dec_bytes + app_bytes) / (step_avg_ms * 1e-3) / 1e9

    # ---- in-library dense decode on the same rotation ----
    dense = {}
    if not args.no_dense:
        dense_fn = lambda i: check(lib.dense_decode(*table[i % copies][0][i % n_pool]["dense"]))
        for i in range(min(Wm, 5)):
            dense_fn(i)
        dense_ms = timed(dense_fn, max(10, K // 4))
        dbytes = T.dense_decode_bytes(seq0.tolist(), w.H, w.H_kv, w.d_h, e)
        dense = {"dense_ms_per_step": round(dense_ms, 4), "dense_GBps": round(dbytes / dense_ms / 1e6, 1),
                 "dense_frac_of_peak": round(dbytes / dense_ms / 1e6 / HBM_PEAK_GBS, 4),
                 "speedup_vs_dense": round(dense_ms / ms_per_step, 3),
                 "transfer_ratio_dense_over_sparq": round(dbytes / (dec_bytes + app_bytes), 3)}

    # ---- plain streaming probes of known size: the attainable HBM rate, and the calibration
    # dispatches for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command ----
    n_probe = 1 << 30
    src = torch.ones(n_probe, dtype=torch.uint8, device=dev); dst = torch.empty_like(src)
    sink = torch.empty(2 << 20, dtype=torch.uint8, device=dev)
    probe = {}
    for name, fn, nbytes in (("read", lambda: B.sparq_read_probe(src, n_probe, sink), n_probe),
                             ("copy", lambda: B.sparq_copy_probe(dst, src, n_probe), 2 * n_probe)):
        fn(); torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for _ in range(5):
            fn()
        p1.record(); torch.cuda.synchronize()
        probe[name + "_GBps"] = round(nbytes * 5 / p0.elapsed_time(p1) / 1e6, 1)
    probe["bytes"] = n_probe
    del src, dst

    # ---- CPU oracle on the host cores, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sparq_oracle as O
        import numpy as np
        restore()
        c = caches[0]
        c.append(kn_pool[0], vn_pool[0]); torch.cuda.synchronize()       # vm[0][0], sl[0][0] are c's own buffers
        # sample: the first n_b sequences of the batch (all heads), sized for roughly cpu-seconds of work
        n_b = w.B
        Kh = W.to_codes(c.K[:n_b]); Vh = W.to_codes(c.V[:n_b]); qh = W.to_codes(q_pool[0][:n_b])
        seq_h = c.seq_lens[:n_b].cpu().numpy(); kk = None if kps is None else kps[:n_b].numpy()
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 50:
            tc = time.perf_counter()
            ref = O.sparq_decode(Kh, Vh, qh, seq_h, r=w.r, k=w.k, dtype=w.dtype_code, k_per_seq=kk)
            spent += time.perf_counter() - tc; reps += 1
        cpu = {"value": round(reps / spent, 4), "unit": "decode steps/s", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"full {args.workload} batch ({n_b} sequences x {w.H} heads), {reps} repetitions of "
                         f"oracle_sparq_decode in {spent:.1f} s (fp64, OpenMP over (sequence, KV head))"}
        # while the data is on the host: the timed kernels' output against the oracle on sampled heads
        got = c.decode(q_pool[0], kps_dev).float().cpu().numpy()
        bad = float(np.abs(got[:n_b] - ref.y).max())
        cpu["max_abs_diff_vs_gpu"] = round(bad, 6)

    rec = {
        "metric": "SparQ decode steps/s and achieved HBM GB/s (% peak) vs dense decode, 1 MI355X",
        "value": round(1e3 / ms_per_step, 2), "unit": "decode steps/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "B": w.B, "H": w.H, "H_kv": w.H_kv, "d_h": w.d_h, "S": int(seq0.max()),
                   "r": w.r, "k": w.k if kps is None else "ceil(S_b/%d)" % w.k_div, "cache_dtype": w.dtype,
                   "step": "sparq_decode_step (append + decode in one launch)", "cache_copies_rotated": copies,
                   "q_pool": n_pool, "S_max": S_max, "untimed_clock_warmup_steps": pre},
        "step_GBps": round((dec_bytes + app_bytes) / ms_per_step / 1e6, 1),
        "step_frac_of_peak": round((dec_bytes + app_bytes) / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
        "two_launch_step_ms": round(two_call_ms, 5), "decode_launch_ms": round(dec_avg_ms, 5),
        "decode_launch_GBps": round(dec_bytes0 / dec_avg_ms / 1e6, 1), "append_launch_ms": round(append_ms, 5),
        "hbm_probe": probe,
        "roofline": {"kernel": "sparq_decode_fused<APPEND> (sparq_decode_step)", "bound": "hbm",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_from_profile(args.workload),
                     "algorithmic_bytes_per_launch": int(dec_bytes + app_bytes), "avg_launch_ms": round(step_avg_ms, 5),
                     "stage_bytes": dict({k2: int(v / K) for k2, v in tot.items() if k2 != "total"}, append=app_bytes)},
        "cpu_baseline": cpu,
    }
    rec.update(dense)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
