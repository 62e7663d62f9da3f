#!/usr/bin/env python3
"""Benchmark of the SparQ decode step on one MI355X.

A "step" is one pass of the whole hot path for one new token of every sequence in the batch:
sparq_kv_append (write k, v, the second key layout, update the mean value vector) followed by
sparq_decode (Steps 1-3 of Section 4 for all B x H heads), issued as the one call sparq_decode_step.
Inputs are synthetic, seeded, shaped like the named workload and resident in HBM before the timed
region.  To keep the timed steps out of the 256 MB last-level cache, the run rotates over several
identical cache copies and a pool of queries.

The headline workload is the largest single-GPU configuration (c4_large_batch); with no --workload the
other named configurations are measured briefly as well and reported under "other_workloads".
Timing follows the paper's protocol (Appendix F: warm-up steps, then timed steps between device
synchronisations; mean and standard error, here also the median, of per-step times).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
CLOCK_WARMUP_STEPS = 300       # untimed steps before the W warm-up steps: the first ~10 ms after idle run at lower clocks
HEADLINE = "c4_large_batch"
OTHERS = ["c1_single_head", "c2_llama2_7b", "c3_llama3_8b_gqa", "c5_gemma_7b_ragged", "paper_table2"]
OUT_TOL = 2e-3                 # max abs error of the 16-bit output against the oracle's fp64 y (the tests' bar)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None, help=f"one named workload (default: {HEADLINE}, plus a brief pass over the others)")
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = enough for > 1 GB touched)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--gqa-shared", action="store_true", help="the paper's grouped-query rule (one selection per KV head)")
    ap.add_argument("--stage-clocks", action="store_true",
                    help="profiling run on libsparq_clocks.so (python -m paper_2312_04985_amd.build --stage-clocks): prints the "
                         "per-stage time stamps of the step kernel's workgroups instead of the benchmark line")
    ap.add_argument("--layout", choices=["two_copies", "single_k", "tiled_k"], default="two_copies",
                    help="key cache layout: K twice (default), once row-major (SPARQ_FLAG_SINGLE_K), once in tiles (SPARQ_FLAG_TILED_K)")
    return ap.parse_args()


def traffic_from_profile(workload: str):
    """HBM bytes per step launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), read from the
    committed counter summary of this workload (profiles/), if there is one."""
    path = os.path.join(ROOT, "profiles", f"sparq_decode_{workload}_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def round_to_format(y, dtype_code):
    """y (float64 array) rounded to nearest-even in the 16-bit output format, as float64."""
    import numpy as np
    if dtype_code == 0:
        return y.astype(np.float16).astype(np.float64)
    u = y.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7fff + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def output_violations(got, y, dtype_code):
    """Elements of the 16-bit output `got` that are not the rounding of some y' within OUT_TOL of the
    oracle's y (for fp16, whose spacing is far below the tolerance at these magnitudes, plainly
    |got - y| <= OUT_TOL).  Returns (count, max abs difference)."""
    import numpy as np
    diff = np.abs(got - y)
    if dtype_code == 0:
        bad = diff > OUT_TOL
    else:
        bad = (got < round_to_format(y - OUT_TOL, dtype_code)) | (got > round_to_format(y + OUT_TOL, dtype_code))
    return int(bad.sum()), float(diff.max())


STAGES = ["stage 0: lengths, query, top-r channels, tau", "Step 1 stream (first wave's share)", "wait: all waves' scores in LDS",
          "Step 2 radix select", "Step 2 compaction, alpha", "Step 2 gather + attention (first wave's share)",
          "wait: all waves' partials in LDS", "merge, blend, output and append stores"]


def stage_clock_summary(caches, B):
    """Per-stage durations from the time stamps a profiling build leaves in every cache copy's workspace (the last
    step launched on that copy)."""
    import numpy as np
    off, n_wg, n_st = B.sparq_stage_clocks(caches[0].shape)
    dur, total, span, starts, drain = [], [], [], [], []
    for c in caches:
        t = c.workspace[off:off + n_wg * n_st * 8].view(torch_int64()).cpu().numpy().reshape(n_wg, n_st).astype(np.float64) * 0.01
        t0 = t[:, 0].min()
        dur.append(np.diff(t, axis=1)); total.append(t[:, -1] - t[:, 0]); span.append(t[:, -1].max() - t0)
        starts.append(np.sort(t[:, 0] - t0))
        ends = np.sort(t[:, -1] - t0)
        drain.append(ends[-1] - np.median(ends[-min(n_wg, 512):]))
    dur = np.concatenate(dur); total = np.concatenate(total)
    q = lambda x: {"median": round(float(np.median(x)), 2), "p10": round(float(np.percentile(x, 10)), 2),
                   "p90": round(float(np.percentile(x, 90)), 2), "mean": round(float(np.mean(x)), 2)}
    st = np.stack(starts)
    return {"unit": "us", "workgroups_per_launch": n_wg, "launches": len(caches),
            "stages": {STAGES[i]: q(dur[:, i]) for i in range(len(STAGES))},
            "workgroup_total": q(total), "launch_span_first_start_to_last_end": q(np.array(span)),
            "workgroups_started_within_2us": int(np.median((st < 2.0).sum(axis=1))),
            "start_of_workgroup_number": {str(n): round(float(np.median(st[:, n])), 2) for n in (0, 511, 512, 1023, 1024, 1535, 1536, n_wg - 1) if n < n_wg},
            "last_end_minus_median_end_of_last_512": q(np.array(drain))}


def torch_int64():
    import torch
    return torch.int64


def measure(name, K, Wm, args, full):
    """One workload: the timed region, per-step statistics, comparison launches; with `full` also the
    bandwidth probes and the CPU oracle leg."""
    import numpy as np
    import torch
    from paper_2312_04985_amd import binding as B
    from paper_2312_04985_amd import traffic as T
    from paper_2312_04985_amd import workloads as W
    from paper_2312_04985_amd.cache import DecodeCache

    dev = torch.device("cuda:0")
    w = W.CONFIGS[name]
    seq0 = W.draw_seq_lens(w)                       # lengths seen by the first timed decode
    kps = W.k_per_seq(w, seq0)
    e = 2
    group_kv = w.H_kv if (args.gqa_shared and w.H != w.H_kv) else None     # bytes per KV head under the grouped-query rule
    step_bytes0 = T.sparq_decode_bytes(seq0.tolist(), w.H, w.d_h, w.r, w.k, e, None if kps is None else kps.tolist(), group_kv)
    copies = args.copies or max(2, -(-(1 << 30) // step_bytes0["total"]))
    pre = max(0, CLOCK_WARMUP_STEPS - Wm)           # untimed extra steps so that the clocks have ramped up
    per_copy = -(-max(K, Wm, pre) // copies) + 1     # appends one copy receives in one pass
    S_max = W.round_up(int(seq0.max()) + per_copy, 64)

    layout_flag = {"two_copies": 0, "single_k": B.SPARQ_FLAG_SINGLE_K, "tiled_k": B.SPARQ_FLAG_TILED_K}[args.layout]
    # ---- build the caches through the library (bulk append of S_b - 1 rows) ----
    K_src, V_src = W.draw_kv(w, dev, n_rows=int(seq0.max()))
    caches = []
    for _ in range(copies):
        c = DecodeCache(w.B, w.H, w.H_kv, S_max, w.d_h, w.r, w.k, w.torch_dtype, device=dev,
                        flags=(B.SPARQ_FLAG_RAGGED_BATCH if w.ragged else 0) | layout_flag |
                              (B.SPARQ_FLAG_GQA_SHARED if args.gqa_shared else 0))
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

    def fused_step(i):            # the step: append + decode in one call
        ci = i % copies
        check(lib.sparq_decode_step(*table[ci][par[ci]][i % n_pool]["step"]))
        par[ci] ^= 1

    def two_call_step(i):         # the same step as two calls (state updated in place)
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

    def per_step_events(fn, n):   # one event after every step: per-step durations (launch gaps included), ms
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(n):
            fn(i)
            evs[i + 1].record()
        torch.cuda.synchronize()
        return np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(n)])

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

    if args.stage_clocks:
        rec = {"workload": name, "step_us_instrumented_build": round(ms_per_step * 1e3, 2),
               "plan": B.sparq_decode_plan(caches[0].shape), "stage_clocks": stage_clock_summary(caches, B)}
        del caches, table, cs, K_src, V_src
        gc.collect()
        torch.cuda.empty_cache()
        return rec

    # ---- average duration of the step's launches over the same K steps, HIP events on their stream;
    # K back-to-back steps, launch gaps included; then once more with an event after every step ----
    restore()
    step_avg_ms = timed_events(fused_step, K)
    restore()
    per = per_step_events(fused_step, K)

    # the decode call alone at the lengths the timed steps ended with (not a multiple of 8 or of 4096: the newest
    # rows come from K, and a few chunks start another round of the stream), so that step minus this is the append
    dec_same_ms = timed_events(lambda i: check(lib.sparq_decode(*table[i % copies][par[i % copies]][i % n_pool]["decode"])), K)

    # for the record: the step as two calls, the decode call alone, the append call alone
    restore()
    two_call_ms = timed(two_call_step, K)
    restore()
    for ci in range(copies):
        check(lib.sparq_kv_append(*table[ci][0][0]["append"]))           # lengths S_b, as in the first timed step
    dec_avg_ms = timed_events(lambda i: check(lib.sparq_decode(*table[i % copies][0][i % n_pool]["decode"])), K)
    restore()
    append_ms = timed(lambda i: check(lib.sparq_kv_append(*table[i % copies][0][i % n_pool]["append"])), K)
    restore()

    # algorithmic bytes of the K timed steps: copy c is visited at steps c, c + copies, ... and holds
    # S_b + (visit number) rows when it is decoded
    tot = {"stage1": 0, "stage3": 0, "blend": 0, "total": 0}
    kk = None if kps is None else kps.tolist()
    for i in range(K):
        bts = T.sparq_decode_bytes((seq0 + (i // copies)).tolist(), w.H, w.d_h, w.r, w.k, e, kk, group_kv)
        for key in tot:
            tot[key] += bts[key]
    dec_bytes = tot["total"] / K
    app_bytes = T.kv_append_bytes(w.B, w.H_kv, w.d_h, e)
    dec_bytes0 = T.sparq_decode_bytes(seq0.tolist(), w.H, w.d_h, w.r, w.k, e, kk, group_kv)["total"]
    achieved = (dec_bytes + app_bytes) / (step_avg_ms * 1e-3) / 1e9
    plan = B.sparq_decode_plan(caches[0].shape)

    rec = {
        "workload": name, "ms_per_step": ms_per_step, "steps_per_s": 1e3 / ms_per_step, "plan": plan,
        "config": {"workload": name, "B": w.B, "H": w.H, "H_kv": w.H_kv, "d_h": w.d_h, "S": int(seq0.max()),
                   "r": w.r, "k": w.k if kps is None else "ceil(S_b/%d)" % w.k_div, "cache_dtype": w.dtype,
                   "step": "sparq_decode_step (append + decode in one call)", "key_layout": args.layout,
                   "gqa_rule": "one selection per KV head (Section 4)" if group_kv else "every query head selects for itself", "cache_copies_rotated": copies,
                   "q_pool": n_pool, "S_max": S_max, "untimed_clock_warmup_steps": pre},
        "step_GBps": round((dec_bytes + app_bytes) / ms_per_step / 1e6, 1),
        "step_frac_of_peak": round((dec_bytes + app_bytes) / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
        "step_us_stats": {"median": round(float(np.median(per)) * 1e3, 2), "mean": round(float(per.mean()) * 1e3, 2),
                          "standard_error": round(float(per.std(ddof=1) / np.sqrt(len(per))) * 1e3, 3), "n": int(len(per)),
                          "how": "one HIP event after every step of a separate pass of K steps"},
        "two_launch_step_ms": round(two_call_ms, 5), "decode_launch_ms": round(dec_avg_ms, 5),
        "decode_launch_at_step_lengths_ms": round(dec_same_ms, 5),
        "decode_launch_GBps": round(dec_bytes0 / dec_avg_ms / 1e6, 1), "append_launch_ms": round(append_ms, 5),
        "roofline": {"kernel": plan + (" with the append built in (sparq_decode_step)" if plan.startswith("sparq_decode_fused") or "digit-bucket" in plan else
                                       "; sparq_decode_step runs append_one_row first"),
                     "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None if group_kv else traffic_from_profile(name),
                     "algorithmic_bytes_per_launch": int(dec_bytes + app_bytes), "avg_launch_ms": round(step_avg_ms, 5),
                     "stage_bytes": dict({k2: int(v / K) for k2, v in tot.items() if k2 != "total"}, append=app_bytes)},
    }

    # ---- in-library dense decode on the same rotation ----
    if not args.no_dense and args.layout != "tiled_k":   # the comparison kernel reads key rows
        dense_fn = lambda i: check(lib.dense_decode(*table[i % copies][0][i % n_pool]["dense"]))
        for i in range(min(Wm, 5)):
            dense_fn(i)
        dense_ms = timed(dense_fn, max(10, K // 4))
        dbytes = T.dense_decode_bytes(seq0.tolist(), w.H, w.H_kv, w.d_h, e)
        rec.update({"dense_ms_per_step": round(dense_ms, 4), "dense_GBps": round(dbytes / dense_ms / 1e6, 1),
                    "dense_frac_of_peak": round(dbytes / dense_ms / 1e6 / HBM_PEAK_GBS, 4),
                    "speedup_vs_dense": round(dense_ms / ms_per_step, 3),
                    "transfer_ratio_dense_over_sparq": round(dbytes / (dec_bytes + app_bytes), 3)})

    if full:
        # ---- plain streaming probes of known size: the attainable HBM rate, and the calibration
        # dispatches for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command ----
        n_probe = 1 << 30
        src = torch.ones(n_probe, dtype=torch.uint8, device=dev); dst = torch.empty_like(src)
        sink = torch.empty(2 << 20, dtype=torch.uint8, device=dev)
        probe = {}
        for pname, fn, nbytes in (("read", lambda: B.sparq_read_probe(src, n_probe, sink), n_probe),
                                  ("copy", lambda: B.sparq_copy_probe(dst, src, n_probe), 2 * n_probe)):
            fn(); torch.cuda.synchronize()
            p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            p0.record()
            for _ in range(5):
                fn()
            p1.record(); torch.cuda.synchronize()
            probe[pname + "_GBps"] = round(nbytes * 5 / p0.elapsed_time(p1) / 1e6, 1)
        probe["bytes"] = n_probe
        rec["hbm_probe"] = probe
        del src, dst

    # ---- CPU oracle on the host cores: timed on the whole batch of this workload, and its result compared
    # with the timed kernels' output on every unit ----
    rec["cpu_baseline"] = None
    if full and not args.no_cpu_baseline:
        from oracle import sparq_oracle as O
        restore()
        c = caches[0]
        c.append(kn_pool[0], vn_pool[0]); torch.cuda.synchronize()       # vm[0][0], sl[0][0] are c's own buffers
        kq_max = int(torch.minimum(kps if kps is not None else torch.full_like(seq0, w.k), seq0).max())
        got_t, _, idx_t, _ = c.decode(q_pool[0], kps_dev, aux=True, idx_stride=kq_max)
        torch.cuda.synchronize()
        Kh = W.to_codes(c.key_rows()); Vh = W.to_codes(c.V); qh = W.to_codes(q_pool[0])
        seq_h = c.seq_lens.cpu().numpy(); kk_h = None if kps is None else kps.numpy()
        oflags = B.SPARQ_FLAG_GQA_SHARED if args.gqa_shared else 0
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 50:
            tc = time.perf_counter()
            ref = O.sparq_decode(Kh, Vh, qh, seq_h, r=w.r, k=w.k, dtype=w.dtype_code, k_per_seq=kk_h, flags=oflags)
            spent += time.perf_counter() - tc; reps += 1
        got = got_t.float().cpu().numpy().astype(np.float64)
        n_bad, max_diff = output_violations(got, ref.y, w.dtype_code)
        same_sets = bool(np.array_equal(idx_t.cpu().numpy()[..., :ref.i2.shape[-1]], ref.i2))
        if n_bad and not same_sets:
            # a position inside the band that the index-set rule leaves open: judge the output on the GPU's own sets
            ref = O.sparq_decode(Kh, Vh, qh, seq_h, r=w.r, k=w.k, dtype=w.dtype_code, k_per_seq=kk_h, flags=oflags,
                                 given_i2=np.ascontiguousarray(idx_t.cpu().numpy()[..., :ref.i2.shape[-1]]))
            n_bad, max_diff = output_violations(got, ref.y, w.dtype_code)
        if n_bad:
            raise RuntimeError(f"{n_bad} output elements of the timed kernel are outside the {OUT_TOL} bar against the oracle "
                               f"(max abs difference {max_diff})")
        rec["cpu_baseline"] = {
            "value": round(reps / spent, 4), "unit": "decode steps/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"whole {name} batch ({w.B} sequences x {w.H} heads), {reps} repetitions of "
                      f"oracle_sparq_decode in {spent:.1f} s (fp64, OpenMP over (sequence, KV head))",
            "max_abs_diff_vs_gpu": round(max_diff, 6), "units_compared": int(w.B * w.H),
            "index_sets_identical": same_sets, "output_tolerance": OUT_TOL}
        del Kh, Vh
    del caches, table, cs, K_src, V_src
    gc.collect()
    torch.cuda.empty_cache()
    return rec


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
    torch.cuda.set_device(0)

    name = args.workload or HEADLINE
    K, Wm = args.steps, args.warmup
    if args.stage_clocks:
        from paper_2312_04985_amd import binding, build
        if not os.path.exists(build.LIB_CLOCKS):
            print("bench.py --stage-clocks needs libsparq_clocks.so: python -m paper_2312_04985_amd.build --stage-clocks", file=sys.stderr)
            sys.exit(1)
        binding.LIB_PATH = build.LIB_CLOCKS
        print(json.dumps(measure(name, K, Wm, args, full=False)))
        return
    main_rec = measure(name, K, Wm, args, full=True)

    rec = {
        "metric": "SparQ decode steps/s and achieved HBM GB/s (% peak) vs dense decode, 1 MI355X",
        "value": round(main_rec["steps_per_s"], 2), "unit": "decode steps/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(main_rec["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
    }
    for key in ("config", "step_GBps", "step_frac_of_peak", "step_us_stats", "two_launch_step_ms", "decode_launch_ms", "decode_launch_at_step_lengths_ms",
                "decode_launch_GBps", "append_launch_ms", "hbm_probe", "roofline", "cpu_baseline", "dense_ms_per_step",
                "dense_GBps", "dense_frac_of_peak", "speedup_vs_dense", "transfer_ratio_dense_over_sparq"):
        if key in main_rec:
            rec[key] = main_rec[key]

    if args.workload is None and not args.no_others:
        # the other named configurations, briefly (parity-test cases; same step, same protocol, fewer steps)
        others = {}
        for other in OTHERS:
            r = measure(other, min(K, 100), min(Wm, 10), args, full=False)
            others[other] = {"step_us": round(r["ms_per_step"] * 1e3, 2), "steps_per_s": round(r["steps_per_s"], 1),
                             "frac_of_peak": r["roofline"]["frac"], "step_us_median": r["step_us_stats"]["median"],
                             "decode_launch_us": round(r["decode_launch_ms"] * 1e3, 2),
                             "dense_us": round(r.get("dense_ms_per_step", float("nan")) * 1e3, 2),
                             "speedup_vs_dense": r.get("speedup_vs_dense"), "plan": r["plan"],
                             "algorithmic_bytes_per_launch": r["roofline"]["algorithmic_bytes_per_launch"]}
        # config 3 once more under the paper's grouped-query rule (a quarter of the bytes: one selection per KV head)
        import copy
        ga = copy.copy(args); ga.gqa_shared = True
        r = measure("c3_llama3_8b_gqa", min(K, 100), min(Wm, 10), ga, full=False)
        others["c3_llama3_8b_gqa, grouped-query rule"] = {
            "step_us": round(r["ms_per_step"] * 1e3, 2), "steps_per_s": round(r["steps_per_s"], 1),
            "frac_of_peak": r["roofline"]["frac"], "step_us_median": r["step_us_stats"]["median"],
            "decode_launch_us": round(r["decode_launch_ms"] * 1e3, 2), "dense_us": round(r.get("dense_ms_per_step", float("nan")) * 1e3, 2),
            "speedup_vs_dense": r.get("speedup_vs_dense"), "plan": r["plan"],
            "algorithmic_bytes_per_launch": r["roofline"]["algorithmic_bytes_per_launch"]}
        rec["other_workloads"] = others
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
