#!/usr/bin/env python3
"""Benchmark of the stateful-session attention path on one MI355X.

A step is one pass of the whole hot path on the Llama-3-8B-shaped layer (bf16, 32 query heads,
8 KV heads, head_dim 128) at 32,768 cached tokens: block allocation, K/V commit of a 256-token
chunk, the chunk's causal attention over cache + chunk (data plane), then a 32-token
non-committing query over 32,768 cached tokens with its cross-split combine (query plane).
The appended session is then truncated back (host metadata only) so every step sees the same
lengths.  Steps rotate over several sessions whose caches together exceed the 256 MB last-level
cache, and the query of a step reads a session half the rotation away from the one the step appends
to, so what it streams comes from HBM ("cold"); --hot keeps one session.

Prints ONE JSON line.  `value` is tokens per second through the whole step; the per-plane
figures the path is judged on (query latency and KV GB/s, append tokens/s and TFLOP/s) are in
"query" and "append"; "roofline" describes the kernel that takes most of the step; "ceilings" holds
what a plain read and a bare matrix loop reach on this device in this run; "extras" the other
workloads and the sweeps (split count, query length, context length).

Every figure comes from this run.  Three kinds of timing are used and named where they appear:
  wall    host clock around a batch of calls bracketed by device synchronisation;
  stream  a pair of HIP events on the launch stream around a batch of back-to-back calls, divided
          by the number of calls (no event between the calls: what a caller issuing them sees);
  kernel  the dispatch's own start and end time stamps, which the library has the runtime write into
          a pair of HIP events per kernel launch (sk_pool_set_profiling), in a repeat of the timed
          steps: the duration rocprofv3 reports for the same launch (profiles/).
HBM bytes per dispatch from hardware counters need rocprofv3 around the process and are therefore
not in this line ("traffic": null); the summaries under profiles/ carry them.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from workloads import synth  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VALU_PEAK_TFLOPS = 157.3

WORKLOADS = {
    # name: (shape, cached tokens at query time, append chunk, query tokens)
    "cfg2_llama3_8b_layer_32k": (synth.CFG2, 32768, 256, 32),
    "cfg3_long_context_128k": (synth.CFG3, 131072, 512, 16),
}


def ramp(fn, ms=100.0, batch=10):
    """Runs fn(i) untimed for `ms` of wall time: the device raises its clocks over tens of milliseconds
    of load, and what the measurements report is the sustained rate."""
    t0, i = time.perf_counter(), 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(batch):
            fn(i); i += 1
        torch.cuda.synchronize()
    return i


def stream_time_us(fn, n, warm=3):
    """Average time of fn(i), i = 0..n-1, issued back to back on the current stream: one pair of HIP
    events around the whole batch, nothing between the calls."""
    for i in range(warm):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n):
        fn(warm + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def build_sessions(pool, shape, n0, n_sessions, gen, piece=1024):
    """Grows n_sessions sessions to n0 cached tokens by commit-only appends of `piece` tokens (same data
    for every session; each session owns different physical blocks, interleaved with the others')."""
    sids = [pool.sk_session_create() for _ in range(n_sessions)]
    done = 0
    while done < n0:
        L = min(piece, n0 - done)
        k = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype).cuda()
        v = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype).cuda()
        for sid in sids:
            pool.sk_session_append(sid, None, k, v)
        done += L
    torch.cuda.synchronize()
    return sids


def query_bytes(shape, n, nq, block_tokens):
    return n * shape.kv_bytes_per_token + nq * shape.n_q_heads * shape.head_dim * (2 + 4) + (n + block_tokens - 1) // block_tokens * 4


def append_flops(shape, n_before, L):
    return 4.0 * shape.head_dim * shape.n_q_heads * L * (n_before + (L + 1) / 2.0)


def rotation_sessions(kv_per_session):
    """Sessions to rotate over so that their caches together exceed 1 GiB (four times the last-level cache)."""
    return max(5, -(-(1 << 30) // kv_per_session) + 1)


def measure_ceilings(sk):
    """What the device itself reaches in this run: a plain streaming read (large buffer, and buffers of
    exactly the bytes a 32K / 128K query streams, launch included), and the bf16 matrix pipe on
    register operands with data-like bit patterns."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").fill_(3)
    res = {}
    ramp(lambda i: sk.sk_probe_read(big, 2048, sink), 60.0, 4)
    best = None
    for nt in (False, True):
        for wgs in (1024, 2048, 4096, 8192, 16384):
            us = stream_time_us(lambda i: sk.sk_probe_read(big, wgs, sink, non_temporal=nt), 8)
            best = us if best is None else min(best, us)
    res["stream_read_GBps"] = big.numel() / (best * 1e-6) / 1e9
    res["stream_read_frac_of_hbm_peak"] = res["stream_read_GBps"] / HBM_PEAK_GBPS
    # buffers of a query's size, rotating through the 2 GiB buffer so that every read is cold
    for name, nbytes in (("read_134MB_us", 32768 * 4096), ("read_537MB_us", 131072 * 4096)):
        n_off = big.numel() // nbytes
        best = None
        for nt in (False, True):
            for wgs in (256, 512, 1024, 2048, 4096):
                t = stream_time_us(lambda i: sk.sk_probe_read(big[(i % n_off) * nbytes:], wgs, sink, nbytes=nbytes, non_temporal=nt), 16)
                best = t if best is None else min(best, t)
        res[name] = best
    del big
    fsink = torch.zeros(4, dtype=torch.float32, device="cuda")
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    # operands: N(0,1) rounded to bf16, like the Q/K/V of the workloads (what the bits do decides the
    # power drawn and with it the clock the pipe holds); and, for contrast, all ones
    data = synth.draw(synth.generator(9), (1 << 20,), "bf16").cuda()
    ones = torch.ones(1 << 20, dtype=torch.bfloat16, device="cuda")
    for key, ops in (("mfma_bf16_TFLOPs", data), ("mfma_bf16_constant_operands_TFLOPs", ones)):
        flops = sk.sk_probe_mfma(n_cus, 5000, fsink, ops)
        ramp(lambda i: sk.sk_probe_mfma(n_cus, 5000, fsink, ops), 100.0, 2)      # 1-2 ms per launch
        us = stream_time_us(lambda i: sk.sk_probe_mfma(n_cus, 5000, fsink, ops), 20)
        res[key] = flops / (us * 1e-6) / 1e12
    res["mfma_bf16_frac_of_published_peak"] = res["mfma_bf16_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    res["how"] = ("sk_probe_read: 16-byte loads, eight in flight per thread, default and non-temporal cache policy, over a 2 GiB buffer "
                  "(best of 1,024-16,384 workgroups) and over 134 / 537 MB pieces of it, never the same piece twice in a row (best of "
                  "256-4,096 workgroups), stream "
                  "timing; sk_probe_mfma: 8 waves per CU x 40,000 v_mfma_f32_32x32x16_bf16 on register operands drawn from N(0,1) "
                  "(or all ones), after 100 ms of the same load")
    return res


def cpu_baseline(shape, n, L, nq, gen, budget_rows):
    """Times the fp64 oracle on a bounded sample of the same step: `budget_rows` output rows
    spread evenly over the append chunk and the query, each against the full cache."""
    import oracle
    o = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    q, k, v = synth.draw_qkv(gen, n - L, shape)
    o.K, o.V = synth.to_raw(k), synth.to_raw(v)
    qa, ka, va = synth.draw_qkv(gen, L, shape)
    qq, _, _ = synth.draw_qkv(gen, nq, shape)
    total_rows = (L + nq) * shape.n_q_heads
    frac = min(1.0, budget_rows / float(total_rows))
    rng = np.random.default_rng(0)
    n_app = max(1, int(round(L * shape.n_q_heads * frac)))
    n_qry = max(1, int(round(nq * shape.n_q_heads * frac)))
    rows_a = [(int(i) // shape.n_q_heads, int(i) % shape.n_q_heads) for i in rng.choice(L * shape.n_q_heads, n_app, replace=False)]
    rows_q = [(int(i) // shape.n_q_heads, int(i) % shape.n_q_heads) for i in rng.choice(nq * shape.n_q_heads, n_qry, replace=False)]
    t0 = time.perf_counter()
    o.append(synth.to_raw(qa), synth.to_raw(ka), synth.to_raw(va), rows=rows_a)
    o.query(synth.to_raw(qq), rows=rows_q)
    dt = time.perf_counter() - t0
    est_step_s = dt * total_rows / float(n_app + n_qry)
    return {
        "value": (L + nq) / est_step_s, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "%d of %d output rows of one step (%d append rows + %d query rows, each over the full %d-token cache), "
                  "%.1f s of CPU work, scaled to the whole step" % (n_app + n_qry, total_rows, n_app, n_qry, n, dt),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--ramp-ms", type=float, default=100.0,
                    help="untimed steps run for this long before the warm-up steps, to bring the device to its sustained clocks")
    ap.add_argument("--workload", default="cfg2_llama3_8b_layer_32k", choices=sorted(WORKLOADS))
    ap.add_argument("--block-tokens", type=int, default=16)
    ap.add_argument("--sessions", type=int, default=0, help="sessions to rotate over (0: enough for > 1 GiB of K/V)")
    ap.add_argument("--hot", action="store_true", help="one session only: K/V may stay in the last-level cache")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads and the sweeps")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the plain-read and matrix-loop probes")
    ap.add_argument("--only", default="", help="comma-separated extras to run instead of all (names as in the output)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times before the steps (a kernel of known "
                         "size against which hardware byte counters are scaled)")
    ap.add_argument("--cpu-rows", type=int, default=0, help="oracle sample size in output rows (0: sized for ~15 s)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (no collectives, no sharding)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    import paper_2605_13784_amd as sk

    ceilings = None if args.no_ceilings else measure_ceilings(sk)
    main_res = stream_workload(sk, args.workload, args, args.steps, args.warmup, ceilings, calibrate=args.copy_calibration,
                               sweeps=not args.no_extras)
    shape, n, L, nq = WORKLOADS[args.workload]
    res = {
        "metric": "stream-step throughput: %d-token append + %d-token query at %d cached tokens" % (L, nq, n),
        "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": main_res["config"], "query": main_res["query"], "append": main_res["append"],
        "roofline": main_res["roofline"], "roofline_query": main_res["roofline_query"],
        "roofline_append": main_res["roofline_append"], "ceilings": ceilings,
    }
    if not args.no_extras:
        only = set(x for x in args.only.split(",") if x)
        want = lambda name: not only or name in only
        extras = {}
        for key in ("split_sweep", "latency_vs_query_tokens"):
            if key in main_res:
                extras[args.workload.split("_")[0] + "_" + key] = main_res[key]
        other = "cfg3_long_context_128k" if "cfg2" in args.workload else "cfg2_llama3_8b_layer_32k"
        if want(other):
            r = stream_workload(sk, other, args, max(10, args.steps // 2), 4, ceilings, sweeps=True)
            extras[other] = {k: r[k] for k in ("ms_per_step", "config", "query", "append", "roofline_query", "roofline_append",
                                               "split_sweep") if k in r}
            if other == "cfg3_long_context_128k" and args.block_tokens != 256:
                # the workload fixes no block size; 256-token blocks are the faster layout for small queries
                big = argparse.Namespace(**vars(args)); big.block_tokens = 256
                r = stream_workload(sk, other, big, max(10, args.steps // 2), 4, ceilings)
                extras[other + "_256_token_blocks"] = {k: r[k] for k in ("ms_per_step", "config", "query", "roofline_query")}
        if want("latency_vs_cached_tokens"):
            extras["latency_vs_cached_tokens"] = latency_vs_cached_tokens(sk, ceilings)
        if want("cfg5_question_batch_64k"):
            extras["cfg5_question_batch_64k"] = question_batch(sk)
        if want("cfg4_multi_tenant_step"):
            extras["cfg4_multi_tenant_step"] = multi_tenant(sk)
        if want("cfg1_fp32_small"):
            extras["cfg1_fp32_small"] = fp32_small(sk)
        if want("head_dim_64_32k"):
            extras["head_dim_64_32k"] = head_dim_64(sk)
        if want("sliding_window_32k"):
            extras["sliding_window_32k"] = sliding_window(sk)
        if want("fork_cost"):
            extras["fork_cost"] = fork_cost(sk)
        if want("top2_sampling"):
            extras["top2_sampling"] = top2_sampling(sk)
        res["extras"] = extras
    if not args.no_cpu_baseline:
        rows = args.cpu_rows or ((L + nq) * shape.n_q_heads if n <= 32768 else 4096)
        res["cpu_baseline"] = cpu_baseline(shape, n, L, nq, synth.generator(7), rows)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


def stream_workload(sk, name, args, steps, warmup, ceilings, calibrate=False, sweeps=False):
    """Times `steps` stream steps (append + query + truncate back) of one workload, then the same steps
    again with the library's HIP-event timing of the kernels switched on, then each plane by itself
    (queries back to back, appends back to back) with nothing between the calls."""
    shape, n, L, nq = WORKLOADS[name]
    B = args.block_tokens
    kv_per_session = n * shape.kv_bytes_per_token
    n_sessions = 1 if args.hot else (args.sessions or rotation_sessions(kv_per_session))
    blocks_per_session = (n + B - 1) // B + 2
    # truncated blocks queue behind the free ones, so keep a margin of free blocks
    n_blocks = n_sessions * blocks_per_session + 4 * (L // B + 2)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_blocks,
                   max_sessions=n_sessions, max_batch_tokens=max(L, nq, 1024))
    gen = synth.generator(2 if "cfg2" in name else 3)
    n0 = n - L
    sids = build_sessions(pool, shape, n0, n_sessions, gen)
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, L, shape)]
    qq = synth.draw(gen, (128, shape.n_q_heads, shape.head_dim), shape.dtype).cuda()
    out_a = torch.empty((L, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((L, shape.n_q_heads), dtype=torch.float32, device="cuda")
    out_q = torch.empty((128, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_q = torch.empty((128, shape.n_q_heads), dtype=torch.float32, device="cuda")
    half = n_sessions // 2

    def do_query(sid, m=nq, S=args.n_splits):
        pool.sk_session_query(sid, qq[:m], out=out_q[:m], lse=lse_q[:m], n_splits=S)

    def step(i, same_session=False):
        sid = sids[i % n_sessions]
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        # the query reads a session the append of this step did not touch: the append has just pulled its
        # own session's cache through the last-level cache
        do_query(sid if same_session else sids[(i + half) % n_sessions])
        pool.sk_session_truncate(sid, n0)

    if calibrate:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # The device raises its clocks over tens of milliseconds of load (after the idle of the session
    # build-up 40 steps measured 0.21 ms each, from 40 ms of load on 0.19 ms, steady over 1,000 steps):
    # the same steps run untimed for --ramp-ms first, so that what is timed is the sustained rate.
    ramp(step, args.ramp_ms, 20)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # same steps again with HIP events around the kernels (recorded by the library on the
    # stream the kernels run on)
    def kernel_times(same_session):
        pool.sk_pool_set_profiling(True)
        for i in range(n_sessions):               # a first pass creates the events and is thrown away (one-off stalls)
            step(warmup + steps + i, same_session)
        torch.cuda.synchronize()
        pool.sk_pool_read_profile()
        for i in range(steps):
            step(warmup + steps + i, same_session)
        torch.cuda.synchronize()
        _, attn_ms, comb_ms = pool.sk_pool_read_profile()
        pool.sk_pool_set_profiling(False)
        return np.array(attn_ms[0::2]), np.array(comb_ms[0::2]), np.array(attn_ms[1::2]), np.array(comb_ms[1::2])
    app_attn, app_comb, qry_attn, qry_comb = kernel_times(False)
    _, _, qry_attn_same, qry_comb_same = kernel_times(True)
    info = pool.sk_pool_last_launch()

    # each plane by itself, calls back to back, nothing between them
    n_rep = max(steps, 3 * n_sessions)
    q_cold_us = stream_time_us(lambda i: do_query(sids[i % n_sessions]), n_rep, warm=n_sessions)
    q_hot_us = stream_time_us(lambda i: do_query(sids[0]), n_rep, warm=4)
    t0 = time.perf_counter()
    for i in range(n_rep):
        do_query(sids[i % n_sessions])
    q_host_us = (time.perf_counter() - t0) * 1e6 / n_rep
    torch.cuda.synchronize()

    def append_only(i):
        sid = sids[i % n_sessions]
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        pool.sk_session_truncate(sid, n0)
    a_us = stream_time_us(append_only, n_rep, warm=n_sessions)

    qb = query_bytes(shape, n, nq, B)
    af = append_flops(shape, n0, L)
    q_kernel_us = float(qry_attn.mean() * 1e3)
    q_comb_us = float(qry_comb.mean() * 1e3)
    a_kernel_us = float(app_attn.mean() * 1e3)
    a_comb_us = float(app_comb.mean() * 1e3)
    same_bytes_key = "read_134MB_us" if n == 32768 else "read_537MB_us"
    roof_q = {"kernel": "sk_attn_bf16_d128 (query, split-KV partial)", "bound": "hbm",
              "achieved": qb / (q_kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
              "frac": qb / (q_kernel_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, "traffic": None,
              "avg_kernel_us": q_kernel_us, "algorithmic_bytes": qb, "timing": "kernel"}
    roof_a = {"kernel": "sk_attn_bf16_d128 (append, causal over cache + chunk)", "bound": "mfma",
              "achieved": af / (a_kernel_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
              "frac": af / (a_kernel_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
              "avg_kernel_us": a_kernel_us, "algorithmic_flops": af, "timing": "kernel"}
    if ceilings:
        roof_q["frac_of_measured_stream_read"] = roof_q["achieved"] / ceilings["stream_read_GBps"]
        roof_q["plain_read_of_the_same_bytes_us"] = ceilings[same_bytes_key]
        roof_a["frac_of_measured_mfma_loop"] = roof_a["achieved"] / ceilings["mfma_bf16_TFLOPs"]
    res = {
        "tokens_per_s": (L + nq) * steps / wall, "ms_per_step": wall * 1e3 / steps,
        "config": {"workload": name, "n_q_heads": shape.n_q_heads, "n_kv_heads": shape.n_kv_heads,
                   "head_dim": shape.head_dim, "cached_tokens": n, "append_tokens": L, "query_tokens": nq,
                   "block_tokens": B, "sessions_rotated": n_sessions, "cache": "hot" if args.hot else "cold",
                   "query_splits": info["n_splits"], "query_workgroups": info["workgroups"]},
        "query": {"latency_us": q_cold_us, "timing": "stream: %d queries back to back, each on the next of %d sessions "
                                                     "(cold), attention + combine + launch gaps" % (n_rep, n_sessions),
                  "latency_hot_us": q_hot_us, "host_call_us": q_host_us,
                  "kv_GBps": qb / (q_cold_us * 1e-6) / 1e9, "hbm_frac": qb / (q_cold_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                  "kv_GBps_hot": qb / (q_hot_us * 1e-6) / 1e9,
                  "kernel_us": q_kernel_us, "combine_us": q_comb_us,
                  "kernel_us_right_after_an_append_to_the_same_session": float(qry_attn_same.mean() * 1e3),
                  "kernel_p50_us": float(np.median(qry_attn) * 1e3), "kernel_max_us": float(qry_attn.max() * 1e3)},
        "append": {"latency_us": a_us, "timing": "stream: %d appends back to back (commit + attention + combine)" % n_rep,
                   "tokens_per_s": L / (a_us * 1e-6), "tflops": af / (a_us * 1e-6) / 1e12,
                   "mfma_frac": af / (a_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                   "kernel_us": a_kernel_us, "combine_us": a_comb_us},
        "roofline": roof_a if a_kernel_us >= q_kernel_us else roof_q, "roofline_query": roof_q, "roofline_append": roof_a,
    }
    if ceilings:
        res["query"]["latency_over_plain_read_of_the_same_bytes"] = q_cold_us / ceilings[same_bytes_key]
        res["append"]["frac_of_measured_mfma_loop"] = res["append"]["tflops"] / ceilings["mfma_bf16_TFLOPs"]
    if sweeps:
        # the query by itself against the number of splits of the cached tokens
        sweep = {}
        for S in (4, 8, 16, 32, 64, 128, 256):
            us = stream_time_us(lambda i: do_query(sids[i % n_sessions], nq, S), 2 * n_sessions + 6, warm=n_sessions)
            sweep[str(S)] = {"latency_us": us, "hbm_frac": qb / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
        sweep["library_choice"] = {"splits": info["n_splits"], "latency_us": q_cold_us}
        res["split_sweep"] = sweep
        if "cfg2" in name:
            # latency against the number of query tokens at a fixed cache (cold and hot)
            curve = {}
            for m in (1, 8, 16, 32, 64, 128):
                c = stream_time_us(lambda i: do_query(sids[i % n_sessions], m, 0), 3 * n_sessions, warm=n_sessions)
                h = stream_time_us(lambda i: do_query(sids[0], m, 0), 3 * n_sessions, warm=4)
                curve[str(m)] = {"cold_us": c, "hot_us": h, "rows_per_kv_head": m * shape.group,
                                 "kv_GBps_cold": query_bytes(shape, n, m, B) / (c * 1e-6) / 1e9}
            res["latency_vs_query_tokens"] = {"cached_tokens": n, "points": curve, "timing": "stream"}
    pool.close()
    return res


def latency_vs_cached_tokens(sk, ceilings, nq=32):
    """Latency of a 32-token (and of a 16-token) query against the cached length (the paper's context
    range, 2,600 and 14,800 tokens, the two workload lengths and 65,536 between them), cold (rotation over sessions that together hold > 1 GiB, at
    most 128 of them) and hot (one session); the bytes a query streams and the rate."""
    shape = synth.CFG2
    B = 16
    qq = synth.draw(synth.generator(2, stream=50), (nq, shape.n_q_heads, shape.head_dim), shape.dtype).cuda()
    out_q = torch.empty((nq, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_q = torch.empty((nq, shape.n_q_heads), dtype=torch.float32, device="cuda")
    points = {}
    q16, out16, lse16 = qq[:16], out_q[:16], lse_q[:16]
    for n in (2600, 14800, 32768, 65536, 131072):
        n_sessions = min(128, rotation_sessions(n * shape.kv_bytes_per_token))
        pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_sessions * ((n + B - 1) // B + 1),
                       max_sessions=n_sessions, max_batch_tokens=1024)
        sids = build_sessions(pool, shape, n, n_sessions, synth.generator(2, stream=51))
        fn_c = lambda i: pool.sk_session_query(sids[i % n_sessions], qq, out=out_q, lse=lse_q)
        fn_h = lambda i: pool.sk_session_query(sids[0], qq, out=out_q, lse=lse_q)
        ramp(fn_c, 30.0, 8)
        reps = max(40, 2 * n_sessions)
        c = stream_time_us(fn_c, reps, warm=min(n_sessions, 16))
        h = stream_time_us(fn_h, reps, warm=4)
        info = pool.sk_pool_last_launch()
        qb = query_bytes(shape, n, nq, B)
        points[str(n)] = {"cold_us": c, "hot_us": h, "sessions_rotated": n_sessions,
                          "rotation_bytes": n_sessions * n * shape.kv_bytes_per_token, "bytes_per_query": qb,
                          "kv_GBps_cold": qb / (c * 1e-6) / 1e9, "hbm_frac_cold": qb / (c * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                          "splits": info["n_splits"], "workgroups": info["workgroups"]}
        # the same with 16 query tokens (64 rows per KV head: the 64-row instance, bound by the stream alone)
        c16 = stream_time_us(lambda i: pool.sk_session_query(sids[i % n_sessions], q16, out=out16, lse=lse16), reps, warm=min(n_sessions, 16))
        h16 = stream_time_us(lambda i: pool.sk_session_query(sids[0], q16, out=out16, lse=lse16), reps, warm=4)
        qb16 = query_bytes(shape, n, 16, B)
        points[str(n)]["16_tokens"] = {"cold_us": c16, "hot_us": h16, "kv_GBps_cold": qb16 / (c16 * 1e-6) / 1e9,
                                       "hbm_frac_cold": qb16 / (c16 * 1e-6) / 1e9 / HBM_PEAK_GBPS}
        pool.close()
    ns = sorted(int(k) for k in points)
    x = np.array([points[str(k)]["bytes_per_query"] for k in ns], dtype=np.float64)
    y = np.array([points[str(k)]["cold_us"] for k in ns])
    slope, icpt = np.polyfit(x, y, 1)
    return {"query_tokens": nq, "points": points, "timing": "stream",
            "fit_cold": {"fixed_us": float(icpt), "us_per_MB": float(slope * 1e6), "implied_GBps": float(1.0 / slope / 1e3)},
            "note": "the 2,600-token rotation holds 1.36 GB in 128 sessions; shorter caches leave most CUs idle (at least 256 keys per workgroup)"}


def head_dim_64(sk, n=32768, L=256, reps=100):
    """A Llama-3.2-1B-shaped layer (bf16, 32/8 heads, head_dim 64) at 32,768 cached tokens: 256-token
    append and 16- / 32-token queries, rotating over sessions that hold more than 1 GiB together.
    Half the bytes and half the matrix work of the headline shape per token; the softmax work is the same."""
    shape = synth.Shape("bf16", 32, 8, 64)
    n_sessions = rotation_sessions(n * shape.kv_bytes_per_token)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n_sessions * (n // 16 + 2),
                   max_sessions=n_sessions, max_batch_tokens=1024)
    sids = build_sessions(pool, shape, n - L, n_sessions, synth.generator(2, stream=70))
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(synth.generator(2, stream=71), L, shape)]
    out_a = torch.empty((L, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((L, shape.n_q_heads), dtype=torch.float32, device="cuda")

    def app(i):
        sid = sids[i % n_sessions]
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        pool.sk_session_truncate(sid, n - L)
    ramp(app, 50.0, 8)
    a_us = stream_time_us(app, reps, warm=n_sessions)
    for sid in sids:
        pool.sk_session_append(sid, None, ka, va)
    res = {"cached_tokens": n, "append_tokens": L, "append_us": a_us,
           "append_tflops": append_flops(shape, n - L, L) / (a_us * 1e-6) / 1e12,
           "append_mfma_frac": append_flops(shape, n - L, L) / (a_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
           "timing": "stream (commit + attention + combine per call; queries cold)"}
    for nq in (16, 32):
        q_us = stream_time_us(lambda i: pool.sk_session_query(sids[i % n_sessions], qa[:nq], out=out_a[:nq], lse=lse_a[:nq]), reps, warm=n_sessions)
        qb = query_bytes(shape, n, nq, 16)
        res["query_%d_tokens" % nq] = {"latency_us": q_us, "kv_GBps": qb / (q_us * 1e-6) / 1e9, "hbm_frac": qb / (q_us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
    pool.close()
    return res


def fp32_small(sk, reps=200):
    """Workload 1's shape (fp32, 4/4 heads, d=64) through the fp32-FMA kernel: a 64-token append at 960
    cached tokens and a 16-token query at 1,024.  This path is the precision gate of the build, not a
    performance path; timed so that its cost is on record.  Bound: fp32 vector ALU."""
    shape = synth.CFG1
    gen = synth.generator(1, stream=60)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, 80, max_sessions=1)
    sid = build_sessions(pool, shape, 960, 1, gen, piece=64)[0]
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, 64, shape)]
    out_a = torch.empty((64, 4, 64), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((64, 4), dtype=torch.float32, device="cuda")

    def app(i):
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        pool.sk_session_truncate(sid, 960)
    a_us = stream_time_us(app, reps, warm=10)
    pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
    q_us = stream_time_us(lambda i: pool.sk_session_query(sid, qa[:16], out=out_a[:16], lse=lse_a[:16]), reps, warm=10)
    fa = append_flops(shape, 960, 64)
    fq = 4.0 * 64 * 4 * 16 * 1024
    pool.close()
    return {"append_64_at_960_us": a_us, "query_16_at_1024_us": q_us, "timing": "stream (commit + attention + combine per call)",
            "roofline": {"kernel": "sk_attn_simple<false>", "bound": "alu", "achieved": fa / (a_us * 1e-6) / 1e12,
                         "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": fa / (a_us * 1e-6) / 1e12 / FP32_VALU_PEAK_TFLOPS,
                         "traffic": None, "algorithmic_flops": fa,
                         "note": "6.5e7 flop per call: launch-bound at this size, the fraction says nothing about the kernel"},
            "query_tflops": fq / (q_us * 1e-6) / 1e12}


def sliding_window(sk, cap=32768, n_frozen=500, L=256, nq=32, n_sessions=9, steps=40):
    """The stream step of the headline workload on sessions that stay at `cap` retained tokens:
    evict the L oldest tokens behind a frozen prefix, append L, query (Alg. 1 with a full Region 1).
    Nothing is truncated back; the sessions really slide."""
    shape = synth.CFG2
    B = 16
    n_blocks = n_sessions * (cap // B + 8) + 64
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_blocks,
                   max_sessions=n_sessions, max_batch_tokens=1024)
    gen = synth.generator(2, stream=40)
    sids = build_sessions(pool, shape, cap, n_sessions, gen)
    for sid in sids:
        pool.sk_session_freeze(sid, n_frozen)
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, L, shape)]
    qq = synth.draw(gen, (nq, shape.n_q_heads, shape.head_dim), shape.dtype).cuda()
    out_a = torch.empty((L, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    out_q = torch.empty((nq, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((L, shape.n_q_heads), dtype=torch.float32, device="cuda")
    lse_q = torch.empty((nq, shape.n_q_heads), dtype=torch.float32, device="cuda")
    evict_host_s = 0.0

    def step(i):
        nonlocal evict_host_s
        sid = sids[i % n_sessions]
        t = time.perf_counter()
        pool.sk_session_evict_oldest(sid, L)
        evict_host_s += time.perf_counter() - t
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        pool.sk_session_query(sids[(i + n_sessions // 2) % n_sessions], qq, out=out_q, lse=lse_q)

    ramp(step)
    for i in range(2 * n_sessions):
        step(i)
    torch.cuda.synchronize()
    evict_host_s = 0.0
    t0 = time.perf_counter()
    for i in range(steps):
        step(2 * n_sessions + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    length = pool.sk_session_length(sids[0])
    blocks = len(pool.sk_session_block_table(sids[0]))
    pool.close()
    return {"retained_tokens": int(length), "frozen_tokens": n_frozen, "evict_append_query_ms_per_step": wall * 1e3 / steps,
            "tokens_per_s": (L + nq) * steps / wall, "evict_call_host_us_incl_wait_for_upload_slot": evict_host_s * 1e6 / steps,
            "blocks_per_session": blocks, "block_table_bytes_copied_per_evict": (blocks - (n_frozen + B - 1) // B) * 4,
            "timing": "wall"}


def fork_cost(sk, n=32768 + 7, reps=20):
    """sk_session_fork of a prefix of a 32K-token session: host call + the device work it enqueues
    (block-table upload, copy of one partly filled block), synchronised; by prefix length."""
    shape = synth.CFG2
    B = 16
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n // B + 64,
                   max_sessions=2, max_batch_tokens=1024)
    gen = synth.generator(2, stream=41)
    (src,) = build_sessions(pool, shape, n, 1, gen)
    res = {}
    for n_prefix in (1000, 8200, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            f = pool.sk_session_fork(src, n_prefix)
            torch.cuda.synchronize()
            pool.sk_session_destroy(f)
        res["prefix_%d_us" % n_prefix] = (time.perf_counter() - t0) * 1e6 / reps
    res["bytes_per_fork_at_32775"] = {"block_table": 4 * ((n + B - 1) // B), "block_copy": B * shape.kv_bytes_per_token,
                                      "kv_shared_not_copied": (n // B) * B * shape.kv_bytes_per_token}
    res["timing"] = "wall, one synchronisation per fork"
    pool.close()
    return res


def top2_sampling(sk, vocab=128256, reps=50):
    """sk_top2 (greedy token, runner-up and logit gap per row) over synthetic fp32 logits N(0, 2.5):
    64 rows (the answers of a question batch) and 1,024 rows (enough bytes to see the rate); outputs
    and workspace allocated once, outside the timing."""
    res = {"vocab": vocab}
    gen = synth.generator(6, stream=1)
    for rows in (64, 1024):
        x = (2.5 * synth.draw(gen, (rows, vocab), "f32")).cuda()
        ws = torch.empty(sk.lib().sk_top2_workspace_bytes(rows, vocab), dtype=torch.uint8, device="cuda")
        outs = sk.top2_outputs(rows, x.device)
        ramp(lambda i: sk.sk_top2(x, workspace=ws, outputs=outs), 50.0)
        us = stream_time_us(lambda i: sk.sk_top2(x, workspace=ws, outputs=outs), reps)
        res["rows_%d" % rows] = {"us_per_call": us, "GBps": rows * vocab * 4 / (us * 1e-6) / 1e9,
                                 "hbm_frac": rows * vocab * 4 / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
        if rows == 64:
            us = stream_time_us(lambda i: sk.sk_top2_static(x, outputs=outs), reps)
            res["rows_64_static_scratch_us_per_call"] = us
    res["timing"] = "stream (two kernels per call)"
    return res


def question_batch(sk, n=65536, L=256, P=16, NQ=64, Sfx=8, cycles=8):
    """Registered-question cycle at the 70B-layer shape: 256-token append, then 64 questions of
    16 shared + 8 own tokens in one batched pass; also the same questions as 64 separate queries."""
    shape = synth.CFG5
    gen = synth.generator(5)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, (n + L * (cycles + 2)) // 16 + 8,
                   max_sessions=1, max_batch_tokens=1024)
    sid = build_sessions(pool, shape, n - L, 1, gen)[0]
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, L, shape)]
    qp, kp, vp = [t.cuda() for t in synth.draw_qkv(gen, P, shape)]
    qs, ks, vs = [t.cuda() for t in synth.draw_qkv(gen, NQ * Sfx, shape)]
    r4 = lambda t: t.reshape(NQ, Sfx, t.shape[1], shape.head_dim)
    batch = lambda: pool.sk_session_query_shared_prefix(sid, qp, kp, vp, r4(qs), r4(ks), r4(vs))
    ramp(lambda i: batch(), 100.0, 4)
    # host side of one batched call (planning, list upload, launches enqueued), device idle
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    batch()
    host_us = (time.perf_counter() - t0) * 1e6
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * (cycles + 1))]
    for c in range(cycles + 1):                         # first cycle is warm-up
        ev[3 * c].record()
        pool.sk_session_append(sid, qa, ka, va)
        ev[3 * c + 1].record()
        batch()
        ev[3 * c + 2].record()
    torch.cuda.synchronize()
    app = [ev[3 * c].elapsed_time(ev[3 * c + 1]) for c in range(1, cycles + 1)]
    bat = [ev[3 * c + 1].elapsed_time(ev[3 * c + 2]) for c in range(1, cycles + 1)]
    n_end = pool.sk_session_length(sid)
    info = pool.sk_pool_last_launch()
    # the batched pass again with the library's per-kernel events
    pool.sk_pool_set_profiling(True)
    for _ in range(2):                              # a first pass creates the events and is thrown away
        batch()
    torch.cuda.synchronize()
    pool.sk_pool_read_profile()
    for _ in range(4):
        batch()
    torch.cuda.synchronize()
    prof, _, _ = pool.sk_pool_read_profile()
    pool.sk_pool_set_profiling(False)
    qfull = torch.cat([qp.expand(1, -1, -1, -1).repeat(NQ, 1, 1, 1), r4(qs)], dim=1).contiguous()
    kfull = torch.cat([kp.expand(1, -1, -1, -1).repeat(NQ, 1, 1, 1), r4(ks)], dim=1).contiguous()
    vfull = torch.cat([vp.expand(1, -1, -1, -1).repeat(NQ, 1, 1, 1), r4(vs)], dim=1).contiguous()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for rep in range(3):
        e0.record()
        for j in range(NQ):
            pool.sk_session_query(sid, qfull[j], kfull[j], vfull[j], want_lse=False)
        e1.record()
        torch.cuda.synchronize()
    indep_ms = e0.elapsed_time(e1)
    flops = 4.0 * shape.head_dim * shape.n_q_heads * (P + NQ * Sfx) * n_end
    bat_ms = float(np.mean(bat))
    attn_ms = prof["attention_ms"] / max(1, prof["calls"])
    pool.close()
    return {"cached_tokens": n, "append_ms": float(np.mean(app)), "question_batch_ms": bat_ms,
            "question_batch_tflops": flops / (bat_ms * 1e-3) / 1e12,
            "question_batch_mfma_frac": flops / (bat_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "host_call_us_device_idle": host_us, "attention_kernels_ms": attn_ms,
            "combine_kernels_ms": prof["combine_ms"] / max(1, prof["calls"]),
            "workgroups": info["workgroups"], "max_splits": info["n_splits"],
            "roofline": {"kernel": "sk_attn_bf16_d128<8,1,4> + <4,1,2> (question batch: prefix rows once, four questions per 256-row tile)",
                         "bound": "mfma", "achieved": flops / (attn_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": flops / (attn_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "algorithmic_flops": flops, "timing": "kernel (both attention launches of a call between one pair of events)"},
            "sixty_four_independent_queries_ms": indep_ms, "speedup_vs_independent": indep_ms / bat_ms,
            "timing": "stream events around each call, host launch overhead included"}


def multi_tenant(sk, n_sessions=48, steps=6):
    """Multi-tenant ragged step: 48 sessions (log-uniform 2K-64K cached tokens, 16-token blocks in a
    seeded random order); each step appends 128-1024 tokens on 16 sessions and queries 8-64 tokens
    (own K/V) on the other 32; the appended tokens are truncated away again after every step."""
    shape = synth.CFG4
    gen = synth.generator(4)
    lengths = synth.loguniform_lengths(gen, n_sessions)
    n_blocks = int(1.25 * sum((x + 15) // 16 for x in lengths)) + 16 * 80
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n_blocks, max_sessions=n_sessions,
                   max_batch_tokens=20480)
    pool.sk_pool_set_alloc_order(synth.permutation(gen, n_blocks))
    sids = [pool.sk_session_create() for _ in range(n_sessions)]
    k = synth.draw(gen, (1024, 8, 128), "bf16").cuda()
    v = synth.draw(gen, (1024, 8, 128), "bf16").cuda()
    done = [0] * n_sessions
    while any(d < x for d, x in zip(done, lengths)):     # round-robin growth: interleaved tables
        for i in range(n_sessions):
            Lp = min(1024, lengths[i] - done[i])
            if Lp > 0:
                pool.sk_session_append(sids[i], None, k[:Lp], v[:Lp])
                done[i] += Lp
    plans = []                                       # inputs of every step, made before anything is timed
    for s in range(steps):
        order = [int(x) for x in synth.permutation(gen, n_sessions)]
        ops = [sk.SK_OP_APPEND] * 16 + [sk.SK_OP_QUERY_B] * 32
        counts = [synth.randint(gen, 128, 1024) for _ in range(16)] + [synth.randint(gen, 8, 64) for _ in range(32)]
        cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        T = int(cu[-1])
        q, kk, vv = [t.cuda() for t in synth.draw_qkv(gen, T, shape)]
        out = torch.empty((T, 32, 128), dtype=torch.float32, device="cuda")
        lse = torch.empty((T, 32), dtype=torch.float32, device="cuda")
        plans.append((order, ops, counts, cu, T, q, kk, vv, out, lse))

    def step(i):
        order, ops, counts, cu, T, q, kk, vv, out, lse = plans[i % steps]
        pool.sk_batch_step([sids[j] for j in order], ops, cu, q, kk, vv, out=out, lse=lse)
        for j in range(16):                              # host only: the appended tokens go away again
            pool.sk_session_truncate(sids[order[j]], lengths[order[j]])

    ramp(step, 100.0, 2)
    # host side of a step (planning, list upload, launches enqueued) with the device idle
    host_us = []
    for i in range(steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step(i)
        host_us.append((time.perf_counter() - t0) * 1e6)
    torch.cuda.synchronize()
    times, toks, kv_bytes, flops = [], [], [], []
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(2 * steps)]
    for i in range(2 * steps):                           # every step twice, back to back, one synchronisation at the end
        evs[i][0].record()
        step(i)
        evs[i][1].record()
    torch.cuda.synchronize()
    for i in range(2 * steps):
        order, ops, counts, cu, T = plans[i % steps][:5]
        times.append(evs[i][0].elapsed_time(evs[i][1])); toks.append(T)
        flops.append(sum(4.0 * 128 * 32 * c * (lengths[j] + (c + 1) / 2.0) for c, j in zip(counts, order)))
        kv_bytes.append(sum(lengths[j] * 4096 for j in order[16:]))
    info = pool.sk_pool_last_launch()
    pool.sk_pool_set_profiling(True)
    for i in range(steps):                          # a first pass creates the events and is thrown away (one-off stalls)
        step(i)
    torch.cuda.synchronize()
    pool.sk_pool_read_profile()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    prof, attn_pc, comb_pc = pool.sk_pool_read_profile()
    pool.sk_pool_set_profiling(False)
    pool.close()
    ms = float(np.mean(times))
    attn_ms = prof["attention_ms"] / max(1, prof["calls"])
    fl = float(np.mean(flops))
    return {"sessions": n_sessions, "cached_tokens_total": int(sum(lengths)), "step_ms": ms,
            "new_tokens_per_step": float(np.mean(toks)), "tokens_per_s": float(np.mean(toks)) / (ms * 1e-3),
            "tflops": fl / (ms * 1e-3) / 1e12, "query_kv_GB_per_step": float(np.mean(kv_bytes)) / 1e9,
            "host_call_us_device_idle": float(np.mean(host_us)), "attention_kernels_ms": attn_ms,
            "combine_kernels_ms": prof["combine_ms"] / max(1, prof["calls"]),
            "per_step_plan": {"step_ms": [float(np.mean(times[i::steps])) for i in range(steps)],
                              "attention_kernels_ms": [float(x) for x in attn_pc], "combine_kernels_ms": [float(x) for x in comb_pc],
                              "append_pflops": [f / 1e15 for f in flops[:steps]]},
            "workgroups_last_step": info["workgroups"], "max_splits_last_step": info["n_splits"],
            "roofline": {"kernel": "sk_attn_bf16_d128<8,1,4> + <4,1,2> + <2,2,2> (one ragged step: 16 appends, 32 queries)",
                         "bound": "mfma", "achieved": fl / (attn_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": fl / (attn_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "algorithmic_flops": fl,
                         "timing": "kernel (the attention launches of a step between one pair of events)"},
            "timing": "stream events around each step, host planning and upload included"}


if __name__ == "__main__":
    main()
