#!/usr/bin/env python3
"""Benchmark of the stateful-session attention path on one MI355X.

A step is one pass of the whole hot path on the Llama-3-8B-shaped layer (bf16, 32 query heads,
8 KV heads, head_dim 128) at 32,768 cached tokens: block allocation, K/V commit of a 256-token
chunk, the chunk's causal attention over cache + chunk (data plane), then a 32-token
non-committing query over the 32,768 cached tokens with its cross-split combine (query plane).
The session is then truncated back (host metadata only) so every step sees the same lengths.
Steps rotate over several sessions whose caches together exceed the 256 MB last-level cache, so
the cached K/V come from HBM ("cold"); --hot keeps one session.

Prints ONE JSON line.  `value` is tokens per second through the whole step; the per-plane
figures the path is judged on (query latency and KV GB/s, append tokens/s and TFLOP/s) are in
"query" and "append"; "roofline" describes the kernel that takes most of the step.
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

# HBM bytes per dispatch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (fetch + write),
# scaled by a 1 GiB device copy; see profiles/bench_cfg2_attention_kernels.md for the runs.
# Keyed by (workload, block_tokens, cache state); other configurations report null.
MEASURED_HBM_TRAFFIC = {
    ("cfg2_llama3_8b_layer_32k", 16, "cold"): {
        "query": {"fetch_bytes": 134.94e6, "write_bytes": 17.04e6, "total_bytes": 151.98e6},
        "append": {"fetch_bytes": 136.93e6, "write_bytes": 34.08e6, "total_bytes": 171.01e6},
    },
}

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


def build_sessions(pool, shape, n0, chunk, n_sessions, gen):
    """Grows n_sessions sessions to n0 cached tokens by `chunk`-token appends (same data for
    every session; each session owns different physical blocks)."""
    sids = [pool.sk_session_create() for _ in range(n_sessions)]
    done = 0
    while done < n0:
        L = min(chunk, n0 - done)
        q, k, v = synth.draw_qkv(gen, L, shape)
        q, k, v = q.cuda(), k.cuda(), v.cuda()
        for sid in sids:
            pool.sk_session_append(sid, q, k, v, want_lse=False)
        done += L
    torch.cuda.synchronize()
    return sids


def query_bytes(shape, n, nq, block_tokens):
    return n * shape.kv_bytes_per_token + nq * shape.n_q_heads * shape.head_dim * (2 + 4) + (n + block_tokens - 1) // block_tokens * 4


def append_flops(shape, n_before, L):
    return 4.0 * shape.head_dim * shape.n_q_heads * L * (n_before + (L + 1) / 2.0)


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
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads (128K context, question batch, multi-tenant step, sliding window)")
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

    main_res = stream_workload(sk, args.workload, args, args.steps, args.warmup, calibrate=args.copy_calibration)
    shape, n, L, nq = WORKLOADS[args.workload]
    res = {
        "metric": "stream-step throughput: %d-token append + %d-token query at %d cached tokens" % (L, nq, n),
        "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": main_res["config"], "query": main_res["query"], "append": main_res["append"],
        "roofline": main_res["roofline"], "roofline_query": main_res["roofline_query"],
        "roofline_append": main_res["roofline_append"],
    }
    if not args.no_extras:
        extras = {}
        other = "cfg3_long_context_128k" if "cfg2" in args.workload else "cfg2_llama3_8b_layer_32k"
        r = stream_workload(sk, other, args, max(10, args.steps // 2), 4)
        extras[other] = {k: r[k] for k in ("ms_per_step", "query", "append", "roofline_query", "roofline_append")}
        if other == "cfg3_long_context_128k" and args.block_tokens != 256:
            # the workload fixes no block size; 256-token blocks are the faster layout for small queries
            big = argparse.Namespace(**vars(args)); big.block_tokens = 256
            r = stream_workload(sk, other, big, max(10, args.steps // 2), 4)
            extras[other + "_256_token_blocks"] = {k: r[k] for k in ("ms_per_step", "config", "query", "roofline_query")}
        extras["cfg5_question_batch_64k"] = question_batch(sk)
        extras["cfg4_multi_tenant_step"] = multi_tenant(sk)
        extras["sliding_window_32k"] = sliding_window(sk)
        extras["fork_cost"] = fork_cost(sk)
        extras["top2_sampling"] = top2_sampling(sk)
        res["extras"] = extras
    if not args.no_cpu_baseline:
        rows = args.cpu_rows or ((L + nq) * shape.n_q_heads if n <= 32768 else 4096)
        res["cpu_baseline"] = cpu_baseline(shape, n, L, nq, synth.generator(7), rows)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


def stream_workload(sk, name, args, steps, warmup, calibrate=False):
    """Times `steps` stream steps (append + query + truncate back) of one workload, then the same
    steps again with the library's HIP-event timing of the kernels switched on."""
    shape, n, L, nq = WORKLOADS[name]
    B = args.block_tokens
    kv_per_session = n * shape.kv_bytes_per_token
    n_sessions = 1 if args.hot else (args.sessions or max(5, -(-(1 << 30) // kv_per_session) + 1))
    blocks_per_session = (n + B - 1) // B + 2
    # truncated blocks queue behind the free ones, so keep a margin of free blocks
    n_blocks = n_sessions * blocks_per_session + 4 * (L // B + 2)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_blocks,
                   max_sessions=n_sessions, max_batch_tokens=max(L, nq, 1024))
    gen = synth.generator(2 if "cfg2" in name else 3)
    n0 = n - L
    sids = build_sessions(pool, shape, n0, 1024, n_sessions, gen)
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, L, shape)]
    qq = synth.draw(gen, (nq, shape.n_q_heads, shape.head_dim), shape.dtype).cuda()
    out_a = torch.empty((L, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((L, shape.n_q_heads), dtype=torch.float32, device="cuda")
    out_q = torch.empty((nq, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device="cuda")
    lse_q = torch.empty((nq, shape.n_q_heads), dtype=torch.float32, device="cuda")

    def step(i):
        sid = sids[i % n_sessions]
        pool.sk_session_append(sid, qa, ka, va, out=out_a, lse=lse_a)
        pool.sk_session_query(sid, qq, out=out_q, lse=lse_q, n_splits=args.n_splits)
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
    pool.sk_pool_set_profiling(True)
    for i in range(steps):
        step(warmup + steps + i)
    torch.cuda.synchronize()
    _, attn_ms, comb_ms = pool.sk_pool_read_profile()
    pool.sk_pool_set_profiling(False)
    app_attn = np.array(attn_ms[0::2]); app_comb = np.array(comb_ms[0::2])
    qry_attn = np.array(attn_ms[1::2]); qry_comb = np.array(comb_ms[1::2])
    info = pool.sk_pool_last_launch()
    pool.close()

    qb = query_bytes(shape, n, nq, B)
    af = append_flops(shape, n0, L)
    q_kernel_us = float(qry_attn.mean() * 1e3)
    q_total_us = float((qry_attn + qry_comb).mean() * 1e3)
    a_kernel_us = float(app_attn.mean() * 1e3)
    a_total_us = float((app_attn + app_comb).mean() * 1e3)
    traffic = MEASURED_HBM_TRAFFIC.get((name, B, "cold" if not args.hot else "hot"), {})
    def hbm(kind):      # "traffic" = measured HBM bytes per launch (fetch + write), null when not measured
        t = traffic.get(kind)
        return {"traffic": None} if t is None else {"traffic": t["total_bytes"], "traffic_fetch_bytes": t["fetch_bytes"],
                                                    "traffic_write_bytes": t["write_bytes"]}
    roof_q = {"kernel": "sk_attn_bf16_d128 (query, split-KV partial)", "bound": "hbm",
              "achieved": qb / (q_kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
              "frac": qb / (q_kernel_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, **hbm("query"),
              "avg_kernel_us": q_kernel_us, "algorithmic_bytes": qb}
    roof_a = {"kernel": "sk_attn_bf16_d128 (append, causal over cache + chunk)", "bound": "mfma",
              "achieved": af / (a_kernel_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
              "frac": af / (a_kernel_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, **hbm("append"),
              "avg_kernel_us": a_kernel_us, "algorithmic_flops": af,
              "timing": "HIP events recorded by the library around the kernel on its stream, in a repeat of the timed "
                        "steps; an event pair adds 3-6 us to what rocprofv3 measures for the same launches"}
    return {
        "tokens_per_s": (L + nq) * steps / wall, "ms_per_step": wall * 1e3 / steps,
        "config": {"workload": name, "n_q_heads": shape.n_q_heads, "n_kv_heads": shape.n_kv_heads,
                   "head_dim": shape.head_dim, "cached_tokens": n, "append_tokens": L, "query_tokens": nq,
                   "block_tokens": B, "sessions_rotated": n_sessions, "cache": "hot" if args.hot else "cold",
                   "query_splits": info["n_splits"], "query_workgroups": info["workgroups"]},
        "query": {"latency_us": q_total_us, "kernel_us": q_kernel_us, "combine_us": q_total_us - q_kernel_us,
                  "kv_GBps": qb / (q_total_us * 1e-6) / 1e9, "hbm_frac_incl_combine": qb / (q_total_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                  "p50_us": float(np.median(qry_attn + qry_comb) * 1e3), "max_us": float((qry_attn + qry_comb).max() * 1e3)},
        "append": {"latency_us": a_total_us, "kernel_us": a_kernel_us, "tokens_per_s": L / (a_total_us * 1e-6),
                   "tflops": af / (a_total_us * 1e-6) / 1e12, "mfma_frac": af / (a_total_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "roofline": roof_a if a_kernel_us >= q_kernel_us else roof_q, "roofline_query": roof_q, "roofline_append": roof_a,
    }


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
    sids = build_sessions(pool, shape, cap, 1024, n_sessions, gen)
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
        pool.sk_session_query(sid, qq, out=out_q, lse=lse_q)

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
            "blocks_per_session": blocks, "block_table_bytes_copied_per_evict": (blocks - (n_frozen + B - 1) // B) * 4}


def fork_cost(sk, n=32768 + 7, reps=20):
    """sk_session_fork of a prefix of a 32K-token session: host call + the device work it enqueues
    (block-table upload, copy of one partly filled block), synchronised; by prefix length."""
    shape = synth.CFG2
    B = 16
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n // B + 64,
                   max_sessions=2, max_batch_tokens=1024)
    gen = synth.generator(2, stream=41)
    (src,) = build_sessions(pool, shape, n, 1024, 1, gen)
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
    pool.close()
    return res


def top2_sampling(sk, vocab=128256, reps=50):
    """sk_top2 (greedy token, runner-up and logit gap per row) over synthetic fp32 logits N(0, 2.5):
    64 rows (the answers of a question batch) and 1,024 rows (enough bytes to see the rate)."""
    res = {"vocab": vocab}
    gen = synth.generator(6, stream=1)
    for rows in (64, 1024):
        x = (2.5 * synth.draw(gen, (rows, vocab), "f32")).cuda()
        ws = torch.empty(sk.lib().sk_top2_workspace_bytes(rows, vocab), dtype=torch.uint8, device="cuda")
        ramp(lambda i: sk.sk_top2(x, workspace=ws), 50.0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            sk.sk_top2(x, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        res["rows_%d" % rows] = {"us_per_call": us, "GBps": rows * vocab * 4 / (us * 1e-6) / 1e9,
                                 "hbm_frac": rows * vocab * 4 / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
    res["timing"] = "torch events on the launch stream around back-to-back calls (two kernels each), output allocation included"
    return res


def question_batch(sk, n=65536, L=256, P=16, NQ=64, Sfx=8, cycles=8):
    """Registered-question cycle at the 70B-layer shape: 256-token append, then 64 questions of
    16 shared + 8 own tokens in one batched pass; also the same questions as 64 separate queries."""
    shape = synth.CFG5
    gen = synth.generator(5)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, (n + L * (cycles + 2)) // 16 + 8,
                   max_sessions=1, max_batch_tokens=1024)
    sid = build_sessions(pool, shape, n - L, 1024, 1, gen)[0]
    qa, ka, va = [t.cuda() for t in synth.draw_qkv(gen, L, shape)]
    qp, kp, vp = [t.cuda() for t in synth.draw_qkv(gen, P, shape)]
    qs, ks, vs = [t.cuda() for t in synth.draw_qkv(gen, NQ * Sfx, shape)]
    r4 = lambda t: t.reshape(NQ, Sfx, t.shape[1], shape.head_dim)
    ramp(lambda i: pool.sk_session_query_shared_prefix(sid, qp, kp, vp, r4(qs), r4(ks), r4(vs)), 100.0, 4)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * (cycles + 1))]
    for c in range(cycles + 1):                         # first cycle is warm-up
        ev[3 * c].record()
        pool.sk_session_append(sid, qa, ka, va)
        ev[3 * c + 1].record()
        pool.sk_session_query_shared_prefix(sid, qp, kp, vp, r4(qs), r4(ks), r4(vs))
        ev[3 * c + 2].record()
    torch.cuda.synchronize()
    app = [ev[3 * c].elapsed_time(ev[3 * c + 1]) for c in range(1, cycles + 1)]
    bat = [ev[3 * c + 1].elapsed_time(ev[3 * c + 2]) for c in range(1, cycles + 1)]
    n_end = pool.sk_session_length(sid)
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
    pool.close()
    return {"cached_tokens": n, "append_ms": float(np.mean(app)), "question_batch_ms": float(np.mean(bat)),
            "question_batch_tflops": flops / (np.mean(bat) * 1e-3) / 1e12,
            "question_batch_mfma_frac": flops / (np.mean(bat) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "sixty_four_independent_queries_ms": indep_ms, "speedup_vs_independent": indep_ms / float(np.mean(bat)),
            "timing": "torch events on the launch stream, host launch overhead included"}


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
    pool.close()
    ms = float(np.mean(times))
    return {"sessions": n_sessions, "cached_tokens_total": int(sum(lengths)), "step_ms": ms,
            "new_tokens_per_step": float(np.mean(toks)), "tokens_per_s": float(np.mean(toks)) / (ms * 1e-3),
            "tflops": float(np.mean(flops)) / (ms * 1e-3) / 1e12, "query_kv_GB_per_step": float(np.mean(kv_bytes)) / 1e9,
            "timing": "torch events on the launch stream, host planning and upload included"}


if __name__ == "__main__":
    main()
