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

WORKLOADS = {
    # name: (shape, cached tokens at query time, append chunk, query tokens)
    "cfg2_llama3_8b_layer_32k": (synth.CFG2, 32768, 256, 32),
    "cfg3_long_context_128k": (synth.CFG3, 131072, 512, 16),
}


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
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg2_llama3_8b_layer_32k", choices=sorted(WORKLOADS))
    ap.add_argument("--block-tokens", type=int, default=16)
    ap.add_argument("--sessions", type=int, default=0, help="sessions to rotate over (0: enough for > 1 GiB of K/V)")
    ap.add_argument("--hot", action="store_true", help="one session only: K/V may stay in the last-level cache")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    shape, n, L, nq = WORKLOADS[args.workload]
    B = args.block_tokens
    kv_per_session = n * shape.kv_bytes_per_token
    n_sessions = 1 if args.hot else (args.sessions or max(5, -(-(1 << 30) // kv_per_session) + 1))
    blocks_per_session = (n + B - 1) // B + 2
    # truncated blocks queue behind the free ones, so keep a margin of free blocks
    n_blocks = n_sessions * blocks_per_session + 4 * (L // B + 2)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_blocks,
                   max_sessions=n_sessions, max_batch_tokens=max(L, nq, 1024))
    gen = synth.generator(2 if "cfg2" in args.workload else 3)
    n0 = n - L
    sids = build_sessions(pool, shape, n0, L, n_sessions, gen)
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

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # same steps again with HIP events around the kernels (recorded by the library on the
    # stream the kernels run on)
    pool.sk_pool_set_profiling(True)
    for i in range(args.steps):
        step(args.warmup + args.steps + i)
    torch.cuda.synchronize()
    _, attn_ms, comb_ms = pool.sk_pool_read_profile()
    pool.sk_pool_set_profiling(False)
    app_attn = np.array(attn_ms[0::2]); app_comb = np.array(comb_ms[0::2])
    qry_attn = np.array(attn_ms[1::2]); qry_comb = np.array(comb_ms[1::2])
    info = pool.sk_pool_last_launch()

    qb = query_bytes(shape, n, nq, B)
    af = append_flops(shape, n0, L)
    q_kernel_us = float(qry_attn.mean() * 1e3)
    q_total_us = float((qry_attn + qry_comb).mean() * 1e3)
    a_kernel_us = float(app_attn.mean() * 1e3)
    a_total_us = float((app_attn + app_comb).mean() * 1e3)
    roof_q = {"kernel": "sk_attn_bf16_d128 (query, split-KV partial)", "bound": "hbm",
              "achieved": qb / (q_kernel_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
              "frac": qb / (q_kernel_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, "traffic": None,
              "avg_kernel_us": q_kernel_us, "algorithmic_bytes": qb}
    roof_a = {"kernel": "sk_attn_bf16_d128 (append, causal over cache + chunk)", "bound": "mfma",
              "achieved": af / (a_kernel_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
              "frac": af / (a_kernel_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
              "avg_kernel_us": a_kernel_us, "algorithmic_flops": af}
    dominant = roof_a if a_kernel_us >= q_kernel_us else roof_q

    res = {
        "metric": "stream-step throughput: %d-token append + %d-token query at %d cached tokens" % (L, nq, n),
        "value": (L + nq) * args.steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "n_q_heads": shape.n_q_heads, "n_kv_heads": shape.n_kv_heads,
                   "head_dim": shape.head_dim, "cached_tokens": n, "append_tokens": L, "query_tokens": nq,
                   "block_tokens": B, "sessions_rotated": n_sessions, "cache": "hot" if args.hot else "cold",
                   "query_splits": info["n_splits"], "query_workgroups": info["workgroups"]},
        "query": {"latency_us": q_total_us, "kernel_us": q_kernel_us, "combine_us": q_total_us - q_kernel_us,
                  "kv_GBps": qb / (q_total_us * 1e-6) / 1e9, "hbm_frac_incl_combine": qb / (q_total_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                  "p50_us": float(np.median(qry_attn + qry_comb) * 1e3), "max_us": float((qry_attn + qry_comb).max() * 1e3)},
        "append": {"latency_us": a_total_us, "kernel_us": a_kernel_us, "tokens_per_s": L / (a_total_us * 1e-6),
                   "tflops": af / (a_total_us * 1e-6) / 1e12, "mfma_frac": af / (a_total_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "roofline": dominant, "roofline_query": roof_q, "roofline_append": roof_a,
    }
    if not args.no_cpu_baseline:
        rows = args.cpu_rows or (1024 if n <= 32768 else 256)
        res["cpu_baseline"] = cpu_baseline(shape, n, L, nq, synth.generator(7), rows)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


if __name__ == "__main__":
    main()
