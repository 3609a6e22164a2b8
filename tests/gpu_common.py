"""Helpers for the GPU parity tests: build a pool and an oracle session side by side, feed both
the same seeded inputs, compare element by element.

Tolerances (written here once, used by every GPU test):
  bf16 inputs, fp32 accumulation: max |gpu - oracle| <= 1e-2 and mean |gpu - oracle| <= 1e-3;
  fp32 inputs: max |gpu - oracle| <= 1e-5.
Because i.i.d. N(0,1) inputs at long context give outputs of magnitude ~sqrt(e/n) (comparable to
those absolute bounds), two tighter checks ride along so that a dropped or duplicated key range
cannot pass: per output row, max |diff| <= 2^-5 (bf16) or 1e-4 (fp32) times the row's rms (the
bf16 rounding of the softmax weights bounds the error of a row by 2^-8 max|v|, about 2^-6 of the
rms of a row that sees two keys, far less of longer rows), and |lse diff| <= 1e-3 (bf16) or 2e-5
(fp32; lse ~ ln n + 1/2 is O(10), so this is ~2 ulp of fp32 at that magnitude).  The kernel
normalises an output row by the sum of its weights as the matrix pipe sees them (rounded to bf16), so
that the row is an exact convex combination of values, and takes the lse from the sum of the
unrounded weights, kept beside it in fp32: what is left in the lse is the hardware exp2/log2 (about
1 ulp each) and the fp32 summation, a few 1e-6 relative to a sum, far inside 1e-3.
"""
import os
import numpy as np
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth

TOL = {
    "bf16": dict(max_abs=1e-2, mean_abs=1e-3, rel=2.0 ** -5, lse=1e-3),
    "f32": dict(max_abs=1e-5, mean_abs=1e-5, rel=1e-4, lse=2e-5),
}


def dev(t):
    return None if t is None else t.to("cuda:0")


def compare(name, out_gpu, lse_gpu, out_ref, lse_ref, dtype, out_is_bf16=False):
    tol = TOL[dtype]
    og = out_gpu.detach().float().cpu().numpy().astype(np.float64).reshape(out_ref.shape)
    diff = np.abs(og - out_ref)
    assert np.isfinite(og).all(), "%s: non-finite output" % name
    d = out_ref.shape[-1]
    row_rms = np.sqrt(np.mean(out_ref.reshape(-1, d) ** 2, axis=1)) + 1e-300
    row_rel = float((diff.reshape(-1, d).max(axis=1) / row_rms).max())
    max_abs, mean_abs = float(diff.max()), float(diff.mean())
    extra = 0.0
    if out_is_bf16:                      # the output itself was rounded to bf16
        extra = float(np.abs(out_ref).max()) * 2.0 ** -8
    assert max_abs <= tol["max_abs"] + extra, "%s: max abs %.3e" % (name, max_abs)
    assert mean_abs <= tol["mean_abs"] + extra, "%s: mean abs %.3e" % (name, mean_abs)
    assert row_rel <= tol["rel"] + (2.0 ** -6 if out_is_bf16 else 0.0), \
        "%s: max over rows of (max abs / row rms) %.3e" % (name, row_rel)
    if lse_gpu is not None:
        lg = lse_gpu.detach().cpu().numpy().astype(np.float64).reshape(lse_ref.shape)
        ld = float(np.abs(lg - lse_ref).max())
        assert ld <= tol["lse"], "%s: lse diff %.3e" % (name, ld)
    return max_abs, mean_abs


class Pair:
    """One GPU pool and, per session, one oracle session fed identically."""

    def __init__(self, shape: synth.Shape, block_tokens=16, n_blocks=256, max_sessions=4, max_batch_tokens=0,
                 alloc_perm=None, kv_fill=None, softmax_scale=0.0, env=None):
        self.shape = shape
        # the library reads its tuning switches from the environment when a pool is created
        old = {k: os.environ.get(k) for k in (env or {})}
        os.environ.update(env or {})
        try:
            self.pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, block_tokens, n_blocks,
                                max_sessions=max_sessions, max_batch_tokens=max_batch_tokens, kv_fill=kv_fill,
                                softmax_scale=softmax_scale)
        finally:
            for k, x in old.items():
                if x is None:
                    os.environ.pop(k, None)
                else:
                    os.environ[k] = x
        if alloc_perm is not None:
            self.pool.sk_pool_set_alloc_order(alloc_perm)
        self.oracles = {}
        self.scale = softmax_scale or None

    def create(self):
        sid = self.pool.sk_session_create()
        s = self.shape
        self.oracles[sid] = oracle.OracleSession(s.dtype, s.n_q_heads, s.n_kv_heads, s.head_dim, self.scale)
        return sid

    def append(self, sid, q, k, v, check=True, name="append", rows=None, **kw):
        out, lse = self.pool.sk_session_append(sid, dev(q), dev(k), dev(v), **kw)
        if check:
            ro, rl = self.oracles[sid].append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
            compare(name, out, lse, ro, rl, self.shape.dtype, kw.get("out_dtype", "f32") == "bf16")
        else:
            self.oracles[sid].K = np.concatenate([self.oracles[sid].K, synth.to_raw(k)])
            self.oracles[sid].V = np.concatenate([self.oracles[sid].V, synth.to_raw(v)])
        return out, lse

    def query(self, sid, q, k=None, v=None, name="query", **kw):
        out, lse = self.pool.sk_session_query(sid, dev(q), dev(k), dev(v), **kw)
        o = self.oracles[sid]
        if k is None:
            ro, rl = o.query(synth.to_raw(q))
        else:
            ro, rl = o.query(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
        compare(name, out, lse, ro, rl, self.shape.dtype, kw.get("out_dtype", "f32") == "bf16")
        return out, lse

    def check_cache(self, sid):
        """Committed K/V read back through the block table equal the oracle's cache bit for bit."""
        k, v = self.pool.sk_session_gather(sid)
        torch.cuda.synchronize()
        Kc, Vc = self.oracles[sid].cache()
        assert self.pool.sk_session_length(sid) == Kc.shape[0]
        np.testing.assert_array_equal(synth.to_raw(k.cpu()), Kc)
        np.testing.assert_array_equal(synth.to_raw(v.cpu()), Vc)

    def freeze(self, sid, n_frozen):
        self.pool.sk_session_freeze(sid, n_frozen)
        self.oracles[sid].freeze(n_frozen)

    def evict(self, sid, n_tokens):
        self.pool.sk_session_evict_oldest(sid, n_tokens)
        self.oracles[sid].evict_oldest(n_tokens)
