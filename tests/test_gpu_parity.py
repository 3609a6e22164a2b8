"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element, on
the same seeded inputs.  Sizes span several key tiles, several row tiles and ragged tails."""
import numpy as np
import pytest
import torch

import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import Pair, compare, dev

pytestmark = pytest.mark.gpu


def test_cfg1_fp32_single_session_every_step():
    """Workload 1: fp32, 4/4 heads, d=64; 16 appends of 64 tokens to 1,024 cached tokens, then 4
    non-committing queries of 16 tokens (cache-only and with own K/V); parity on every step."""
    shape = synth.CFG1
    gen = synth.generator(1)
    pr = Pair(shape, block_tokens=16, n_blocks=80, kv_fill=0xFF)       # 0xFF bytes = NaN canaries
    sid = pr.create()
    for step in range(16):
        q, k, v = synth.draw_qkv(gen, 64, shape)
        pr.append(sid, q, k, v, name="cfg1 append %d" % step)
    pr.check_cache(sid)
    before = pr.pool.kv_mem.clone()
    for i in range(4):
        q, k, v = synth.draw_qkv(gen, 16, shape)
        pr.query(sid, q, name="cfg1 query A %d" % i)
        pr.query(sid, q, k, v, name="cfg1 query B %d" % i)
        pr.query(sid, q, n_splits=3, name="cfg1 query A splits=3 %d" % i)
    torch.cuda.synchronize()
    assert torch.equal(before, pr.pool.kv_mem)
    assert pr.pool.sk_session_length(sid) == 1024


# the instances and the cache policy that the library keeps for long caches, taken at any length
LONG_CACHE_PATHS = {"SK_P128_MIN_TOKENS": "0", "SK_STREAM_MIN_TOKENS": "0"}


@pytest.mark.parametrize("block_tokens,env", [(16, None), (64, None), (16, LONG_CACHE_PATHS)])
def test_bf16_gqa_ragged_appends_and_queries(block_tokens, env):
    """Llama-3-8B-shaped layer (32/8 heads, d=128, bf16) at a size the oracle finishes in seconds:
    appends of ragged lengths (several row tiles, partial tiles, single tokens, block-straddling),
    then queries of several lengths in both modes with several split counts; once more with the
    eight-wave 128-row instance and the non-temporal loads that single-session calls of 65-128 rows
    otherwise only take from 30,720 / 65,536 cached tokens on."""
    shape = synth.CFG2
    gen = synth.generator(2, stream=1)
    pr = Pair(shape, block_tokens=block_tokens, n_blocks=4096 // block_tokens + 8, kv_fill=0xFF, max_batch_tokens=1024, env=env)
    sid = pr.create()
    for i, L in enumerate([256, 100, 7, 1, 333, 64, 15, 1000]):
        q, k, v = synth.draw_qkv(gen, L, shape)
        pr.append(sid, q, k, v, name="append %d (L=%d)" % (i, L))
    pr.check_cache(sid)
    n = pr.pool.sk_session_length(sid)
    assert n == 1776
    before = pr.pool.kv_mem.clone()
    for nq in [32, 16, 1, 5, 64, 100]:
        q, k, v = synth.draw_qkv(gen, nq, shape)
        pr.query(sid, q, name="query A nq=%d" % nq)
        pr.query(sid, q, k, v, name="query B nq=%d" % nq)
        for S in (1, 2, 7):
            pr.query(sid, q, n_splits=S, name="query A nq=%d S=%d" % (nq, S))
            pr.query(sid, q, k, v, n_splits=S, name="query B nq=%d S=%d" % (nq, S))
    torch.cuda.synchronize()
    assert torch.equal(before, pr.pool.kv_mem)


def test_bf16_first_tokens_short_context():
    """Short contexts (n < 16), where the bf16 rounding of the softmax weights weighs most, and
    the very first token of an empty session (output = its own value, to fp32 rounding)."""
    shape = synth.CFG2
    gen = synth.generator(2, stream=2)
    pr = Pair(shape, n_blocks=16, kv_fill=0xFF)
    sid = pr.create()
    q, k, v = synth.draw_qkv(gen, 1, shape)
    out, lse = pr.append(sid, q, k, v, name="first token")
    G = shape.group
    torch.cuda.synchronize()
    expect = v.float().repeat_interleave(G, dim=1)
    # one key: the weight is exp2(fma(s, c, -round(s*c))), which is 1 up to one rounding of s*c
    assert torch.allclose(out.cpu(), expect, rtol=1e-6, atol=0)
    for L in [1, 2, 3, 5]:
        q, k, v = synth.draw_qkv(gen, L, shape)
        pr.append(sid, q, k, v, name="short append L=%d" % L)
    q, k, v = synth.draw_qkv(gen, 3, shape)
    pr.query(sid, q, name="short query A")
    pr.query(sid, q, k, v, name="short query B")
    pr.check_cache(sid)


def test_bf16_output_dtype_bf16_and_no_lse():
    shape = synth.CFG2
    gen = synth.generator(2, stream=3)
    pr = Pair(shape, n_blocks=64)
    sid = pr.create()
    q, k, v = synth.draw_qkv(gen, 300, shape)
    out, lse = pr.append(sid, q, k, v, out_dtype="bf16", want_lse=False)
    assert out.dtype == torch.bfloat16 and lse is None
    q, k, v = synth.draw_qkv(gen, 32, shape)
    pr.query(sid, q, out_dtype="bf16", n_splits=4, name="bf16 out, split")
    pr.query(sid, q, out_dtype="bf16", n_splits=1, name="bf16 out, direct")


@pytest.mark.parametrize("shape", [synth.Shape("bf16", 8, 8, 64), synth.Shape("bf16", 12, 4, 128),
                                   synth.Shape("f32", 8, 2, 128), synth.Shape("bf16", 64, 8, 128),
                                   synth.Shape("bf16", 8, 8, 128), synth.Shape("bf16", 32, 2, 128),
                                   synth.Shape("bf16", 32, 1, 128)])
def test_other_shapes(shape):
    """fp32 goes through the fp32-FMA kernel; bf16 with G = 32, 16, 8, 3 and 1 through the MFMA kernel
    (a wave's 32 rows are then one token's heads, two tokens, four tokens, ten tokens and two thirds
    of another, 32 tokens), head_dim 64 included."""
    gen = synth.generator(9, stream=shape.n_q_heads)
    pr = Pair(shape, n_blocks=64)
    sid = pr.create()
    for L in [70, 3, 130]:
        q, k, v = synth.draw_qkv(gen, L, shape)
        pr.append(sid, q, k, v, name="append L=%d" % L)
    pr.check_cache(sid)
    q, k, v = synth.draw_qkv(gen, 9, shape)
    pr.query(sid, q, name="query A")
    pr.query(sid, q, k, v, n_splits=2, name="query B")


@pytest.mark.parametrize("hq,hkv,d", [(28, 4, 128), (12, 4, 128), (40, 8, 128), (6, 1, 128),
                                      (32, 8, 64), (14, 2, 64), (8, 8, 64), (16, 1, 64),
                                      (48, 1, 128), (71, 1, 64), (128, 1, 128)])
def test_group_sizes_and_head_dim_64_on_the_matrix_pipe(hq, hkv, d):
    """G = 7, 3, 5 and 6 on the matrix-pipe kernels: a tile holds floor(rows / G) tokens, its last rows
    idle, and a token's heads can lie in two waves.  head_dim 64 (G = 4, 7, 1, 16) on the same kernels:
    half of every K row and of the V^T dims of a tile.  Multi-query shapes with 48, 71 and 128 heads on one
    KV head: a token then fills most of a tile, or two waves and more.  Appends over several row tiles, queries that
    take the 64-, 128- and 256-row instances in both modes and with several split counts, a sliding
    window, a batched step and a question batch."""
    shape = synth.Shape("bf16", hq, hkv, d)
    G = hq // hkv
    gen = synth.generator(9, stream=100 + hq)
    pr = Pair(shape, n_blocks=200, max_sessions=3, max_batch_tokens=1024, kv_fill=0xFF)
    sid = pr.create()
    for L in [300, 1, 37, 150]:
        q, k, v = synth.draw_qkv(gen, L, shape)
        pr.append(sid, q, k, v, name="append L=%d" % L)
        assert pr.pool.sk_pool_last_launch()["kernel_variant"] != 0
    pr.check_cache(sid)
    for rows in (64, 128, 256, 300):
        nq = max(1, rows // G)
        q, k, v = synth.draw_qkv(gen, nq, shape)
        pr.query(sid, q, name="query A nq=%d" % nq)
        assert pr.pool.sk_pool_last_launch()["kernel_variant"] != 0
        for S in (1, 3):
            pr.query(sid, q, k, v, n_splits=S, name="query B nq=%d S=%d" % (nq, S))
    pr.freeze(sid, 33)
    pr.evict(sid, 101)
    q, k, v = synth.draw_qkv(gen, 21, shape)
    pr.query(sid, q, name="query A behind a hole")
    pr.append(sid, q, k, v, name="append behind a hole")
    pr.check_cache(sid)
    # batched step: an append on a second session and a query on the first
    other = pr.create()
    counts = [90, 17]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    q, k, v = synth.draw_qkv(gen, int(cu[-1]), shape)
    out, lse = pr.pool.sk_batch_step([other, sid], [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B], cu, dev(q), dev(k), dev(v))
    qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
    ro0, rl0 = pr.oracles[other].append(qr[:90], kr[:90], vr[:90])
    ro1, rl1 = pr.oracles[sid].query(qr[90:], kr[90:], vr[90:])
    compare("batch step", out, lse, np.concatenate([ro0, ro1]), np.concatenate([rl0, rl1]), shape.dtype)
    pr.check_cache(other)
    # question batch
    P_, NQ, Sfx = 16, 5, 8
    qp, kp, vp = synth.draw_qkv(gen, P_, shape)
    qs, ks, vs = [t.reshape(NQ, Sfx, t.shape[1], d) for t in synth.draw_qkv(gen, NQ * Sfx, shape)]
    op, lp, os_, ls = pr.pool.sk_session_query_shared_prefix(sid, dev(qp), dev(kp), dev(vp), dev(qs), dev(ks), dev(vs))
    rop, rlp, ros, rls = pr.oracles[sid].query_shared_prefix(synth.to_raw(qp), synth.to_raw(kp), synth.to_raw(vp),
                                                             synth.to_raw(qs), synth.to_raw(ks), synth.to_raw(vs))
    compare("question batch, prefix", op, lp, rop, rlp, shape.dtype)
    compare("question batch, suffixes", os_.reshape(NQ * Sfx, hq, d), ls.reshape(NQ * Sfx, hq),
            ros.reshape(NQ * Sfx, hq, d), rls.reshape(NQ * Sfx, hq), shape.dtype)


def test_large_logits_and_needle():
    """Queries scaled by 8 (scores of magnitude ~8 sigma) prove the max subtraction; a planted key
    aligned with the query at several positions (first, last, block and split boundaries) must
    return that key's value: exact retrieval from mid-context (the paper's Q6 idea, Sec. 4.3)."""
    shape = synth.CFG2
    gen = synth.generator(2, stream=4)
    n = 2048
    for pos in [0, 15, 16, 511, 512, 1023, 1024, n - 1]:
        pr = Pair(shape, n_blocks=n // 16 + 4)
        sid = pr.create()
        q, k, v = synth.draw_qkv(gen, n, shape)
        qq, _, _ = synth.draw_qkv(gen, 4, shape, scale=8.0)
        # plant: key at `pos` of KV head 2 is 4x query row (token 1, head 9); head 9 reads KV head 2
        k[pos, 2] = (4.0 * qq[1, 9].float()).to(torch.bfloat16)
        pr.append(sid, q[:1024], k[:1024], v[:1024], check=False)
        pr.append(sid, q[1024:], k[1024:], v[1024:], check=False)
        out, _ = pr.query(sid, qq, n_splits=4, name="needle pos=%d" % pos)
        torch.cuda.synchronize()
        got = out[1, 9].cpu()
        assert torch.allclose(got, v[pos, 2].float(), atol=1e-2), "needle at %d not retrieved" % pos


@pytest.mark.parametrize("scale", [0.05, 0.2])
def test_custom_softmax_scale(scale):
    """Eq. 1's 1/sqrt(d_k) is the default, not the only scale: a pool created with softmax_scale set
    (0.05 flattens the weights, 0.2 sharpens them well beyond 1/sqrt(128) = 0.088) against an oracle
    given the same number, through every entry point: appends (several row tiles, split merge),
    cache-only and own-K/V queries with several split counts, a ragged multi-session step and a
    shared-prefix question batch; fp32 pool once as well."""
    import oracle
    import paper_2605_13784_amd as sk
    shape = synth.CFG2
    gen = synth.generator(2, stream=300 + int(scale * 100))
    pr = Pair(shape, block_tokens=16, n_blocks=400, max_sessions=3, max_batch_tokens=1024, softmax_scale=scale)
    a, b = pr.create(), pr.create()
    for sid, Ls in ((a, [300, 700, 41]), (b, [90, 1])):
        for L in Ls:
            q, k, v = synth.draw_qkv(gen, L, shape)
            pr.append(sid, q, k, v, name="scale %.2f append %d" % (scale, L))
    for nq in (32, 5):
        q, k, v = synth.draw_qkv(gen, nq, shape)
        for S in (0, 1, 5):
            pr.query(a, q, n_splits=S, name="scale %.2f query A nq=%d S=%d" % (scale, nq, S))
            pr.query(a, q, k, v, n_splits=S, name="scale %.2f query B nq=%d S=%d" % (scale, nq, S))
    # ragged step: append on b, own-K/V query on a
    counts = [130, 20]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    q, k, v = synth.draw_qkv(gen, int(cu[-1]), shape)
    out, lse = pr.pool.sk_batch_step([b, a], [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B], cu, dev(q), dev(k), dev(v))
    qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
    ro, rl = pr.oracles[b].append(qr[:130], kr[:130], vr[:130])
    compare("scale %.2f step append" % scale, out[:130], lse[:130], ro, rl, shape.dtype)
    ro, rl = pr.oracles[a].query(qr[130:], kr[130:], vr[130:])
    compare("scale %.2f step query" % scale, out[130:], lse[130:], ro, rl, shape.dtype)
    pr.check_cache(b)
    # question batch on a
    P, NQ, Sfx = 16, 6, 8
    qp, kp, vp = synth.draw_qkv(gen, P, shape)
    qs, ks, vs = synth.draw_qkv(gen, NQ * Sfx, shape)
    r4 = lambda t: t.reshape(NQ, Sfx, t.shape[1], shape.head_dim)
    op, lp, os_, ls = pr.pool.sk_session_query_shared_prefix(a, dev(qp), dev(kp), dev(vp), dev(r4(qs)), dev(r4(ks)), dev(r4(vs)))
    rop, rlp, ros, rls = pr.oracles[a].query_shared_prefix(synth.to_raw(qp), synth.to_raw(kp), synth.to_raw(vp),
                                                           synth.to_raw(r4(qs)), synth.to_raw(r4(ks)), synth.to_raw(r4(vs)))
    compare("scale %.2f prefix" % scale, op, lp, rop, rlp, shape.dtype)
    compare("scale %.2f suffixes" % scale, os_, ls, ros, rls, shape.dtype)
    # the fp32 path takes the scale the same way
    pf = Pair(synth.CFG1, block_tokens=16, n_blocks=40, softmax_scale=scale)
    s = pf.create()
    q, k, v = synth.draw_qkv(gen, 100, synth.CFG1)
    pf.append(s, q, k, v, name="fp32 scale %.2f append" % scale)
    q, k, v = synth.draw_qkv(gen, 9, synth.CFG1)
    pf.query(s, q, n_splits=3, name="fp32 scale %.2f query A" % scale)
    pf.query(s, q, k, v, name="fp32 scale %.2f query B" % scale)
