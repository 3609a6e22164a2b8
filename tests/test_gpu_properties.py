"""Properties the paper fixes for the stateful path, checked on the GPU:
  I1  appending chunk by chunk == one causal pass over the whole stream (Sec. 2, Sec. 3.4);
  I2  a query leaves the cache untouched (Sec. 3.3 Region 2; Sec. 3.9.3);
  I3  a query does not depend on how the cache was built (Sec. 3.2 "complexity profile");
  I4  Extend-then-Clear == a non-committing query with own K/V (Sec. 3.9.3);
plus what this implementation promises on top: run-to-run determinism and independence of the
physical block placement."""
import numpy as np
import pytest
import torch

import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import TOL, Pair, compare, dev

pytestmark = pytest.mark.gpu
SHAPE = synth.CFG2


def _stream(gen, T):
    return synth.draw_qkv(gen, T, SHAPE)


def test_chunking_history_does_not_matter():
    """I1 + I3: three histories of the same 1,500-token stream give a bit-identical cache, outputs
    within tolerance of the oracle for every token, a bit-identical query result and the same
    launch geometry."""
    gen = synth.generator(2, stream=10)
    T = 1500
    q, k, v = _stream(gen, T)
    qq, kq, vq = _stream(gen, 32)
    results = []
    for cuts in ([0, 1500], [0, 256, 512, 768, 1024, 1280, 1500], [0, 1, 17, 300, 301, 900, 1499, 1500]):
        pr = Pair(SHAPE, n_blocks=128, max_batch_tokens=2048)
        sid = pr.create()
        for a, b in zip(cuts[:-1], cuts[1:]):
            pr.append(sid, q[a:b], k[a:b], v[a:b], name="append [%d,%d)" % (a, b))
        pr.check_cache(sid)
        kc, vc = pr.pool.sk_session_gather(sid)
        oa, la = pr.query(sid, qq, name="query A")
        geo_a = pr.pool.sk_pool_last_launch()
        ob, lb = pr.query(sid, qq, kq, vq, name="query B")
        torch.cuda.synchronize()
        results.append((kc.cpu(), vc.cpu(), oa.cpu(), la.cpu(), ob.cpu(), lb.cpu(), geo_a))
    for r in results[1:]:
        for x, y in zip(r[:6], results[0][:6]):
            assert torch.equal(x, y)
        assert r[6] == results[0][6]


def test_query_is_pure_and_deterministic():
    """I2 + determinism: kv_mem, tables and lengths are unchanged by queries of both kinds and by a
    question batch; the same call twice gives the same bits."""
    gen = synth.generator(2, stream=11)
    pr = Pair(SHAPE, n_blocks=200, max_sessions=2)
    a, b = pr.create(), pr.create()
    for sid, T in ((a, 1111), (b, 700)):
        q, k, v = _stream(gen, T)
        pr.append(sid, q, k, v, check=False)
    torch.cuda.synchronize()
    mem0 = pr.pool.kv_mem.clone()
    tab0 = [pr.pool.sk_session_block_table(s) for s in (a, b)]
    qq, kq, vq = (dev(t) for t in _stream(gen, 48))
    outs = []
    for rep in range(2):
        o1, l1 = pr.pool.sk_session_query(a, qq)
        o2, l2 = pr.pool.sk_session_query(a, qq, kq, vq, n_splits=3)
        o3 = pr.pool.sk_session_query_shared_prefix(a, qq[:16], kq[:16], vq[:16], qq[16:].reshape(4, 8, 32, 128),
                                                    kq[16:].reshape(4, 8, 8, 128), vq[16:].reshape(4, 8, 8, 128))
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (o1, l1, o2, l2, o3[0], o3[2])])
    for x, y in zip(outs[0], outs[1]):
        assert torch.equal(x, y)
    assert torch.equal(mem0, pr.pool.kv_mem)
    assert tab0 == [pr.pool.sk_session_block_table(s) for s in (a, b)]
    assert [pr.pool.sk_session_length(s) for s in (a, b)] == [1111, 700]


def test_physical_block_placement_does_not_matter():
    """Same logical cache, blocks handed out in order vs in a seeded random order: identical bits out."""
    gen = synth.generator(2, stream=12)
    q, k, v = _stream(gen, 2000)
    qq, kq, vq = _stream(gen, 40)
    res = []
    for perm in (None, synth.permutation(synth.generator(2, stream=13), 160)):
        pr = Pair(SHAPE, n_blocks=160, alloc_perm=perm, max_batch_tokens=2048)
        sid = pr.create()
        o1, l1 = pr.append(sid, q[:900], k[:900], v[:900])
        o2, l2 = pr.append(sid, q[900:], k[900:], v[900:])
        o3, l3 = pr.query(sid, qq, n_splits=4)
        o4, l4 = pr.query(sid, qq, kq, vq)
        torch.cuda.synchronize()
        res.append([t.cpu() for t in (o1, l1, o2, l2, o3, l3, o4, l4)])
        if perm is not None:
            assert pr.pool.sk_session_block_table(sid) != sorted(pr.pool.sk_session_block_table(sid))
    for x, y in zip(*res):
        assert torch.equal(x, y)


def test_extend_then_clear_equals_noncommitting_query():
    """I4: append the question tokens, read the output, SeqRemove them (truncate) - the paper's literal
    cycle - against the query that never commits.  Outputs agree (different tile alignment, so within
    a tight tolerance rather than bit for bit) and the cache is back to its bytes."""
    gen = synth.generator(2, stream=14)
    pr = Pair(SHAPE, n_blocks=100)
    sid = pr.create()
    q, k, v = _stream(gen, 1000)
    pr.append(sid, q, k, v, check=False)
    qq, kq, vq = _stream(gen, 24)
    ob, lb = pr.query(sid, qq, kq, vq, name="non-committing")
    k0, v0 = pr.pool.sk_session_gather(sid)
    free0 = pr.pool.sk_pool_blocks_free()
    oa, la = pr.pool.sk_session_append(sid, dev(qq), dev(kq), dev(vq))
    assert pr.pool.sk_session_length(sid) == 1024
    pr.pool.sk_session_truncate(sid, 1000)
    k1, v1 = pr.pool.sk_session_gather(sid)
    torch.cuda.synchronize()
    assert pr.pool.sk_session_length(sid) == 1000 and pr.pool.sk_pool_blocks_free() == free0
    assert torch.equal(k0, k1) and torch.equal(v0, v1)
    # two evaluations in different key orders: each LSE carries its own rounding of the weights
    assert float((oa - ob).abs().max()) <= 2e-3 and float((la - lb).abs().max()) <= TOL[SHAPE.dtype]["lse"]
    # the session keeps working after the truncate: next append lands on the same positions
    q2, k2, v2 = _stream(gen, 50)
    pr.append(sid, q2, k2, v2, name="append after truncate")
    pr.check_cache(sid)


def test_latency_scales_with_bytes_not_with_history():
    """Not a timing test: the work the library launches for a query is a function of (n, |q|, splits)
    only - same workgroups, same splits - whether the cache came from 2 or from 40 appends."""
    gen = synth.generator(2, stream=15)
    geos = []
    for pieces in (2, 40):
        pr = Pair(SHAPE, n_blocks=300, max_batch_tokens=4096)
        sid = pr.create()
        _, k, v = _stream(gen, 4000)
        step = 4000 // pieces
        for a in range(0, 4000, step):
            pr.pool.sk_session_append(sid, None, dev(k[a:a + step]), dev(v[a:a + step]))
        qq = dev(synth.draw(gen, (32, 32, 128), "bf16"))
        pr.pool.sk_session_query(sid, qq)
        geos.append(pr.pool.sk_pool_last_launch())
        st = pr.pool.sk_pool_get_stats()
        assert st["tokens_appended"] == 4000 and st["tokens_queried"] == 32
    assert geos[0] == geos[1]


def test_two_pools_on_two_streams():
    """The library enqueues on the caller's stream and orders its own uploads and copies there: two
    pools driven alternately on two non-default streams (appends with eviction and a fork on one,
    batched steps on the other, while the default stream is kept busy) give what the oracle gives."""
    gen = synth.generator(2, stream=15)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    busy = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    p1 = Pair(SHAPE, n_blocks=300, max_sessions=3, max_batch_tokens=2048)
    p2 = Pair(SHAPE, block_tokens=64, n_blocks=100, max_sessions=3, max_batch_tokens=2048)
    a = p1.create()
    b, c = p2.create(), p2.create()
    results, keep_alive = [], []          # inputs stay allocated until both streams have drained
    for rnd in range(4):
        busy.fill_(rnd)                                        # unrelated work on the default stream
        q, k, v = _stream(gen, 300)
        q2, k2, v2 = _stream(gen, 200)
        qd, kd, vd, q2d, k2d, v2d = (dev(t) for t in (q, k, v, q2, k2, v2))
        keep_alive.append((qd, kd, vd, q2d, k2d, v2d))
        s1.wait_stream(torch.cuda.current_stream()); s2.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s1):
            o1, l1 = p1.pool.sk_session_append(a, qd, kd, vd)
            if rnd == 1:
                p1.pool.sk_session_evict_oldest(a, 133)
            if rnd == 2:
                f = p1.pool.sk_session_fork(a, 250)
            oq, lq = p1.pool.sk_session_query(a, qd[:24])
        with torch.cuda.stream(s2):
            cu = np.array([0, 150, 200], dtype=np.int32)
            ops = [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B if rnd % 2 else sk.SK_OP_APPEND]
            o2, l2 = p2.pool.sk_batch_step([b, c], ops, cu, q2d, k2d, v2d)
        results.append((rnd, q, k, v, q2, k2, v2, ops, o1, l1, oq, lq, o2, l2))
    s1.synchronize(); s2.synchronize()
    for rnd, q, k, v, q2, k2, v2, ops, o1, l1, oq, lq, o2, l2 in results:
        qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
        compare("stream 1 append, round %d" % rnd, o1, l1, *p1.oracles[a].append(qr, kr, vr), SHAPE.dtype)
        if rnd == 1:
            p1.oracles[a].evict_oldest(133)
        if rnd == 2:
            p1.oracles[f] = p1.oracles[a].fork(250)
        compare("stream 1 query, round %d" % rnd, oq, lq, *p1.oracles[a].query(qr[:24]), SHAPE.dtype)
        q2r, k2r, v2r = synth.to_raw(q2), synth.to_raw(k2), synth.to_raw(v2)
        ro0, rl0 = p2.oracles[b].append(q2r[:150], k2r[:150], v2r[:150])
        if ops[1] == sk.SK_OP_APPEND:
            ro1, rl1 = p2.oracles[c].append(q2r[150:], k2r[150:], v2r[150:])
        else:
            ro1, rl1 = p2.oracles[c].query(q2r[150:], k2r[150:], v2r[150:])
        compare("stream 2 batch step, round %d" % rnd, o2, l2, np.concatenate([ro0, ro1]), np.concatenate([rl0, rl1]), SHAPE.dtype)
    with torch.cuda.stream(s1):
        p1.check_cache(a); p1.check_cache(f)
    with torch.cuda.stream(s2):
        p2.check_cache(b); p2.check_cache(c)


def _pool_with_env(env, shape, **kw):
    """The tuning switches are read when a pool is created."""
    import os
    old = {k: os.environ.get(k) for k in env}
    os.environ.update(env)
    try:
        return sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, **kw)
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


def test_merge_inside_the_kernel_equals_the_separate_combine_bit_for_bit():
    """The split partials of a call are merged by a second kernel (the default) or, with SK_FUSE=1, by
    whichever workgroups of the attention kernel happen to do it: all of a row tile's workgroups
    sharing the rows (they waited for each other), or the last one alone (nobody waits:
    SK_WAIT_POLLS=0).  One function merges a row in split order in all of them, so outputs and
    log-sum-exps must agree to the last bit, call after call (the counters the workgroups meet at are
    left at zero by every launch); also for a batched step and a question batch with SK_FUSE_LIST=1."""
    shape = synth.CFG2
    gen = synth.generator(2, stream=77)
    kw = dict(block_tokens=16, n_blocks=700, max_sessions=3, max_batch_tokens=2048)
    pools = [_pool_with_env({"SK_FUSE": "1"}, shape, **kw), _pool_with_env({"SK_FUSE": "1", "SK_WAIT_POLLS": "0"}, shape, **kw),
             _pool_with_env({}, shape, **kw), _pool_with_env({"SK_FUSE": "1", "SK_FUSE_LIST": "1"}, shape, **kw),
             _pool_with_env({"SK_FUSE": "1", "SK_MERGE_FENCES": "1"}, shape, **kw)]
    sids = [(p.sk_session_create(), p.sk_session_create()) for p in pools]

    def same(results, what):
        for r in results[1:]:
            for x, y in zip(results[0], r):
                assert torch.equal(x, y), what

    for L in (600, 256, 1, 2000, 77, 1300):
        q, k, v = [dev(t) for t in synth.draw_qkv(gen, L, shape)]
        same([p.sk_session_append(s[0], q, k, v) for p, s in zip(pools, sids)], "append %d" % L)
    assert pools[0].sk_pool_last_launch()["fused_merge"] == 1 and pools[2].sk_pool_last_launch()["fused_merge"] == 0
    for nq in (32, 16, 100, 3):
        q, k, v = [dev(t) for t in synth.draw_qkv(gen, nq, shape)]
        for S in (0, 3, 40):
            same([p.sk_session_query(s[0], q, n_splits=S) for p, s in zip(pools, sids)], "query A %d S=%d" % (nq, S))
            same([p.sk_session_query(s[0], q, k, v, n_splits=S) for p, s in zip(pools, sids)], "query B %d S=%d" % (nq, S))
    # batched step (append on the second session, queries on the first) and a question batch
    counts = [700, 40]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    q, k, v = [dev(t) for t in synth.draw_qkv(gen, int(cu[-1]), shape)]
    for rep in range(2):
        same([p.sk_batch_step([s[1], s[0]], [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B], cu, q, k, v) for p, s in zip(pools, sids)],
             "batch step %d" % rep)
    assert pools[3].sk_pool_last_launch()["fused_merge"] == 1
    P, NQ, Sfx = 16, 8, 8
    qp, kp, vp = [dev(t) for t in synth.draw_qkv(gen, P, shape)]
    qs, ks, vs = [dev(t.reshape(NQ, Sfx, t.shape[1], shape.head_dim)) for t in synth.draw_qkv(gen, NQ * Sfx, shape)]
    same([p.sk_session_query_shared_prefix(s[0], qp, kp, vp, qs, ks, vs) for p, s in zip(pools, sids)], "question batch")
    torch.cuda.synchronize()
    for p in pools:
        p.close()


def test_query_replays_from_a_hip_graph():
    """A single-session query enqueues kernels only (its decomposition and its short scatter list
    travel in the kernel arguments), so a caller can capture it in a HIP graph and replay it: every
    replay, with new query contents in the captured buffers and eager calls and synchronisations
    in between, equals the eager call on the same inputs bit for bit, and the oracle within
    tolerance.  The greedy sampler's entry point that allocates nothing is captured along."""
    gen = synth.generator(2, stream=91)
    pr = Pair(SHAPE, block_tokens=16, n_blocks=300, kv_fill=0xFF, max_batch_tokens=2048)
    sid = pr.create()
    q, k, v = synth.draw_qkv(gen, 1500, SHAPE)
    pr.append(sid, q, k, v, check=False)
    nq, vocab = 20, 8192 * 3 + 4
    qs = torch.zeros((nq, SHAPE.n_q_heads, SHAPE.head_dim), dtype=torch.bfloat16, device="cuda")
    ks = torch.zeros((nq, SHAPE.n_kv_heads, SHAPE.head_dim), dtype=torch.bfloat16, device="cuda")
    vs = torch.zeros_like(ks)
    logits = torch.zeros((nq, vocab), dtype=torch.float32, device="cuda")
    out_a = torch.empty((nq, SHAPE.n_q_heads, SHAPE.head_dim), dtype=torch.float32, device="cuda")
    lse_a = torch.empty((nq, SHAPE.n_q_heads), dtype=torch.float32, device="cuda")
    out_b, lse_b = torch.empty_like(out_a), torch.empty_like(lse_a)
    tops = sk.top2_outputs(nq, "cuda")
    sk.sk_top2_static(logits[:0])                         # set-up call (no rows): resolves the scratch address outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        pr.pool.sk_session_query(sid, qs, out=out_a, lse=lse_a)
        pr.pool.sk_session_query(sid, qs, ks, vs, out=out_b, lse=lse_b)
        sk.sk_top2_static(logits, outputs=tops)
        graph.capture_end()
    torch.cuda.synchronize()
    before = pr.pool.kv_mem.clone()
    for rep in range(4):
        q1, k1, v1 = synth.draw_qkv(gen, nq, SHAPE)
        lg = synth.draw(gen, (nq, vocab), "f32")
        qs.copy_(dev(q1)); ks.copy_(dev(k1)); vs.copy_(dev(v1)); logits.copy_(dev(lg))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out_a, lse_a, out_b, lse_b)] + [t.clone() for t in tops]
        # eager work of the program's own between the replays, then the same calls eagerly
        ea = pr.pool.sk_session_query(sid, qs)
        eb = pr.pool.sk_session_query(sid, qs, ks, vs)
        et = sk.sk_top2(logits)
        torch.cuda.synchronize()
        for x, y in zip(got, list(ea) + list(eb) + list(et)):
            assert torch.equal(x, y), "replay %d differs from the eager call" % rep
        o = pr.oracles[sid]
        ro, rl = o.query(synth.to_raw(q1))
        compare("graph replay %d, query A" % rep, got[0], got[1], ro, rl, SHAPE.dtype)
        ro, rl = o.query(synth.to_raw(q1), synth.to_raw(k1), synth.to_raw(v1))
        compare("graph replay %d, query B" % rep, got[2], got[3], ro, rl, SHAPE.dtype)
    assert torch.equal(before, pr.pool.kv_mem)
