"""Parity at the full sizes of the workloads, in the launch configuration bench.py times: the oracle
computes a sample of output rows one by one (each against the whole cache), the GPU computes
everything; the cache is checked bit for bit on sampled token ranges."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import TOL, compare, dev

pytestmark = pytest.mark.gpu


def _tile_rows(T, shape):
    """Height of the row tile the library gives a call of T tokens (rows per KV head = T x group):
    256 rows above 128, else 128 above 64, else 64."""
    rows = T * shape.group
    return 256 if rows > 128 else 128 if rows > 64 else 64


def _sample_rows(rng, n_tok, shape, extra=0, always=(), tile_rows=None):
    """Rows (token, query head) to check against the oracle, stratified over the launch: for every
    (row tile, KV head) - one workgroup column of the kernel - the tile's first row, its last row and
    one row drawn at random inside it, so that a fault confined to one tile of one head cannot go
    unsampled; plus `extra` rows drawn uniformly."""
    G, Hkv = shape.group, shape.n_kv_heads
    tpt = max(1, (tile_rows or _tile_rows(n_tok, shape)) // G)
    rows = set(always)
    for t0 in range(0, n_tok, tpt):
        t1 = min(t0 + tpt, n_tok) - 1
        for g in range(Hkv):
            rows.add((t0, g * G))
            rows.add((t1, g * G + G - 1))
            rows.add((int(rng.integers(t0, t1 + 1)), g * G + int(rng.integers(G))))
    for _ in range(extra):
        rows.add((int(rng.integers(n_tok)), int(rng.integers(shape.n_q_heads))))
    return sorted(rows)


def _check_rows(name, out, lse, rows, ro, rl, dtype):
    tol = TOL[dtype]
    og = torch.stack([out[i, h] for i, h in rows]).float().cpu().numpy().astype(np.float64)
    lg = torch.stack([lse[i, h] for i, h in rows]).cpu().numpy().astype(np.float64)
    diff = np.abs(og - ro)
    rms = np.sqrt((ro ** 2).mean(axis=1)) + 1e-300
    assert np.isfinite(og).all(), name
    assert diff.max() <= tol["max_abs"] and diff.mean() <= tol["mean_abs"], "%s: max %.3e mean %.3e" % (name, diff.max(), diff.mean())
    assert (diff.max(axis=1) / rms).max() <= tol["rel"], "%s: rel %.3e" % (name, (diff.max(axis=1) / rms).max())
    assert np.abs(lg - rl).max() <= tol["lse"], "%s: lse %.3e" % (name, np.abs(lg - rl).max())


def _build(pool, sid, ref, n, shape, gen, piece=2048):
    """Commits n tokens (K/V only) into the GPU session and mirrors them in the oracle."""
    Ks, Vs = [], []
    for a in range(0, n, piece):
        L = min(piece, n - a)
        k = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype)
        v = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype)
        pool.sk_session_append(sid, None, dev(k), dev(v))
        Ks.append(synth.to_raw(k)); Vs.append(synth.to_raw(v))
    ref.K = np.concatenate([ref.K] + Ks); ref.V = np.concatenate([ref.V] + Vs)


@pytest.mark.parametrize("n,L,nq,n_rows,B", [(32768, 256, 32, 64, 16), (131072, 512, 16, 24, 16), (131072, 512, 16, 24, 256)])
def test_single_session_full_context(n, L, nq, n_rows, B):
    """Workloads 2 and 3: one Llama-3-8B-shaped layer at 32,768 / 131,072 cached tokens; the append
    that reaches that length, then queries with the library's own split choice (what bench.py times)."""
    shape = synth.CFG2
    gen = synth.generator(2 if n == 32768 else 3, stream=20)
    rng = np.random.default_rng(n)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n // B + 8, max_sessions=1,
                   max_batch_tokens=2048)
    ref = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    sid = pool.sk_session_create()
    _build(pool, sid, ref, n - L, shape, gen)
    q, k, v = synth.draw_qkv(gen, L, shape)
    out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
    rows = _sample_rows(rng, L, shape, extra=n_rows)
    ro, rl = ref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v), rows=rows)
    _check_rows("append at %d" % (n - L), out, lse, rows, ro, rl, shape.dtype)
    assert pool.sk_session_length(sid) == n
    # commit, bit for bit, on the first, a middle and the last 1,024 tokens
    for first in (0, n // 2 - 512, n - 1024):
        kc, vc = pool.sk_session_gather(sid, first, 1024)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(synth.to_raw(kc.cpu()), ref.K[first:first + 1024])
        np.testing.assert_array_equal(synth.to_raw(vc.cpu()), ref.V[first:first + 1024])
    qq, kq, vq = synth.draw_qkv(gen, nq, shape)
    rows = _sample_rows(rng, nq, shape, extra=n_rows)
    out, lse = pool.sk_session_query(sid, dev(qq))
    geo = pool.sk_pool_last_launch()
    assert geo["workgroups"] >= 256                      # the configuration bench.py times fills the chip
    ro, rl = ref.query(synth.to_raw(qq), rows=rows)
    _check_rows("query A at %d" % n, out, lse, rows, ro, rl, shape.dtype)
    out, lse = pool.sk_session_query(sid, dev(qq), dev(kq), dev(vq))
    ro, rl = ref.query(synth.to_raw(qq), synth.to_raw(kq), synth.to_raw(vq), rows=rows)
    _check_rows("query B at %d" % n, out, lse, rows, ro, rl, shape.dtype)
    for S in (7, 128):
        out, lse = pool.sk_session_query(sid, dev(qq), n_splits=S)
        ro, rl = ref.query(synth.to_raw(qq), rows=rows[:8])
        _check_rows("query A S=%d" % S, out, lse, rows[:8], ro, rl, shape.dtype)
    if n > 65536 and B == 16:
        # 32 tokens (128 rows per KV head) at this length: the eight-wave 128-row instance, which from
        # 65,536 cached tokens on loads the cache with the non-temporal policy
        q2, k2, v2 = synth.draw_qkv(gen, 32, shape)
        rows2 = _sample_rows(rng, 32, shape, extra=4)[:12]
        out, lse = pool.sk_session_query(sid, dev(q2))
        ro, rl = ref.query(synth.to_raw(q2), rows=rows2)
        _check_rows("32-token query A at %d" % n, out, lse, rows2, ro, rl, shape.dtype)
        out, lse = pool.sk_session_query(sid, dev(q2), dev(k2), dev(v2))
        ro, rl = ref.query(synth.to_raw(q2), synth.to_raw(k2), synth.to_raw(v2), rows=rows2)
        _check_rows("32-token query B at %d" % n, out, lse, rows2, ro, rl, shape.dtype)


def test_head_dim_64_at_70000_cached_tokens():
    """A Llama-3.2-1B-shaped layer (32/8 heads, head_dim 64, bf16) at a length where the library takes
    the launch configurations of the long caches (one workgroup per CU, the eight-wave 128-row instance,
    non-temporal loads): a 256-token append, then 16-, 32- and 100-token queries on sampled rows."""
    shape = synth.Shape("bf16", 32, 8, 64)
    n, L = 70000, 256
    gen = synth.generator(6, stream=21)
    rng = np.random.default_rng(64)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n // 16 + 8, max_sessions=1,
                   max_batch_tokens=2048)
    ref = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    sid = pool.sk_session_create()
    _build(pool, sid, ref, n - L, shape, gen)
    q, k, v = synth.draw_qkv(gen, L, shape)
    out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
    assert pool.sk_pool_last_launch()["kernel_variant"] != 0
    rows = _sample_rows(rng, L, shape, extra=16, tile_rows=128)      # head_dim 64 has no 256-row tile
    ro, rl = ref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v), rows=rows)
    _check_rows("append at %d" % (n - L), out, lse, rows, ro, rl, shape.dtype)
    for first in (0, n - 1024):
        kc, vc = pool.sk_session_gather(sid, first, 1024)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(synth.to_raw(kc.cpu()), ref.K[first:first + 1024])
        np.testing.assert_array_equal(synth.to_raw(vc.cpu()), ref.V[first:first + 1024])
    for nq in (16, 32, 100):
        qq, kq, vq = synth.draw_qkv(gen, nq, shape)
        rows = _sample_rows(rng, nq, shape, extra=4, tile_rows=min(128, _tile_rows(nq, shape)))
        rows = [rows[i] for i in sorted(rng.choice(len(rows), size=min(16, len(rows)), replace=False))]
        out, lse = pool.sk_session_query(sid, dev(qq))
        assert pool.sk_pool_last_launch()["workgroups"] >= 256
        ro, rl = ref.query(synth.to_raw(qq), rows=rows)
        _check_rows("query A, %d tokens" % nq, out, lse, rows, ro, rl, shape.dtype)
        out, lse = pool.sk_session_query(sid, dev(qq), dev(kq), dev(vq))
        ro, rl = ref.query(synth.to_raw(qq), synth.to_raw(kq), synth.to_raw(vq), rows=rows)
        _check_rows("query B, %d tokens" % nq, out, lse, rows, ro, rl, shape.dtype)


def test_registered_question_batch_at_65536():
    """Workload 5: 64 questions of 16 + 8 tokens against a 65,536-token session at the 70B-layer shape,
    after a 256-token append; sampled rows of the prefix and of several questions."""
    shape = synth.CFG5
    gen = synth.generator(5, stream=20)
    rng = np.random.default_rng(5)
    n, L, P, NQ, Sfx = 65536, 256, 16, 64, 8
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n // 16 + 8, max_sessions=1,
                   max_batch_tokens=1024)
    ref = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    sid = pool.sk_session_create()
    _build(pool, sid, ref, n - L, shape, gen, piece=1024)
    q, k, v = synth.draw_qkv(gen, L, shape)
    out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
    rows = _sample_rows(rng, L, shape, extra=8)
    ro, rl = ref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v), rows=rows)
    _check_rows("append", out, lse, rows, ro, rl, shape.dtype)
    qp, kp, vp = synth.draw_qkv(gen, P, shape)
    qs, ks, vs = synth.draw_qkv(gen, NQ * Sfx, shape)
    r4 = lambda t, H: t.reshape(NQ, Sfx, H, shape.head_dim)
    op, lp, os_, ls = pool.sk_session_query_shared_prefix(sid, dev(qp), dev(kp), dev(vp), dev(r4(qs, 64)),
                                                          dev(r4(ks, 8)), dev(r4(vs, 8)))
    rows = _sample_rows(rng, P, shape, extra=4)
    ro, rl = ref.query(synth.to_raw(qp), synth.to_raw(kp), synth.to_raw(vp), rows=rows)
    _check_rows("prefix rows", op, lp, rows, ro, rl, shape.dtype)
    # every question (four of them share a 256-row tile): first and last row of every KV head, one at random
    for j in range(NQ):
        sl = slice(j * Sfx, (j + 1) * Sfx)
        qj = np.concatenate([synth.to_raw(qp), synth.to_raw(qs[sl])])
        kj = np.concatenate([synth.to_raw(kp), synth.to_raw(ks[sl])])
        vj = np.concatenate([synth.to_raw(vp), synth.to_raw(vs[sl])])
        rows = _sample_rows(rng, Sfx, shape, tile_rows=Sfx * shape.group)
        ro, rl = ref.query(qj, kj, vj, rows=[(P + i, h) for i, h in rows])
        _check_rows("question %d" % j, os_[j], ls[j], rows, ro, rl, shape.dtype)
    assert pool.sk_session_length(sid) == n


def test_multi_tenant_step_at_full_size():
    """Workload 4: 48 sessions, lengths log-uniform over 2K-64K, 16-token blocks in a seeded random
    order; one step appends 128-1024 tokens on 16 sessions and queries 8-64 tokens on 32; three rows of
    every (row tile, KV head) of every item against the oracle, commits checked bit for bit on the
    appended ranges."""
    shape = synth.CFG4
    gen = synth.generator(4, stream=20)
    rng = np.random.default_rng(4)
    NS = 48
    lengths = synth.loguniform_lengths(gen, NS)
    n_blocks = int(1.25 * sum((x + 15) // 16 for x in lengths)) + 16 * 70
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n_blocks, max_sessions=NS,
                   max_batch_tokens=20480)
    pool.sk_pool_set_alloc_order(synth.permutation(gen, n_blocks))
    refs = [oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim) for _ in range(NS)]
    sids = [pool.sk_session_create() for _ in range(NS)]
    # round-robin growth in 1,024-token pieces so that the tables interleave
    done = [0] * NS
    Kl, Vl = [[] for _ in range(NS)], [[] for _ in range(NS)]
    while any(d < n for d, n in zip(done, lengths)):
        for i in range(NS):
            Lp = min(1024, lengths[i] - done[i])
            if Lp <= 0:
                continue
            k = synth.draw(gen, (Lp, 8, 128), "bf16"); v = synth.draw(gen, (Lp, 8, 128), "bf16")
            pool.sk_session_append(sids[i], None, dev(k), dev(v))
            Kl[i].append(synth.to_raw(k)); Vl[i].append(synth.to_raw(v))
            done[i] += Lp
    for i in range(NS):
        refs[i].K, refs[i].V = np.concatenate(Kl[i]), np.concatenate(Vl[i])
    del Kl, Vl
    order = [int(x) for x in synth.permutation(gen, NS)]
    ops = [sk.SK_OP_APPEND] * 16 + [sk.SK_OP_QUERY_B if j % 2 else sk.SK_OP_QUERY_A for j in range(32)]
    counts = [synth.randint(gen, 128, 1024) for _ in range(16)] + [synth.randint(gen, 8, 64) for _ in range(32)]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    q, k, v = synth.draw_qkv(gen, int(cu[-1]), shape)
    out, lse = pool.sk_batch_step([sids[i] for i in order], ops, cu, dev(q), dev(k), dev(v))
    torch.cuda.synchronize()
    qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
    for j, i in enumerate(order):
        a, b = int(cu[j]), int(cu[j + 1])
        rows = _sample_rows(rng, b - a, shape)
        if ops[j] == sk.SK_OP_APPEND:
            ro, rl = refs[i].append(qr[a:b], kr[a:b], vr[a:b], rows=rows)
            kc, vc = pool.sk_session_gather(sids[i], lengths[i], b - a)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(synth.to_raw(kc.cpu()), kr[a:b])
            np.testing.assert_array_equal(synth.to_raw(vc.cpu()), vr[a:b])
        elif ops[j] == sk.SK_OP_QUERY_A:
            ro, rl = refs[i].query(qr[a:b], rows=rows)
        else:
            ro, rl = refs[i].query(qr[a:b], kr[a:b], vr[a:b], rows=rows)
        _check_rows("item %d (op %d, n=%d)" % (j, ops[j], lengths[i]), out[a:b], lse[a:b], rows, ro, rl, shape.dtype)
        assert pool.sk_session_length(sids[i]) == refs[i].length


def test_pool_of_160_gib_serves_a_session_from_its_last_blocks():
    """Largest pool a test can afford (160 GiB of the 288 GB; nothing in it is initialised beyond what
    the session writes): the session's blocks are the pool's highest-numbered ones, in a shuffled
    order, so every byte offset the kernels form is beyond 2^37 for the last KV head.  Ragged
    appends and both kinds of query against the oracle element by element, cache bit for bit."""
    shape = synth.CFG2
    n_blocks = 160 * (1 << 30) // (16 * shape.n_kv_heads * shape.head_dim * 2 * 2)
    torch.cuda.empty_cache()
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n_blocks, max_sessions=2,
                   max_session_tokens=4096, max_batch_tokens=1024)
    assert pool.kv_mem.numel() == 160 * (1 << 30)
    gen = synth.generator(2, stream=40)
    top = n_blocks - 1 - synth.permutation(gen, 256).astype(np.int64)
    perm = np.concatenate([top, np.arange(n_blocks - 256, dtype=np.int64)]).astype(np.int32)
    pool.sk_pool_set_alloc_order(perm)
    sid = pool.sk_session_create()
    ref = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    for L in (300, 1, 411, 200):
        q, k, v = synth.draw_qkv(gen, L, shape)
        out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
        ro, rl = ref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
        compare("append %d" % L, out, lse, ro, rl, shape.dtype)
    table = pool.sk_session_block_table(sid)
    assert min(table) >= n_blocks - 256 and table != sorted(table)
    qq, kq, vq = synth.draw_qkv(gen, 24, shape)
    out, lse = pool.sk_session_query(sid, dev(qq))
    compare("query A", out, lse, *ref.query(synth.to_raw(qq)), shape.dtype)
    out, lse = pool.sk_session_query(sid, dev(qq), dev(kq), dev(vq))
    compare("query B", out, lse, *ref.query(synth.to_raw(qq), synth.to_raw(kq), synth.to_raw(vq)), shape.dtype)
    kc, vc = pool.sk_session_gather(sid)
    torch.cuda.synchronize()
    Kc, Vc = ref.cache()
    assert np.array_equal(synth.to_raw(kc.cpu()), Kc) and np.array_equal(synth.to_raw(vc.cpu()), Vc)
    # fork at a prefix that ends inside a block: the one block copy of a fork, here between two of the
    # pool's highest blocks; then a cut of the source into a block it shares, whose next append copies
    # that block first
    fid = pool.sk_session_fork(sid, 700)
    fref = ref.fork(700)
    q, k, v = synth.draw_qkv(gen, 90, shape)
    out, lse = pool.sk_session_append(fid, dev(q), dev(k), dev(v))
    compare("append to the fork", out, lse, *fref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)), shape.dtype)
    pool.sk_session_truncate(sid, 650)
    ref.truncate(650)
    q, k, v = synth.draw_qkv(gen, 40, shape)
    out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
    compare("append to the source after the cut", out, lse, *ref.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)), shape.dtype)
    assert min(pool.sk_session_block_table(fid)) >= n_blocks - 256
    for s_, r_ in ((sid, ref), (fid, fref)):
        kc, vc = pool.sk_session_gather(s_)
        torch.cuda.synchronize()
        Kc, Vc = r_.cache()
        assert np.array_equal(synth.to_raw(kc.cpu()), Kc) and np.array_equal(synth.to_raw(vc.cpu()), Vc)
    del pool
    torch.cuda.empty_cache()
