"""A call that fails half way on a real pool: the failure is forced by the library's test hook right
before a HIP call (nothing faulty reaches the device), the call reports an error, and afterwards the
session behaves as if the call had never been made: lengths, committed K/V bit for bit, and the results
of later appends and queries against the fp64 oracle, which never saw the failed call (Alg. 1: an
append either happens or does not)."""
import numpy as np
import pytest
import torch

import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import Pair, compare, dev

pytestmark = pytest.mark.gpu
SHAPE = synth.CFG2


def _fail(pool, site, fn):
    pool.sk_pool_inject_failure(site, 1)
    with pytest.raises(sk.SkError) as e:
        fn()
    pool.sk_pool_inject_failure(0, 0)
    return e.value.status


@pytest.mark.parametrize("site", [sk.SK_SITE_SCATTER, sk.SK_SITE_ATTENTION, sk.SK_SITE_COMBINE, sk.SK_SITE_RING, sk.SK_SITE_UPLOAD])
def test_failed_append_leaves_the_session_as_it_was(site):
    gen = synth.generator(2, stream=500 + site)
    pr = Pair(SHAPE, block_tokens=16, n_blocks=600, max_sessions=2, max_batch_tokens=2048)
    sid = pr.create()
    for L in (700, 45):
        q, k, v = synth.draw_qkv(gen, L, SHAPE)
        pr.append(sid, q, k, v)
    free0, n0 = pr.pool.sk_pool_blocks_free(), pr.pool.sk_session_length(sid)
    long_list = site in (sk.SK_SITE_RING, sk.SK_SITE_UPLOAD)        # only a long scatter list is uploaded
    q, k, v = synth.draw_qkv(gen, 1500 if long_list else 300, SHAPE)
    assert _fail(pr.pool, site, lambda: pr.pool.sk_session_append(sid, dev(q), dev(k), dev(v))) == sk.SK_E_HIP
    assert pr.pool.sk_session_length(sid) == n0 and pr.pool.sk_pool_blocks_free() == free0
    pr.check_cache(sid)
    qq, kq, vq = synth.draw_qkv(gen, 20, SHAPE)
    pr.query(sid, qq, name="query after the failed append")
    pr.query(sid, qq, kq, vq, name="query with own K/V after the failed append")
    q, k, v = synth.draw_qkv(gen, 333, SHAPE)
    pr.append(sid, q, k, v, name="append after the failed append")
    pr.check_cache(sid)


@pytest.mark.parametrize("site", [sk.SK_SITE_PLAN, sk.SK_SITE_UPLOAD, sk.SK_SITE_SCATTER, sk.SK_SITE_ATTENTION])
def test_failed_batch_step_leaves_every_session_as_it_was(site):
    gen = synth.generator(4, stream=600 + site)
    pr = Pair(SHAPE, block_tokens=16, n_blocks=900, max_sessions=4, max_batch_tokens=4096)
    sids = [pr.create() for _ in range(3)]
    for sid, L in zip(sids, (400, 90, 1200)):
        q, k, v = synth.draw_qkv(gen, L, SHAPE)
        pr.append(sid, q, k, v, check=False)
    state0 = [(pr.pool.sk_session_length(s), pr.pool.sk_session_block_table(s)) for s in sids], pr.pool.sk_pool_blocks_free()
    ops = [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B, sk.SK_OP_APPEND]
    counts = [260, 30, 100]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    q, k, v = synth.draw_qkv(gen, int(cu[-1]), SHAPE)
    st = _fail(pr.pool, site, lambda: pr.pool.sk_batch_step(sids, ops, cu, dev(q), dev(k), dev(v)))
    assert st == (sk.SK_E_WORKSPACE if site == sk.SK_SITE_PLAN else sk.SK_E_HIP)
    assert ([(pr.pool.sk_session_length(s), pr.pool.sk_session_block_table(s)) for s in sids], pr.pool.sk_pool_blocks_free()) == state0
    for sid in sids:
        pr.check_cache(sid)
    # the same step now goes through and matches the oracle, which only sees this one
    out, lse = pr.pool.sk_batch_step(sids, ops, cu, dev(q), dev(k), dev(v))
    qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
    for j, sid in enumerate(sids):
        a, b = int(cu[j]), int(cu[j + 1])
        o = pr.oracles[sid]
        ro, rl = o.append(qr[a:b], kr[a:b], vr[a:b]) if ops[j] == sk.SK_OP_APPEND else o.query(qr[a:b], kr[a:b], vr[a:b])
        compare("item %d after the failed step" % j, out[a:b], lse[a:b], ro, rl, SHAPE.dtype)
        pr.check_cache(sid)


def test_failed_fork_and_evict_change_nothing_and_a_kept_copy_is_harmless():
    gen = synth.generator(2, stream=700)
    pr = Pair(SHAPE, block_tokens=16, n_blocks=400, max_sessions=3, max_batch_tokens=1024)
    a = pr.create()
    q, k, v = synth.draw_qkv(gen, 500, SHAPE)
    pr.append(a, q, k, v, check=False)
    for site in (sk.SK_SITE_RING, sk.SK_SITE_UPLOAD, sk.SK_SITE_BLOCK_COPY):
        free0 = pr.pool.sk_pool_blocks_free()
        assert _fail(pr.pool, site, lambda: pr.pool.sk_session_fork(a, 205)) == sk.SK_E_HIP
        assert pr.pool.sk_pool_blocks_free() == free0
    f = pr.pool.sk_session_fork(a, 205)
    pr.oracles[f] = pr.oracles[a].fork(205)
    qq, _, _ = synth.draw_qkv(gen, 16, SHAPE)
    # f ends inside a block of its own (the copy the fork made); cut it back into a block it shares with
    # the source, then make the append that must first take a private copy of that block fail after the
    # commit kernel is enqueued: the copy is kept, nothing else changes
    pr.pool.sk_session_truncate(f, 100); pr.oracles[f].truncate(100)
    q, k, v = synth.draw_qkv(gen, 60, SHAPE)
    free0 = pr.pool.sk_pool_blocks_free()
    assert _fail(pr.pool, sk.SK_SITE_ATTENTION, lambda: pr.pool.sk_session_append(f, dev(q), dev(k), dev(v))) == sk.SK_E_HIP
    assert pr.pool.sk_session_length(f) == 100 and pr.pool.sk_pool_blocks_free() == free0 - 1
    pr.check_cache(f)
    pr.check_cache(a)
    pr.query(f, qq, name="fork after its failed append")
    pr.append(f, q, k, v, name="append to the fork after the failed one")
    pr.query(a, qq, name="source after the fork's append")
    pr.check_cache(f)
    # eviction that frees whole blocks rewrites the device table: force its copy to fail
    pr.freeze(a, 40)
    for site in (sk.SK_SITE_RING, sk.SK_SITE_UPLOAD):
        assert _fail(pr.pool, site, lambda: pr.pool.sk_session_evict_oldest(a, 200)) == sk.SK_E_HIP
        assert pr.pool.sk_session_length(a) == 500
    pr.evict(a, 200)
    pr.query(a, qq, name="source after eviction")
    pr.query(f, qq, name="fork after the source's eviction")
    pr.check_cache(a)
