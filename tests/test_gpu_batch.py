"""GPU parity of the batched entry points: the ragged multi-session step and the shared-prefix
question batch, against the fp64 oracle (which defines them as "the same calls one by one")."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import compare, dev

pytestmark = pytest.mark.gpu


def _grow(pool, ref, sids, lengths, shape, gen):
    """Round-robin growth in 64-token pieces so that block tables interleave."""
    done = [0] * len(sids)
    while any(d < n for d, n in zip(done, lengths)):
        for i, sid in enumerate(sids):
            L = min(64, lengths[i] - done[i])
            if L <= 0:
                continue
            q, k, v = synth.draw_qkv(gen, L, shape)
            pool.sk_session_append(sid, None, dev(k), dev(v))
            o = ref.sessions[sid]
            o.K = np.concatenate([o.K, synth.to_raw(k)])
            o.V = np.concatenate([o.V, synth.to_raw(v)])
            done[i] += L


def _check_caches(pool, ref, sids):
    for sid in sids:
        k, v = pool.sk_session_gather(sid)
        torch.cuda.synchronize()
        K, V = ref.sessions[sid].cache()
        np.testing.assert_array_equal(synth.to_raw(k.cpu()), K)
        np.testing.assert_array_equal(synth.to_raw(v.cpu()), V)


@pytest.mark.parametrize("shape,n_sessions,lo,hi", [(synth.CFG4, 8, 40, 3000), (synth.CFG1, 5, 10, 400)])
def test_ragged_multi_session_steps(shape, n_sessions, lo, hi):
    """Multi-tenant workload in small: sessions of log-uniform lengths in one pool with 16-token
    blocks handed out in a seeded random order; every step mixes appends on some sessions with
    queries (cache-only and with own K/V) on others."""
    gen = synth.generator(4, stream=n_sessions)
    lengths = synth.loguniform_lengths(gen, n_sessions, lo, hi)
    n_blocks = sum((n + 15) // 16 for n in lengths) + 400
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n_blocks,
                   max_sessions=n_sessions, max_batch_tokens=4096, kv_fill=0xFF)
    pool.sk_pool_set_alloc_order(synth.permutation(gen, n_blocks))
    ref = oracle.OraclePool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    sids = [pool.sk_session_create() for _ in range(n_sessions)]
    for _ in sids:
        ref.create()
    _grow(pool, ref, sids, lengths, shape, gen)
    _check_caches(pool, ref, sids)
    for step in range(3):
        order = [int(x) for x in synth.permutation(gen, n_sessions)]
        n_app = max(1, n_sessions // 3)
        ops, counts = [], []
        for j, s in enumerate(order):
            if j < n_app:
                ops.append(sk.SK_OP_APPEND); counts.append(synth.randint(gen, 128, 300))
            else:
                ops.append(sk.SK_OP_QUERY_B if j % 2 else sk.SK_OP_QUERY_A); counts.append(synth.randint(gen, 8, 64))
        if step == 2:
            counts[-1] = 0                      # an empty item is legal
        cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        q, k, v = synth.draw_qkv(gen, int(cu[-1]), shape)
        out, lse = pool.sk_batch_step(order, ops, cu, dev(q), dev(k), dev(v))
        ro, rl = ref.batch_step(order, ops, cu, synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
        compare("step %d" % step, out, lse, ro, rl, shape.dtype)
        for s in order:
            assert pool.sk_session_length(s) == ref.sessions[s].length
    _check_caches(pool, ref, sids)
    # blocks no session owns still hold the canary bytes; so does nothing else get written
    owned = set()
    for sid in sids:
        owned.update(pool.sk_session_block_table(sid))
    torch.cuda.synchronize()
    mem = pool.kv_mem
    free = [b for b in range(n_blocks) if b not in owned][:50]
    for b in free:
        for h in (0, shape.n_kv_heads - 1):
            a = pool.sk_pool_element_offset(b, h, False, 0, 0)
            e = pool.sk_pool_element_offset(b, h, True, 15, shape.head_dim - 1)
            assert bool((mem[a:e] == 0xFF).all()), "block %d was written" % b


def test_batch_errors_leave_state_unchanged():
    shape = synth.CFG4
    gen = synth.generator(4, stream=77)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, 12, max_sessions=3,
                   max_batch_tokens=512)
    a, b, c = (pool.sk_session_create() for _ in range(3))
    q, k, v = (dev(t) for t in synth.draw_qkv(gen, 200, shape))
    pool.sk_session_append(a, q[:64], k[:64], v[:64])            # 4 blocks
    state = lambda: ([pool.sk_session_length(s) for s in (a, b, c)], pool.sk_pool_blocks_free())
    before = state()
    with pytest.raises(sk.SkError) as e:                          # needs 5 + 5 blocks, 8 free
        pool.sk_batch_step([a, b], [sk.SK_OP_APPEND, sk.SK_OP_APPEND], [0, 80, 160], q, k, v)
    assert e.value.status == sk.SK_E_NOMEM and state() == before
    with pytest.raises(sk.SkError) as e:                          # same session twice
        pool.sk_batch_step([a, a], [sk.SK_OP_QUERY_A, sk.SK_OP_QUERY_A], [0, 8, 16], q, k, v)
    assert e.value.status == sk.SK_E_INVAL and state() == before
    with pytest.raises(sk.SkError) as e:                          # cache-only query on an empty session
        pool.sk_batch_step([a, b], [sk.SK_OP_APPEND, sk.SK_OP_QUERY_A], [0, 16, 24], q, k, v)
    assert e.value.status == sk.SK_E_EMPTY and state() == before
    with pytest.raises(sk.SkError) as e:
        pool.sk_batch_step([a, 7], [sk.SK_OP_QUERY_A, sk.SK_OP_QUERY_A], [0, 8, 16], q, k, v)
    assert e.value.status == sk.SK_E_BADSESSION and state() == before
    pool.sk_batch_step([b, a], [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B], [0, 100, 130], q, k, v)
    assert state() == ([64, 100, 0], 1)


@pytest.mark.parametrize("n,P,NQ,Sfx", [(700, 16, 6, 8), (1300, 5, 3, 3), (130, 0, 4, 8), (0, 16, 2, 8), (900, 40, 2, 20)])
def test_shared_prefix_question_batch(n, P, NQ, Sfx):
    """Registered-question batch at the 70B-layer shape (64/8 heads): prefix rows once, suffix rows
    per question; equal to the oracle's independent evaluations, and nothing is committed."""
    shape = synth.CFG5
    gen = synth.generator(5, stream=n + P)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 16, n // 16 + 8, max_sessions=1,
                   kv_fill=0xFF)
    ref = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    sid = pool.sk_session_create()
    if n:
        q, k, v = synth.draw_qkv(gen, n, shape)
        pool.sk_session_append(sid, None, dev(k), dev(v))
        ref.K, ref.V = synth.to_raw(k), synth.to_raw(v)
    qp, kp, vp = synth.draw_qkv(gen, P, shape)
    qs, ks, vs = synth.draw_qkv(gen, NQ * Sfx, shape)
    r4 = lambda t, H: t.reshape(NQ, Sfx, H, shape.head_dim)
    before = pool.kv_mem.clone()
    op, lp, os_, ls = pool.sk_session_query_shared_prefix(
        sid, dev(qp) if P else None, dev(kp) if P else None, dev(vp) if P else None,
        dev(r4(qs, shape.n_q_heads)), dev(r4(ks, shape.n_kv_heads)), dev(r4(vs, shape.n_kv_heads)))
    rop, rlp, ros, rls = ref.query_shared_prefix(
        synth.to_raw(qp), synth.to_raw(kp), synth.to_raw(vp),
        synth.to_raw(qs).reshape(NQ, Sfx, shape.n_q_heads, -1), synth.to_raw(ks).reshape(NQ, Sfx, shape.n_kv_heads, -1),
        synth.to_raw(vs).reshape(NQ, Sfx, shape.n_kv_heads, -1))
    if P:
        compare("prefix rows", op, lp, rop, rlp, shape.dtype)
    compare("suffix rows", os_, ls, ros.reshape(NQ * Sfx, shape.n_q_heads, -1), rls.reshape(NQ * Sfx, -1), shape.dtype)
    torch.cuda.synchronize()
    assert torch.equal(before, pool.kv_mem) and pool.sk_session_length(sid) == n
