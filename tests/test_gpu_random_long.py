"""Seeded random operations at long contexts (3,000 to 70,000 cached tokens, where calls are cut into
many splits and row tiles): appends of up to 1,024 tokens, both kinds of query with free and forced
split counts, evictions of up to half a session, truncations, forks and batched steps over up to
three sessions, each checked on sampled output rows that the oracle computes one by one against
the whole cache; sampled cache ranges are read back bit for bit at the end."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import dev
from test_gpu_fullsize import _sample_rows, _check_rows

pytestmark = pytest.mark.gpu

SHAPES = [synth.CFG2, synth.Shape("bf16", 8, 2, 128), synth.Shape("bf16", 64, 8, 128), synth.Shape("bf16", 16, 8, 128)]
OPS = [sk.SK_OP_APPEND, sk.SK_OP_QUERY_A, sk.SK_OP_QUERY_B]


def _rows(rng, n_tok, shape, count):
    return _sample_rows(rng, n_tok, shape, extra=count)


def _build(pool, sid, ref, n, shape, gen):
    left = n
    while left:
        L = min(2048, left)
        left -= L
        k = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype)
        v = synth.draw(gen, (L, shape.n_kv_heads, shape.head_dim), shape.dtype)
        pool.sk_session_append(sid, None, dev(k), dev(v))
        ref.K = np.concatenate([ref.K, synth.to_raw(k)])
        ref.V = np.concatenate([ref.V, synth.to_raw(v)])


@pytest.mark.parametrize("seed", list(range(7000, 7024)))
def test_random_operations_at_long_context(seed):
    rng = np.random.default_rng(seed)
    gen = synth.generator(7, stream=seed)
    shape = SHAPES[int(rng.integers(len(SHAPES)))]
    B = int(rng.choice([16, 64, 256]))
    n0 = int(np.exp(rng.uniform(np.log(3000), np.log(70000))))
    n_blocks = 2 * ((n0 + 6000) // B + 8)
    pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, B, n_blocks, max_sessions=3,
                   max_batch_tokens=2048)
    pool.sk_pool_set_alloc_order(synth.permutation(gen, n_blocks))
    refs = {}
    first = pool.sk_session_create()
    refs[first] = oracle.OracleSession(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    _build(pool, first, refs[first], n0, shape, gen)
    for step in range(14):
        sid = sorted(refs)[int(rng.integers(len(refs)))]
        o = refs[sid]
        kind = int(rng.integers(7))
        if kind == 0:                                           # append
            L = int(rng.choice([1, 64, 200, 256, 512, 777, 1024]))
            q, k, v = synth.draw_qkv(gen, L, shape)
            name = "seed %d: append %d to session %d at %d" % (seed, L, sid, o.length)
            out, lse = pool.sk_session_append(sid, dev(q), dev(k), dev(v))
            rows = _rows(rng, L, shape, 10)
            ro, rl = o.append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v), rows=rows)
            _check_rows(name, out, lse, rows, ro, rl, shape.dtype)
        elif kind in (1, 2):                                    # query, cache only / with own K/V
            nq = int(rng.choice([1, 8, 16, 32, 64, 128]))
            S = int(rng.choice([0, 0, 1, 3, 7, 32, 128]))
            q, k, v = synth.draw_qkv(gen, nq, shape)
            name = "seed %d: query %s, %d tokens, session %d at %d, n_splits %d" % (seed, "AB"[kind - 1], nq, sid, o.length, S)
            rows = _rows(rng, nq, shape, 8)
            if kind == 1:
                if o.length == 0:
                    continue
                out, lse = pool.sk_session_query(sid, dev(q), n_splits=S)
                ro, rl = o.query(synth.to_raw(q), rows=rows)
            else:
                out, lse = pool.sk_session_query(sid, dev(q), dev(k), dev(v), n_splits=S)
                ro, rl = o.query(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v), rows=rows)
            _check_rows(name, out, lse, rows, ro, rl, shape.dtype)
        elif kind == 3:                                         # evict up to half of what is not frozen
            room = o.length - o.n_frozen
            if room < 2:
                continue
            n = int(rng.integers(1, room // 2 + 1))
            pool.sk_session_evict_oldest(sid, n)
            o.evict_oldest(n)
        elif kind == 4:                                         # truncate
            p = int(rng.integers(o.length // 2, o.length + 1))
            pool.sk_session_truncate(sid, p)
            o.truncate(p)
        elif kind == 5 and len(refs) < 3:                       # fork
            n = int(rng.integers(0, o.length + 1))
            refs[pool.sk_session_fork(sid, n)] = o.fork(n)
        elif kind == 6:                                         # one batched step over every session
            ids, ops, counts = sorted(refs), [], []
            for s in ids:
                kk = int(rng.integers(3))
                if kk == 1 and refs[s].length == 0:
                    kk = 2
                ops.append(OPS[kk])
                counts.append(int(rng.choice([1, 16, 64, 300, 600])) if kk == 0 else int(rng.choice([1, 16, 64])))
            cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
            q, k, v = synth.draw_qkv(gen, int(cu[-1]), shape)
            name = "seed %d: batch step sessions %s ops %s counts %s" % (seed, ids, ops, counts)
            out, lse = pool.sk_batch_step(ids, ops, cu, dev(q), dev(k), dev(v))
            qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
            for i, (s, op) in enumerate(zip(ids, ops)):
                a, b = int(cu[i]), int(cu[i + 1])
                rows = _rows(rng, b - a, shape, 6)
                if op == sk.SK_OP_APPEND:
                    ro, rl = refs[s].append(qr[a:b], kr[a:b], vr[a:b], rows=rows)
                elif op == sk.SK_OP_QUERY_A:
                    ro, rl = refs[s].query(qr[a:b], rows=rows)
                else:
                    ro, rl = refs[s].query(qr[a:b], kr[a:b], vr[a:b], rows=rows)
                _check_rows(name + ", item %d" % i, out[a:b], lse[a:b], rows, ro, rl, shape.dtype)
    for sid, o in refs.items():
        n = o.length
        assert pool.sk_session_length(sid) == n
        if n == 0:
            continue
        start = int(rng.integers(0, max(1, n - 1000)))
        count = min(1000, n - start)
        kc, vc = pool.sk_session_gather(sid, start, count)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(synth.to_raw(kc.cpu()), o.K[start:start + count])
        np.testing.assert_array_equal(synth.to_raw(vc.cpu()), o.V[start:start + count])
    pool.close()
