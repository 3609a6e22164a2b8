"""Seeded random walks over the whole session API: appends, both kinds of query, ragged batch steps,
question batches, freeze / evict, truncate, fork, destroy and re-create, in any order over several
sessions of one pool.  Every output is compared with the oracle session that received the same
calls (Sec. 3.3 regions, Sec. 3.4 isolation, Sec. 3.7 batching, Sec. 3.9.3 SeqRemove), every cache
is read back bit for bit at the end of each walk and at random points in it."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth
from gpu_common import compare, dev

pytestmark = pytest.mark.gpu

MAX_LEN = 2600          # a session that grows beyond this is cut back (evict or truncate)


class Walk:
    def __init__(self, shape, block_tokens, max_sessions, seed, tight=False):
        self.shape, self.B = shape, block_tokens
        self.rng = np.random.default_rng(seed)
        self.gen = synth.generator(6, stream=seed)
        n_blocks = max_sessions * ((MAX_LEN + 1400) // block_tokens + 3)
        if tight:               # a pool that runs out: refused calls must change nothing
            n_blocks = max(8, (MAX_LEN + 600) // block_tokens)
        self.refused = 0
        self.pool = sk.Pool(shape.dtype, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, block_tokens, n_blocks,
                            max_sessions=max_sessions, max_batch_tokens=2048, kv_fill=0xFF)
        self.pool.sk_pool_set_alloc_order(synth.permutation(self.gen, n_blocks))
        self.max_sessions = max_sessions
        self.ref = {}            # session id -> OracleSession
        self.may_freeze = {}     # no eviction behind the frozen region yet
        self.log = []
        self.count = {}

    def new_oracle(self):
        s = self.shape
        return oracle.OracleSession(s.dtype, s.n_q_heads, s.n_kv_heads, s.head_dim)

    def draw(self, n):
        return synth.draw_qkv(self.gen, n, self.shape)

    def pick(self, nonempty=False):
        ids = [s for s in sorted(self.ref) if not nonempty or self.ref[s].length > 0]
        return ids[int(self.rng.integers(len(ids)))] if ids else None

    def check_cache(self, sid):
        k, v = self.pool.sk_session_gather(sid)
        torch.cuda.synchronize()
        K, V = self.ref[sid].cache()
        assert self.pool.sk_session_length(sid) == K.shape[0], self.log[-8:]
        np.testing.assert_array_equal(synth.to_raw(k.cpu()), K)
        np.testing.assert_array_equal(synth.to_raw(v.cpu()), V)

    # ---- operations; each returns a short description for the failure message ----
    def op_create(self):
        if len(self.ref) >= self.max_sessions:
            return None
        sid = self.pool.sk_session_create()
        assert sid not in self.ref
        self.ref[sid] = self.new_oracle(); self.may_freeze[sid] = True
        return "create %d" % sid

    def op_destroy(self):
        if len(self.ref) < 2:
            return None
        sid = self.pick()
        self.pool.sk_session_destroy(sid)
        del self.ref[sid], self.may_freeze[sid]
        return "destroy %d" % sid

    def op_append(self):
        sid = self.pick()
        L = int(self.rng.choice([1, 7, 16, 33, 64, 100, 129, 256, 300]))
        q, k, v = self.draw(L)
        odt = "bf16" if self.shape.dtype == "bf16" and self.rng.integers(4) == 0 else "f32"
        name = "append %d tokens to session %d at %d, out %s" % (L, sid, self.ref[sid].length, odt)
        try:
            out, lse = self.pool.sk_session_append(sid, dev(q), dev(k), dev(v), out_dtype=odt)
        except sk.SkError as e:
            return self.was_refused(e, name)
        ro, rl = self.ref[sid].append(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
        compare(name, out, lse, ro, rl, self.shape.dtype, odt == "bf16")
        return name

    def was_refused(self, e, name):
        """The pool is out of blocks: the call must have changed nothing (checked by every later
        comparison and cache read-back, since the oracle was not told about it)."""
        assert e.status == sk.SK_E_NOMEM, name
        self.refused += 1
        for sid in sorted(self.ref):
            assert self.pool.sk_session_length(sid) == self.ref[sid].length, name
        return name + " (refused: no blocks)"

    def op_query(self):
        mode_b = bool(self.rng.integers(2))
        sid = self.pick(nonempty=not mode_b)
        if sid is None:
            return None
        nq = int(self.rng.choice([1, 3, 8, 16, 17, 32, 40, 64]))
        q, k, v = self.draw(nq)
        kw = {"n_splits": int(self.rng.choice([0, 0, 1, 2, 5]))}
        name = "query %s, %d tokens, session %d at %d, n_splits %d" % ("B" if mode_b else "A", nq, sid, self.ref[sid].length, kw["n_splits"])
        if self.shape.dtype == "bf16" and self.rng.integers(4) == 0:
            kw["out_dtype"] = "bf16"
        if self.rng.integers(5) == 0:
            kw["want_lse"] = False
        if mode_b:
            out, lse = self.pool.sk_session_query(sid, dev(q), dev(k), dev(v), **kw)
            ro, rl = self.ref[sid].query(synth.to_raw(q), synth.to_raw(k), synth.to_raw(v))
        else:
            out, lse = self.pool.sk_session_query(sid, dev(q), **kw)
            ro, rl = self.ref[sid].query(synth.to_raw(q))
        compare(name + " %s" % sorted(kw.items()), out, lse, ro, rl, self.shape.dtype, kw.get("out_dtype") == "bf16")
        return name

    def op_batch(self):
        ids = [int(s) for s in self.rng.permutation(sorted(self.ref))]
        ids = ids[:max(1, int(self.rng.integers(1, len(ids) + 1)))]
        ops, counts = [], []
        for s in ids:
            kind = int(self.rng.integers(3))
            if kind == 1 and self.ref[s].length == 0:
                kind = 2
            ops.append([sk.SK_OP_APPEND, sk.SK_OP_QUERY_A, sk.SK_OP_QUERY_B][kind])
            counts.append(int(self.rng.choice([0, 1, 5, 16, 31, 64, 130, 260]) if kind == 0 else self.rng.choice([1, 4, 16, 24, 64])))
        cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        T = int(cu[-1])
        if T == 0:
            return None
        q, k, v = self.draw(T)
        name = "batch step sessions %s ops %s counts %s" % (ids, ops, counts)
        try:
            out, lse = self.pool.sk_batch_step(ids, ops, cu, dev(q), dev(k), dev(v))
        except sk.SkError as e:
            return self.was_refused(e, name)
        qr, kr, vr = synth.to_raw(q), synth.to_raw(k), synth.to_raw(v)
        ro = np.zeros((T, self.shape.n_q_heads, self.shape.head_dim)); rl = np.zeros((T, self.shape.n_q_heads))
        for i, (s, op) in enumerate(zip(ids, ops)):
            a, b = int(cu[i]), int(cu[i + 1])
            if a == b:
                continue
            if op == sk.SK_OP_APPEND:
                ro[a:b], rl[a:b] = self.ref[s].append(qr[a:b], kr[a:b], vr[a:b])
            elif op == sk.SK_OP_QUERY_A:
                ro[a:b], rl[a:b] = self.ref[s].query(qr[a:b])
            else:
                ro[a:b], rl[a:b] = self.ref[s].query(qr[a:b], kr[a:b], vr[a:b])
        compare(name, out, lse, ro, rl, self.shape.dtype)
        return name

    def op_questions(self):
        sid = self.pick()
        P = int(self.rng.choice([0, 5, 16]))
        NQ, Sfx = int(self.rng.choice([1, 3, 8])), int(self.rng.choice([1, 8, 11]))
        s = self.shape
        qp, kp, vp = self.draw(P)
        qs, ks, vs = self.draw(NQ * Sfx)
        r4 = lambda t, H: t.reshape(NQ, Sfx, H, s.head_dim)
        name = "question batch P=%d NQ=%d Sfx=%d session %d at %d" % (P, NQ, Sfx, sid, self.ref[sid].length)
        op_, lp_, os_, ls_ = self.pool.sk_session_query_shared_prefix(
            sid, dev(qp) if P else None, dev(kp) if P else None, dev(vp) if P else None,
            dev(r4(qs, s.n_q_heads)), dev(r4(ks, s.n_kv_heads)), dev(r4(vs, s.n_kv_heads)))
        rop, rlp, ros, rls = self.ref[sid].query_shared_prefix(
            synth.to_raw(qp), synth.to_raw(kp), synth.to_raw(vp),
            synth.to_raw(qs).reshape(NQ, Sfx, s.n_q_heads, -1), synth.to_raw(ks).reshape(NQ, Sfx, s.n_kv_heads, -1),
            synth.to_raw(vs).reshape(NQ, Sfx, s.n_kv_heads, -1))
        if P:
            compare(name + " (prefix rows)", op_, lp_, rop, rlp, self.shape.dtype)
        compare(name + " (suffix rows)", os_, ls_, ros, rls, self.shape.dtype)
        return name

    def op_freeze(self):
        sid = self.pick(nonempty=True)
        if sid is None or not self.may_freeze[sid]:
            return None
        o = self.ref[sid]
        nf = int(self.rng.integers(o.n_frozen, min(o.length, o.n_frozen + 200) + 1))
        self.pool.sk_session_freeze(sid, nf); o.freeze(nf)
        return "freeze session %d at %d" % (sid, nf)

    def op_evict(self, sid=None, n=None):
        sid = self.pick(nonempty=True) if sid is None else sid
        if sid is None:
            return None
        o = self.ref[sid]
        room = o.length - o.n_frozen
        if room == 0:
            return None
        n = int(self.rng.integers(1, min(room, 700) + 1)) if n is None else min(n, room)
        self.pool.sk_session_evict_oldest(sid, n); o.evict_oldest(n)
        self.may_freeze[sid] = False
        return "evict %d from session %d (frozen %d, now %d)" % (n, sid, o.n_frozen, o.length)

    def op_truncate(self):
        sid = self.pick(nonempty=True)
        if sid is None:
            return None
        o = self.ref[sid]
        p = int(self.rng.integers(0, o.length + 1)) if self.rng.integers(4) else int(max(0, o.length - self.rng.integers(1, 40)))
        self.pool.sk_session_truncate(sid, p); o.truncate(p)
        if p <= o.n_frozen:
            self.may_freeze[sid] = True
        return "truncate session %d to %d" % (sid, p)

    def op_fork(self):
        if len(self.ref) >= self.max_sessions:
            return None
        src = self.pick()
        o = self.ref[src]
        n = int(self.rng.integers(0, o.length + 1)) if self.rng.integers(3) else o.length
        try:
            new = self.pool.sk_session_fork(src, n)
        except sk.SkError as e:
            return self.was_refused(e, "fork session %d at %d" % (src, n))
        assert new not in self.ref
        self.ref[new] = o.fork(n)
        self.may_freeze[new] = self.may_freeze[src] or n <= o.n_frozen
        self.check_cache(new)
        return "fork session %d at %d of %d -> %d" % (src, n, o.length, new)

    def run(self, n_ops):
        table = [(self.op_append, 30), (self.op_query, 22), (self.op_batch, 10), (self.op_questions, 6), (self.op_freeze, 4),
                 (self.op_evict, 8), (self.op_truncate, 6), (self.op_fork, 6), (self.op_create, 4), (self.op_destroy, 4)]
        w = np.array([x[1] for x in table], dtype=np.float64); w /= w.sum()
        self.log.append(self.op_create())
        done = 0
        while done < n_ops:
            op = table[int(self.rng.choice(len(table), p=w))][0]
            try:
                what = op()
            except Exception:
                print("\n".join(str(x) for x in self.log[-12:]), flush=True)
                raise
            if what is None:
                continue
            self.log.append(what); done += 1
            self.count[op.__name__] = self.count.get(op.__name__, 0) + 1
            for sid in sorted(self.ref):               # keep the oracle fast: cut long sessions back
                if self.ref[sid].length > MAX_LEN:
                    o = self.ref[sid]
                    if o.length - o.n_frozen > 1500:
                        self.log.append(self.op_evict(sid, 1500))
                    else:
                        self.pool.sk_session_truncate(sid, 800); o.truncate(800)
                        self.may_freeze[sid] = self.may_freeze[sid] or 800 <= o.n_frozen
                        self.log.append("truncate session %d to 800 (cap)" % sid)
            if done % 25 == 0:
                for sid in sorted(self.ref):
                    self.check_cache(sid)
        for sid in sorted(self.ref):
            self.check_cache(sid)
        # every block is owned by a live session or free
        owned = set()
        for sid in self.ref:
            owned.update(self.pool.sk_session_block_table(sid))
        assert self.pool.sk_pool_blocks_free() == self.pool.desc.n_blocks - len(owned)
        assert all(self.count.get(f.__name__, 0) > 0 for f, _ in table), self.count      # the walk reached every operation
        return self.refused


@pytest.mark.parametrize("shape,block_tokens,max_sessions,seed,n_ops", [
    (synth.Shape("bf16", 8, 2, 128), 16, 5, 101, 400),
    (synth.CFG2, 64, 4, 102, 250),
    (synth.Shape("bf16", 16, 2, 128), 32, 4, 103, 300),
    (synth.CFG1, 16, 5, 104, 400),
    (synth.Shape("bf16", 8, 8, 128), 16, 6, 105, 300),
    (synth.Shape("bf16", 12, 4, 128), 128, 3, 106, 200),
    (synth.Shape("bf16", 8, 1, 128), 16, 4, 107, 300),
    (synth.Shape("f32", 8, 2, 128), 32, 4, 108, 200),
    (synth.Shape("bf16", 14, 2, 64), 16, 4, 109, 400),       # head_dim 64, seven query heads per KV head
    (synth.Shape("bf16", 32, 8, 64), 64, 4, 110, 200),
])
def test_random_walk_over_the_session_api(shape, block_tokens, max_sessions, seed, n_ops):
    Walk(shape, block_tokens, max_sessions, seed).run(n_ops)


@pytest.mark.parametrize("shape,block_tokens,max_sessions,seed,n_ops", [
    (synth.Shape("bf16", 8, 2, 128), 16, 5, 201, 400),
    (synth.CFG1, 64, 4, 202, 300),
])
def test_random_walk_in_a_pool_that_runs_out_of_blocks(shape, block_tokens, max_sessions, seed, n_ops):
    """Same walk with blocks for about one long session in all: appends, batch steps and forks are
    refused now and then (all or nothing), and everything keeps agreeing with the oracle, which never
    hears of a refused call."""
    assert Walk(shape, block_tokens, max_sessions, seed, tight=True).run(n_ops) > 0
