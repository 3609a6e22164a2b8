"""fp64 oracle of the stateful-session attention path.  TEST INFRASTRUCTURE ONLY.

A session is the persistent per-stream state of the paper (Sec. 3.4): the keys
and values of everything ingested so far.  Two operations act on it:

  append  (data plane, Alg. 1: K.append(Forward(tokens, K))): the chunk's K/V are
          committed and every chunk token attends over cache + chunk, causally;
  query   (query plane, Alg. 2; Sec. 3.2 Eq. 2): query tokens attend over the
          cache and nothing is committed (Region 2 is ephemeral, Sec. 3.3;
          Flash Query evaluation restores the cache, Sec. 3.9.3).

Arrays are numpy; "f32" data is np.float32, "bf16" data is np.uint16 holding the
raw bf16 bit patterns.  Outputs are float64.  The arithmetic lives in
attention_oracle.c; this file only keeps the cache and says which keys each row
may see.

Readings where the paper is silent (listed again in the design notes):
  * causal alignment: chunk token i (absolute position n + i) sees positions
    0 .. n + i inclusive;
  * a query may carry its own keys/values (mode B: Alg. 2's Forward(tokens_q, K),
    Sec. 3.9.3 Extend) or not (mode A: the literal Eq. 2);
  * softmax scale 1/sqrt(d_k) unless given.
"""
import ctypes
import math

import numpy as np

from . import _lib

_DT = {"f32": (0, np.float32), "bf16": (1, np.uint16)}


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(a, np_dtype, shape_tail, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np_dtype:
        raise TypeError("%s: expected %s, got %s" % (name, np_dtype, a.dtype))
    if a.ndim != 3 or tuple(a.shape[1:]) != tuple(shape_tail):
        raise ValueError("%s: expected [*, %d, %d], got %s" % (name, shape_tail[0], shape_tail[1], a.shape))
    return a


def attention(dtype, q, kc, vc, ke, ve, vis, n_q_heads, n_kv_heads, head_dim, scale, rows=None):
    """softmax(q K^T * scale) V per row, K/V = cache ++ leading vis[i] extra keys.

    rows=None: all rows -> (out [m,Hq,d], lse [m,Hq]).
    rows=[(i,h),...]: only those -> (out [len,d], lse [len]).
    Raises ZeroDivisionError if some requested row sees no key at all.
    """
    code, npdt = _DT[dtype]
    Hq, Hkv, d = n_q_heads, n_kv_heads, head_dim
    q = _check(q, npdt, (Hq, d), "q")
    m = q.shape[0]
    n = 0 if kc is None else kc.shape[0]
    if n:
        kc = _check(kc, npdt, (Hkv, d), "kc")
        vc = _check(vc, npdt, (Hkv, d), "vc")
    else:
        kc = vc = None
    ne = 0 if ke is None else ke.shape[0]
    if ne:
        ke = _check(ke, npdt, (Hkv, d), "ke")
        ve = _check(ve, npdt, (Hkv, d), "ve")
        vis = np.ascontiguousarray(vis, dtype=np.int64)
        assert vis.shape == (m,)
    else:
        ke = ve = vis = None
    L = _lib.lib()
    if rows is None:
        out = np.zeros((m, Hq, d), dtype=np.float64)
        lse = np.zeros((m, Hq), dtype=np.float64)
        rc = L.oracle_attention(code, _ptr(q), m, _ptr(kc), _ptr(vc), n, _ptr(ke), _ptr(ve), ne,
                                _ptr(vis), Hq, Hkv, d, float(scale), _ptr(out), _ptr(lse))
    else:
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 2))
        out = np.zeros((rows.shape[0], d), dtype=np.float64)
        lse = np.zeros((rows.shape[0],), dtype=np.float64)
        rc = L.oracle_attention_rows(code, _ptr(q), m, _ptr(kc), _ptr(vc), n, _ptr(ke), _ptr(ve), ne,
                                     _ptr(vis), Hq, Hkv, d, float(scale),
                                     _ptr(rows), rows.shape[0], _ptr(out), _ptr(lse))
    if rc == -1:
        raise ZeroDivisionError("softmax over zero keys")
    if rc != 0:
        raise RuntimeError("oracle_attention failed: %d" % rc)
    return out, lse


class OracleSession:
    """Cache of one session plus the two planes acting on it."""

    def __init__(self, dtype, n_q_heads, n_kv_heads, head_dim, scale=None):
        if dtype not in _DT:
            raise ValueError(dtype)
        if n_q_heads % n_kv_heads:
            raise ValueError("n_q_heads must be a multiple of n_kv_heads")
        self.dtype = dtype
        self.Hq, self.Hkv, self.d = n_q_heads, n_kv_heads, head_dim
        self.scale = (1.0 / math.sqrt(head_dim)) if not scale else float(scale)
        npdt = _DT[dtype][1]
        self.K = np.zeros((0, n_kv_heads, head_dim), dtype=npdt)
        self.V = np.zeros((0, n_kv_heads, head_dim), dtype=npdt)
        self.n_frozen = 0

    def freeze(self, n_frozen):
        """Region 0 (Sec. 3.3): the first n_frozen tokens are never evicted."""
        if not (self.n_frozen <= n_frozen <= self.length):
            raise ValueError("n_frozen")
        self.n_frozen = int(n_frozen)

    def evict_oldest(self, n_tokens):
        """Region-1 FIFO eviction (Sec. 3.3; Alg. 1 evict_oldest): the n_tokens oldest tokens behind
        the frozen region leave the cache; attention over them is lost (Sec. 5.3 discussion of the
        sliding window), the order of the rest is kept."""
        if not (0 <= n_tokens <= self.length - self.n_frozen):
            raise ValueError("n_tokens")
        a, b = self.n_frozen, self.n_frozen + int(n_tokens)
        self.K = np.concatenate([self.K[:a], self.K[b:]], axis=0)
        self.V = np.concatenate([self.V[:a], self.V[b:]], axis=0)

    def fork(self, n_prefix):
        """A new session holding the first n_prefix tokens of this one (Sec. 3.7 followers aliasing the
        leader's state; Sec. 3.10 sequence aliasing): by value here, the two never interact."""
        if not (0 <= n_prefix <= self.length):
            raise ValueError("n_prefix")
        t = OracleSession(self.dtype, self.Hq, self.Hkv, self.d, self.scale)
        t.K, t.V = self.K[:n_prefix].copy(), self.V[:n_prefix].copy()
        t.n_frozen = min(self.n_frozen, int(n_prefix))
        return t

    @property
    def length(self):
        return self.K.shape[0]

    def _attend(self, q, k, v, vis, rows):
        return attention(self.dtype, q, self.K, self.V, k, v, vis,
                         self.Hq, self.Hkv, self.d, self.scale, rows)

    def append(self, q, k, v, rows=None):
        """Data plane.  Token i of the chunk sees the cache and chunk[0..i]; then the
        chunk's K/V bits are committed behind the cache."""
        L = q.shape[0]
        if L == 0:
            return (np.zeros((0, self.Hq, self.d)), np.zeros((0, self.Hq)))
        vis = np.arange(1, L + 1, dtype=np.int64)
        res = self._attend(q, k, v, vis, rows)
        self.K = np.concatenate([self.K, np.ascontiguousarray(k)], axis=0)
        self.V = np.concatenate([self.V, np.ascontiguousarray(v)], axis=0)
        return res

    def query(self, q, k=None, v=None, rows=None):
        """Query plane; the cache is not touched.
        k is None: mode A, keys = cache only, no mask (Sec. 3.2 Eq. 2).
        k given:   mode B, the query's own K/V follow the cache causally and are
                   dropped afterwards (Sec. 3.3 Region 2; Sec. 3.9.3)."""
        if k is None:
            return self._attend(q, None, None, None, rows)
        vis = np.arange(1, q.shape[0] + 1, dtype=np.int64)
        return self._attend(q, k, v, vis, rows)

    def query_shared_prefix(self, qp, kp, vp, qs, ks, vs):
        """A batch of questions that share a prefix (Sec. 3.7 grouped prefill applied to
        the registered questions of Alg. 3).  Question j is prefix ++ suffix_j and is
        evaluated like a mode-B query.  Returns the prefix rows (identical for every
        question, so computed from the prefix alone) and each question's suffix rows.
          qp,kp,vp [P,H,d]; qs,ks,vs [NQ,Sfx,H,d]
          -> out_prefix [P,Hq,d], lse_prefix [P,Hq], out_suffix [NQ,Sfx,Hq,d], lse_suffix [NQ,Sfx,Hq]
        """
        P = qp.shape[0]
        NQ, Sfx = qs.shape[0], qs.shape[1]
        out_p, lse_p = self.query(qp, kp, vp)
        out_s = np.zeros((NQ, Sfx, self.Hq, self.d))
        lse_s = np.zeros((NQ, Sfx, self.Hq))
        for j in range(NQ):
            q = np.concatenate([qp, qs[j]], axis=0)
            k = np.concatenate([kp, ks[j]], axis=0)
            v = np.concatenate([vp, vs[j]], axis=0)
            o, l = self.query(q, k, v)
            out_s[j] = o[P:]
            lse_s[j] = l[P:]
        return out_p, lse_p, out_s, lse_s

    def truncate(self, new_length):
        """SeqRemove(s, p, infinity) of Sec. 3.9.3: forget every token at position >= new_length."""
        if new_length < 0 or new_length > self.length:
            raise ValueError("new_length out of range")
        self.K = self.K[:new_length].copy()
        self.V = self.V[:new_length].copy()
        self.n_frozen = min(self.n_frozen, int(new_length))

    def cache(self):
        """Copies of the committed keys and values, [n,Hkv,d] raw bits."""
        return self.K.copy(), self.V.copy()


OP_APPEND, OP_QUERY_A, OP_QUERY_B = 0, 1, 2


class OraclePool:
    """Several isolated sessions (Sec. 3.4) and the ragged step
    that the multi-tenant scheduler of Sec. 3.7 issues: a mix of appends and queries
    over distinct sessions, equal by definition to issuing them one at a time."""

    def __init__(self, dtype, n_q_heads, n_kv_heads, head_dim, scale=None):
        self.args = (dtype, n_q_heads, n_kv_heads, head_dim, scale)
        self.sessions = {}
        self._next = 0

    def create(self):
        sid = self._next
        self._next += 1
        self.sessions[sid] = OracleSession(*self.args)
        return sid

    def destroy(self, sid):
        del self.sessions[sid]

    def batch_step(self, session_ids, ops, cu_tokens, q, k, v):
        """Packed rows cu_tokens[i]:cu_tokens[i+1] belong to item i.
        Returns out [T,Hq,d], lse [T,Hq]."""
        if len(set(session_ids)) != len(session_ids):
            raise ValueError("a session may appear once per step")
        T = int(cu_tokens[-1])
        dtype, Hq, Hkv, d, _ = self.args
        out = np.zeros((T, Hq, d))
        lse = np.zeros((T, Hq))
        for i, (sid, op) in enumerate(zip(session_ids, ops)):
            a, b = int(cu_tokens[i]), int(cu_tokens[i + 1])
            s = self.sessions[sid]
            if op == OP_APPEND:
                o, l = s.append(q[a:b], k[a:b], v[a:b])
            elif op == OP_QUERY_A:
                o, l = s.query(q[a:b])
            elif op == OP_QUERY_B:
                o, l = s.query(q[a:b], k[a:b], v[a:b])
            else:
                raise ValueError("bad op")
            out[a:b] = o
            lse[a:b] = l
        return out, lse


def num_threads():
    return int(_lib.lib().oracle_num_threads())
