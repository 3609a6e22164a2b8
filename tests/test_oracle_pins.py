"""Pins for the fp64 oracle: everything here is fixed by the paper's definition
(Sec. 3.2 Eq. 1/2) or by mathematics, none of it by the oracle's own code.

A plausible mistake in the oracle (dropped scale, wrong GQA mapping, off-by-one in the
causal limit, transposed operand, keys and values swapped, missing max subtraction)
fails at least one test below.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import OracleSession, OraclePool, OP_APPEND, OP_QUERY_A, OP_QUERY_B
from workloads import synth


def _rand(rng, shape, dtype):
    x = torch.from_numpy(rng.standard_normal(shape).astype(np.float32))
    return synth.to_raw(x.to(synth.torch_dtype(dtype)))


def _brute_row(q, keys, vals, scale):
    """Pure-Python softmax(q.k*scale) v for one row; lists of floats."""
    s = [scale * sum(a * b for a, b in zip(q, k)) for k in keys]
    mx = max(s)
    p = [math.exp(x - mx) for x in s]
    l = sum(p)
    d = len(vals[0])
    out = [sum(p[j] * vals[j][t] for j in range(len(keys))) / l for t in range(d)]
    return out, mx + math.log(l)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Hq,Hkv,d,n,L", [(1, 1, 1, 0, 1), (2, 1, 3, 5, 3), (4, 2, 4, 8, 4), (4, 4, 2, 3, 2), (6, 2, 4, 1, 5)])
def test_brute_force_tiny(dtype, Hq, Hkv, d, n, L):
    rng = np.random.default_rng(100 + Hq * 7 + n)
    s = OracleSession(dtype, Hq, Hkv, d)
    if n:
        s.append(_rand(rng, (n, Hq, d), dtype), _rand(rng, (n, Hkv, d), dtype), _rand(rng, (n, Hkv, d), dtype))
    q, k, v = _rand(rng, (L, Hq, d), dtype), _rand(rng, (L, Hkv, d), dtype), _rand(rng, (L, Hkv, d), dtype)
    Kc, Vc = s.cache()
    qf, kf, vf = synth.raw_to_f64(q), synth.raw_to_f64(k), synth.raw_to_f64(v)
    Kf, Vf = synth.raw_to_f64(Kc), synth.raw_to_f64(Vc)
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d)
    # mode B == append output: causal over cache + own tokens
    ob, lb = s.query(q, k, v)
    for i in range(L):
        for h in range(Hq):
            g = h // G
            keys = [list(Kf[j, g]) for j in range(n)] + [list(kf[j, g]) for j in range(i + 1)]
            vals = [list(Vf[j, g]) for j in range(n)] + [list(vf[j, g]) for j in range(i + 1)]
            eo, el = _brute_row(list(qf[i, h]), keys, vals, scale)
            np.testing.assert_allclose(ob[i, h], eo, rtol=0, atol=1e-13)
            assert abs(lb[i, h] - el) < 1e-13
    # mode A: cache only, no mask
    if n:
        oa, la = s.query(q)
        for i in range(L):
            for h in range(Hq):
                g = h // G
                eo, el = _brute_row(list(qf[i, h]), [list(Kf[j, g]) for j in range(n)],
                                    [list(Vf[j, g]) for j in range(n)], scale)
                np.testing.assert_allclose(oa[i, h], eo, rtol=0, atol=1e-13)
                assert abs(la[i, h] - el) < 1e-13


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_torch_sdpa_fp64_explicit_mask(dtype):
    """Second opinion from a library routine: torch SDPA in fp64 with an explicit boolean
    mask (bottom-right aligned) and KV heads expanded by repeat_interleave."""
    rng = np.random.default_rng(7)
    Hq, Hkv, d, n, L = 8, 2, 16, 37, 11
    s = OracleSession(dtype, Hq, Hkv, d)
    s.append(_rand(rng, (n, Hq, d), dtype), _rand(rng, (n, Hkv, d), dtype), _rand(rng, (n, Hkv, d), dtype))
    q, k, v = _rand(rng, (L, Hq, d), dtype), _rand(rng, (L, Hkv, d), dtype), _rand(rng, (L, Hkv, d), dtype)
    Kc, Vc = s.cache()
    out, lse = s.query(q, k, v)
    G = Hq // Hkv
    Q = torch.from_numpy(synth.raw_to_f64(q)).permute(1, 0, 2)                       # [Hq,L,d]
    Kall = torch.from_numpy(np.concatenate([synth.raw_to_f64(Kc), synth.raw_to_f64(k)])).permute(1, 0, 2)
    Vall = torch.from_numpy(np.concatenate([synth.raw_to_f64(Vc), synth.raw_to_f64(v)])).permute(1, 0, 2)
    Kall = Kall.repeat_interleave(G, dim=0)
    Vall = Vall.repeat_interleave(G, dim=0)
    pos_q = torch.arange(L)[:, None] + n
    pos_k = torch.arange(n + L)[None, :]
    mask = pos_k <= pos_q
    ref = torch.nn.functional.scaled_dot_product_attention(Q[None], Kall[None], Vall[None], attn_mask=mask)[0]
    np.testing.assert_allclose(out, ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)
    # and the log-sum-exp from the same scores
    sc = (Q @ Kall.transpose(1, 2)) / math.sqrt(d)
    sc = sc.masked_fill(~mask, float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(sc, dim=-1).permute(1, 0).numpy(), rtol=0, atol=1e-12)


def test_first_token_of_empty_session_returns_its_value():
    s = OracleSession("f32", 2, 1, 4)
    q = np.array([[[1, 2, 3, 4], [0.5, 0, 0, 0]]], dtype=np.float32)
    k = np.array([[[1, 0, 1, 0]]], dtype=np.float32)
    v = np.array([[[9, 8, 7, 6]]], dtype=np.float32)
    o, l = s.append(q, k, v)
    np.testing.assert_array_equal(o[0, 0], [9, 8, 7, 6])
    np.testing.assert_array_equal(o[0, 1], [9, 8, 7, 6])
    assert l[0, 0] == pytest.approx((1 + 3) / 2.0, abs=1e-15)     # single score, scale 1/sqrt(4)
    assert l[0, 1] == pytest.approx(0.25, abs=1e-15)


def test_scale_is_one_over_sqrt_dk_two_key_closed_form():
    """Two keys, scores a*b/sqrt(d) and 0 -> weights are a logistic function."""
    d = 16
    s = OracleSession("f32", 1, 1, d)
    k = np.zeros((2, 1, d), np.float32)
    v = np.zeros((2, 1, d), np.float32)
    k[0, 0, 0] = 3.0
    v[0, 0, :] = 1.0
    v[1, 0, :] = -1.0
    s.append(np.zeros((2, 1, d), np.float32), k, v)
    q = np.zeros((1, 1, d), np.float32)
    q[0, 0, 0] = 2.0
    o, l = s.query(q)
    x = 2.0 * 3.0 / math.sqrt(d)
    p0 = 1.0 / (1.0 + math.exp(-x))
    np.testing.assert_allclose(o[0, 0], np.full(d, p0 - (1 - p0)), atol=1e-15)
    assert l[0, 0] == pytest.approx(math.log(math.exp(x) + 1.0), abs=1e-14)
    # an explicit scale overrides the default
    s2 = OracleSession("f32", 1, 1, d, scale=0.5)
    s2.append(np.zeros((2, 1, d), np.float32), k, v)
    o2, _ = s2.query(q)
    p0 = 1.0 / (1.0 + math.exp(-3.0))
    np.testing.assert_allclose(o2[0, 0], np.full(d, 2 * p0 - 1), atol=1e-15)


def test_zero_query_gives_causal_running_mean_of_positions():
    """q = 0 -> uniform weights.  With V[j] = position j the output of chunk token i is the
    mean of 0..n+i, which fixes the causal limit to 'absolute position, inclusive'."""
    Hq, Hkv, d, n, L = 2, 2, 4, 6, 5
    s = OracleSession("f32", Hq, Hkv, d)
    pos = np.arange(n + L, dtype=np.float32)
    V = np.broadcast_to(pos[:, None, None], (n + L, Hkv, d)).copy()
    K = np.random.default_rng(1).standard_normal((n + L, Hkv, d)).astype(np.float32)
    s.append(np.zeros((n, Hq, d), np.float32), K[:n], V[:n])
    o, l = s.append(np.zeros((L, Hq, d), np.float32), K[n:], V[n:])
    for i in range(L):
        np.testing.assert_allclose(o[i], (n + i) / 2.0, atol=1e-13)
        np.testing.assert_allclose(l[i], math.log(n + i + 1), atol=1e-13)
    # mode A sees exactly the cache, all of it, whatever the row
    o, l = s.query(np.zeros((3, Hq, d), np.float32))
    np.testing.assert_allclose(o, (n + L - 1) / 2.0, atol=1e-13)
    np.testing.assert_allclose(l, math.log(n + L), atol=1e-13)


def test_gqa_head_h_reads_kv_head_h_div_group():
    Hq, Hkv, d, n = 8, 2, 4, 5
    rng = np.random.default_rng(2)
    s = OracleSession("bf16", Hq, Hkv, d)
    V = np.zeros((n, Hkv, d), np.float32)
    V[:, 0, :] = 1.0
    V[:, 1, :] = 2.0
    s.append(_rand(rng, (n, Hq, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"),
             synth.to_raw(torch.from_numpy(V).to(torch.bfloat16)))
    o, _ = s.query(_rand(rng, (3, Hq, d), "bf16"))
    for h in range(Hq):
        np.testing.assert_allclose(o[:, h, :], 1.0 + (h // 4), atol=1e-14)


def test_identical_keys_give_mean_of_values_and_lse_s_plus_log_count():
    Hq, Hkv, d, n = 2, 1, 8, 9
    rng = np.random.default_rng(3)
    krow = rng.standard_normal(d).astype(np.float32)
    K = np.broadcast_to(krow, (n, Hkv, d)).copy()
    V = rng.standard_normal((n, Hkv, d)).astype(np.float32)
    s = OracleSession("f32", Hq, Hkv, d)
    s.append(np.zeros((n, Hq, d), np.float32), K, V)
    q = rng.standard_normal((2, Hq, d)).astype(np.float32)
    o, l = s.query(q)
    for i in range(2):
        for h in range(Hq):
            np.testing.assert_allclose(o[i, h], V[:, 0, :].astype(np.float64).mean(0), atol=1e-14)
            sc = float(q[i, h].astype(np.float64) @ krow.astype(np.float64)) / math.sqrt(d)
            assert l[i, h] == pytest.approx(sc + math.log(n), abs=1e-13)


def test_value_scaling_and_cached_row_permutation():
    Hq, Hkv, d, n = 4, 2, 8, 33
    rng = np.random.default_rng(4)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (5, Hq, d), "f32")
    zq = np.zeros((n, Hq, d), np.float32)
    a = OracleSession("f32", Hq, Hkv, d)
    a.append(zq, K, V)
    o1, l1 = a.query(q)
    b = OracleSession("f32", Hq, Hkv, d)
    b.append(zq, K, 2.0 * V)                      # exact in fp32
    o2, l2 = b.query(q)
    np.testing.assert_allclose(o2, 2.0 * o1, rtol=0, atol=1e-14)
    np.testing.assert_array_equal(l1, l2)
    perm = rng.permutation(n)
    c = OracleSession("f32", Hq, Hkv, d)
    c.append(zq, K[perm], V[perm])
    o3, l3 = c.query(q)
    np.testing.assert_allclose(o3, o1, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l3, l1, rtol=0, atol=1e-13)


def test_large_scores_need_max_subtraction_and_needle_retrieval():
    """One cached key aligned with the query at a score of several hundred: the result is that
    key's value (exact value retrieval from mid-context, the paper's Q6 idea, Sec. 4.3); a
    softmax without max subtraction would overflow."""
    Hq, Hkv, d, n = 2, 1, 16, 50
    rng = np.random.default_rng(5)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (1, Hq, d), "f32")
    pos = 23
    K[pos, 0] = 400.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    s = OracleSession("f32", Hq, Hkv, d)
    s.append(np.zeros((n, Hq, d), np.float32), K, V)
    o, l = s.query(q)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    np.testing.assert_allclose(o[0, 0], V[pos, 0].astype(np.float64), atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_incremental_append_equals_one_shot_bit_identical(dtype):
    """Appending D_1..D_k one at a time gives every token the output of one causal pass over
    [S; D_1; ..; D_k] (Sec. 2 (i)-(iii); Sec. 3.4)."""
    Hq, Hkv, d, T = 4, 2, 8, 40
    rng = np.random.default_rng(6)
    q, k, v = _rand(rng, (T, Hq, d), dtype), _rand(rng, (T, Hkv, d), dtype), _rand(rng, (T, Hkv, d), dtype)
    one = OracleSession(dtype, Hq, Hkv, d)
    o_ref, l_ref = one.append(q, k, v)
    for cuts in ([0, 1, 2, 40], [0, 16, 32, 40], [0, 7, 8, 9, 39, 40], list(range(41))):
        s = OracleSession(dtype, Hq, Hkv, d)
        outs, lses = [], []
        for a, b in zip(cuts[:-1], cuts[1:]):
            o, l = s.append(q[a:b], k[a:b], v[a:b])
            outs.append(o)
            lses.append(l)
        np.testing.assert_array_equal(np.concatenate(outs), o_ref)
        np.testing.assert_array_equal(np.concatenate(lses), l_ref)
        Kc, Vc = s.cache()
        np.testing.assert_array_equal(Kc, k)
        np.testing.assert_array_equal(Vc, v)


def test_query_leaves_cache_untouched_and_equals_append_output():
    """Region 2 is cleared between queries (Sec. 3.3); evaluation returns the cache to its
    pre-evaluation state (Sec. 3.9.3).  Extend-then-Clear == append output minus the commit."""
    Hq, Hkv, d, n, L = 4, 2, 8, 19, 6
    rng = np.random.default_rng(8)
    s = OracleSession("bf16", Hq, Hkv, d)
    s.append(_rand(rng, (n, Hq, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"))
    K0, V0 = s.cache()
    q, k, v = _rand(rng, (L, Hq, d), "bf16"), _rand(rng, (L, Hkv, d), "bf16"), _rand(rng, (L, Hkv, d), "bf16")
    oa, la = s.query(q)
    ob, lb = s.query(q, k, v)
    ob2, lb2 = s.query(q, k, v)
    K1, V1 = s.cache()
    np.testing.assert_array_equal(K0, K1)
    np.testing.assert_array_equal(V0, V1)
    assert s.length == n
    np.testing.assert_array_equal(ob, ob2)
    o_app, l_app = s.append(q, k, v)
    np.testing.assert_array_equal(ob, o_app)
    np.testing.assert_array_equal(lb, l_app)
    assert s.length == n + L
    assert not np.array_equal(oa, ob)


def test_partition_of_keys_merges_by_log_sum_exp():
    """Softmax attention over a union of key ranges is the LSE-weighted mean of the per-range
    results; any partition reproduces the unsplit result."""
    Hq, Hkv, d, n = 4, 2, 8, 101
    rng = np.random.default_rng(9)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (3, Hq, d), "f32")
    full = OracleSession("f32", Hq, Hkv, d)
    full.append(np.zeros((n, Hq, d), np.float32), K, V)
    o_ref, l_ref = full.query(q)
    for cuts in ([0, 50, 101], [0, 1, 17, 64, 100, 101], [0, 33, 66, 101]):
        outs, lses = [], []
        for a, b in zip(cuts[:-1], cuts[1:]):
            part = OracleSession("f32", Hq, Hkv, d)
            part.append(np.zeros((b - a, Hq, d), np.float32), K[a:b], V[a:b])
            o, l = part.query(q)
            outs.append(o)
            lses.append(l)
        lses = np.stack(lses)
        M = lses.max(0)
        w = np.exp(lses - M)
        o = (np.stack(outs) * w[..., None]).sum(0) / w.sum(0)[..., None]
        np.testing.assert_allclose(o, o_ref, rtol=0, atol=1e-12)
        np.testing.assert_allclose(M + np.log(w.sum(0)), l_ref, rtol=0, atol=1e-12)


def test_shared_prefix_batch_equals_independent_queries():
    """Grouped prefill turns N redundant passes into one (Sec. 3.7); the results are those of
    the N independent evaluations of Alg. 3."""
    Hq, Hkv, d, n, P, NQ, Sfx = 4, 2, 8, 21, 3, 4, 2
    rng = np.random.default_rng(10)
    s = OracleSession("bf16", Hq, Hkv, d)
    s.append(_rand(rng, (n, Hq, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"))
    qp, kp, vp = _rand(rng, (P, Hq, d), "bf16"), _rand(rng, (P, Hkv, d), "bf16"), _rand(rng, (P, Hkv, d), "bf16")
    qs = _rand(rng, (NQ * Sfx, Hq, d), "bf16").reshape(NQ, Sfx, Hq, d)
    ks = _rand(rng, (NQ * Sfx, Hkv, d), "bf16").reshape(NQ, Sfx, Hkv, d)
    vs = _rand(rng, (NQ * Sfx, Hkv, d), "bf16").reshape(NQ, Sfx, Hkv, d)
    op, lp, os_, ls = s.query_shared_prefix(qp, kp, vp, qs, ks, vs)
    assert s.length == n
    for j in range(NQ):
        o, l = s.query(np.concatenate([qp, qs[j]]), np.concatenate([kp, ks[j]]), np.concatenate([vp, vs[j]]))
        np.testing.assert_array_equal(o[:P], op)
        np.testing.assert_array_equal(l[:P], lp)
        np.testing.assert_array_equal(o[P:], os_[j])
        np.testing.assert_array_equal(l[P:], ls[j])
    # brute force of one suffix row: it sees cache, whole prefix, own suffix up to itself,
    # and nothing of the other questions
    Kc, Vc = s.cache()
    j, t, h = 2, 1, 3
    g = h // (Hq // Hkv)
    keys = np.concatenate([synth.raw_to_f64(Kc)[:, g], synth.raw_to_f64(kp)[:, g], synth.raw_to_f64(ks[j])[: t + 1, g]])
    vals = np.concatenate([synth.raw_to_f64(Vc)[:, g], synth.raw_to_f64(vp)[:, g], synth.raw_to_f64(vs[j])[: t + 1, g]])
    eo, el = _brute_row(list(synth.raw_to_f64(qs[j])[t, h]), [list(x) for x in keys], [list(x) for x in vals],
                        1 / math.sqrt(d))
    np.testing.assert_allclose(os_[j, t, h], eo, atol=1e-13)
    assert abs(ls[j, t, h] - el) < 1e-13


def test_batch_step_equals_one_by_one_and_sessions_are_isolated():
    Hq, Hkv, d = 4, 2, 8
    rng = np.random.default_rng(11)
    pool, ref = OraclePool("f32", Hq, Hkv, d), OraclePool("f32", Hq, Hkv, d)
    ids = [pool.create() for _ in range(3)]
    for p in (pool, ref):
        if p is ref:
            [p.create() for _ in range(3)]
    lens = [5, 9, 2]
    init = [(_rand(rng, (n, Hq, d), "f32"), _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")) for n in lens]
    for p in (pool, ref):
        for sid, (q, k, v) in zip(ids, init):
            p.sessions[sid].append(q, k, v)
    cu = np.array([0, 4, 7, 9])
    q, k, v = _rand(rng, (9, Hq, d), "f32"), _rand(rng, (9, Hkv, d), "f32"), _rand(rng, (9, Hkv, d), "f32")
    ops = [OP_APPEND, OP_QUERY_B, OP_QUERY_A]
    before = ref.sessions[ids[1]].cache()
    out, lse = pool.batch_step(ids, ops, cu, q, k, v)
    o0, l0 = ref.sessions[ids[0]].append(q[0:4], k[0:4], v[0:4])
    o1, l1 = ref.sessions[ids[1]].query(q[4:7], k[4:7], v[4:7])
    o2, l2 = ref.sessions[ids[2]].query(q[7:9])
    np.testing.assert_array_equal(out, np.concatenate([o0, o1, o2]))
    np.testing.assert_array_equal(lse, np.concatenate([l0, l1, l2]))
    assert [pool.sessions[i].length for i in ids] == [9, 9, 2]
    np.testing.assert_array_equal(pool.sessions[ids[1]].cache()[0], before[0])
    with pytest.raises(ValueError):
        pool.batch_step([ids[0], ids[0]], [OP_QUERY_A, OP_QUERY_A], np.array([0, 1, 2]), q, k, v)


def test_mode_a_on_empty_session_is_an_error():
    s = OracleSession("f32", 2, 1, 4)
    with pytest.raises(ZeroDivisionError):
        s.query(np.zeros((1, 2, 4), np.float32))


def test_selected_rows_match_full_evaluation():
    Hq, Hkv, d, n, L = 8, 2, 16, 70, 9
    rng = np.random.default_rng(12)
    s = OracleSession("bf16", Hq, Hkv, d)
    s.append(_rand(rng, (n, Hq, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"))
    q, k, v = _rand(rng, (L, Hq, d), "bf16"), _rand(rng, (L, Hkv, d), "bf16"), _rand(rng, (L, Hkv, d), "bf16")
    o, l = s.query(q, k, v)
    rows = [(0, 0), (8, 7), (3, 5), (4, 2)]
    orow, lrow = s.query(q, k, v, rows=rows)
    for r, (i, h) in enumerate(rows):
        np.testing.assert_array_equal(orow[r], o[i, h])
        assert lrow[r] == l[i, h]


def test_bf16_inputs_are_widened_exactly():
    """bf16 -> fp64 is exact, so the oracle on bf16 bits equals the oracle on the same values
    held in fp32."""
    Hq, Hkv, d, n = 4, 1, 8, 12
    rng = np.random.default_rng(13)
    k16, v16, q16 = _rand(rng, (n, Hkv, d), "bf16"), _rand(rng, (n, Hkv, d), "bf16"), _rand(rng, (2, Hq, d), "bf16")
    a = OracleSession("bf16", Hq, Hkv, d)
    a.append(np.zeros((n, Hq, d), np.uint16), k16, v16)
    b = OracleSession("f32", Hq, Hkv, d)
    f = lambda x: synth.raw_to_f64(x).astype(np.float32)
    b.append(np.zeros((n, Hq, d), np.float32), f(k16), f(v16))
    oa, la = a.query(q16)
    ob, lb = b.query(f(q16))
    np.testing.assert_array_equal(oa, ob)
    np.testing.assert_array_equal(la, lb)


def test_eviction_attends_over_frozen_prefix_and_retained_window_only():
    """Region 0 frozen, Region 1 FIFO-evicted (Sec. 3.3; Alg. 1 evict_oldest): after evicting, every
    row equals a pure-Python softmax over [frozen tokens ; retained tokens] in their original order;
    a needle in the frozen region is still retrieved, one in the evicted range is lost (Sec. 5.3:
    evicted data can no longer be attended to), evicting nothing changes nothing."""
    Hq, Hkv, d, n, nf, ne = 2, 1, 4, 20, 5, 7
    rng = np.random.default_rng(11)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (2, Hq, d), "f32")
    s = OracleSession("f32", Hq, Hkv, d)
    s.append(np.zeros((n, Hq, d), np.float32), K, V)
    before = s.query(q)
    s.freeze(nf)
    s.evict_oldest(0)
    np.testing.assert_array_equal(s.query(q)[0], before[0])
    s.evict_oldest(ne)
    assert s.length == n - ne
    keep = list(range(nf)) + list(range(nf + ne, n))
    np.testing.assert_array_equal(s.cache()[0], K[keep])
    o, l = s.query(q)
    for i in range(2):
        for h in range(Hq):
            ro, rl = _brute_row(q[i, h].tolist(), [K[t, 0].tolist() for t in keep], [V[t, 0].tolist() for t in keep], 0.5)
            np.testing.assert_allclose(o[i, h], ro, rtol=1e-12, atol=1e-13)
            assert abs(l[i, h] - rl) < 1e-12
    # appended tokens go behind the retained window and see all of it
    k2, v2, q2 = _rand(rng, (3, Hkv, d), "f32"), _rand(rng, (3, Hkv, d), "f32"), _rand(rng, (3, Hq, d), "f32")
    o2, _ = s.append(q2, k2, v2)
    ro, _ = _brute_row(q2[0, 1].tolist(), [K[t, 0].tolist() for t in keep] + [k2[0, 0].tolist()],
                       [V[t, 0].tolist() for t in keep] + [v2[0, 0].tolist()], 0.5)
    np.testing.assert_allclose(o2[0, 1], ro, rtol=1e-12, atol=1e-13)
    # needles: frozen survives, evicted is lost
    for pos, survives in ((2, True), (8, False)):
        t = OracleSession("f32", Hq, Hkv, d)
        K2 = K.copy(); K2[pos, 0] = 300.0 * q[0, 0] / np.linalg.norm(q[0, 0])
        t.append(np.zeros((n, Hq, d), np.float32), K2, V)
        t.freeze(nf); t.evict_oldest(ne)
        got = t.query(q)[0][0, 0]
        assert np.allclose(got, V[pos, 0].astype(np.float64), atol=1e-9) == survives
    with pytest.raises(ValueError):
        s.evict_oldest(s.length - nf + 1)              # more than Region 1 holds
    with pytest.raises(ValueError):
        s.freeze(nf - 1)                               # the frozen region only grows


def test_fork_is_a_prefix_by_value():
    """fork(n) reads like the source cut at n tokens (brute force on the first n tokens), and the
    two sessions are isolated afterwards (the session isolation of Sec. 3.4)."""
    Hq, Hkv, d, n, n_prefix = 2, 2, 3, 9, 6
    rng = np.random.default_rng(12)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (1, Hq, d), "f32")
    s = OracleSession("f32", Hq, Hkv, d)
    s.append(np.zeros((n, Hq, d), np.float32), K, V)
    t = s.fork(n_prefix)
    o, l = t.query(q)
    for h in range(Hq):
        ro, rl = _brute_row(q[0, h].tolist(), [K[j, h].tolist() for j in range(n_prefix)],
                            [V[j, h].tolist() for j in range(n_prefix)], 1.0 / math.sqrt(d))
        np.testing.assert_allclose(o[0, h], ro, rtol=1e-12, atol=1e-13)
        assert abs(l[0, h] - rl) < 1e-12
    before = s.query(q)
    t.append(_rand(rng, (2, Hq, d), "f32"), _rand(rng, (2, Hkv, d), "f32"), _rand(rng, (2, Hkv, d), "f32"))
    t.evict_oldest(3)
    np.testing.assert_array_equal(s.query(q)[0], before[0])
    assert s.length == n and t.length == n_prefix + 2 - 3


def test_truncate_keeps_exactly_the_first_p_tokens():
    """SeqRemove(s, p, infinity) of Sec. 3.9.3: after truncate(p) every row equals a pure-Python
    softmax over the first p committed tokens (an off-by-one in the cut fails: p-1 and p+1 keys give
    other numbers), appends continue at position p, and the literal Strip / Extend / Clear cycle
    (append, read, truncate back) returns what the non-committing query returns and leaves the cache
    as it was."""
    Hq, Hkv, d, n = 2, 1, 3, 11
    rng = np.random.default_rng(13)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (2, Hq, d), "f32")
    scale = 1.0 / math.sqrt(d)
    for p in (n, 7, 1):
        s = OracleSession("f32", Hq, Hkv, d)
        s.append(np.zeros((n, Hq, d), np.float32), K, V)
        s.truncate(p)
        assert s.length == p
        np.testing.assert_array_equal(s.cache()[0], K[:p])
        np.testing.assert_array_equal(s.cache()[1], V[:p])
        o, l = s.query(q)
        for i in range(2):
            for h in range(Hq):
                ro, rl = _brute_row(q[i, h].tolist(), [K[j, 0].tolist() for j in range(p)],
                                    [V[j, 0].tolist() for j in range(p)], scale)
                np.testing.assert_allclose(o[i, h], ro, rtol=1e-12, atol=1e-13)
                assert abs(l[i, h] - rl) < 1e-12
                if 1 < p < n:      # the neighbours of the cut are different numbers, so the check can fail
                    for wrong in (p - 1, p + 1):
                        wo, _ = _brute_row(q[i, h].tolist(), [K[j, 0].tolist() for j in range(wrong)],
                                           [V[j, 0].tolist() for j in range(wrong)], scale)
                        assert np.abs(np.array(wo) - o[i, h]).max() > 1e-6
        # the next append lands at position p: its first row sees p + 1 keys
        k2, v2, q2 = _rand(rng, (2, Hkv, d), "f32"), _rand(rng, (2, Hkv, d), "f32"), _rand(rng, (2, Hq, d), "f32")
        o2, _ = s.append(q2, k2, v2)
        ro, _ = _brute_row(q2[0, 1].tolist(), [K[j, 0].tolist() for j in range(p)] + [k2[0, 0].tolist()],
                           [V[j, 0].tolist() for j in range(p)] + [v2[0, 0].tolist()], scale)
        np.testing.assert_allclose(o2[0, 1], ro, rtol=1e-12, atol=1e-13)
        assert s.length == p + 2
    # Extend then Clear == non-committing query (Sec. 3.9.3), cache restored bit for bit
    s = OracleSession("f32", Hq, Hkv, d)
    s.append(np.zeros((n, Hq, d), np.float32), K, V)
    qq, kq, vq = _rand(rng, (3, Hq, d), "f32"), _rand(rng, (3, Hkv, d), "f32"), _rand(rng, (3, Hkv, d), "f32")
    pure = s.query(qq, kq, vq)
    lit = s.append(qq, kq, vq)
    s.truncate(n)
    np.testing.assert_array_equal(pure[0], lit[0])
    np.testing.assert_array_equal(pure[1], lit[1])
    np.testing.assert_array_equal(s.cache()[0], K)
    with pytest.raises(ValueError):
        s.truncate(n + 1)
    with pytest.raises(ValueError):
        s.truncate(-1)
    s.truncate(0)
    assert s.length == 0
    with pytest.raises(ZeroDivisionError):
        s.query(q)


def test_truncate_and_fork_below_the_frozen_length_clip_it():
    """Region 0 cannot be longer than the session (Sec. 3.3): cutting a session, or forking a prefix,
    below n_frozen leaves a frozen region of the new length, so a later eviction starts behind it
    (brute force over the expected survivors); cutting above n_frozen leaves it alone."""
    Hq, Hkv, d, n, nf = 1, 1, 2, 12, 6
    rng = np.random.default_rng(14)
    K, V = _rand(rng, (n, Hkv, d), "f32"), _rand(rng, (n, Hkv, d), "f32")
    q = _rand(rng, (1, Hq, d), "f32")
    k2, v2 = _rand(rng, (5, Hkv, d), "f32"), _rand(rng, (5, Hkv, d), "f32")
    scale = 1.0 / math.sqrt(d)

    def fresh():
        s = OracleSession("f32", Hq, Hkv, d)
        s.append(np.zeros((n, Hq, d), np.float32), K, V)
        s.freeze(nf)
        return s

    def expect(s, keys, vals):
        o, l = s.query(q)
        ro, rl = _brute_row(q[0, 0].tolist(), [x.tolist() for x in keys], [x.tolist() for x in vals], scale)
        np.testing.assert_allclose(o[0, 0], ro, rtol=1e-12, atol=1e-13)
        assert abs(l[0, 0] - rl) < 1e-12

    # cut below the frozen length: frozen becomes 4; five new tokens, evict two -> the new tokens 0,1 go
    for make in (lambda: (lambda s: (s.truncate(4), s)[1])(fresh()), lambda: fresh().fork(4)):
        s = make()
        assert s.n_frozen == 4 and s.length == 4
        s.append(np.zeros((5, Hq, d), np.float32), k2, v2)
        s.evict_oldest(2)
        expect(s, list(K[:4, 0]) + list(k2[2:, 0]), list(V[:4, 0]) + list(v2[2:, 0]))
        with pytest.raises(ValueError):
            s.evict_oldest(4)                      # only three unfrozen tokens are left
    # cut above it: frozen stays 6; evicting two drops tokens 6 and 7
    for make in (lambda: (lambda s: (s.truncate(9), s)[1])(fresh()), lambda: fresh().fork(9)):
        s = make()
        assert s.n_frozen == nf and s.length == 9
        s.evict_oldest(2)
        expect(s, list(K[:6, 0]) + list(K[8:9, 0]), list(V[:6, 0]) + list(V[8:9, 0]))
    # the source of a fork keeps its own frozen length
    s = fresh(); s.fork(2)
    assert s.n_frozen == nf and s.length == n


def test_pool_destroy_forgets_the_session_and_nothing_else():
    """Sec. 3.4 session life cycle: a destroyed session is gone (its id is no longer served), the
    others still read exactly what they read before, and a new session starts empty."""
    pool = OraclePool("f32", 2, 1, 2)
    a, b = pool.create(), pool.create()
    rng = np.random.default_rng(15)
    for sid in (a, b):
        pool.sessions[sid].append(_rand(rng, (3, 2, 2), "f32"), _rand(rng, (3, 1, 2), "f32"), _rand(rng, (3, 1, 2), "f32"))
    q = _rand(rng, (1, 2, 2), "f32")
    before = pool.sessions[b].query(q)
    pool.destroy(a)
    assert a not in pool.sessions and b in pool.sessions
    with pytest.raises(KeyError):
        pool.batch_step([a], [OP_QUERY_A], [0, 1], q, None, None)
    with pytest.raises(KeyError):
        pool.destroy(a)
    after = pool.sessions[b].query(q)
    np.testing.assert_array_equal(before[0], after[0])
    c = pool.create()
    assert c != b and pool.sessions[c].length == 0
