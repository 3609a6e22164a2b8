"""Host-side logic of the library, exercised without a GPU through a metadata-only pool:
C-ABI exports, sizes, the block allocator (all-or-nothing, reuse, permuted order), session
life cycle, argument checks."""
import ctypes
import os
import re

import pytest

import paper_2605_13784_amd as sk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def meta_pool(**kw):
    args = dict(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, block_tokens=16, n_blocks=64,
                max_sessions=4, metadata_only=True)
    args.update(kw)
    return sk.Pool(**args)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sk.h")).read()
    declared = set(re.findall(r"\b(sk_[a-z0-9_]+)\s*\(", header))
    declared -= {"sk_pool_desc", "sk_pool_stats", "sk_launch_info", "sk_status", "sk_pool", "sk_profile"}
    assert declared == set(sk.EXPORTS)
    L = sk.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert L.sk_version() >= 1


def test_memory_model_matches_paper_formula():
    """Sec. 5.3: M_KV = 2 * L * d * n_ctx * sizeof.  Per layer, with d = n_kv_heads*head_dim = 4096,
    32K tokens, 2-byte elements: 2*4096*32768*2 bytes; times L = 32 layers is the printed ~17 GB."""
    golden = open(os.path.join(ROOT, "tests", "golden", "memory_model.txt")).read()
    per_session = int(re.search(r"M_KV_bytes\s*=\s*(\d+)", golden).group(1))
    assert per_session == 2 * 32 * 4096 * 32768 * 2
    desc = sk.make_desc("bf16", 32, 32, 128, 16, 32768 // 16)
    assert sk.sk_pool_kv_bytes(desc) * 32 == per_session
    assert round(per_session / 1e9) == 17
    # grouped-query shape of the workloads: 8 KV heads -> a quarter of that, 4096 bytes per token
    desc = sk.make_desc("bf16", 32, 8, 128, 16, 32768 // 16)
    assert sk.sk_pool_kv_bytes(desc) == 32768 * 4096


def test_bad_descriptions_are_rejected():
    assert sk.sk_pool_kv_bytes(sk.make_desc("bf16", 32, 5, 128, 16, 8)) == 0      # heads not divisible
    assert sk.sk_pool_kv_bytes(sk.make_desc("bf16", 32, 8, 96, 16, 8)) == 0       # head_dim
    assert sk.sk_pool_kv_bytes(sk.make_desc("bf16", 32, 8, 128, 24, 8)) == 0      # block not power of two
    assert sk.sk_pool_kv_bytes(sk.make_desc("bf16", 32, 8, 128, 8, 8)) == 0       # block too small
    assert sk.sk_pool_kv_bytes(sk.make_desc("bf16", 32, 8, 128, 16, 0)) == 0
    with pytest.raises(sk.SkError):
        meta_pool(head_dim=100)
    # a device pool needs memory
    d = sk.make_desc("f32", 4, 4, 64, 16, 8)
    h = ctypes.c_void_p()
    assert sk.lib().sk_pool_create(ctypes.byref(d), ctypes.byref(h)) == sk.SK_E_INVAL
    assert not h.value


def test_allocator_all_or_nothing_and_reuse():
    p = meta_pool(n_blocks=10, block_tokens=16)
    a, b = p.sk_session_create(), p.sk_session_create()
    assert p.sk_pool_blocks_free() == 10
    p.reserve(a, 17)                       # 2 blocks
    assert p.sk_session_length(a) == 17 and p.sk_session_block_table(a) == [0, 1]
    p.reserve(a, 15)                       # fills block 1 exactly
    assert p.sk_session_length(a) == 32 and len(p.sk_session_block_table(a)) == 2
    p.reserve(b, 1)
    assert p.sk_session_block_table(b) == [2]
    p.reserve(a, 1)
    assert p.sk_session_block_table(a) == [0, 1, 3]
    assert p.sk_pool_blocks_free() == 6
    # needs 7 blocks, 6 free: refused, nothing changes
    before = (p.sk_session_length(a), p.sk_session_block_table(a), p.sk_pool_blocks_free())
    with pytest.raises(sk.SkError) as e:
        p.reserve(a, 15 + 16 * 6 + 1)
    assert e.value.status == sk.SK_E_NOMEM
    assert before == (p.sk_session_length(a), p.sk_session_block_table(a), p.sk_pool_blocks_free())
    p.reserve(a, 15 + 16 * 6)              # exactly fits
    assert p.sk_pool_blocks_free() == 0
    with pytest.raises(sk.SkError):
        p.reserve(b, 16)                   # b has 15 slots left in its block, 16 needs one more
    p.reserve(b, 15)
    # destroy returns blocks; they are reused in return order
    p.sk_session_destroy(a)
    assert p.sk_pool_blocks_free() == 9
    c = p.sk_session_create()
    assert c == a                          # ids are reused
    assert p.sk_session_length(c) == 0
    p.reserve(c, 16)
    assert p.sk_session_block_table(c) == [0]
    with pytest.raises(sk.SkError) as e:
        p.sk_session_length(3)
    assert e.value.status == sk.SK_E_BADSESSION


def test_permuted_alloc_order_and_its_checks():
    p = meta_pool(n_blocks=8)
    p.sk_pool_set_alloc_order([7, 3, 5, 1, 0, 2, 4, 6])
    a, b = p.sk_session_create(), p.sk_session_create()
    p.reserve(a, 16); p.reserve(b, 16); p.reserve(a, 16); p.reserve(b, 32)
    assert p.sk_session_block_table(a) == [7, 5]
    assert p.sk_session_block_table(b) == [3, 1, 0]
    with pytest.raises(sk.SkError):
        p.sk_pool_set_alloc_order(list(range(8)))          # blocks in use
    q = meta_pool(n_blocks=4)
    with pytest.raises(sk.SkError):
        q.sk_pool_set_alloc_order([0, 1, 2])                # wrong length
    with pytest.raises(sk.SkError):
        q.sk_pool_set_alloc_order([0, 1, 1, 2])             # not a permutation


def test_session_limits():
    p = meta_pool(max_sessions=2, n_blocks=100, max_session_tokens=40, max_batch_tokens=64)
    a, b = p.sk_session_create(), p.sk_session_create()
    with pytest.raises(sk.SkError) as e:
        p.sk_session_create()
    assert e.value.status == sk.SK_E_NOMEM
    p.reserve(a, 40)
    with pytest.raises(sk.SkError) as e:
        p.reserve(a, 1)                                      # longest session reached
    assert e.value.status == sk.SK_E_NOMEM
    with pytest.raises(sk.SkError) as e:
        p.reserve(b, 65)                                     # more than max_batch_tokens in one call
    assert e.value.status == sk.SK_E_WORKSPACE
    p.reserve(b, 0)                                          # no-op
    assert p.sk_session_length(b) == 0
    # compute calls on a metadata-only pool say so
    h = p.h
    rc = sk.lib().sk_session_query(h, a, None, None, None, 4, None, 0, None, 0, None)
    assert rc == sk.SK_E_NODEVICE
    assert sk.lib().sk_session_query(h, a, None, None, None, -1, None, 0, None, 0, None) == sk.SK_E_INVAL
    assert sk.lib().sk_strerror(sk.SK_E_NOMEM).decode() == "pool exhausted"


def test_element_offsets_describe_the_layout():
    p = meta_pool(n_blocks=4, block_tokens=16)
    e = 2
    blk = 2 * 16 * 128 * e                         # one (head, block): K then V
    assert p.sk_pool_element_offset(0, 0, False, 0, 0) == 0
    assert p.sk_pool_element_offset(1, 0, False, 0, 0) == blk
    assert p.sk_pool_element_offset(0, 1, False, 0, 0) == 4 * blk          # heads are outermost
    assert p.sk_pool_element_offset(0, 0, False, 3, 5) == (3 * 128 + 5) * e
    assert p.sk_pool_element_offset(0, 0, True, 3, 5) == 16 * 128 * e + (5 * 16 + 3) * e    # V is [dim][token] per 16-token group
    big = meta_pool(n_blocks=4, block_tokens=64)
    v0 = 64 * 128 * e
    assert big.sk_pool_element_offset(0, 0, True, 3, 5) == v0 + (5 * 16 + 3) * e
    assert big.sk_pool_element_offset(0, 0, True, 16 + 3, 5) == v0 + (128 * 16 + 5 * 16 + 3) * e   # next group: 4 KiB on
    assert big.sk_pool_element_offset(0, 0, True, 63, 127) == v0 + (3 * 128 * 16 + 127 * 16 + 15) * e == 2 * v0 - e
    assert p.sk_pool_element_offset(4, 0, False, 0, 0) == -1
    f = meta_pool(dtype="f32", n_q_heads=4, n_kv_heads=4, head_dim=64, n_blocks=4)
    assert f.sk_pool_element_offset(0, 0, True, 3, 5) == 16 * 64 * 4 + (3 * 64 + 5) * 4       # V is [token][dim]


def test_truncate_returns_whole_blocks_only():
    p = meta_pool(n_blocks=8)
    a = p.sk_session_create()
    p.reserve(a, 40)                        # blocks 0,1,2
    p.sk_session_truncate(a, 33)
    assert p.sk_session_length(a) == 33 and p.sk_session_block_table(a) == [0, 1, 2]
    p.sk_session_truncate(a, 32)
    assert p.sk_session_block_table(a) == [0, 1] and p.sk_pool_blocks_free() == 6
    p.sk_session_truncate(a, 0)
    assert p.sk_session_block_table(a) == [] and p.sk_pool_blocks_free() == 8
    with pytest.raises(sk.SkError):
        p.sk_session_truncate(a, 1)         # cannot grow
    p.reserve(a, 16)
    assert p.sk_session_block_table(a) == [3]          # freed blocks queue behind the untouched ones


def test_eviction_metadata():
    """Region-1 FIFO eviction behind a frozen prefix: lengths count retained tokens, blocks that
    hold only evicted tokens return to the pool at once, the table is compacted, appends continue
    behind the window, truncate and freeze respect the frozen region."""
    p = meta_pool(n_blocks=16, block_tokens=16)
    a = p.sk_session_create()
    p.reserve(a, 100)                                   # blocks 0..6
    p.sk_session_freeze(a, 20)                          # frozen: block 0 and 4 tokens of block 1
    assert p.sk_session_length(a) == 100
    p.sk_session_evict_oldest(a, 10)                    # storage [20,30): inside block 1, nothing freed
    assert p.sk_session_length(a) == 90 and p.sk_session_block_table(a) == [0, 1, 2, 3, 4, 5, 6]
    p.sk_session_evict_oldest(a, 30)                    # storage [20,60): blocks 2 and 3... block 2 = [32,48) goes, block 3 = [48,64) stays
    assert p.sk_session_length(a) == 60 and p.sk_session_block_table(a) == [0, 1, 3, 4, 5, 6]
    assert p.sk_pool_blocks_free() == 10
    p.sk_session_evict_oldest(a, 4)                     # up to the end of block 3: it goes too
    assert p.sk_session_block_table(a) == [0, 1, 4, 5, 6] and p.sk_session_length(a) == 56
    with pytest.raises(sk.SkError) as e:
        p.sk_session_evict_oldest(a, 37)                # only 36 tokens left behind the frozen region
    assert e.value.status == sk.SK_E_INVAL and p.sk_session_length(a) == 56
    with pytest.raises(sk.SkError):
        p.sk_session_freeze(a, 30)                      # not after an eviction
    p.reserve(a, 20)                                    # 4 tokens fill block 6, one new block
    assert p.sk_session_length(a) == 76 and len(p.sk_session_block_table(a)) == 6
    p.sk_session_truncate(a, 25)                        # 20 frozen + 5 of the window
    assert p.sk_session_length(a) == 25
    p.sk_session_truncate(a, 7)                         # into the frozen region
    assert p.sk_session_length(a) == 7 and p.sk_session_block_table(a) == [0]
    p.sk_session_evict_oldest(a, 0)
    with pytest.raises(sk.SkError):
        p.sk_session_evict_oldest(a, 1)                 # nothing behind the frozen region
    st = p.sk_pool_get_stats()
    assert st["tokens_evicted"] == 44


def test_fork_shares_blocks_by_reference_count():
    """Fork = table copy + one block at most: full blocks of the prefix are shared, a partly filled
    last block is replaced by a fresh one; a shared block returns to the free list only when its last
    holder lets go, whichever way (destroy, truncate, evict)."""
    p = meta_pool(n_blocks=12, block_tokens=16, max_sessions=4)
    a = p.sk_session_create()
    p.reserve(a, 70)                                     # blocks 0..4
    b = p.sk_session_fork(a, 48)                         # three full blocks, shared
    assert p.sk_session_block_table(b) == [0, 1, 2] and p.sk_session_length(b) == 48
    assert p.sk_pool_blocks_free() == 7
    c = p.sk_session_fork(a, 40)                         # 2 shared + a copy of the third
    assert p.sk_session_block_table(c) == [0, 1, 5] and p.sk_pool_blocks_free() == 6
    p.reserve(b, 10)                                     # b's next tokens go to a block of its own
    assert p.sk_session_block_table(b) == [0, 1, 2, 6]
    p.sk_session_destroy(a)                              # blocks 3, 4 free; 0, 1, 2 still held
    assert p.sk_pool_blocks_free() == 7
    p.sk_session_truncate(b, 16)                         # b drops 1, 2, 6: 2 and 6 free, 1 still held by c
    assert p.sk_pool_blocks_free() == 9
    p.sk_session_evict_oldest(c, 32)                     # c drops 0 and 1: 1 free now, 0 still held by b
    assert p.sk_session_block_table(c) == [5] and p.sk_pool_blocks_free() == 10
    p.sk_session_destroy(b)
    p.sk_session_destroy(c)
    assert p.sk_pool_blocks_free() == 12
    # the hole travels with the prefix
    a = p.sk_session_create()
    p.reserve(a, 100)
    p.sk_session_freeze(a, 10)
    p.sk_session_evict_oldest(a, 25)                     # retained 75: [0,10) + storage [19,84) after dropping one block
    d = p.sk_session_fork(a, 30)
    assert p.sk_session_length(d) == 30
    p.sk_session_evict_oldest(d, 20)
    assert p.sk_session_length(d) == 10
    with pytest.raises(sk.SkError):
        p.sk_session_evict_oldest(d, 1)                  # only the frozen tokens are left
    with pytest.raises(sk.SkError) as e:
        p.sk_session_fork(a, 76)
    assert e.value.status == sk.SK_E_INVAL
    e2 = p.sk_session_fork(a, 0)
    assert p.sk_session_length(e2) == 0 and p.sk_session_block_table(e2) == []
    assert p.sk_pool_get_stats()["forks"] == 4


def test_append_into_a_shared_block_takes_a_copy_first():
    """After a fork, a truncation can leave a session's end inside a block that another session still
    reads.  The next append must not write there: the session swaps that block for a fresh one (one
    extra block, counted in the all-or-nothing check), the other holder keeps the old one."""
    p = meta_pool(n_blocks=8, block_tokens=16, max_sessions=3)
    a = p.sk_session_create()
    p.reserve(a, 64)                                     # blocks 0..3, all full
    b = p.sk_session_fork(a, 64)                         # all four shared
    assert p.sk_session_block_table(b) == [0, 1, 2, 3] and p.sk_pool_blocks_free() == 4
    p.sk_session_truncate(a, 40)                         # a ends inside block 2, which b still reads
    assert p.sk_session_block_table(a) == [0, 1, 2] and p.sk_pool_blocks_free() == 4
    p.reserve(a, 4)                                      # stays inside the block: still needs the copy
    assert p.sk_session_block_table(a) == [0, 1, 4] and p.sk_session_block_table(b) == [0, 1, 2, 3]
    assert p.sk_pool_blocks_free() == 3
    p.reserve(a, 4)                                      # the block is a's alone now: nothing more to take
    assert p.sk_session_block_table(a) == [0, 1, 4] and p.sk_pool_blocks_free() == 3
    # the fork side: b truncates into block 1 (shared with a) and grows past it
    p.sk_session_truncate(b, 20)                         # b lets go of 2 and 3 (nobody else holds them now)
    assert p.sk_pool_blocks_free() == 5
    p.reserve(b, 30)                                     # copy of block 1 + two more blocks
    tb = p.sk_session_block_table(b)
    assert tb[0] == 0 and tb[1] not in (1, 4) and len(tb) == 4 and p.sk_pool_blocks_free() == 2
    assert p.sk_session_block_table(a) == [0, 1, 4]
    # all-or-nothing: the copy counts
    c = p.sk_session_fork(a, 32)                         # shares 0 and 1 with a
    p.sk_session_truncate(c, 17)
    p.reserve(a, 16 * 2 - 8)                             # a fills its last block and takes the two free ones
    assert p.sk_pool_blocks_free() == 0
    with pytest.raises(sk.SkError) as e:
        p.reserve(c, 1)                                  # would need a copy of block 1: no block left
    assert e.value.status == sk.SK_E_NOMEM and p.sk_session_length(c) == 17 and p.sk_session_block_table(c) == [0, 1]
    for s in (a, b, c):
        p.sk_session_destroy(s)
    assert p.sk_pool_blocks_free() == 8


# ---- a call that fails half way leaves the pool as it was (Alg. 1: an append is one step) ----

def _state(p, sids):
    return ([(p.sk_session_length(s), p.sk_session_block_table(s)) for s in sids], p.sk_pool_blocks_free())


def _grow_to_next_blocks(p, sid, n_tokens):
    """Blocks the next n_tokens-token append of `sid` would take, read off a run that is then undone."""
    before = p.sk_session_block_table(sid)
    n0 = p.sk_session_length(sid)
    p.reserve(sid, n_tokens)
    got = p.sk_session_block_table(sid)[len(before):]
    p.sk_session_truncate(sid, n0)
    return got


SITES_APPEND = [sk.SK_SITE_SCATTER, sk.SK_SITE_ATTENTION]


@pytest.mark.parametrize("site", SITES_APPEND + [sk.SK_SITE_RING, sk.SK_SITE_UPLOAD])
def test_append_that_fails_late_changes_nothing(site):
    """Every failure site of an append, forced by the test hook on a metadata-only pool (which walks
    the same steps without the HIP calls): status is an error, lengths, block tables and the number
    and ORDER of free blocks are as before (the next append gets the blocks it would have got)."""
    long_list = site in (sk.SK_SITE_RING, sk.SK_SITE_UPLOAD)      # only a list too long for the kernel arguments is uploaded
    L = 16 * 100 if long_list else 40
    p, twin = (meta_pool(n_blocks=400, max_batch_tokens=2048) for _ in range(2))
    for q in (p, twin):
        q.sk_pool_set_alloc_order(list(range(399, -1, -1)))
        a, b = q.sk_session_create(), q.sk_session_create()
        q.reserve(a, 21); q.reserve(b, 5)
    before = _state(p, [a, b])
    p.sk_pool_inject_failure(site, 1)
    with pytest.raises(sk.SkError) as e:
        p.reserve(a, L)
    assert e.value.status == sk.SK_E_HIP
    assert _state(p, [a, b]) == before
    # the hook is spent: the same call now succeeds and takes exactly the blocks the twin's takes
    p.reserve(a, L); twin.reserve(a, L)
    assert _state(p, [a, b]) == _state(twin, [a, b])


def test_append_into_a_shared_tail_that_fails_late_keeps_or_returns_the_copy():
    """A session whose last block is shared with a fork gets a copy of it before it appends.  If the
    call fails before the commit kernel is enqueued the copy is given back (nothing changed at all);
    if it fails after, the device block table already names the copy, so the session keeps it: its
    length and every other block are as before, and one block fewer is free."""
    for site, keeps_copy in ((sk.SK_SITE_BLOCK_COPY, False), (sk.SK_SITE_SCATTER, False), (sk.SK_SITE_ATTENTION, True)):
        p = meta_pool(n_blocks=32)
        a = p.sk_session_create()
        p.reserve(a, 40)                       # blocks 0,1,2; 8 tokens in block 2
        f = p.sk_session_fork(a, 40)           # f gets its own copy of block 2 (block 3)
        p.sk_session_truncate(f, 20)           # f now ends inside block 1, which a also holds
        before = _state(p, [a, f])
        p.sk_pool_inject_failure(site, 1)
        with pytest.raises(sk.SkError):
            p.reserve(f, 30)
        after = _state(p, [a, f])
        assert after[0][0] == before[0][0]                         # the source session never changes
        assert after[0][1][0] == before[0][1][0]                   # same length for f
        if keeps_copy:
            assert after[1] == before[1] - 1
            assert after[0][1][1][:-1] == before[0][1][1][:-1] and after[0][1][1][-1] != before[0][1][1][-1]
        else:
            assert after == before
        p.reserve(f, 30)                       # and the append still works afterwards
        assert p.sk_session_length(f) == 50 and p.sk_session_length(a) == 40


@pytest.mark.parametrize("site", [sk.SK_SITE_PLAN, sk.SK_SITE_RING, sk.SK_SITE_UPLOAD, sk.SK_SITE_SCATTER, sk.SK_SITE_ATTENTION])
def test_batch_step_that_fails_late_changes_no_session(site):
    """A multi-session step that is stopped after some (or all) of its appends were booked - the lists
    do not fit, the upload slot, the upload, a launch - takes every one of them back, in order."""
    import ctypes
    p, twin = (meta_pool(n_blocks=200, max_sessions=6, max_batch_tokens=4096) for _ in range(2))
    sids = None
    for q in (p, twin):
        sids = [q.sk_session_create() for _ in range(5)]
        for i, s in enumerate(sids):
            q.reserve(s, 7 + 13 * i)
    ops = [sk.SK_OP_APPEND, sk.SK_OP_QUERY_B, sk.SK_OP_APPEND, sk.SK_OP_QUERY_A, sk.SK_OP_APPEND]
    counts = [100, 9, 33, 5, 260]
    cu = [0]
    for c in counts:
        cu.append(cu[-1] + c)

    def step(q):
        n = len(sids)
        return sk.lib().sk_batch_step(q.h, n, (ctypes.c_int32 * n)(*sids), (ctypes.c_int32 * n)(*ops),
                                      (ctypes.c_int32 * (n + 1))(*cu), None, None, None, None, sk.SK_F32, None, None)

    before = _state(p, sids)
    p.sk_pool_inject_failure(site, 1)
    rc = step(p)
    assert rc == (sk.SK_E_WORKSPACE if site == sk.SK_SITE_PLAN else sk.SK_E_HIP)
    assert _state(p, sids) == before
    assert step(p) == sk.SK_OK and step(twin) == sk.SK_OK
    assert _state(p, sids) == _state(twin, sids)
    assert [p.sk_session_length(s) for s in sids] == [7 + 100, 20, 33 + 33, 46, 59 + 260]


def test_batch_step_too_large_for_the_upload_region_is_refused_up_front():
    """Thousands of one-token items need more list space than a small pool's region holds at the finest
    decomposition; the planner coarsens it until it fits, and a step that cannot fit is refused with
    every session unchanged (here the region is sized from max_batch_tokens, so it always fits)."""
    import ctypes
    n = 3000
    p = meta_pool(n_blocks=4096, max_sessions=n, max_batch_tokens=4096, block_tokens=16)
    sids = [p.sk_session_create() for _ in range(n)]
    for s in sids:
        p.reserve(s, 3)
    cu = list(range(n + 1))
    ops = [sk.SK_OP_APPEND] * n
    rc = sk.lib().sk_batch_step(p.h, n, (ctypes.c_int32 * n)(*sids), (ctypes.c_int32 * n)(*ops),
                                (ctypes.c_int32 * (n + 1))(*cu), None, None, None, None, sk.SK_F32, None, None)
    assert rc == sk.SK_OK
    assert all(p.sk_session_length(s) == 4 for s in sids[:50])


@pytest.mark.parametrize("site", [sk.SK_SITE_RING, sk.SK_SITE_UPLOAD])
def test_evict_that_fails_changes_nothing(site):
    p = meta_pool(n_blocks=64)
    a = p.sk_session_create()
    p.reserve(a, 200)
    p.sk_session_freeze(a, 20)
    before = _state(p, [a])
    p.sk_pool_inject_failure(site, 1)
    with pytest.raises(sk.SkError):
        p.sk_session_evict_oldest(a, 100)          # frees whole blocks: the device table would be rewritten
    assert _state(p, [a]) == before
    p.sk_session_evict_oldest(a, 100)
    assert p.sk_session_length(a) == 100
    assert p.sk_pool_blocks_free() > before[1]


@pytest.mark.parametrize("site", [sk.SK_SITE_RING, sk.SK_SITE_UPLOAD, sk.SK_SITE_BLOCK_COPY])
def test_fork_that_fails_changes_nothing(site):
    p = meta_pool(n_blocks=64, max_sessions=3)
    a = p.sk_session_create()
    p.reserve(a, 70)
    before = _state(p, [a])
    p.sk_pool_inject_failure(site, 1)
    with pytest.raises(sk.SkError):
        p.sk_session_fork(a, 41)                   # ends inside a block: table upload + one block copy
    assert _state(p, [a]) == before
    f = p.sk_session_fork(a, 41)                   # the session id was not consumed either
    g = p.sk_session_create()
    assert sorted([a, f, g]) == [0, 1, 2]
    assert p.sk_session_length(f) == 41 and p.sk_pool_blocks_free() == before[1] - 1


def test_table_offsets_must_fit_32_bits():
    """max_sessions x blocks per session is the extent of the device block tables, addressed with
    32-bit offsets: a description beyond that is refused instead of overflowing."""
    ok = sk.make_desc("bf16", 32, 8, 128, 16, 1 << 20, max_sessions=2047)
    bad = sk.make_desc("bf16", 32, 8, 128, 16, 1 << 20, max_sessions=2048)
    assert sk.sk_pool_workspace_bytes(ok) > 0
    assert sk.sk_pool_workspace_bytes(bad) == 0
