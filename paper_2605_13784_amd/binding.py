"""ctypes binding of libsk.so: the same entry points as include/sk.h, argument marshalling
only.  PyTorch appears here for device memory and streams, nothing else; every step of the
path runs in the library's HIP kernels.  There is no CPU fallback: if libsk.so is missing or
a call fails, an exception is raised.
"""
import ctypes
import os
import numpy as np

import torch

from . import _build

SK_F32, SK_BF16 = 0, 1
SK_OP_APPEND, SK_OP_QUERY_A, SK_OP_QUERY_B = 0, 1, 2
SK_POOL_METADATA_ONLY = 1

SK_SITE_RING, SK_SITE_UPLOAD, SK_SITE_BLOCK_COPY, SK_SITE_SCATTER, SK_SITE_ATTENTION, SK_SITE_COMBINE, SK_SITE_PLAN = 1, 2, 3, 4, 5, 6, 7
SK_TOP2_STATIC_BYTES = 1 << 20

SK_OK = 0
SK_E_INVAL, SK_E_SHAPE, SK_E_DTYPE, SK_E_NOMEM, SK_E_BADSESSION = -1, -2, -3, -4, -5
SK_E_EMPTY, SK_E_WORKSPACE, SK_E_HIP, SK_E_NODEVICE = -6, -7, -8, -9


class SkError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s: %s (%d)" % (where, lib().sk_strerror(status).decode(), status)
        if status == SK_E_HIP:
            msg += " hipError=%d" % lib().sk_last_hip_error()
        super().__init__(msg)


class sk_pool_desc(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("max_sessions", ctypes.c_int32),
        ("n_blocks", ctypes.c_int64), ("max_session_tokens", ctypes.c_int64),
        ("max_batch_tokens", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("reserved", ctypes.c_int32),
        ("kv_mem", ctypes.c_void_p), ("kv_bytes", ctypes.c_size_t),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


class sk_pool_stats(ctypes.Structure):
    _fields_ = [("tokens_appended", ctypes.c_int64), ("tokens_queried", ctypes.c_int64),
                ("launches", ctypes.c_int64), ("kv_bytes_streamed", ctypes.c_int64),
                ("tokens_evicted", ctypes.c_int64), ("forks", ctypes.c_int64)]


class sk_launch_info(ctypes.Structure):
    _fields_ = [("workgroups", ctypes.c_int32), ("n_splits", ctypes.c_int32),
                ("row_tiles", ctypes.c_int32), ("kernel_variant", ctypes.c_int32),
                ("fused_merge", ctypes.c_int32), ("reserved", ctypes.c_int32 * 3)]


class sk_profile(ctypes.Structure):
    _fields_ = [("calls", ctypes.c_int64), ("attention_ms", ctypes.c_double), ("combine_ms", ctypes.c_double)]


EXPORTS = [
    "sk_pool_kv_bytes", "sk_pool_workspace_bytes", "sk_pool_create", "sk_pool_destroy",
    "sk_pool_blocks_free", "sk_pool_set_alloc_order", "sk_session_create", "sk_session_destroy",
    "sk_session_length", "sk_session_block_table", "sk_session_append", "sk_session_query",
    "sk_batch_step", "sk_session_query_shared_prefix", "sk_session_gather",
    "sk_session_truncate", "sk_session_freeze", "sk_session_evict_oldest", "sk_session_fork",
    "sk_pool_set_profiling", "sk_pool_read_profile",
    "sk_pool_element_offset", "sk_pool_get_stats", "sk_pool_last_launch", "sk_strerror",
    "sk_last_hip_error", "sk_version", "sk_top2_workspace_bytes", "sk_top2", "sk_top2_static",
    "sk_pool_inject_failure", "sk_probe_read", "sk_probe_mfma",
]

_lib = None


def lib_path():
    return _build.LIB


def lib():
    """Loads libsk.so (building it only if no built library is there)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    elif _build.is_stale():
        import warnings
        warnings.warn("%s is older than its sources; run paper_2605_13784_amd._build.build()" % _build.LIB, RuntimeWarning)
    L = ctypes.CDLL(_build.LIB)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    P = ctypes.POINTER
    L.sk_pool_kv_bytes.restype = sz
    L.sk_pool_kv_bytes.argtypes = [P(sk_pool_desc)]
    L.sk_pool_workspace_bytes.restype = sz
    L.sk_pool_workspace_bytes.argtypes = [P(sk_pool_desc)]
    L.sk_pool_create.argtypes = [P(sk_pool_desc), P(vp)]
    L.sk_pool_destroy.argtypes = [vp]
    L.sk_pool_blocks_free.argtypes = [vp, P(i64)]
    L.sk_pool_set_alloc_order.argtypes = [vp, P(i32), i64]
    L.sk_session_create.argtypes = [vp, P(i32)]
    L.sk_session_destroy.argtypes = [vp, i32]
    L.sk_session_length.argtypes = [vp, i32, P(i64)]
    L.sk_session_block_table.argtypes = [vp, i32, P(P(i32)), P(i64)]
    L.sk_session_append.argtypes = [vp, i32, vp, vp, vp, i32, vp, ctypes.c_int, vp, vp]
    L.sk_session_query.argtypes = [vp, i32, vp, vp, vp, i32, vp, ctypes.c_int, vp, i32, vp]
    L.sk_batch_step.argtypes = [vp, i32, P(i32), P(i32), P(i32), vp, vp, vp, vp, ctypes.c_int, vp, vp]
    L.sk_session_query_shared_prefix.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp, i32, i32,
                                                 vp, vp, ctypes.c_int, vp, vp, vp]
    L.sk_session_gather.argtypes = [vp, i32, i64, i64, vp, vp, vp]
    L.sk_session_truncate.argtypes = [vp, i32, i64]
    L.sk_session_freeze.argtypes = [vp, i32, i64]
    L.sk_session_evict_oldest.argtypes = [vp, i32, i64, vp]
    L.sk_session_fork.argtypes = [vp, i32, i64, P(i32), vp]
    L.sk_top2_workspace_bytes.restype = ctypes.c_size_t
    L.sk_top2_workspace_bytes.argtypes = [i32, i32]
    L.sk_top2.argtypes = [vp, i32, i32, i64, vp, ctypes.c_size_t, vp, vp, vp, vp, vp, vp]
    L.sk_top2_static.argtypes = [vp, i32, i32, i64, vp, vp, vp, vp, vp, vp]
    L.sk_pool_inject_failure.argtypes = [vp, i32, i32]
    L.sk_probe_read.argtypes = [vp, ctypes.c_size_t, i32, i32, vp, vp]
    L.sk_probe_mfma.argtypes = [i32, i32, vp, ctypes.c_size_t, vp, P(ctypes.c_double), vp]
    L.sk_pool_set_profiling.argtypes = [vp, ctypes.c_int]
    L.sk_pool_read_profile.argtypes = [vp, P(sk_profile), P(ctypes.c_float), P(ctypes.c_float), i32]
    L.sk_pool_element_offset.restype = i64
    L.sk_pool_element_offset.argtypes = [vp, i64, i32, i32, i32, i32]
    L.sk_pool_get_stats.argtypes = [vp, P(sk_pool_stats)]
    L.sk_pool_last_launch.argtypes = [vp, P(sk_launch_info)]
    L.sk_strerror.restype = ctypes.c_char_p
    L.sk_strerror.argtypes = [ctypes.c_int]
    L.sk_last_hip_error.argtypes = []
    L.sk_version.argtypes = []
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is ctypes.c_int:
            fn.restype = ctypes.c_int
    _lib = L
    return L


def _dt(dtype):
    if dtype in ("f32", torch.float32, SK_F32):
        return SK_F32
    if dtype in ("bf16", torch.bfloat16, SK_BF16):
        return SK_BF16
    raise ValueError(dtype)


def _p(t):
    if t is None:
        return None
    assert t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(stream)


def _ck(status, where):
    if status != SK_OK:
        raise SkError(status, where)


def make_desc(dtype, n_q_heads, n_kv_heads, head_dim, block_tokens, n_blocks, max_sessions=1,
              max_session_tokens=0, max_batch_tokens=0, softmax_scale=0.0, flags=0):
    d = sk_pool_desc()
    d.dtype = _dt(dtype)
    d.n_q_heads, d.n_kv_heads, d.head_dim = n_q_heads, n_kv_heads, head_dim
    d.block_tokens, d.n_blocks, d.max_sessions = block_tokens, n_blocks, max_sessions
    d.max_session_tokens, d.max_batch_tokens = max_session_tokens, max_batch_tokens
    d.softmax_scale, d.flags = softmax_scale, flags
    return d


def sk_pool_kv_bytes(desc):
    return int(lib().sk_pool_kv_bytes(ctypes.byref(desc)))


def sk_pool_workspace_bytes(desc):
    return int(lib().sk_pool_workspace_bytes(ctypes.byref(desc)))


class Pool:
    """A pool handle plus the torch tensors that back it (allocation only)."""

    def __init__(self, dtype, n_q_heads, n_kv_heads, head_dim, block_tokens, n_blocks, max_sessions=1,
                 max_session_tokens=0, max_batch_tokens=0, softmax_scale=0.0, metadata_only=False,
                 device="cuda:0", kv_fill=None):
        self.desc = make_desc(dtype, n_q_heads, n_kv_heads, head_dim, block_tokens, n_blocks, max_sessions,
                              max_session_tokens, max_batch_tokens, softmax_scale,
                              SK_POOL_METADATA_ONLY if metadata_only else 0)
        self.dtype = "f32" if self.desc.dtype == SK_F32 else "bf16"
        self.torch_dtype = torch.float32 if self.desc.dtype == SK_F32 else torch.bfloat16
        self.Hq, self.Hkv, self.d = n_q_heads, n_kv_heads, head_dim
        self.device = device
        kvb, wsb = sk_pool_kv_bytes(self.desc), sk_pool_workspace_bytes(self.desc)
        if kvb == 0 or wsb == 0:
            raise SkError(SK_E_SHAPE, "pool description")
        self.kv_mem = self.workspace = None
        if not metadata_only:
            self.kv_mem = torch.empty(kvb, dtype=torch.uint8, device=device)
            if kv_fill is not None:
                self.kv_mem.fill_(kv_fill)
            self.workspace = torch.empty(wsb, dtype=torch.uint8, device=device)
            self.desc.kv_mem, self.desc.kv_bytes = self.kv_mem.data_ptr(), kvb
            self.desc.workspace, self.desc.workspace_bytes = self.workspace.data_ptr(), wsb
        h = ctypes.c_void_p()
        _ck(lib().sk_pool_create(ctypes.byref(self.desc), ctypes.byref(h)), "sk_pool_create")
        self.h = h

    def close(self):
        if self.h:
            if self.kv_mem is not None:
                torch.cuda.synchronize()
            lib().sk_pool_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- bookkeeping -----------------------------------------------------------------------
    def sk_pool_blocks_free(self):
        out = ctypes.c_int64()
        _ck(lib().sk_pool_blocks_free(self.h, ctypes.byref(out)), "sk_pool_blocks_free")
        return out.value

    def sk_pool_set_alloc_order(self, perm):
        arr = np.ascontiguousarray(perm, dtype=np.int32)
        _ck(lib().sk_pool_set_alloc_order(self.h, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), arr.size),
            "sk_pool_set_alloc_order")

    def sk_session_create(self):
        out = ctypes.c_int32()
        _ck(lib().sk_session_create(self.h, ctypes.byref(out)), "sk_session_create")
        return out.value

    def sk_session_destroy(self, sid):
        _ck(lib().sk_session_destroy(self.h, sid), "sk_session_destroy")

    def sk_session_length(self, sid):
        out = ctypes.c_int64()
        _ck(lib().sk_session_length(self.h, sid, ctypes.byref(out)), "sk_session_length")
        return out.value

    def sk_session_block_table(self, sid):
        tbl = ctypes.POINTER(ctypes.c_int32)()
        n = ctypes.c_int64()
        _ck(lib().sk_session_block_table(self.h, sid, ctypes.byref(tbl), ctypes.byref(n)), "sk_session_block_table")
        return [tbl[i] for i in range(n.value)]

    def sk_session_truncate(self, sid, new_length):
        _ck(lib().sk_session_truncate(self.h, sid, int(new_length)), "sk_session_truncate")

    def sk_session_freeze(self, sid, n_frozen):
        _ck(lib().sk_session_freeze(self.h, sid, int(n_frozen)), "sk_session_freeze")

    def sk_session_fork(self, src, n_prefix, stream=None):
        out = ctypes.c_int32()
        _ck(lib().sk_session_fork(self.h, src, int(n_prefix), ctypes.byref(out),
                                  _stream(stream) if self.kv_mem is not None else None), "sk_session_fork")
        return out.value

    def sk_session_evict_oldest(self, sid, n_tokens, stream=None):
        _ck(lib().sk_session_evict_oldest(self.h, sid, int(n_tokens), _stream(stream) if self.kv_mem is not None else None),
            "sk_session_evict_oldest")

    def sk_pool_set_profiling(self, enable):
        _ck(lib().sk_pool_set_profiling(self.h, int(bool(enable))), "sk_pool_set_profiling")

    def sk_pool_read_profile(self):
        """-> (sums dict, per-call attention ms list, per-call combine ms list)"""
        s = sk_profile()
        cap = 4096
        a = (ctypes.c_float * cap)()
        c = (ctypes.c_float * cap)()
        _ck(lib().sk_pool_read_profile(self.h, ctypes.byref(s), a, c, cap), "sk_pool_read_profile")
        n = min(cap, s.calls)
        return {k: getattr(s, k) for k, _ in s._fields_}, list(a[:n]), list(c[:n])

    def sk_pool_get_stats(self):
        s = sk_pool_stats()
        _ck(lib().sk_pool_get_stats(self.h, ctypes.byref(s)), "sk_pool_get_stats")
        return {k: getattr(s, k) for k, _ in s._fields_}

    def sk_pool_last_launch(self):
        s = sk_launch_info()
        _ck(lib().sk_pool_last_launch(self.h, ctypes.byref(s)), "sk_pool_last_launch")
        return {k: getattr(s, k) for k, _ in s._fields_ if k != "reserved"}

    def sk_pool_inject_failure(self, site, countdown=1):
        _ck(lib().sk_pool_inject_failure(self.h, int(site), int(countdown)), "sk_pool_inject_failure")

    def sk_pool_element_offset(self, block, kv_head, is_v, slot, dim):
        return int(lib().sk_pool_element_offset(self.h, block, kv_head, int(is_v), slot, dim))

    # -- compute ---------------------------------------------------------------------------
    def _out(self, T, out_dtype, want_lse):
        odt = torch.float32 if _dt(out_dtype) == SK_F32 else torch.bfloat16
        out = torch.empty((T, self.Hq, self.d), dtype=odt, device=self.device)
        lse = torch.empty((T, self.Hq), dtype=torch.float32, device=self.device) if want_lse else None
        return out, lse

    def sk_session_append(self, sid, q, k, v, out=None, lse=None, out_dtype="f32", want_lse=True, stream=None,
                          n_tokens=None):
        L = int(k.shape[0]) if n_tokens is None else int(n_tokens)
        if q is not None and out is None and self.kv_mem is not None:
            out, lse = self._out(L, out_dtype, want_lse)
        _ck(lib().sk_session_append(self.h, sid, _p(q), _p(k), _p(v), L, _p(out), _dt(out_dtype), _p(lse),
                                    _stream(stream) if self.kv_mem is not None else None), "sk_session_append")
        return out, lse

    def reserve(self, sid, n_tokens):
        """Metadata-only pools: the allocation half of an append."""
        _ck(lib().sk_session_append(self.h, sid, None, None, None, int(n_tokens), None, SK_F32, None, None),
            "sk_session_append")

    def sk_session_query(self, sid, q, k=None, v=None, out=None, lse=None, out_dtype="f32", want_lse=True,
                         n_splits=0, stream=None):
        nq = int(q.shape[0])
        if out is None:
            out, lse = self._out(nq, out_dtype, want_lse)
        _ck(lib().sk_session_query(self.h, sid, _p(q), _p(k), _p(v), nq, _p(out), _dt(out_dtype), _p(lse),
                                   int(n_splits), _stream(stream)), "sk_session_query")
        return out, lse

    def sk_batch_step(self, session_ids, ops, cu_tokens, q, k, v, out=None, lse=None, out_dtype="f32",
                      want_lse=True, stream=None):
        n = len(session_ids)
        T = int(cu_tokens[-1])
        if out is None:
            out, lse = self._out(T, out_dtype, want_lse)
        sid = (ctypes.c_int32 * n)(*[int(x) for x in session_ids])
        op = (ctypes.c_int32 * n)(*[int(x) for x in ops])
        cu = (ctypes.c_int32 * (n + 1))(*[int(x) for x in cu_tokens])
        _ck(lib().sk_batch_step(self.h, n, sid, op, cu, _p(q), _p(k), _p(v), _p(out), _dt(out_dtype), _p(lse),
                                _stream(stream)), "sk_batch_step")
        return out, lse

    def sk_session_query_shared_prefix(self, sid, qp, kp, vp, qs, ks, vs, out_dtype="f32", want_lse=True,
                                       stream=None):
        P = 0 if qp is None else int(qp.shape[0])
        NQ, Sfx = int(qs.shape[0]), int(qs.shape[1])
        out_p, lse_p = self._out(P, out_dtype, want_lse)
        out_s, lse_s = self._out(NQ * Sfx, out_dtype, want_lse)
        _ck(lib().sk_session_query_shared_prefix(self.h, sid, _p(qp), _p(kp), _p(vp), P, _p(qs), _p(ks), _p(vs),
                                                 NQ, Sfx, _p(out_p), _p(out_s), _dt(out_dtype), _p(lse_p),
                                                 _p(lse_s), _stream(stream)), "sk_session_query_shared_prefix")
        out_s = out_s.view(NQ, Sfx, self.Hq, self.d)
        if lse_s is not None:
            lse_s = lse_s.view(NQ, Sfx, self.Hq)
        return out_p, lse_p, out_s, lse_s

    def sk_session_gather(self, sid, first=0, count=None, stream=None):
        if count is None:
            count = self.sk_session_length(sid) - first
        k = torch.empty((count, self.Hkv, self.d), dtype=self.torch_dtype, device=self.device)
        v = torch.empty_like(k)
        _ck(lib().sk_session_gather(self.h, sid, first, count, _p(k), _p(v), _stream(stream)), "sk_session_gather")
        return k, v


def top2_outputs(rows, device):
    """Output tensors of sk_top2 / sk_top2_static for `rows` rows: (idx1, idx2, val1, val2, gap)."""
    idx1 = torch.empty(rows, dtype=torch.int32, device=device)
    val1 = torch.empty(rows, dtype=torch.float32, device=device)
    return idx1, torch.empty_like(idx1), val1, torch.empty_like(val1), torch.empty_like(val1)


def sk_top2_static(logits, outputs=None, stream=None):
    """sk_top2 through the entry point that allocates nothing: `outputs` (see top2_outputs) are the
    caller's; they are only made here when left out."""
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
    rows, vocab = logits.shape
    if outputs is None:
        outputs = top2_outputs(rows, logits.device)
    idx1, idx2, val1, val2, gap = outputs
    _ck(lib().sk_top2_static(ctypes.c_void_p(logits.data_ptr()) if rows else None, rows, vocab,
                             logits.stride(0) if rows else vocab, _p(idx1), _p(idx2), _p(val1), _p(val2), _p(gap),
                             _stream(stream)), "sk_top2_static")
    return outputs


def sk_top2(logits, stream=None, workspace=None, outputs=None):
    """logits: CUDA float32 tensor [rows, vocab] (rows may be strided by a multiple of 4 elements).
    Returns (idx1, idx2, val1, val2, gap), each [rows]."""
    assert logits.is_cuda and logits.dtype == torch.float32 and logits.dim() == 2 and logits.stride(1) == 1
    rows, vocab = logits.shape
    need = lib().sk_top2_workspace_bytes(rows, vocab)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=logits.device)
    idx1, idx2, val1, val2, gap = outputs if outputs is not None else top2_outputs(rows, logits.device)
    _ck(lib().sk_top2(ctypes.c_void_p(logits.data_ptr()) if rows else None, rows, vocab, logits.stride(0) if rows else vocab, _p(workspace),
                      workspace.numel(), _p(idx1), _p(idx2), _p(val1), _p(val2), _p(gap), _stream(stream)), "sk_top2")
    return idx1, idx2, val1, val2, gap


def sk_probe_read(buf, n_workgroups, sink, stream=None, nbytes=None, non_temporal=False):
    """Plain streaming read of a CUDA tensor (measurement probe)."""
    nbytes = buf.numel() * buf.element_size() if nbytes is None else int(nbytes)
    _ck(lib().sk_probe_read(_p(buf), nbytes, int(n_workgroups), int(bool(non_temporal)), _p(sink), _stream(stream)), "sk_probe_read")


def sk_probe_mfma(n_workgroups, iters, sink, operands=None, stream=None):
    """Back-to-back bf16 matrix products on register operands (measurement probe), the operands taken
    from the bf16 CUDA tensor `operands` if given; returns the flops of the launch."""
    f = ctypes.c_double()
    nb = 0 if operands is None else operands.numel() * operands.element_size()
    _ck(lib().sk_probe_mfma(int(n_workgroups), int(iters), _p(operands), nb, _p(sink), ctypes.byref(f), _stream(stream)),
        "sk_probe_mfma")
    return f.value
