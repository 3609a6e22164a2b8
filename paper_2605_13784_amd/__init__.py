"""Stateful-session attention for MI355X: ctypes binding over libsk.so (HIP, gfx950)."""
from .binding import (Pool, SkError, lib, lib_path, make_desc, sk_pool_kv_bytes, sk_pool_workspace_bytes, sk_top2, sk_top2_static, top2_outputs, sk_probe_read, sk_probe_mfma,
                      SK_TOP2_STATIC_BYTES, SK_SITE_RING, SK_SITE_UPLOAD, SK_SITE_BLOCK_COPY, SK_SITE_SCATTER,
                      SK_SITE_ATTENTION, SK_SITE_COMBINE, SK_SITE_PLAN,
                      SK_F32, SK_BF16, SK_OP_APPEND, SK_OP_QUERY_A, SK_OP_QUERY_B, SK_POOL_METADATA_ONLY,
                      SK_OK, SK_E_INVAL, SK_E_SHAPE, SK_E_DTYPE, SK_E_NOMEM, SK_E_BADSESSION, SK_E_EMPTY,
                      SK_E_WORKSPACE, SK_E_HIP, SK_E_NODEVICE, EXPORTS)
from ._build import build

__all__ = [n for n in dir() if not n.startswith("_")]
