"""fp64 CPU oracle (test infrastructure only; the product path never imports it)."""
from .session import (OracleSession, OraclePool, attention, num_threads,
                      OP_APPEND, OP_QUERY_A, OP_QUERY_B)
from ._lib import build

__all__ = ["OracleSession", "OraclePool", "attention", "num_threads", "build",
           "OP_APPEND", "OP_QUERY_A", "OP_QUERY_B"]
