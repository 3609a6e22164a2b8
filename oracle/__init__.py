"""fp64 CPU oracle (test infrastructure only; the product path never imports it)."""
from .session import (OracleSession, OraclePool, attention, num_threads,
                      OP_APPEND, OP_QUERY_A, OP_QUERY_B)
from ._lib import build
from .sampling import top2

__all__ = ["OracleSession", "OraclePool", "attention", "num_threads", "build", "top2",
           "OP_APPEND", "OP_QUERY_A", "OP_QUERY_B"]
