"""Seeded synthetic inputs shared by the oracle-side tests and the GPU-side harness.

Holds no attention arithmetic: only random draws, dtype rounding, workload shapes
and the bookkeeping that turns a torch CPU tensor into the raw numpy arrays the
oracle takes.  The draws stand in for projected, position-encoded Q/K/V
activations of one attention layer: i.i.d. N(0,1) in fp32 from a CPU generator,
rounded to bf16 (round-to-nearest-even) where the workload is bf16.
"""
import dataclasses
import math

import numpy as np
import torch

SEED_BASE = 0x5EED0000


@dataclasses.dataclass(frozen=True)
class Shape:
    dtype: str          # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def kv_bytes_per_token(self):
        return 2 * self.n_kv_heads * self.head_dim * (4 if self.dtype == "f32" else 2)


# The five workload shapes (single small fp32 session; Llama-3-8B-shaped layer at 32K;
# the same at 128K; multi-tenant ragged batch; 70B-shaped registered-question batch).
CFG1 = Shape("f32", 4, 4, 64)
CFG2 = Shape("bf16", 32, 8, 128)
CFG3 = CFG2
CFG4 = CFG2
CFG5 = Shape("bf16", 64, 8, 128)


def generator(cfg_id, stream=0):
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + cfg_id + (stream << 8))
    return g


def torch_dtype(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def draw(gen, shape, dtype, scale=1.0):
    """N(0,1)*scale in fp32, then rounded to the workload dtype.  CPU tensor."""
    x = torch.randn(shape, generator=gen, dtype=torch.float32)
    if scale != 1.0:
        x = x * scale
    return x.to(torch_dtype(dtype)).contiguous()


def draw_qkv(gen, n_tokens, shape: Shape, scale=1.0):
    q = draw(gen, (n_tokens, shape.n_q_heads, shape.head_dim), shape.dtype, scale)
    k = draw(gen, (n_tokens, shape.n_kv_heads, shape.head_dim), shape.dtype, scale)
    v = draw(gen, (n_tokens, shape.n_kv_heads, shape.head_dim), shape.dtype, scale)
    return q, k, v


def to_raw(t: torch.Tensor) -> np.ndarray:
    """CPU torch tensor -> numpy array of the same bits (bf16 -> uint16, f32 -> float32)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype == torch.float32:
        return t.numpy().copy()
    raise TypeError(t.dtype)


def from_raw(a: np.ndarray) -> torch.Tensor:
    """Inverse of to_raw."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
    if a.dtype == np.float32:
        return torch.from_numpy(a.copy())
    raise TypeError(a.dtype)


def raw_to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of raw bits to float64 (for brute-force checks in the tests)."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def loguniform_lengths(gen, n_sessions, lo=2048, hi=65536):
    """Cached lengths of the multi-tenant workload: floor(lo * (hi/lo)**u), u ~ U[0,1)."""
    u = torch.rand(n_sessions, generator=gen, dtype=torch.float64)
    return [int(math.floor(lo * (hi / lo) ** float(x))) for x in u]


def randint(gen, lo, hi_inclusive, n=None):
    r = torch.randint(lo, hi_inclusive + 1, (1 if n is None else n,), generator=gen)
    return int(r[0]) if n is None else [int(x) for x in r]


def permutation(gen, n):
    return torch.randperm(n, generator=gen).to(torch.int32).numpy()
