"""Seeded synthetic batches for multi-token paged attention.

This module only draws *inputs*: request lengths, page tables and random
element values.  It contains none of the attention / append arithmetic and
knows nothing about how a pool stores a page, so that the CPU oracle and the
HIP path can both be fed from it without sharing any method code.

The five named recipes follow the serving batches the paper describes
(Section 4.2: new-turn prompts and single-token generation steps share one
batch; Table "models": 40-head MHA and 64/8-head GQA layers with head size
128; Section 6.4: 32 requests x 8 query tokens over a context sweep).  The
paper's conversation datasets are not used; only the shapes are.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

PAGE_SIZE = 16


@dataclass
class Batch:
    """Integer structure of one batch (all host numpy, int32)."""

    name: str
    dtype: str  # "f16" | "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    ctx_lens: np.ndarray  # [R] past tokens already in the cache
    q_lens: np.ndarray  # [R] new tokens in this batch
    q_start: np.ndarray  # [R] exclusive prefix sum of q_lens
    page_table: np.ndarray  # [R, max_pages] physical page of each logical page, -1 = unused
    num_pages: int  # pool size in pages
    seed: int
    value_std: float = 1.0
    meta: Dict[str, object] = field(default_factory=dict)

    @property
    def num_reqs(self) -> int:
        return int(self.ctx_lens.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.q_lens.sum())

    @property
    def max_pages_per_req(self) -> int:
        return int(self.page_table.shape[1])

    @property
    def kv_lens(self) -> np.ndarray:
        return (self.ctx_lens + self.q_lens).astype(np.int64)

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    # ---- algorithmic counts used by bench / reports (pure counting) ----
    def causal_pairs(self) -> int:
        c = self.ctx_lens.astype(np.int64)
        n = self.q_lens.astype(np.int64)
        return int((n * c + n * (n + 1) // 2).sum())

    def flops(self) -> int:
        return 4 * self.head_dim * self.num_q_heads * self.causal_pairs()

    def kv_bytes(self) -> int:
        return int(2 * self.kv_lens.sum() * self.num_kv_heads * self.head_dim * 2)

    def qo_bytes(self) -> int:
        return int(2 * self.total_q * self.num_q_heads * self.head_dim * 2)

    def page_table_bytes(self) -> int:
        return int(4 * np.ceil(self.kv_lens / self.page_size).sum())

    def algorithmic_bytes(self) -> int:
        return self.kv_bytes() + self.qo_bytes() + self.page_table_bytes()


def _finish(name, dtype, hq, hkv, d, ctx, qn, rng, seed, pool_pages=None,
            pool_factor=1.5, value_std=1.0, identity_pages=False, meta=None) -> Batch:
    ctx = np.asarray(ctx, dtype=np.int32)
    qn = np.asarray(qn, dtype=np.int32)
    q_start = np.zeros_like(qn)
    if len(qn):
        q_start[1:] = np.cumsum(qn)[:-1]
    pages_per_req = (ctx.astype(np.int64) + qn + PAGE_SIZE - 1) // PAGE_SIZE
    needed = int(pages_per_req.sum())
    if pool_pages is None:
        pool_pages = max(1, int(np.ceil(needed * pool_factor)))
    assert pool_pages >= needed
    order = np.arange(pool_pages) if identity_pages else rng.permutation(pool_pages)
    max_pages = int(pages_per_req.max()) if len(qn) else 1
    max_pages = max(max_pages, 1)
    table = np.full((len(qn), max_pages), -1, dtype=np.int32)
    at = 0
    for r, npg in enumerate(pages_per_req):
        table[r, :npg] = order[at:at + npg]
        at += int(npg)
    return Batch(name=name, dtype=dtype, num_q_heads=hq, num_kv_heads=hkv, head_dim=d,
                 page_size=PAGE_SIZE, ctx_lens=ctx, q_lens=qn, q_start=q_start,
                 page_table=table, num_pages=int(pool_pages), seed=seed,
                 value_std=value_std, meta=dict(meta or {}))


def _split_counts(rng, total: int, frac_first: float) -> np.ndarray:
    """Boolean mask with round(frac_first*total) True entries at random places."""
    k = int(round(frac_first * total))
    mask = np.zeros(total, dtype=bool)
    mask[rng.permutation(total)[:k]] = True
    return mask


def tiny(seed: int = 1000) -> Batch:
    rng = np.random.default_rng(seed)
    return _finish("tiny", "f16", 4, 4, 64, [37, 100], [5, 12], rng, seed,
                   pool_pages=64, value_std=0.5)


def mha13b(seed: int = 1001, num_reqs: int = 32) -> Batch:
    rng = np.random.default_rng(seed)
    ctx = rng.integers(200, 1801, size=num_reqs)
    decode = _split_counts(rng, num_reqs, 0.5)
    turn = rng.integers(20, 301, size=num_reqs)
    qn = np.where(decode, 1, turn)
    return _finish("mha13b", "f16", 40, 40, 128, ctx, qn, rng, seed)


def gqa70b(seed: int = 1002, num_reqs: int = 64) -> Batch:
    rng = np.random.default_rng(seed)
    ctx = np.exp(rng.normal(np.log(1000.0), 1.0, size=num_reqs))
    ctx = np.clip(np.rint(ctx), 16, 4096).astype(np.int64)
    decode = _split_counts(rng, num_reqs, 0.7)
    turn = rng.integers(16, 513, size=num_reqs)
    qn = np.where(decode, 1, turn)
    return _finish("gqa70b", "bf16", 64, 8, 128, ctx, qn, rng, seed)


def long_history(seed: int = 1003, num_reqs: int = 8, q_len: int = 512,
                 ctx_lo: int = 16384, ctx_hi: int = 32768) -> Batch:
    rng = np.random.default_rng(seed)
    ctx = rng.integers(ctx_lo, ctx_hi + 1, size=num_reqs)
    qn = np.full(num_reqs, q_len)
    return _finish("long_history", "bf16", 64, 8, 128, ctx, qn, rng, seed)


def decode_heavy(seed: int = 1004, num_reqs: int = 256, ctx_lo: int = 512,
                 ctx_hi: int = 4096) -> Batch:
    rng = np.random.default_rng(seed)
    ctx = rng.integers(ctx_lo, ctx_hi + 1, size=num_reqs)
    qn = np.ones(num_reqs, dtype=np.int64)
    return _finish("decode_heavy", "f16", 40, 40, 128, ctx, qn, rng, seed)


def microbench(ctx: int, seed: int = 1005, num_reqs: int = 32, q_len: int = 8,
               identity_pages: bool = False) -> Batch:
    """Shape of the paper's kernel microbenchmark (Section 6.4)."""
    rng = np.random.default_rng(seed)
    return _finish(f"micro_c{ctx}", "f16", 40, 40, 128, np.full(num_reqs, ctx),
                   np.full(num_reqs, q_len), rng, seed, identity_pages=identity_pages)


def custom(ctx_lens, q_lens, *, num_q_heads, num_kv_heads, head_dim, dtype="f16", seed=7,
           pool_pages: Optional[int] = None, pool_factor: float = 1.5, value_std: float = 1.0,
           identity_pages: bool = False, name: str = "custom") -> Batch:
    rng = np.random.default_rng(seed)
    return _finish(name, dtype, num_q_heads, num_kv_heads, head_dim, ctx_lens, q_lens, rng,
                   seed, pool_pages=pool_pages, pool_factor=pool_factor, value_std=value_std,
                   identity_pages=identity_pages)


CONFIGS = {
    "tiny": tiny,
    "mha13b": mha13b,
    "gqa70b": gqa70b,
    "long_history": long_history,
    "decode_heavy": decode_heavy,
}
CONFIG_ORDER: List[str] = ["tiny", "mha13b", "gqa70b", "long_history", "decode_heavy"]


# ---------------------------------------------------------------------------
# random element values (16-bit patterns)
# ---------------------------------------------------------------------------

def _torch_dtype(dtype: str):
    import torch
    return {"f16": torch.float16, "bf16": torch.bfloat16}[dtype]


def random_values(shape, dtype: str, seed: int, std: float = 1.0, device: str = "cpu"):
    """N(0, std^2) drawn in fp32 then rounded to the 16-bit type.  Returns a torch tensor."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(_torch_dtype(dtype))


def as_u16(t) -> np.ndarray:
    """Bit patterns of a CPU 16-bit float torch tensor as a numpy uint16 array."""
    import torch
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def nan_pattern(dtype: str) -> int:
    return 0x7E00 if dtype == "f16" else 0x7FC0


def pool_elems(b: Batch) -> int:
    """Number of 16-bit elements in one pool (K or V)."""
    return b.num_pages * b.num_kv_heads * b.page_size * b.head_dim
