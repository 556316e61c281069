"""Paged K/V pools, page tables and random Q/K/V values for a prefix forest.

Only input plumbing lives here: page assignment, random draws, 16-bit rounding
and exact 16-bit -> float64 widening for reports.  Nothing of the attention
method itself.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

from .trees import Forest

DTYPE_FP16 = 0
DTYPE_BF16 = 1
_TORCH_DTYPE = {DTYPE_FP16: torch.float16, DTYPE_BF16: torch.bfloat16}


@dataclass
class HeadConfig:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int = 128
    dtype: int = DTYPE_BF16
    page_size: int = 16
    scale: float = 0.0          # 0 -> 1/sqrt(head_dim)

    def __post_init__(self):
        if self.scale == 0.0:
            self.scale = float(np.float32(1.0 / np.sqrt(np.float32(self.head_dim))))

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def torch_dtype(self):
        return _TORCH_DTYPE[self.dtype]

    @property
    def bytes_per_token(self) -> int:
        """K and V bytes one token occupies over all KV heads."""
        return self.num_kv_heads * self.head_dim * 2 * 2


@dataclass
class PagedKV:
    page_size: int
    node_page_off: np.ndarray     # int32 [N+1] into page_ids
    page_ids: np.ndarray          # int32, physical page of each logical page of each node
    num_pages: int                # pool size (>= pages referenced)
    layout: str                   # "thd": [page][token][kv_head][d];  "htd": [page][kv_head][token][d];
                                  # "hktd": one pool [page][kv_head][K|V][token][d], K and V of a page and
                                  # head side by side (8 KB of consecutive memory with 16-token pages)
    page_stride: int = 0          # in elements
    token_stride: int = 0
    head_stride: int = 0


@dataclass
class Workload:
    name: str
    forest: Forest
    head: HeadConfig
    paged: PagedKV
    q: torch.Tensor               # [B, h_q, d]
    k_pool: torch.Tensor          # [num_pages, ...] per layout
    v_pool: torch.Tensor
    seed: int = 0
    notes: dict = field(default_factory=dict)
    kv_pool: Optional[torch.Tensor] = None    # "hktd": the pool k_pool and v_pool are views of

    # raw 16-bit patterns, host side, for the CPU oracle
    def q_bits(self) -> np.ndarray:
        return self.q.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def _pool_bits(self) -> np.ndarray:
        return self.kv_pool.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).reshape(-1)

    def k_bits(self) -> np.ndarray:
        if self.kv_pool is not None:            # addressed with the pool's strides from K's first element
            return self._pool_bits()
        return self.k_pool.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def v_bits(self) -> np.ndarray:
        if self.kv_pool is not None:            # the same strides from V's first element
            return self._pool_bits()[self.paged.page_size * self.head.head_dim:]
        return self.v_pool.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    @property
    def unique_kv_bytes(self) -> int:
        from .trees import forest_stats
        return forest_stats(self.forest)["unique_tokens"] * self.head.bytes_per_token

    def to(self, device) -> "Workload":
        if self.kv_pool is not None:
            pool = self.kv_pool.to(device)
            return Workload(self.name, self.forest, self.head, self.paged, self.q.to(device),
                            pool[:, :, 0], pool[:, :, 1], self.seed, dict(self.notes), pool)
        return Workload(self.name, self.forest, self.head, self.paged, self.q.to(device),
                        self.k_pool.to(device), self.v_pool.to(device), self.seed, dict(self.notes))


def build_paged_kv(forest: Forest, head: HeadConfig, seed: int, spare_pages: int = 64,
                   layout: str = "thd", shuffle: bool = True) -> PagedKV:
    """Give every node its own whole pages; physical order is a seeded permutation.

    Tokens fill a node's pages in order, so only its last page can be partly
    filled.  ``spare_pages`` extra pages are never referenced.
    """
    ps = head.page_size
    n_pages_node = (forest.node_len.astype(np.int64) + ps - 1) // ps
    off = np.zeros(forest.num_nodes + 1, dtype=np.int64)
    np.cumsum(n_pages_node, out=off[1:])
    used = int(off[-1])
    total = used + spare_pages
    assert total < 2**31
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
    perm = rng.permutation(total) if shuffle else np.arange(total)
    page_ids = perm[:used].astype(np.int32)
    d, h = head.head_dim, head.num_kv_heads
    if layout == "thd":
        token_stride, head_stride = h * d, d
    elif layout == "htd":
        token_stride, head_stride = d, ps * d
    elif layout == "hktd":
        token_stride, head_stride = d, 2 * ps * d
    else:
        raise ValueError(layout)
    page_stride = (2 if layout == "hktd" else 1) * ps * h * d
    return PagedKV(ps, off.astype(np.int32), page_ids, total, layout,
                   page_stride=page_stride, token_stride=token_stride, head_stride=head_stride)


def _randn_into(dst: torch.Tensor, gen: torch.Generator, chunk: int = 1 << 26) -> None:
    """Fill ``dst`` (16-bit) with N(0,1) drawn in fp32 and rounded once to dst's dtype."""
    flat = dst.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        flat[s:e] = torch.randn(e - s, dtype=torch.float32, device=dst.device, generator=gen).to(dst.dtype)


def make_workload(name: str, forest: Forest, head: HeadConfig, seed: int,
                  device: str = "cpu", layout: str = "thd", poison: bool = False,
                  spare_pages: int = 64, q_scale: float = 1.0,
                  paged: Optional[PagedKV] = None) -> Workload:
    """Random Q, K, V ~ N(0,1) (seeded on ``device``) in a shuffled page pool.

    With ``poison`` the unreferenced pages and the unused tail of every partly
    filled page hold NaN, so that a kernel that reads a masked position shows.
    """
    if paged is None:
        paged = build_paged_kv(forest, head, seed, spare_pages, layout)
    dt = head.torch_dtype
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    b = forest.num_requests
    q = torch.empty((b, head.num_q_heads, head.head_dim), dtype=dt, device=device)
    _randn_into(q, gen)
    if q_scale != 1.0:
        q = (q.float() * q_scale).to(dt)
    ps, h, d = head.page_size, head.num_kv_heads, head.head_dim
    shape = (paged.num_pages, ps, h, d) if paged.layout == "thd" else (paged.num_pages, h, ps, d)
    k_pool = torch.empty(shape, dtype=dt, device=device)
    v_pool = torch.empty(shape, dtype=dt, device=device)
    _randn_into(k_pool, gen)
    _randn_into(v_pool, gen)
    kv_pool = None
    if paged.layout == "hktd":                  # the values of "htd", K and V of a (page, head) side by side
        kv_pool = torch.empty((paged.num_pages, h, 2, ps, d), dtype=dt, device=device)
        kv_pool[:, :, 0] = k_pool
        kv_pool[:, :, 1] = v_pool
        k_pool, v_pool = kv_pool[:, :, 0], kv_pool[:, :, 1]
    if poison:
        nan = float("nan")
        referenced = torch.zeros(paged.num_pages, dtype=torch.bool)
        referenced[torch.from_numpy(paged.page_ids.astype(np.int64))] = True
        spare = (~referenced).nonzero().flatten().to(device)
        k_pool[spare] = nan
        v_pool[spare] = nan
        tail = forest.node_len.astype(np.int64) % ps
        for n in np.nonzero(tail)[0]:
            last = int(paged.page_ids[paged.node_page_off[n + 1] - 1])
            t0 = int(tail[n])
            if paged.layout == "thd":
                k_pool[last, t0:] = nan
                v_pool[last, t0:] = nan
            else:
                k_pool[last, :, t0:] = nan
                v_pool[last, :, t0:] = nan
    return Workload(name, forest, head, paged, q, k_pool, v_pool, seed, kv_pool=kv_pool)


def bits_to_float64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of raw fp16/bf16 bit patterns to float64 (reporting helper)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == DTYPE_FP16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def float_to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round float values to fp16/bf16 (nearest even) and return the raw bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(_TORCH_DTYPE[dtype])
    return t.view(torch.int16).numpy().view(np.uint16).copy()
