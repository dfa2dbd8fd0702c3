"""Seeded synthetic inputs for paged GQA decode attention.

This module only *draws inputs*: context lengths, block tables and bf16 tensor
values.  It holds none of the attention arithmetic and is the one module that
both the CPU oracle's tests and the GPU path's tests/benchmark may use, so that
both sides see the same bits.  It imports neither of them.

The five workloads stand in for the request mixes of the paper's evaluation
(short compute-bound requests mixed with long memory-bound ones, section 1 (i)
and section 2 "Workload heterogeneity"; the production traces of section 6.1
are not available): the length mixture of workload 3 plays the role of the
short-vs-long request mix, workloads 1/2 take the head geometry of a Llama-3-8B
replica and of one tensor-parallel (TP=4) shard of a 70B model (section 6.2
deploys 70B replicas at TP=4).

Integer structure (lengths, page permutations) comes from a counter-based
splitmix64 hash implemented here, so it does not depend on any library's random
stream.  Tensor values are N(0,1) samples drawn by torch's seeded generator on
the device where the tensor lives, rounded to bf16 (round-to-nearest-even); the
other side always receives a *copy* of those bits, never a regeneration.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

PAGE_SIZE = 16
BASE_SEED = 20260212

_U64 = np.uint64
_MASK = (1 << 64) - 1


# --------------------------------------------------------------------------
# counter-based integer generator (splitmix64 finaliser over seed + counter)
# --------------------------------------------------------------------------
def _splitmix64(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x += _U64(0x9E3779B97F4A7C15)
        x ^= x >> _U64(30)
        x *= _U64(0xBF58476D1CE4E5B9)
        x ^= x >> _U64(27)
        x *= _U64(0x94D049BB133111EB)
        x ^= x >> _U64(31)
    return x


class CounterRng:
    """Stateless-per-draw stream: value i of stream s is hash(hash(seed, s), i)."""

    def __init__(self, seed: int):
        self.seed = int(seed) & _MASK
        self._stream = 0

    def _next_key(self) -> np.uint64:
        self._stream += 1
        base = np.array([(self.seed * 0x100000001B3 + self._stream) & _MASK], dtype=np.uint64)
        return _splitmix64(base)[0]

    def raw(self, n: int) -> np.ndarray:
        key = self._next_key()
        ctr = np.arange(n, dtype=np.uint64)
        with np.errstate(over="ignore"):
            return _splitmix64(ctr * _U64(0xD1342543DE82EF95) + key)

    def uniform(self, n: int) -> np.ndarray:
        """float64 in (0, 1): 53 random bits, never exactly 0."""
        return ((self.raw(n) >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)

    def integers(self, lo: int, hi: int, n: int) -> np.ndarray:
        """Uniform integers in [lo, hi], both ends included."""
        span = hi - lo + 1
        return (lo + np.floor(self.uniform(n) * span)).astype(np.int64).clip(lo, hi)

    def normal(self, n: int) -> np.ndarray:
        """Box-Muller on two uniform streams."""
        u1 = self.uniform(n)
        u2 = self.uniform(n)
        return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)

    def permutation(self, n: int) -> np.ndarray:
        """A permutation of 0..n-1: stable argsort of hashed keys."""
        return np.argsort(self.raw(n), kind="stable").astype(np.int64)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int = PAGE_SIZE
    # pool sizing: either a factor over the pages needed, or a fixed page count
    pool_factor: float = 1.25
    pool_pages_fixed: Optional[int] = None
    # which config's context-length recipe to draw from (None: the workload's own index)
    recipe: Optional[int] = None

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def scale(self) -> float:
        """1/sqrt(head_dim) rounded to fp32 (the value both sides must use)."""
        return float(np.float32(1.0 / math.sqrt(self.head_dim)))

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS = (
    Workload(0, "tiny", batch=4, num_q_heads=8, num_kv_heads=2, head_dim=64,
             pool_pages_fixed=64),
    Workload(1, "llama3-8b", batch=64, num_q_heads=32, num_kv_heads=8, head_dim=128),
    Workload(2, "llama3-70b-tp4-shard", batch=128, num_q_heads=16, num_kv_heads=2, head_dim=128),
    Workload(3, "heterogeneous-mix", batch=256, num_q_heads=32, num_kv_heads=8, head_dim=128),
    Workload(4, "long-context", batch=16, num_q_heads=32, num_kv_heads=8, head_dim=128,
             pool_pages_fixed=1 << 21),
    # Shape variants of the heterogeneous mix: per-GPU head geometries of the paper's other models
    # (section 6.1: OPT-30B is MHA with 56 heads, Llama2-70B has 64 query / 8 kv heads) at
    # tensor-parallel degrees its deployments use, and larger cache pages.
    Workload(5, "mix-opt30b-tp2-mha", batch=128, num_q_heads=28, num_kv_heads=28, head_dim=128, recipe=3),
    Workload(6, "mix-llama2-70b-tp8", batch=256, num_q_heads=8, num_kv_heads=1, head_dim=128, recipe=3),
    Workload(7, "mix-page32", batch=256, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=32, recipe=3),
    Workload(8, "mix-page64", batch=256, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=64, recipe=3),
)


def context_lens(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    """int32 [batch] context lengths of workload `w` (the recipe of each config)."""
    rng = CounterRng(w.seed if seed is None else seed)
    recipe = w.index if w.recipe is None else w.recipe
    if recipe == 0:
        lens = np.array([17, 64, 200, 513], dtype=np.int64)
    elif recipe == 1:
        lens = rng.integers(128, 2048, w.batch)
    elif recipe == 2:
        lens = rng.integers(1024, 16384, w.batch)
    elif recipe == 3:
        n_short = int(round(0.7 * w.batch))
        n_long = w.batch - n_short
        z = rng.normal(n_short)
        short = np.clip(np.rint(np.exp(math.log(512.0) + 0.8 * z)), 16, 4096).astype(np.int64)
        long_ = rng.integers(8192, 32768, n_long)
        lens = np.concatenate([short, long_])[rng.permutation(w.batch)]
    elif recipe == 4:
        lens = rng.integers(65536, 131072, w.batch)
    else:
        raise ValueError(f"unknown workload {w.index}")
    return lens.astype(np.int32)


PREFILL_WORKLOAD_NAMES = (
    "16 whole prompts of 4096 tokens",
    "8 chunks of 2048 tokens ending 32768-token contexts",
    "64 chunks of 512 tokens ending contexts uniform in [8192, 32768]",
)


def prefill_workload(which: int):
    """(Workload, context lengths, query lengths) of chunked-prefill workload `which` (Llama-3-8B heads):
    request b brings the last qlens[b] of its lens[b] cached tokens as query tokens."""
    if which == 0:
        lens, qlens = np.full(16, 4096), np.full(16, 4096)
    elif which == 1:
        lens, qlens = np.full(8, 32768), np.full(8, 2048)
    elif which == 2:
        lens, qlens = CounterRng(20260212 + 100 + which).integers(8192, 32768, 64), np.full(64, 512)
    else:
        raise ValueError(f"unknown prefill workload {which}")
    w = Workload(100 + which, "prefill", batch=len(lens), num_q_heads=32, num_kv_heads=8, head_dim=128)
    return w, lens.astype(np.int32), qlens.astype(np.int32)


def mixed_workload():
    """(Workload, context lengths, query lengths) of the mixed prefill + decode benchmark batch: the 256 decode
    requests of the heterogeneous mix (one query token each) followed by 8 prefill chunks of 512 tokens that end
    contexts uniform in [2048, 16384] - one step of a serving engine that runs chunked prefill next to its decodes."""
    w3 = WORKLOADS[3]
    dec = context_lens(w3)
    ctx = CounterRng(BASE_SEED + 200).integers(2048, 16384, 8)
    lens = np.concatenate([dec, ctx]).astype(np.int32)
    qlens = np.concatenate([np.ones(len(dec), dtype=np.int64), np.full(8, 512)]).astype(np.int32)
    w = Workload(200, "mixed-prefill-decode", batch=len(lens), num_q_heads=32, num_kv_heads=8, head_dim=128)
    return w, lens, qlens


def pages_needed(lens: np.ndarray, page_size: int = PAGE_SIZE) -> np.ndarray:
    return (lens.astype(np.int64) + page_size - 1) // page_size


def pool_pages(w: Workload, lens: np.ndarray) -> int:
    need = int(pages_needed(lens, w.page_size).sum())
    if w.pool_pages_fixed is not None:
        if w.pool_pages_fixed < need:
            raise ValueError("fixed pool smaller than the pages needed")
        return w.pool_pages_fixed
    return int(math.ceil(w.pool_factor * need))


def make_block_table(lens: np.ndarray, num_pool_pages: int, rng: CounterRng,
                     page_size: int = PAGE_SIZE, pad_cols: int = 0):
    """Scatter each request's logical pages over the pool.

    Returns (block_table int32 [batch, max_pages + pad_cols], used_ids int64
    [total pages]) where used_ids lists the physical ids in (request, logical
    page) order.  Unused block-table entries are -1 and must never be read.
    """
    n = pages_needed(lens, page_size)
    total = int(n.sum())
    if total > num_pool_pages:
        raise ValueError("pool too small")
    used = rng.permutation(num_pool_pages)[:total]
    width = int(n.max()) + pad_cols if len(n) else pad_cols
    bt = np.full((len(lens), max(width, 1)), -1, dtype=np.int32)
    off = 0
    for b, nb in enumerate(n):
        bt[b, :nb] = used[off:off + nb]
        off += nb
    return bt, used


def kv_bytes(lens: np.ndarray, num_kv_heads: int, head_dim: int) -> int:
    """Algorithmic K+V bytes one decode step must read: valid tokens only."""
    return int(lens.astype(np.int64).sum()) * num_kv_heads * head_dim * 2 * 2


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
@dataclass
class Inputs:
    workload: Workload
    q: torch.Tensor            # bf16 [B, Hq, D]
    k_pages: torch.Tensor      # bf16 [P, Hkv, page, D]
    v_pages: torch.Tensor      # bf16 [P, Hkv, page, D]
    block_table: torch.Tensor  # int32 [B, max_pages]
    context_lens: torch.Tensor  # int32 [B] (on the tensors' device)
    context_lens_host: np.ndarray  # int32 [B]
    scale: float
    used_pages: np.ndarray = field(repr=False, default=None)  # int64 physical ids in use

    @property
    def kv_bytes(self) -> int:
        w = self.workload
        return kv_bytes(self.context_lens_host, w.num_kv_heads, w.head_dim)


def _randn_bf16(shape, gen: torch.Generator, device, chunk_elems: int = 1 << 26) -> torch.Tensor:
    """bf16 RNE of fp32 N(0,1) samples, drawn in bounded chunks to cap the fp32 temporary."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk_elems):
        e = min(n, s + chunk_elems)
        flat[s:e] = torch.randn(e - s, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    return out


def make_inputs(w: Workload, device="cpu", seed: Optional[int] = None,
                lens: Optional[np.ndarray] = None, fill_unused: bool = True,
                pool_pages_override: Optional[int] = None) -> Inputs:
    """Draw the tensors of workload `w` on `device`.

    `lens` overrides the recipe's context lengths (same head geometry).  With
    `fill_unused=False` only the pages named by the block table receive N(0,1)
    values and the rest of the pool is left as allocated (used for pools far
    larger than the pages needed).
    """
    seed = w.seed if seed is None else seed
    lens = context_lens(w, seed) if lens is None else np.asarray(lens, dtype=np.int32)
    rng = CounterRng(seed ^ 0x5EED)
    if pool_pages_override is not None:
        npool = pool_pages_override
    elif w.pool_pages_fixed is not None and int(pages_needed(lens, w.page_size).sum()) <= w.pool_pages_fixed:
        npool = w.pool_pages_fixed
    else:
        npool = int(math.ceil(w.pool_factor * int(pages_needed(lens, w.page_size).sum())))
    bt, used = make_block_table(lens, npool, rng, w.page_size)

    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    q = _randn_bf16((len(lens), w.num_q_heads, w.head_dim), gen, dev)
    page_shape = (w.num_kv_heads, w.page_size, w.head_dim)
    if fill_unused:
        k_pages = _randn_bf16((npool,) + page_shape, gen, dev)
        v_pages = _randn_bf16((npool,) + page_shape, gen, dev)
    else:
        k_pages = torch.empty((npool,) + page_shape, dtype=torch.bfloat16, device=dev)
        v_pages = torch.empty((npool,) + page_shape, dtype=torch.bfloat16, device=dev)
        ids = torch.from_numpy(used).to(dev)
        step = 4096
        for s in range(0, len(used), step):
            sel = ids[s:s + step]
            k_pages[sel] = _randn_bf16((len(sel),) + page_shape, gen, dev)
            v_pages[sel] = _randn_bf16((len(sel),) + page_shape, gen, dev)
    return Inputs(
        workload=w, q=q, k_pages=k_pages, v_pages=v_pages,
        block_table=torch.from_numpy(bt).to(dev),
        context_lens=torch.from_numpy(lens.copy()).to(dev),
        context_lens_host=lens, scale=w.scale, used_pages=used,
    )
