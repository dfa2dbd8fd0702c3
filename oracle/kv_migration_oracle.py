"""Plain numpy statement of the KV-block migration copies.  TEST INFRASTRUCTURE ONLY.

What is computed (paper section 5.2, "KV cache transmission": the KV blocks of
long requests are migrated in layer-aligned chunks into buffers pre-allocated
on the target): one layer's chunk is a gather of the pages a block table names
for the migrating requests (and of a range of their kv heads) into a contiguous
staging array, and a scatter of such an array into the pages a target table
names.  Written as explicit loops over requests and pages, one assignment per
(page, head) unit, so that it can be checked by eye; shares nothing with the GPU
library.  Arrays hold bf16 bit patterns as uint16; the copies are bit-exact.

Pins (tests/test_kv_migration.py): a hand-written two-request example; gather of
every page in table order with all heads is the pool itself re-indexed; scatter
after gather through the same table restores exactly the gathered pages and
leaves every other page and head untouched; head ranges compose (two half-range
gathers equal the halves of a full-range gather).
"""
from __future__ import annotations

import numpy as np


def staging_offsets(context_lens, page_size: int) -> np.ndarray:
    """First staging page of each migrating request, and the total (last entry)."""
    off = [0]
    for L in context_lens:
        off.append(off[-1] + (int(L) + page_size - 1) // page_size)
    return np.asarray(off, dtype=np.int64)


def gather(pool: np.ndarray, block_table: np.ndarray, table_rows, context_lens, head_begin: int, num_heads: int):
    """pool: [pages, heads, page_size, D] uint16 -> staging [n, num_heads, page_size, D]."""
    page_size = pool.shape[2]
    off = staging_offsets(context_lens, page_size)
    stage = np.zeros((int(off[-1]), num_heads) + pool.shape[2:], dtype=pool.dtype)
    for r, row in enumerate(table_rows):
        for pg in range(int(off[r + 1] - off[r])):
            pid = int(block_table[row, pg])
            for j in range(num_heads):
                stage[off[r] + pg, j] = pool[pid, head_begin + j]
    return stage


def scatter(stage: np.ndarray, pool: np.ndarray, target_table: np.ndarray, context_lens, head_begin: int):
    """Writes stage [n, num_heads, page_size, D] into a copy of pool [pages, heads, page_size, D]; returns it."""
    out = pool.copy()
    page_size = pool.shape[2]
    off = staging_offsets(context_lens, page_size)
    for r in range(len(context_lens)):
        for pg in range(int(off[r + 1] - off[r])):
            pid = int(target_table[r, pg])
            for j in range(stage.shape[1]):
                out[pid, head_begin + j] = stage[off[r] + pg, j]
    return out
