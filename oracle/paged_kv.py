"""Oracle: paged KV cache addressing.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

A serving stack keeps the committed keys/values of all sequences in one pool of
fixed-size pages, `pool[n_pages, page_size, Hkv, D]`, and a per-sequence table
of page ids: token t of sequence b lives in page `block_table[b, t // page_size]`
at slot `t % page_size`.  (The paper does not discuss cache layout; this is the
layout of the serving systems its method is meant to run in, and a library
convention.)  Verification attention over a paged cache is, by definition, the
attention of oracle/tree_attention.py over the cache one obtains by reading the
pages back in table order; committing the accepted path writes the same rows
oracle/commit_path.py writes, at the paged addresses.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np


def gather_pages(pool: np.ndarray, block_table: np.ndarray, page_size: int, length: int) -> np.ndarray:
    """pool [n_pages, page_size, Hkv, D], block_table [B, max_blocks] -> contiguous [B, length, Hkv, D]."""
    B = block_table.shape[0]
    out = np.zeros((B, length) + pool.shape[2:], dtype=pool.dtype)
    for b in range(B):
        for t in range(length):
            out[b, t] = pool[int(block_table[b, t // page_size]), t % page_size]
    return out


def scatter_rows(pool: np.ndarray, block_table: np.ndarray, page_size: int, b: int, positions: Sequence[int],
                 rows: np.ndarray) -> None:
    """In place: token positions of sequence b receive rows [len(positions), Hkv, D]."""
    for i, t in enumerate(positions):
        pool[int(block_table[b, t // page_size]), t % page_size] = rows[i]
