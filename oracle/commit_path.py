"""Oracle: committing the accepted path to the KV cache.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

What is computed (Section 2.1 step 3 of the paper: the accepted tokens are
appended to the sequence and everything else the draft proposed is dropped).
For the attention state of one layer this means: the key/value rows of the
accepted tree nodes, in path order, become the next rows of the cache, and the
prefix grows by their number,

    for every sequence b and i < n_b:
        cache[b, L_b + i] = tree[b, path[b, i]]       (keys and values, all KV heads)
    L_b <- L_b + n_b          (only when `advance` is set: the caches of all
                               layers share one length, the caller advances
                               it with the last layer)

n_b is accept_len[b] cut down where the library must not follow it: negative
lengths (a walk that gave up reports -1) count as 0, the path array holds
max_depth entries, a node id outside [0, T) ends the commit in front of it,
and rows that would land beyond the cache capacity are dropped.  (These cuts
are this library's error behaviour, not the paper's.)  The token the target
model adds itself after the last accepted node has no key/value yet: it is the
root of the next round.

Parity pin that does not restate the copy: the attention output of the last
accepted node before the commit (prefix + its ancestors, which are exactly
the path) equals plain one-token decoding attention of the same query over
the first L_b + n_b rows of the committed cache (tests/test_oracle_commit.py).
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def committed_rows(path_b: Sequence[int], accept_len_b: int, n_tree: int, prefix_len_b: int, capacity: int) -> int:
    """Number of leading path entries that are committed for one sequence."""
    n = max(0, int(accept_len_b))
    n = min(n, len(path_b))
    for i in range(n):
        if not (0 <= int(path_b[i]) < n_tree):
            n = i
            break
    room = max(0, capacity - max(0, int(prefix_len_b)))
    return min(n, room)


def commit_path(k_cache: np.ndarray, v_cache: np.ndarray, k_tree: np.ndarray, v_tree: np.ndarray,
                path: np.ndarray, accept_len: Sequence[int], prefix_len: Sequence[int],
                advance: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """k_cache, v_cache [B,Lcap,Hkv,D]; k_tree, v_tree [B,T,Hkv,D]; path [B,max_depth] node ids;
    accept_len, prefix_len [B].  Returns (k_cache', v_cache', prefix_len') as new arrays."""
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    B, cap = k_out.shape[0], k_out.shape[1]
    T = k_tree.shape[1]
    new_len = np.array(prefix_len, dtype=np.int64, copy=True)
    for b in range(B):
        L = int(prefix_len[b])
        n = committed_rows(path[b], accept_len[b], T, L, cap)
        for i in range(n):
            node = int(path[b][i])
            k_out[b, L + i] = k_tree[b, node]
            v_out[b, L + i] = v_tree[b, node]
        if advance:
            new_len[b] = L + n
    return k_out, v_out, new_len
