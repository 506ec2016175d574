"""Oracle: tree-masked verification attention, written out as its definition.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

What is computed (Section 2.1 step 2: the target model scores every candidate
of the draft in one forward pass; Section 3.1.2 and its tree-attention-mask
figure: candidates form a tree, and a candidate must see exactly the context
it would see if its own root-to-node path were decoded token by token):

  for every sequence b, tree node i and query head h
      kv   = h // G                      (G = Hq // Hkv consecutive query heads share a KV head)
      keys = cache positions 0 .. L_b-1  together with  A(i) = {i, parent[i], parent[parent[i]], ...}
      s_j  = scale * <Q[b,i,h,:], K_j[kv,:]>        for every key j
      w_j  = exp(s_j - max_j s_j)
      out[b,i,h,:] = sum_j w_j V_j[kv,:] / sum_j w_j

Everything is fp64, two-pass softmax, no blocking, no running max.  The mask
figure is missing from the paper's text; the rule above (prefix + self +
strict ancestors, nothing else) is the reading under which each candidate's
conditional equals the autoregressive one.  Parity pins: chain tree == causal
attention (checked against torch's scaled_dot_product_attention), single node
== decode attention, per-node linearisation, sibling independence, closed
forms (equal V rows, equal K rows), GQA == expanded MHA, relabelling.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np


def ancestor_sets(parent: Sequence[int]) -> List[List[int]]:
    """A(i) for every node: the node itself followed by its ancestors, nearest
    first, stopping at -1 (the committed prefix)."""
    n = len(parent)
    out: List[List[int]] = []
    for i in range(n):
        chain = []
        a = i
        while a >= 0:
            if not (-1 <= parent[a] < a):
                raise ValueError(f"parent[{a}]={parent[a]} violates -1 <= parent[i] < i")
            chain.append(a)
            a = int(parent[a])
        out.append(chain)
    return out


def tree_verify_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                          k_tree: np.ndarray, v_tree: np.ndarray, parent: np.ndarray,
                          prefix_len: Sequence[int], scale: Optional[float] = None) -> np.ndarray:
    """q [B,T,Hq,D]; k_cache, v_cache [B,Lcap,Hkv,D]; k_tree, v_tree [B,T,Hkv,D];
    parent [B,T] (int, -1 = child of the prefix); prefix_len [B].
    Returns out [B,T,Hq,D] in float64.  scale defaults to 1/sqrt(D)."""
    q = np.asarray(q, dtype=np.float64)
    k_cache = np.asarray(k_cache, dtype=np.float64)
    v_cache = np.asarray(v_cache, dtype=np.float64)
    k_tree = np.asarray(k_tree, dtype=np.float64)
    v_tree = np.asarray(v_tree, dtype=np.float64)
    B, T, Hq, D = q.shape
    Hkv = k_cache.shape[2]
    if Hq % Hkv:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    out = np.zeros((B, T, Hq, D), dtype=np.float64)
    for b in range(B):
        L = int(prefix_len[b])
        if L < 0 or L > k_cache.shape[1]:
            raise ValueError("prefix_len out of range")
        anc = ancestor_sets([int(p) for p in parent[b]])
        for i in range(T):
            idx = anc[i]
            for h in range(Hq):
                kv = h // G
                # scores of the prefix keys followed by the scores of the visible tree keys
                s = scale * np.concatenate([k_cache[b, :L, kv, :] @ q[b, i, h, :],
                                            k_tree[b, idx, kv, :] @ q[b, i, h, :]])
                w = np.exp(s - s.max())
                num = w[:L] @ v_cache[b, :L, kv, :] + w[L:] @ v_tree[b, idx, kv, :]
                out[b, i, h, :] = num / w.sum()
    return out
