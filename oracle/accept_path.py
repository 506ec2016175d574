"""Oracle: token acceptance over a draft tree, step by step.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

The paper states acceptance for one drafted chain (Section 2.1): step 2
accepts candidate t with probability min(1, p(t)/q(t)), testing candidates in
order; step 3 appends accepted tokens and, at the first rejection, draws the
replacement from norm(max(0, p - q)) and drops the rest of the draft.  Greedy
decoding is "strict top-1 verification" (Section 3.2).  For a tree (Section
2.3: branches let verification fall back to an alternative continuation when
a token is rejected) the same rule is applied sibling by sibling, left to
right (Section 3.1.2: the higher-scoring expert's candidates sit on the left):
after a sibling is rejected the target distribution at that position is
replaced by the normalised residual before the next sibling is tried.  Every
node k carries its own draft distribution q_k.  These are readings of the paper,
as are the tie rules below.

Rows: logits row 0 is the distribution after the committed prefix, row k+1
the distribution after node k.  Node k is therefore judged with the row of
its parent, row(parent[k]) = parent[k] + 1.

Parity pins: greedy full/zero acceptance, 1-node tree == textbook speculative
sampling with P(accept) = sum_x min(p_x, q_x), exact enumeration and
Monte-Carlo of the emitted-token distribution on tiny vocabularies, q == p
accepts every first child.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np


@dataclass
class AcceptResult:
    path: List[int]                 # accepted node ids, root-most first
    accept_len: int
    bonus_token: int
    # sampling mode only: every threshold decision taken on the walk
    #   (kind, node, lhs, rhs, margin) with kind in {"accept", "reject", "bonus"}
    decisions: List[tuple] = field(default_factory=list)
    min_margin: float = float("inf")


def _children(parent: Sequence[int], c: int) -> List[int]:
    return [k for k in range(len(parent)) if parent[k] == c]


def _greedy(tokens, parent, logits, max_depth) -> AcceptResult:
    c = -1
    path: List[int] = []
    while True:
        t_star = int(np.argmax(logits[c + 1]))          # first maximum = lowest id on ties
        if max_depth is not None and len(path) >= max_depth:
            return AcceptResult(path, len(path), t_star)  # the walk may go no deeper: c's own row gives the token
        nxt = None
        for k in _children(parent, c):                   # left to right
            if int(tokens[k]) == t_star:
                nxt = k
                break
        if nxt is None:
            return AcceptResult(path, len(path), t_star)
        path.append(nxt)
        c = nxt


def _sample(tokens, parent, logits, draft_probs, uniforms, temperature, ftype, max_depth) -> AcceptResult:
    n = len(parent)
    res = AcceptResult([], 0, -1)

    def note(kind, node, lhs, rhs, margin):
        res.decisions.append((kind, node, float(lhs), float(rhs), float(margin)))
        res.min_margin = min(res.min_margin, float(margin))

    c = -1
    while True:
        z = np.asarray(logits[c + 1], dtype=ftype) / ftype(temperature)
        e = np.exp(z - z.max())
        p = e / e.sum()
        accepted = None
        if max_depth is not None and len(res.path) >= max_depth:
            break                                        # no deeper: the token after c comes from c's untouched row
        for k in _children(parent, c):
            x = int(tokens[k])
            qk = np.asarray(draft_probs[k], dtype=ftype)
            lhs = ftype(uniforms[k]) * qk[x]
            rhs = p[x]
            big = max(float(lhs), float(rhs))
            margin = abs(float(lhs) - float(rhs)) / big if big > 0 else 0.0
            if lhs < rhs:                                # u < min(1, p/q) for q > 0
                note("accept", k, lhs, rhs, margin)
                accepted = k
                break
            note("reject", k, lhs, rhs, margin)
            r = np.maximum(ftype(0), p - qk)
            s = r.sum()
            if s > 0:
                p = r / s                                # else: keep p
        if accepted is None:
            break
        res.path.append(accepted)
        c = accepted
    # replacement / extra token: inverse CDF of the distribution left at the stop
    cdf = np.cumsum(p)
    tot = cdf[-1]
    target = ftype(uniforms[n]) * tot
    above = np.nonzero(cdf > target)[0]
    if len(above):
        v = int(above[0])
        lo = float(cdf[v - 1]) if v > 0 else 0.0
        margin = min(float(target) - lo, float(cdf[v]) - float(target)) / float(tot)
    else:
        v = int(np.nonzero(p > 0)[0][-1])
        margin = 0.0
    note("bonus", -1, target, cdf[v], margin)
    res.accept_len = len(res.path)
    res.bonus_token = v
    return res


def accept_path(tree_tokens: np.ndarray, parent: np.ndarray, target_logits: np.ndarray,
                mode: str = "greedy", draft_probs: Optional[np.ndarray] = None,
                uniforms: Optional[np.ndarray] = None, temperature: float = 1.0,
                ftype=np.float64, max_depth: Optional[int] = None) -> AcceptResult:
    """One tree.  tree_tokens [N], parent [N], target_logits [N+1, V];
    mode "greedy" or "sample"; sample also needs draft_probs [N, V] and
    uniforms [N+1] (entry k tests node k, entry N draws the final token).
    ftype is the arithmetic type of the sampling walk (float64; float32 only to
    show that decisions do not hinge on precision).  max_depth (optional) stops
    the descent after that many accepted nodes: the children of the last one are
    not examined, and the final token is taken from that node's own row, exactly
    as if the tree had been cut below that depth (which is how the cap is pinned)."""
    parent = [int(x) for x in parent]
    for i, pa in enumerate(parent):
        if not (-1 <= pa < i):
            raise ValueError(f"parent[{i}]={pa} violates -1 <= parent[i] < i")
    if max_depth is not None and max_depth < 1:
        raise ValueError("max_depth must be at least 1")
    if mode == "greedy":
        return _greedy(tree_tokens, parent, np.asarray(target_logits), max_depth)
    if mode == "sample":
        if draft_probs is None or uniforms is None:
            raise ValueError("sample mode needs draft_probs and uniforms")
        if not temperature > 0:
            raise ValueError("temperature must be positive")
        return _sample(tree_tokens, parent, target_logits, draft_probs, uniforms,
                       temperature, ftype, max_depth)
    raise ValueError(f"unknown mode {mode!r}")
