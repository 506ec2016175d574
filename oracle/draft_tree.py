"""Oracle: growing the draft token tree from the two experts' candidate lists.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

What is computed (Section 3.1.2 of the paper: at every depth both activated
experts propose their own top-k candidates for each expanded node, the expert
with the larger router score on the left, the other on the right; the process
follows the top-k construction principle of the Eagle tree and can be combined
with a dynamically constructed tree).  The paper gives no further rule, so the
growth and the final cut below are this library's reading of "dynamic tree
with two candidate lists per node":

  grow (one depth, one sequence)
      for every frontier node f (in node order), for expert e = left, right,
      for rank j = 0..k-1:  a new node with token cand_tok[f][e][j], parent f and
      score = score(f) * cand_p[f][e][j]   (fp32 product; the root has score 1),
      numbered in exactly that order, so that the children of a node are ordered
      left to right by index with the left expert's list first.
      Nodes beyond the capacity are dropped.
      Next frontier: the `width` new nodes with the largest scores (ties to the
      lower index), listed in increasing index.
  finalize (one sequence)
      keep the n_keep nodes with the largest scores (ties to the lower index);
      a candidate probability is at most 1, so a node never scores higher than
      its parent and the kept set contains every kept node's ancestors;
      renumber the kept nodes in increasing old index (still parents first,
      siblings left to right) and translate the parents.

Scores are products of fp32 numbers taken in fp32, in path order, on both
sides, so the integer results (frontiers, kept sets, numbering) can be
compared exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np


@dataclass
class TreeState:
    tokens: List[int] = field(default_factory=list)
    parent: List[int] = field(default_factory=list)
    score: List[np.float32] = field(default_factory=list)
    q_row: List[int] = field(default_factory=list)   # row of the draft distribution the node's token came from


def grow(state: TreeState, frontier: Sequence[int], cand_tok: np.ndarray, cand_p: np.ndarray, width: int,
         max_nodes: int, q_row_base: int) -> List[int]:
    """One depth.  frontier: node ids (or [-1] for the root); cand_tok, cand_p [len(frontier)][2][k].
    The distribution of (frontier slot f, expert e) has row number q_row_base + 2 f + e.
    Appends the new nodes to `state` and returns the next frontier."""
    new = []
    k = cand_tok.shape[2]
    for f, pid in enumerate(frontier):
        ps = np.float32(1.0) if pid < 0 else state.score[pid]
        for e in range(2):
            for j in range(k):
                if len(state.tokens) >= max_nodes:
                    continue
                new.append(len(state.tokens))
                state.tokens.append(int(cand_tok[f, e, j]))
                state.parent.append(int(pid))
                state.score.append(np.float32(ps * np.float32(cand_p[f, e, j])))
                state.q_row.append(q_row_base + 2 * f + e)
    best = sorted(new, key=lambda i: (-float(state.score[i]), i))[:width]
    return sorted(best)


def finalize(state: TreeState, n_keep: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Cut to the n_keep best nodes.  Returns (tokens, parent, q_row, old_index) of the kept nodes, renumbered."""
    n = len(state.tokens)
    order = sorted(range(n), key=lambda i: (-float(state.score[i]), i))[:n_keep]
    kept = sorted(order)
    new_id = {-1: -1}
    for i, old in enumerate(kept):
        new_id[old] = i
    return (np.asarray([state.tokens[i] for i in kept], dtype=np.int64),
            np.asarray([new_id[state.parent[i]] for i in kept], dtype=np.int64),
            np.asarray([state.q_row[i] for i in kept], dtype=np.int64),
            np.asarray(kept, dtype=np.int64))


def grow_parallel_tail(state: TreeState, frontier: Sequence[int], cand_tok: np.ndarray, cand_p: np.ndarray,
                       k1: int, k2: int, width: int, max_nodes: int, q_row_base: int) -> None:
    """The last draft pass when the two heads are the mixture head and the contrastive head (Section 3.2,
    Eq. 6-8): the mixture head's candidates are the next level as usual, and the contrastive head, which
    predicts one position further from the same features, supplies the level after it without another pass
    of the draft model.

    Reading: every frontier node f gets the first k1 candidates of its mixture list (cand_*[f][0]) as
    children; then each of the `width` best children (ties to the lower index), in index order, gets the
    first k2 candidates of its parent's contrastive list (cand_*[f][1]) as children.  All children are
    numbered before all grandchildren.  Scores multiply as in `grow`; the distribution rows are
    q_row_base + 2 f for children and q_row_base + 2 f + 1 for grandchildren."""
    children, slot_of = [], {}
    for f, pid in enumerate(frontier):
        ps = np.float32(1.0) if pid < 0 else state.score[pid]
        for j in range(k1):
            if len(state.tokens) >= max_nodes:
                continue
            c = len(state.tokens)
            children.append(c)
            slot_of[c] = f
            state.tokens.append(int(cand_tok[f, 0, j]))
            state.parent.append(int(pid))
            state.score.append(np.float32(ps * np.float32(cand_p[f, 0, j])))
            state.q_row.append(q_row_base + 2 * f)
    best = sorted(sorted(children, key=lambda i: (-float(state.score[i]), i))[:width])
    for c in best:
        f = slot_of[c]
        for j in range(k2):
            if len(state.tokens) >= max_nodes:
                continue
            state.tokens.append(int(cand_tok[f, 1, j]))
            state.parent.append(c)
            state.score.append(np.float32(state.score[c] * np.float32(cand_p[f, 1, j])))
            state.q_row.append(q_row_base + 2 * f + 1)


def fill_static(state: TreeState, frontier: Sequence[int], cand_tok: np.ndarray, cand_p: np.ndarray,
                slot: Sequence[int], expert: Sequence[int], rank: Sequence[int], max_nodes: int,
                q_row_base: int) -> List[int]:
    """One depth of a predefined (static) tree shape (Section 3.1.2: the two candidate lists can also fill a
    predefined tree): new node j hangs under frontier node frontier[slot[j]] and takes candidate rank[j] of
    that node's list of expert[j] (0 = left, 1 = right).  The shape is the caller's; nodes are appended in
    the order given.  Returns the indices of the appended nodes (-1 for nodes dropped at the capacity)."""
    ids = []
    for j in range(len(slot)):
        f, e, r = int(slot[j]), int(expert[j]), int(rank[j])
        pid = int(frontier[f])
        ps = np.float32(1.0) if pid < 0 else state.score[pid]
        if len(state.tokens) >= max_nodes:
            ids.append(-1)
            continue
        ids.append(len(state.tokens))
        state.tokens.append(int(cand_tok[f, e, r]))
        state.parent.append(pid)
        state.score.append(np.float32(ps * np.float32(cand_p[f, e, r])))
        state.q_row.append(q_row_base + 2 * f + e)
    return ids
