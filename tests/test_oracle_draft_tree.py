"""Pins for the draft-tree growth oracle (Section 3.1.2: two candidate lists per expanded node, left
expert first; top-k construction): hand-worked example, chain special case, structural invariants."""
import numpy as np

from oracle import draft_tree as dt


def _grow_random(rng, depth, k, width, max_nodes, vocab=1000):
    st = dt.TreeState()
    frontier = [-1]
    base = 0
    for d in range(depth):
        nf = len(frontier)
        p = np.sort(rng.random((nf, 2, k)).astype(np.float32), axis=2)[:, :, ::-1] * np.float32(0.9)
        tok = rng.integers(0, vocab, size=(nf, 2, k))
        frontier = dt.grow(st, frontier, tok, p, width, max_nodes, base)
        base += 2 * nf
    return st


def test_hand_worked_two_depths():
    st = dt.TreeState()
    tok0 = np.array([[[11, 12], [21, 22]]])
    p0 = np.array([[[0.5, 0.2], [0.25, 0.05]]], dtype=np.float32)
    fr = dt.grow(st, [-1], tok0, p0, width=2, max_nodes=64, q_row_base=0)
    assert st.tokens == [11, 12, 21, 22] and st.parent == [-1] * 4 and st.q_row == [0, 0, 1, 1]
    assert fr == [0, 2]                                   # scores 0.5 and 0.25
    tok1 = np.array([[[31, 32], [41, 42]], [[51, 52], [61, 62]]])
    p1 = np.array([[[0.5, 0.25], [0.125, 0.0625]], [[1.0, 0.5], [0.25, 0.125]]], dtype=np.float32)
    fr = dt.grow(st, fr, tok1, p1, width=2, max_nodes=64, q_row_base=2)
    assert st.parent[4:] == [0, 0, 0, 0, 2, 2, 2, 2]
    assert [float(s) for s in st.score[4:]] == [0.25, 0.125, 0.0625, 0.03125, 0.25, 0.125, 0.0625, 0.03125]
    assert st.q_row[4:] == [2, 2, 3, 3, 4, 4, 5, 5]
    assert fr == [4, 8]                                   # 0.25 twice: both kept, in index order
    tokens, parent, q_row, old = dt.finalize(st, 6)
    # best six: 0 (.5), 2 (.25), 4 (.25), 8 (.25), 1 (.2), then .125 twice: the lower index (5) wins
    assert old.tolist() == [0, 1, 2, 4, 5, 8]
    assert parent.tolist() == [-1, -1, -1, 0, 0, 2]
    assert tokens.tolist() == [11, 12, 21, 31, 32, 51]
    assert q_row.tolist() == [0, 0, 1, 2, 2, 4]


def test_single_candidate_single_slot_is_a_chain():
    st = dt.TreeState()
    fr = [-1]
    for d in range(5):
        tok = np.array([[[100 + d], [200 + d]]])
        p = np.array([[[0.9], [0.3]]], dtype=np.float32)
        fr = dt.grow(st, fr, tok, p, width=1, max_nodes=64, q_row_base=2 * d)
        assert fr == [2 * d]                              # the left expert's candidate
    tokens, parent, q_row, old = dt.finalize(st, 5)
    assert old.tolist() == [0, 2, 4, 6, 8] and parent.tolist() == [-1, 0, 1, 2, 3]
    assert tokens.tolist() == [100, 101, 102, 103, 104]


def test_invariants_on_random_trees():
    rng = np.random.default_rng(0)
    for trial in range(20):
        k, width, depth = int(rng.integers(1, 6)), int(rng.integers(1, 6)), int(rng.integers(1, 7))
        width = min(width, 2 * k)
        st = _grow_random(rng, depth, k, width, max_nodes=500)
        n = len(st.tokens)
        par = np.array(st.parent)
        assert (par < np.arange(n)).all() and (par >= -1).all()
        # score = product of the candidate probabilities along the path: never above the parent's
        for i in range(n):
            if par[i] >= 0:
                assert st.score[i] <= st.score[par[i]]
        # children of one parent: contiguous, left expert's rows (even q_row) before the right's, each list
        # by non-increasing score
        for pnode in set(par.tolist()):
            ch = np.nonzero(par == pnode)[0]
            assert (np.diff(ch) == 1).all() and len(ch) == 2 * k
            assert [st.q_row[c] % 2 for c in ch] == [0] * k + [1] * k
            for half in (ch[:k], ch[k:]):
                sc = [float(st.score[c]) for c in half]
                assert sc == sorted(sc, reverse=True)
        for n_keep in (1, n // 2, n):
            if n_keep < 1:
                continue
            tokens, parent, q_row, old = dt.finalize(st, n_keep)
            assert len(old) == n_keep and (np.diff(old) > 0).all()
            kept = set(old.tolist())
            assert all(st.parent[o] in kept or st.parent[o] < 0 for o in old)          # closed under ancestors
            assert (parent < np.arange(n_keep)).all()
            worst_kept = min(float(st.score[o]) for o in old)
            assert all(float(st.score[i]) <= worst_kept for i in range(n) if i not in kept)
            assert [st.tokens[o] for o in old] == tokens.tolist()
            # the renumbering keeps the tree: parents map to parents
            back = {o: i for i, o in enumerate(old.tolist())}
            assert all((parent[i] == -1 and st.parent[o] < 0) or back[st.parent[o]] == parent[i]
                       for i, o in enumerate(old.tolist()))
        if n_keep == n:
            assert old.tolist() == list(range(n))


def test_ties_go_to_the_lower_index_and_capacity_drops_the_tail():
    st = dt.TreeState()
    tok = np.arange(8).reshape(1, 2, 4)
    p = np.full((1, 2, 4), 0.5, dtype=np.float32)
    fr = dt.grow(st, [-1], tok, p, width=3, max_nodes=6, q_row_base=0)
    assert len(st.tokens) == 6 and fr == [0, 1, 2]
    assert dt.finalize(st, 4)[3].tolist() == [0, 1, 2, 3]


def test_parallel_tail_hand_worked_and_invariants():
    st = dt.TreeState()
    fr = dt.grow(st, [-1], np.array([[[1, 2], [3, 4]]]), np.array([[[0.5, 0.25], [0.125, 0.0625]]], dtype=np.float32),
                 width=2, max_nodes=64, q_row_base=0)
    assert fr == [0, 1]
    tok = np.array([[[10, 11, 12], [20, 21, 22]], [[30, 31, 32], [40, 41, 42]]])
    p = np.array([[[0.5, 0.25, 0.125], [0.5, 0.5, 0.25]], [[1.0, 0.5, 0.25], [0.25, 0.125, 0.0625]]], dtype=np.float32)
    dt.grow_parallel_tail(st, fr, tok, p, k1=2, k2=2, width=3, max_nodes=64, q_row_base=2)
    # children: 4,5 under node 0 (0.25, 0.125), 6,7 under node 1 (0.25, 0.125); best three: 4, 6, 5
    assert st.tokens[4:8] == [10, 11, 30, 31] and st.parent[4:8] == [0, 0, 1, 1] and st.q_row[4:8] == [2, 2, 4, 4]
    assert [float(s) for s in st.score[4:8]] == [0.25, 0.125, 0.25, 0.125]
    # grandchildren in index order of the chosen children 4, 5, 6, each with its parent's contrastive list
    assert st.parent[8:] == [4, 4, 5, 5, 6, 6]
    assert st.tokens[8:] == [20, 21, 20, 21, 40, 41]
    assert st.q_row[8:] == [3, 3, 3, 3, 5, 5]
    assert [float(s) for s in st.score[8:]] == [0.125, 0.125, 0.0625, 0.0625, 0.0625, 0.03125]
    # invariants on a random case
    rng = np.random.default_rng(3)
    st = dt.TreeState()
    fr = dt.grow(st, [-1], rng.integers(0, 99, (1, 2, 4)), np.sort(rng.random((1, 2, 4)).astype(np.float32))[:, :, ::-1],
                 3, 200, 0)
    n0 = len(st.tokens)
    tok = rng.integers(0, 99, (3, 2, 5))
    p = np.sort(rng.random((3, 2, 5)).astype(np.float32), axis=2)[:, :, ::-1]
    dt.grow_parallel_tail(st, fr, tok, p, 4, 3, 5, 200, 2)
    par = np.array(st.parent)
    kids = [i for i in range(n0, len(par)) if par[i] in fr]
    grand = [i for i in range(n0, len(par)) if par[i] >= n0]
    assert len(kids) == 12 and len(grand) == 15 and max(kids) < min(grand)
    assert all(st.q_row[i] % 2 == 0 for i in kids) and all(st.q_row[i] % 2 == 1 for i in grand)
    for g in grand:                                # a grandchild's list is its grandparent's contrastive list
        f = fr.index(par[par[g]])
        assert st.tokens[g] in tok[f, 1, :3] and st.q_row[g] == st.q_row[par[g]] + 1
        assert st.score[g] <= st.score[par[g]]
    expanded = sorted(set(par[g] for g in grand))
    rest = [c for c in kids if c not in expanded]
    assert all(float(st.score[c]) <= min(float(st.score[e]) for e in expanded) for c in rest)


def test_static_fill_reduces_to_growth_for_the_full_shape_and_follows_a_given_shape():
    rng = np.random.default_rng(5)
    k, nf = 3, 2
    tok0, p0 = rng.integers(0, 99, (1, 2, k)), np.sort(rng.random((1, 2, k)).astype(np.float32))[:, :, ::-1]
    tok1, p1 = rng.integers(0, 99, (nf, 2, k)), np.sort(rng.random((nf, 2, k)).astype(np.float32), axis=2)[:, :, ::-1]
    a, b = dt.TreeState(), dt.TreeState()
    fr_a = dt.grow(a, [-1], tok0, p0, nf, 100, 0)
    ids = dt.fill_static(b, [-1], tok0, p0, [0] * (2 * k), [0] * k + [1] * k, list(range(k)) * 2, 100, 0)
    assert ids == list(range(2 * k)) and (a.tokens, a.parent, a.q_row) == (b.tokens, b.parent, b.q_row)
    assert [float(x) for x in a.score] == [float(x) for x in b.score]
    # the full shape under the same frontier gives the same nodes as growth
    dt.grow(a, fr_a, tok1, p1, nf, 100, 2)
    full = [(f, e, r) for f in range(nf) for e in range(2) for r in range(k)]
    dt.fill_static(b, fr_a, tok1, p1, [s[0] for s in full], [s[1] for s in full], [s[2] for s in full], 100, 2)
    assert (a.tokens, a.parent, a.q_row) == (b.tokens, b.parent, b.q_row)
    # a sparse shape: second frontier node only, right expert's best, then left expert's third
    c = dt.TreeState()
    dt.grow(c, [-1], tok0, p0, nf, 100, 0)
    ids = dt.fill_static(c, fr_a, tok1, p1, [1, 1], [1, 0], [0, 2], 100, 2)
    assert ids == [2 * k, 2 * k + 1]
    assert c.tokens[-2:] == [int(tok1[1, 1, 0]), int(tok1[1, 0, 2])] and c.parent[-2:] == [fr_a[1]] * 2
    assert c.q_row[-2:] == [2 + 3, 2 + 2]
    assert float(c.score[-1]) == float(np.float32(c.score[fr_a[1]] * p1[1, 0, 2]))
    # capacity
    d = dt.TreeState()
    assert dt.fill_static(d, [-1], tok0, p0, [0, 0, 0], [0, 0, 1], [0, 1, 0], 2, 0) == [0, 1, -1]
