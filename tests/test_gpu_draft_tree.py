"""GPU parity: jk_tree_grow / jk_tree_finalize / jk_gather_draft_probs (through the C ABI) against the
tree-growth oracle, bit for bit (integer results; scores are single fp32 products on both sides), and one
whole round on the device: experts -> heads -> tree -> verification attention -> acceptance."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from gpu_util import reset_tuning, tune
from oracle import accept_path as oracle_accept, draft_tree as dt
from workloads import draft_head_inputs, moe_inputs

pytestmark = pytest.mark.gpu


def _cands(rng, rows, k, vocab=5000, ties=False):
    p = np.sort(rng.random((rows, 2, k)).astype(np.float32), axis=2)[:, :, ::-1] * np.float32(0.9)
    if ties:
        p = np.round(p * 4) / 4
    tok = rng.integers(0, vocab, size=(rows, 2, k)).astype(np.int32)
    return tok, np.ascontiguousarray(p, dtype=np.float32)


def _run_round(seed, B, depth, k, width, max_nodes, n_keep, ties=False):
    rng = np.random.default_rng(seed)
    state = jk.TreeState(B, max_nodes)
    oracles = [dt.TreeState() for _ in range(B)]
    fronts = [[-1] for _ in range(B)]
    frontier = None
    base = 0
    for d in range(depth):
        nf = 1 if frontier is None else frontier.shape[1]
        tok, p = _cands(rng, B * nf, k, ties=ties)
        frontier = jk.tree_grow(state, frontier, torch.from_numpy(tok).cuda(), torch.from_numpy(p).cuda(), width, base)
        torch.cuda.synchronize()
        got = frontier.cpu().numpy()
        for b in range(B):
            fronts[b] = dt.grow(oracles[b], fronts[b], tok[b * nf:(b + 1) * nf], p[b * nf:(b + 1) * nf], width,
                                max_nodes, base + 2 * b * nf)
            ref = fronts[b] + [fronts[b][0] if fronts[b] else -1] * (width - len(fronts[b]))
            assert got[b].tolist() == ref, (d, b)
            fronts[b] = ref
        base += 2 * B * nf
    n_nodes = state.n_nodes.cpu().numpy()
    for b in range(B):
        n = len(oracles[b].tokens)
        assert n_nodes[b] == n
        assert state.tokens[b, :n].cpu().tolist() == oracles[b].tokens
        assert state.parent[b, :n].cpu().tolist() == oracles[b].parent
        assert state.q_row[b, :n].cpu().tolist() == oracles[b].q_row
        np.testing.assert_array_equal(state.score[b, :n].cpu().numpy(), np.asarray(oracles[b].score, dtype=np.float32))
    tokens, parent, q_row, old, n_valid = jk.tree_finalize(state, n_keep)
    torch.cuda.synchronize()
    for b in range(B):
        rt, rp, rq, ro = dt.finalize(oracles[b], n_keep)
        nv = len(ro)
        assert int(n_valid[b]) == nv
        assert tokens[b, :nv].cpu().tolist() == rt.tolist()
        assert parent[b, :nv].cpu().tolist() == rp.tolist()
        assert q_row[b, :nv].cpu().tolist() == rq.tolist()
        assert old[b, :nv].cpu().tolist() == ro.tolist()
        assert (tokens[b, nv:] == -1).all() and (parent[b, nv:] == -1).all()
        if nv == n_keep:
            assert jk.validate_tree(parent[b].cpu().numpy()) == 0
    return state, tokens, parent, q_row


@pytest.mark.parametrize("B,depth,k,width,max_nodes,n_keep", [(3, 4, 5, 5, 512, 60), (1, 6, 5, 5, 1024, 100),
                                                            (4, 3, 1, 1, 64, 3), (2, 5, 16, 8, 1024, 128),
                                                            (2, 3, 2, 3, 256, 20)])
def test_growth_and_cut_match_the_oracle(B, depth, k, width, max_nodes, n_keep):
    _run_round(B * 100 + depth, B, depth, k, width, max_nodes, n_keep)


def test_equal_scores_and_capacity():
    _run_round(7, 2, 4, 4, 4, 512, 40, ties=True)
    _run_round(8, 2, 4, 5, 5, 40, 40)        # the node arrays fill up: the tail of the last depths is dropped
    _run_round(9, 1, 2, 2, 3, 64, 30)        # fewer nodes than asked for: the rest of the output says so


def test_gather_draft_probs():
    rng = np.random.default_rng(1)
    q_all = rng.random((37, 1003)).astype(np.float32)
    rows = rng.integers(0, 37, size=(3, 11)).astype(np.int32)
    out = jk.gather_draft_probs(torch.from_numpy(q_all).cuda(), torch.from_numpy(rows).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), q_all[rows])
    bad = rows.copy()
    bad[0, 0], bad[1, 1] = -5, 99                      # clamped, must not fault
    out = jk.gather_draft_probs(torch.from_numpy(q_all).cuda(), torch.from_numpy(bad).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), q_all[np.clip(bad, 0, 36)])
    q4 = rng.random((5, 1024)).astype(np.float32)      # vector path
    r4 = rng.integers(0, 5, size=(2, 3)).astype(np.int32)
    out = jk.gather_draft_probs(torch.from_numpy(q4).cuda(), torch.from_numpy(r4).cuda())
    np.testing.assert_array_equal(out.cpu().numpy(), q4[r4])


def test_whole_round_on_the_device():
    """Random weights: hidden states -> experts -> heads -> tree (3 depths) -> cut -> dense draft distributions ->
    speculative-sampling acceptance.  Every node's token is one of its distribution's top-k, its draft probability
    is positive, the tree is a valid input of the verification calls, and the acceptance result equals the
    oracle's on the same tree."""
    B, d, F, N, V, k, width, depth, n_keep = 2, 256, 384, 4, 2000, 4, 3, 3, 20
    w_head = torch.from_numpy(draft_head_inputs(1, d, V, seed=3)["w_head"]).cuda().to(torch.bfloat16)
    state = jk.TreeState(B, 256)
    frontier, base = None, 0
    q_bufs, cand_toks = [], []
    for dep in range(depth):
        nf = 1 if frontier is None else frontier.shape[1]
        x = moe_inputs(B * nf, d, F, N, seed=10 + dep)     # (the draft layer's attention is not part of the library)
        dev = lambda key: torch.from_numpy(x[key]).cuda().to(torch.bfloat16)
        f_top, s_top, idx, _ = jk.moe_experts(dev("u"), dev("centroids"), dev("w_gate"), dev("w_up"), dev("w_down"), False)
        lg, q, tk, tp = jk.draft_heads(f_top, s_top, w_head, jk.JK_HEADS_DECOUPLED, 1.0, k)
        frontier = jk.tree_grow(state, frontier, tk.reshape(B * nf, 2, k), tp.reshape(B * nf, 2, k), width, base)
        q_bufs.append(q.reshape(-1, V))
        cand_toks.append(tk.reshape(-1, k))
        base += 2 * B * nf
    q_all = torch.cat(q_bufs, 0).contiguous()
    tokens, parent, q_row, old, n_valid = jk.tree_finalize(state, n_keep)
    draft_probs = jk.gather_draft_probs(q_all, q_row)
    torch.cuda.synchronize()
    assert n_valid.cpu().tolist() == [n_keep] * B
    all_cands = torch.cat(cand_toks, 0).cpu().numpy()
    tok_h, par_h, qr_h, dp_h = tokens.cpu().numpy(), parent.cpu().numpy(), q_row.cpu().numpy(), draft_probs.cpu().numpy()
    for b in range(B):
        assert jk.validate_tree(par_h[b]) == 0
        for i in range(n_keep):
            assert tok_h[b, i] in all_cands[qr_h[b, i]]
            assert dp_h[b, i, tok_h[b, i]] > 0
            np.testing.assert_allclose(dp_h[b, i].sum(), 1.0, rtol=1e-4)
    rng = np.random.default_rng(5)
    logits = (rng.standard_normal((B, n_keep + 1, V)) * 2).astype(np.float32)
    for b in range(B):                                   # make the drafts plausible for the target
        for i in range(n_keep):
            logits[b, par_h[b, i] + 1, tok_h[b, i]] += 6.0
    uni = rng.random((B, n_keep + 1)).astype(np.float32)
    path, alen, bonus = jk.accept_path(tokens, parent, torch.from_numpy(logits).cuda(), jk.JK_SAMPLE, 1.0,
                                       draft_probs, torch.from_numpy(uni).cuda(), max_depth=depth)
    torch.cuda.synchronize()
    checked = 0
    for b in range(B):
        r = oracle_accept(tok_h[b], par_h[b], logits[b], "sample", temperature=1.0, draft_probs=dp_h[b], uniforms=uni[b])
        if r.min_margin > 1e-9:
            assert path[b, : int(alen[b])].cpu().tolist() == r.path[:depth] and int(bonus[b]) == r.bonus_token
            checked += 1
    assert checked >= 1


def test_argument_errors():
    state = jk.TreeState(1, 64)
    tok = torch.zeros((1, 2, 200), dtype=torch.int32, device="cuda")
    p = torch.zeros((1, 2, 200), dtype=torch.float32, device="cuda")
    with pytest.raises(jk.JakiroError) as e:           # 400 candidates in one call
        jk.tree_grow(state, None, tok, p, 4, 0)
    assert e.value.status == 3
    with pytest.raises(jk.JakiroError) as e:
        jk.tree_finalize(state, 65)
    assert e.value.status == 1
    big = jk.TreeState(1, 2048)
    with pytest.raises(jk.JakiroError) as e:
        jk.tree_grow(big, None, tok[:, :, :4].contiguous(), p[:, :, :4].contiguous(), 4, 0)
    assert e.value.status == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("B,k,k1,k2,width,max_nodes", [(2, 5, 5, 5, 5, 512), (3, 4, 2, 3, 7, 256), (1, 8, 8, 8, 32, 1024),
                                                      (2, 6, 6, 4, 4, 60)])
def test_parallel_tail_matches_the_oracle(B, k, k1, k2, width, max_nodes):
    rng = np.random.default_rng(B * 10 + k)
    state = jk.TreeState(B, max_nodes)
    oracles = [dt.TreeState() for _ in range(B)]
    tok, p = _cands(rng, B, k)
    front_w = 4
    frontier = jk.tree_grow(state, None, torch.from_numpy(tok).cuda(), torch.from_numpy(p).cuda(), front_w, 0)
    fronts = [dt.grow(oracles[b], [-1], tok[b:b + 1], p[b:b + 1], front_w, max_nodes, 2 * b) for b in range(B)]
    tok, p = _cands(rng, B * front_w, k)
    base = 2 * B
    jk.tree_grow_tail(state, frontier, torch.from_numpy(tok).cuda(), torch.from_numpy(p).cuda(), k1, k2, width, base)
    torch.cuda.synchronize()
    for b in range(B):
        dt.grow_parallel_tail(oracles[b], fronts[b], tok[b * front_w:(b + 1) * front_w], p[b * front_w:(b + 1) * front_w],
                              k1, k2, width, max_nodes, base + 2 * b * front_w)
        n = len(oracles[b].tokens)
        assert int(state.n_nodes[b]) == n
        assert state.tokens[b, :n].cpu().tolist() == oracles[b].tokens
        assert state.parent[b, :n].cpu().tolist() == oracles[b].parent
        assert state.q_row[b, :n].cpu().tolist() == oracles[b].q_row
        np.testing.assert_array_equal(state.score[b, :n].cpu().numpy(), np.asarray(oracles[b].score, dtype=np.float32))
    n_keep = min(40, max_nodes)
    tokens, parent, q_row, old, n_valid = jk.tree_finalize(state, n_keep)
    torch.cuda.synchronize()
    for b in range(B):
        rt, rp, rq, ro = dt.finalize(oracles[b], n_keep)
        nv = len(ro)
        assert int(n_valid[b]) == nv and parent[b, :nv].cpu().tolist() == rp.tolist()
        assert tokens[b, :nv].cpu().tolist() == rt.tolist() and q_row[b, :nv].cpu().tolist() == rq.tolist()


def test_example_round_runs_and_is_consistent():
    """The example that strings all calls of a round together (draft passes, tree, verification, acceptance,
    commit): the tree it builds is valid, the accepted path follows tree edges, lengths advance by accept_len.
    The draft layer's attention gets the partial draft tree (Eq. 1, Section 3.1.1): its slot parents are the
    growing tree's own edges, and its output is the oracle's tree attention over the draft cache and those slots."""
    from oracle import tree_verify_attention as oracle_attention
    from paper_2502_06282_amd import example_round
    r = example_round.run(batch=2, seed=1, verbose=False)
    par = r["parent"].cpu().numpy()
    path, alen = r["path"].cpu().numpy(), r["accept_len"].cpu().numpy()
    for b in range(2):
        assert jk.validate_tree(par[b]) == 0
        prev = -1
        for i in range(int(alen[b])):
            assert par[b, path[b, i]] == prev
            prev = path[b, i]
        assert int(r["prefix_len"][b]) == 256 + int(alen[b])
        assert 0 <= int(r["bonus"][b]) < 8000
    assert all(torch.isfinite(o.float()).all() for o in r["outs"])
    # the partial tree of the draft passes
    rd = r["round"]
    dpar, node = r["draft_parent"].cpu().numpy(), r["draft_slot_node"].cpu().numpy()
    st_parent = rd.state.parent.cpu().numpy()
    t_all = dpar.shape[1]
    assert t_all == rd.t_max == 1 + 4 * 3 and node.shape == dpar.shape
    for b in range(2):
        assert jk.validate_tree(dpar[b]) == 0 and dpar[b, 0] == -1 and node[b, 0] == -1
        assert (dpar[b, 1:] >= 0).all(), "every expanded node descends from the last committed token's slot"
        for s_ in range(1, t_all):
            assert st_parent[b, node[b, s_]] == node[b, dpar[b, s_]]
        assert len(set(node[b, 1:].tolist())) == t_all - 1
    assert (dpar[:, 5:].max(axis=1) >= 1).all(), "later passes must hang below earlier passes' nodes, not only the root"
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    ref = oracle_attention(f64(rd.q_acc), f64(rd.dk_cache), f64(rd.dv_cache), f64(rd.k_acc), f64(rd.v_acc), dpar, [256, 256])
    got = f64(rd.o_acc)
    # (slots of the last pass hold that pass's output; earlier slots were recomputed by every later pass with the
    # same inputs, so all of them must agree with the oracle)
    assert np.abs(got - ref).max() <= 2e-2 * np.abs(ref).max()


def test_example_round_phases_replay_as_graphs():
    """The three phases captured as HIP graphs: every replay of the round gives the eager round's results."""
    from paper_2502_06282_amd import example_round
    rd = example_round.Round(seed=3, **example_round.SHAPES["small"])
    eager = {k: v.clone() for k, v in rd.run().items() if k in ("tokens", "parent", "path", "accept_len", "bonus", "prefix_len")}
    outs = [o.clone() for o in rd.result["outs"]]
    torch.cuda.synchronize()
    graphs = rd.capture()
    replayed = dict(rd.result)         # the tensors the graphs write (an eager round makes new ones)
    for _ in range(3):
        for t_ in replayed["outs"]:
            t_.zero_()
        for name in ("draft", "verify", "refine"):
            graphs[name].replay()
        torch.cuda.synchronize()
        for k, v in eager.items():
            assert torch.equal(replayed[k], v), k
        for a, b in zip(outs, replayed["outs"]):
            assert torch.equal(a, b)
        rd.run()                       # eager work between replays
        torch.cuda.synchronize()
    t = rd.time_phases(reps=3)
    assert t["round_us"] > 0 and t["draft_us"] > 0 and t["verify_us"] > 0 and t["refine_us"] > 0


def test_acceptance_through_the_row_table_equals_the_dense_call():
    """jk_accept_path_rows on (q_all, q_row) gives exactly what jk_accept_path gives on the gathered dense array,
    for the cooperative walk (large vocabulary) and the single-workgroup walk (forced), bad row numbers clamped."""
    import os
    rng = np.random.default_rng(4)
    for V, B, N in ((5000, 3, 17), (40000, 2, 30)):
        n_rows = 23
        q_all = rng.dirichlet(np.full(V, 0.05), size=n_rows).astype(np.float32)
        q_row = rng.integers(0, n_rows, size=(B, N)).astype(np.int32)
        q_row[0, 0] = n_rows + 5                       # clamped to the last row
        parent = np.stack([np.concatenate([[-1], rng.integers(-1, np.arange(1, N))]) for _ in range(B)]).astype(np.int32)
        dense = q_all[np.clip(q_row, 0, n_rows - 1)]
        tokens = np.zeros((B, N), dtype=np.int32)
        for b in range(B):
            for i in range(N):
                tokens[b, i] = rng.choice(V, p=dense[b, i].astype(np.float64) / dense[b, i].astype(np.float64).sum())
        logits = (rng.standard_normal((B, N + 1, V)) * 2).astype(np.float32)
        for b in range(B):
            for i in range(N):
                logits[b, parent[b, i] + 1, tokens[b, i]] += 5.0
        uni = rng.random((B, N + 1)).astype(np.float32)
        t = lambda a: torch.from_numpy(a).cuda()
        for single in ("0", "1"):
            tune("accept_single", single)
            try:
                ref = jk.accept_path(t(tokens), t(parent), t(logits), jk.JK_SAMPLE, 0.9, t(dense), t(uni))
                got = jk.accept_path_rows(t(tokens), t(parent), t(logits), t(q_all), t(q_row), t(uni), 0.9)
                torch.cuda.synchronize()
            finally:
                reset_tuning()
            for a, b_ in zip(ref, got):
                assert torch.equal(a, b_)
            assert int(ref[1].min()) >= 0


def test_static_shape_fill_matches_the_oracle_and_rebuilds_the_predefined_tree():
    """The predefined 28-node tree of workload c7, filled depth by depth from random candidate lists: the first
    half of a node's children (rounded up) take the left expert's best candidates, the rest the right expert's."""
    from workloads import static_tree, tree_depths
    shape_parent = static_tree()
    depth_of = tree_depths(shape_parent)
    N, B, k = len(shape_parent), 3, 4
    rng = np.random.default_rng(6)
    state = jk.TreeState(B, 64)
    oracles = [dt.TreeState() for _ in range(B)]
    frontier_nodes = [-1]                       # shape nodes whose children come next (-1: the root)
    frontier_dev, fronts = None, [[-1] for _ in range(B)]
    base = 0
    t32 = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda")
    for d in range(1, int(depth_of.max()) + 1):
        new = [i for i in range(N) if depth_of[i] == d]
        slot, expert, rank = [], [], []
        for p in frontier_nodes:
            ch = [i for i in new if shape_parent[i] == p]
            n_left = (len(ch) + 1) // 2
            for j, _ in enumerate(ch):
                slot.append(frontier_nodes.index(p))
                expert.append(0 if j < n_left else 1)
                rank.append(j if j < n_left else j - n_left)
        nxt_nodes = [i for i in new if (shape_parent == i).any()]
        next_index = [new.index(i) for i in nxt_nodes]
        nf = len(frontier_nodes)
        tok, p = _cands(rng, B * nf, k)
        fo, ids = jk.tree_fill_static(state, frontier_dev, torch.from_numpy(tok).cuda(), torch.from_numpy(p).cuda(),
                                      t32(slot), t32(expert), t32(rank), t32(next_index) if next_index else None, base)
        torch.cuda.synchronize()
        for b in range(B):
            got_ids = dt.fill_static(oracles[b], fronts[b], tok[b * nf:(b + 1) * nf], p[b * nf:(b + 1) * nf], slot, expert,
                                     rank, 64, base + 2 * b * nf)
            assert ids[b].cpu().tolist() == got_ids
            fronts[b] = [got_ids[j] for j in next_index]
            if next_index:
                assert fo[b].cpu().tolist() == fronts[b]
        frontier_nodes, frontier_dev = nxt_nodes, fo
        base += 2 * B * nf
    tokens, parent, q_row, old, n_valid = jk.tree_finalize(state, N)
    torch.cuda.synchronize()
    for b in range(B):
        assert int(state.n_nodes[b]) == N and int(n_valid[b]) == N
        assert state.tokens[b, :N].cpu().tolist() == oracles[b].tokens
        assert state.q_row[b, :N].cpu().tolist() == oracles[b].q_row
        np.testing.assert_array_equal(state.score[b, :N].cpu().numpy(), np.asarray(oracles[b].score, dtype=np.float32))
        assert parent[b].cpu().tolist() == shape_parent.tolist()       # the predefined tree, as the verification takes it
        assert old[b].cpu().tolist() == list(range(N))
