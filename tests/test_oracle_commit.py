"""Pins for the commit oracle (oracle/commit_path.py): facts that do not restate its copy loop."""
import numpy as np
import pytest

from oracle import accept_path, commit_path, committed_rows, tree_verify_attention
from workloads import CONFIGS, accept_inputs, attention_inputs, tree_for_config


def _setup(seed=3, L=37, cap=64):
    cfg = CONFIGS["c1_tiny"].with_(batch=2, prefix_len=cap, n_q_heads=4, n_kv_heads=2, head_dim=16)
    par = tree_for_config(cfg, seed=seed)
    x = attention_inputs(cfg, seed=seed)
    return cfg, par, x, [L, L - 9]


def _paths(par, depth_wanted):
    """A root-to-node chain of the wanted length (or the longest there is) per sequence."""
    out, lens = [], []
    for b in range(par.shape[0]):
        best = []
        for i in range(par.shape[1]):
            chain, a = [], i
            while a >= 0:
                chain.append(a)
                a = int(par[b, a])
            chain.reverse()
            if len(chain) > len(best) and len(chain) <= depth_wanted:
                best = chain
        lens.append(len(best))
        out.append(best + [-1] * (8 - len(best)))
    return np.array(out, dtype=np.int32), lens


def test_last_accepted_node_sees_the_committed_cache_as_plain_decoding():
    """Verification attention of the last accepted node before the commit == one-token decode
    attention over the committed cache: fixes which rows go where, in which order, and the new length."""
    cfg, par, x, plen = _setup()
    path, lens = _paths(par, 3)
    before = tree_verify_attention(**x, parent=par, prefix_len=plen)
    kc, vc, new_len = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, lens, plen)
    for b in range(cfg.batch):
        assert lens[b] >= 2 and new_len[b] == plen[b] + lens[b]
        last = path[b, lens[b] - 1]
        # the last accepted node as a lone query whose own key/value already sit in the cache:
        # decode attention over new_len rows = a single tree node with prefix new_len - 1
        xb = {"q": x["q"][b:b + 1, last:last + 1], "k_cache": kc[b:b + 1], "v_cache": vc[b:b + 1],
              "k_tree": x["k_tree"][b:b + 1, last:last + 1], "v_tree": x["v_tree"][b:b + 1, last:last + 1]}
        after = tree_verify_attention(**xb, parent=np.array([[-1]]), prefix_len=[new_len[b] - 1])
        np.testing.assert_allclose(after[0, 0], before[b, last], rtol=1e-12, atol=1e-14)


def test_everything_else_is_untouched_and_order_matters():
    cfg, par, x, plen = _setup()
    path, lens = _paths(par, 3)
    kc, vc, new_len = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, lens, plen)
    for b in range(cfg.batch):
        lo, hi = plen[b], plen[b] + lens[b]
        np.testing.assert_array_equal(kc[b, :lo], x["k_cache"][b, :lo])
        np.testing.assert_array_equal(vc[b, hi:], x["v_cache"][b, hi:])
        # reversing the path changes the committed block (the rows are distinct random vectors)
        rev = path.copy()
        rev[b, :lens[b]] = rev[b, :lens[b]][::-1]
        kr, _, _ = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], rev, lens, plen)
        assert not np.array_equal(kr[b, lo:hi], kc[b, lo:hi])
    # inputs are not modified in place
    assert not np.shares_memory(kc, x["k_cache"])


@pytest.mark.parametrize("alen,expect", [(0, 0), (-1, 0), (2, 2), (99, 8)])
def test_length_cuts(alen, expect):
    assert committed_rows([0, 1, 2, 3, 4, 5, 6, 7], alen, 10, 5, 64) == expect


def test_bad_node_id_and_capacity_end_the_commit():
    assert committed_rows([0, 1, 12, 3], 4, 10, 5, 64) == 2      # node 12 does not exist
    assert committed_rows([0, -1, 2, 3], 4, 10, 5, 64) == 1      # padding inside the counted part
    assert committed_rows([0, 1, 2, 3], 4, 10, 62, 64) == 2      # two rows of room
    assert committed_rows([0, 1, 2, 3], 4, 10, 64, 64) == 0
    cfg, par, x, plen = _setup(L=62, cap=64)
    path = np.array([[0, 1, 2, 3, -1, -1, -1, -1]] * 2, dtype=np.int32)
    # make the ids a valid chain irrespective of the tree: only existence matters to the commit
    kc, vc, new_len = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, [4, 4], [62, 53])
    assert list(new_len) == [64, 57]
    np.testing.assert_array_equal(kc[0, 63], x["k_tree"][0, 1])
    kc2, _, keep = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, [4, 4], [62, 53],
                               advance=False)
    assert list(keep) == [62, 53]
    np.testing.assert_array_equal(kc2, kc)


def test_greedy_round_trip_walk_then_commit():
    """The walk's own output feeds the commit: accepted nodes form a root-to-node chain, so after the
    commit the cache holds prefix ++ tokens' rows in exactly the order the walk accepted them."""
    cfg = CONFIGS["c1_tiny"].with_(batch=3, prefix_len=20)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg)
    acc = accept_inputs(cfg, par)
    paths, lens = [], []
    for b in range(cfg.batch):
        r = accept_path(acc["tokens"][b], par[b], acc["logits"][b], "greedy")
        p = list(r.path) + [-1] * (cfg.depth - len(r.path))
        paths.append(p[:cfg.depth])
        lens.append(r.accept_len)
        for i in range(1, r.accept_len):
            assert par[b, r.path[i]] == r.path[i - 1]
    cap = x["k_cache"].shape[1]
    kc, _, new_len = commit_path(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], np.array(paths), lens,
                                 [cap - 8] * cfg.batch)
    for b in range(cfg.batch):
        for i in range(lens[b]):
            np.testing.assert_array_equal(kc[b, cap - 8 + i], x["k_tree"][b, paths[b][i]])
        assert new_len[b] == cap - 8 + lens[b]
