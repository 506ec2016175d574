"""Pins for the attention oracle: every check compares it with something that is
not itself -- torch's scaled_dot_product_attention (a library routine), closed
forms, or structural invariants of the tree mask (Section 2.1 step 2; Section
3.1.2, tree attention mask)."""
import numpy as np
import pytest
import torch

from oracle import ancestor_sets, tree_verify_attention
from workloads import CONFIGS, attention_inputs, coin_tree, tree_for_config, two_expert_tree


def _rand(rng, B, T, Hq, Hkv, D, L):
    return dict(
        q=rng.standard_normal((B, T, Hq, D)),
        k_cache=rng.standard_normal((B, L, Hkv, D)),
        v_cache=rng.standard_normal((B, L, Hkv, D)),
        k_tree=rng.standard_normal((B, T, Hkv, D)),
        v_tree=rng.standard_normal((B, T, Hkv, D)),
    )


def _sdpa(q, k, v, mask=None, causal=False, scale=None):
    """q [H,Tq,D], k/v [H,Tk,D] float64 -> [H,Tq,D] via torch (library routine)."""
    o = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        attn_mask=None if mask is None else torch.from_numpy(mask), is_causal=causal, scale=scale)
    return o[0].numpy()


def test_hand_computed_two_keys():
    # D=1, scale=1, q=1: prefix key 0 (value 0), the node's own key ln 3 (value 1)
    # -> weights 1 : 3 -> 0.75.  Second node (child): keys 0, ln3, ln4 -> (3*1 + 4*2)/8.
    q = np.ones((1, 2, 1, 1))
    kc = np.zeros((1, 1, 1, 1)); vc = np.zeros((1, 1, 1, 1))
    kt = np.log(np.array([3.0, 4.0])).reshape(1, 2, 1, 1)
    vt = np.array([1.0, 2.0]).reshape(1, 2, 1, 1)
    out = tree_verify_attention(q, kc, vc, kt, vt, np.array([[-1, 0]]), [1], scale=1.0)
    assert out[0, 0, 0, 0] == pytest.approx(0.75, abs=1e-15)
    assert out[0, 1, 0, 0] == pytest.approx(11.0 / 8.0, abs=1e-15)
    # siblings instead of a chain: the second node no longer sees the first
    out = tree_verify_attention(q, kc, vc, kt, vt, np.array([[-1, -1]]), [1], scale=1.0)
    assert out[0, 1, 0, 0] == pytest.approx(8.0 / 5.0, abs=1e-15)


def test_default_scale_is_inverse_sqrt_d():
    rng = np.random.default_rng(5)
    x = _rand(rng, 1, 3, 2, 2, 16, 7)
    par = np.array([[-1, 0, 0]])
    a = tree_verify_attention(**x, parent=par, prefix_len=[7])
    b = tree_verify_attention(**x, parent=par, prefix_len=[7], scale=0.25)
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("G", [1, 4])
def test_chain_tree_equals_causal_attention(G):
    """P1: parent = [-1,0,1,...] is ordinary causal attention over prefix ++ tree."""
    rng = np.random.default_rng(11)
    B, T, Hkv, D, L = 2, 9, 2, 32, 37
    Hq = Hkv * G
    x = _rand(rng, B, T, Hq, Hkv, D, L)
    par = np.tile(np.arange(-1, T - 1), (B, 1))
    out = tree_verify_attention(**x, parent=par, prefix_len=[L, L])
    for b in range(B):
        k = np.concatenate([x["k_cache"][b], x["k_tree"][b]], 0).transpose(1, 0, 2)
        v = np.concatenate([x["v_cache"][b], x["v_tree"][b]], 0).transpose(1, 0, 2)
        k = np.repeat(k, G, axis=0); v = np.repeat(v, G, axis=0)
        # (i) explicit mask on the T tree queries
        mask = (np.arange(L + T)[None, :] <= (L + np.arange(T))[:, None])
        ref = _sdpa(np.ascontiguousarray(x["q"][b].transpose(1, 0, 2)), k, v, mask=mask)
        np.testing.assert_allclose(out[b].transpose(1, 0, 2), ref, rtol=0, atol=1e-12)
        # (ii) is_causal on the full sequence with arbitrary queries at prefix positions
        qfull = np.concatenate([rng.standard_normal((Hq, L, D)), x["q"][b].transpose(1, 0, 2)], 1)
        ref2 = _sdpa(qfull, k, v, causal=True)[:, L:, :]
        np.testing.assert_allclose(out[b].transpose(1, 0, 2), ref2, rtol=0, atol=1e-12)


def test_single_node_equals_decode_attention():
    """P2: T=1 is one-token decode attention over L+1 keys."""
    rng = np.random.default_rng(12)
    x = _rand(rng, 1, 1, 4, 2, 64, 50)
    out = tree_verify_attention(**x, parent=np.array([[-1]]), prefix_len=[50])
    k = np.repeat(np.concatenate([x["k_cache"][0], x["k_tree"][0]], 0).transpose(1, 0, 2), 2, 0)
    v = np.repeat(np.concatenate([x["v_cache"][0], x["v_tree"][0]], 0).transpose(1, 0, 2), 2, 0)
    ref = _sdpa(np.ascontiguousarray(x["q"][0].transpose(1, 0, 2)), k, v)
    np.testing.assert_allclose(out[0].transpose(1, 0, 2), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_per_node_linearisation(seed):
    """P3: out[i] == plain attention of q_i over prefix ++ path(root -> i)."""
    rng = np.random.default_rng(100 + seed)
    tree = two_expert_tree(rng, depth=4, topk=2, frontier=2, budget=14)
    par = tree["parent"]
    T = len(par)
    Hq, Hkv, D, L = 4, 2, 16, 13
    x = _rand(rng, 1, T, Hq, Hkv, D, L)
    out = tree_verify_attention(**x, parent=par[None], prefix_len=[L])
    for i in range(T):
        path = []
        a = i
        while a >= 0:
            path.append(a); a = par[a]
        path = path[::-1]
        k = np.concatenate([x["k_cache"][0, :L], x["k_tree"][0, path]], 0).transpose(1, 0, 2)
        v = np.concatenate([x["v_cache"][0, :L], x["v_tree"][0, path]], 0).transpose(1, 0, 2)
        k = np.repeat(k, 2, 0); v = np.repeat(v, 2, 0)
        ref = _sdpa(np.ascontiguousarray(x["q"][0, i][:, None, :]), k, v)[:, 0, :]
        np.testing.assert_allclose(out[0, i], ref, rtol=0, atol=1e-12)


def test_sibling_independence_bitwise():
    """P4: nodes outside A(i) cannot influence out[i], not even with NaN/huge values."""
    rng = np.random.default_rng(13)
    par = two_expert_tree(rng, depth=3, topk=2, frontier=2, budget=10)["parent"]
    T = len(par)
    x = _rand(rng, 1, T, 2, 1, 8, 5)
    base = tree_verify_attention(**x, parent=par[None], prefix_len=[5])
    anc = ancestor_sets(par)
    for i in range(T):
        y = {k: v.copy() for k, v in x.items()}
        others = [j for j in range(T) if j not in anc[i]]
        y["k_tree"][0, others] = np.nan
        y["v_tree"][0, others] = 1e300
        y["q"][0, [j for j in range(T) if j != i]] = np.nan
        with np.errstate(all="ignore"):
            pert = tree_verify_attention(**y, parent=par[None], prefix_len=[5])
        np.testing.assert_array_equal(pert[0, i], base[0, i])
    # and a visible ancestor does matter
    y = {k: v.copy() for k, v in x.items()}
    leaf = T - 1
    y["v_tree"][0, anc[leaf][-1]] += 1.0
    pert = tree_verify_attention(**y, parent=par[None], prefix_len=[5])
    assert np.abs(pert[0, leaf] - base[0, leaf]).max() > 1e-6


def test_star_tree_is_independent_decodes():
    """P5: all parents -1 -> every node is a decode over L keys + itself."""
    rng = np.random.default_rng(14)
    T, L = 6, 21
    x = _rand(rng, 1, T, 2, 2, 16, L)
    out = tree_verify_attention(**x, parent=np.full((1, T), -1), prefix_len=[L])
    for i in range(T):
        one = tree_verify_attention(x["q"][:, i:i + 1], x["k_cache"], x["v_cache"],
                                    x["k_tree"][:, i:i + 1], x["v_tree"][:, i:i + 1],
                                    np.array([[-1]]), [L])
        np.testing.assert_allclose(out[0, i], one[0, 0], rtol=0, atol=1e-14)


def test_closed_forms():
    """P6: equal V rows -> that row; equal K rows -> mean of visible V rows
    (count = L + depth); empty prefix + root -> its own V row."""
    rng = np.random.default_rng(15)
    par = coin_tree(rng, 10, 3)
    T, L = len(par), 9
    x = _rand(rng, 1, T, 2, 2, 8, L)
    y = dict(x)
    row = rng.standard_normal(8)
    y["v_cache"] = np.broadcast_to(row, x["v_cache"].shape).copy()
    y["v_tree"] = np.broadcast_to(row, x["v_tree"].shape).copy()
    out = tree_verify_attention(**y, parent=par[None], prefix_len=[L])
    np.testing.assert_allclose(out, np.broadcast_to(row, out.shape), rtol=0, atol=1e-14)

    y = dict(x)
    krow = rng.standard_normal(8)
    y["k_cache"] = np.broadcast_to(krow, x["k_cache"].shape).copy()
    y["k_tree"] = np.broadcast_to(krow, x["k_tree"].shape).copy()
    out = tree_verify_attention(**y, parent=par[None], prefix_len=[L])
    anc = ancestor_sets(par)
    for i in range(T):
        for h in range(2):
            mean = (x["v_cache"][0, :L, h].sum(0) + x["v_tree"][0, anc[i], h].sum(0)) / (L + len(anc[i]))
            np.testing.assert_allclose(out[0, i, h], mean, rtol=0, atol=1e-13)

    out = tree_verify_attention(**x, parent=par[None], prefix_len=[0])
    roots = [i for i in range(T) if par[i] < 0]
    for i in roots:
        np.testing.assert_allclose(out[0, i], x["v_tree"][0, i], rtol=0, atol=1e-15)


def test_prefix_len_hides_cache_tail():
    rng = np.random.default_rng(16)
    x = _rand(rng, 1, 3, 2, 2, 8, 12)
    par = np.array([[-1, 0, 0]])
    a = tree_verify_attention(**x, parent=par, prefix_len=[7])
    y = {k: v.copy() for k, v in x.items()}
    y["k_cache"][0, 7:] = np.nan
    y["v_cache"][0, 7:] = np.nan
    b = tree_verify_attention(**y, parent=par, prefix_len=[7])
    np.testing.assert_array_equal(a, b)


def test_gqa_equals_expanded_mha():
    """P7: consecutive query heads share a KV head (kv = h // G)."""
    rng = np.random.default_rng(17)
    par = coin_tree(rng, 10, 3)
    x = _rand(rng, 1, 10, 8, 2, 16, 11)
    a = tree_verify_attention(**x, parent=par[None], prefix_len=[11])
    y = dict(x)
    for n in ("k_cache", "v_cache", "k_tree", "v_tree"):
        y[n] = np.repeat(x[n], 4, axis=2)
    b = tree_verify_attention(**y, parent=par[None], prefix_len=[11])
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_relabelling_permutes_rows():
    """P8: another topological numbering of the same tree permutes the output rows."""
    rng = np.random.default_rng(18)
    par = two_expert_tree(rng, depth=4, topk=2, frontier=2, budget=12)["parent"]
    T = len(par)
    x = _rand(rng, 1, T, 2, 1, 8, 6)
    base = tree_verify_attention(**x, parent=par[None], prefix_len=[6])
    # DFS preorder is topological too
    order = []
    def dfs(c):
        for k in range(T):
            if par[k] == c:
                order.append(k); dfs(k)
    dfs(-1)
    new_of = {old: new for new, old in enumerate(order)}
    new_of[-1] = -1
    par2 = np.array([new_of[par[old]] for old in order])
    y = dict(x)
    for n in ("q", "k_tree", "v_tree"):
        y[n] = x[n][:, order]
    out2 = tree_verify_attention(**y, parent=par2[None], prefix_len=[6])
    np.testing.assert_allclose(out2[0], base[0, order], rtol=0, atol=1e-14)


def test_bad_tree_rejected():
    x = _rand(np.random.default_rng(0), 1, 2, 1, 1, 4, 2)
    with pytest.raises(ValueError):
        tree_verify_attention(**x, parent=np.array([[0, -1]]), prefix_len=[2])
    with pytest.raises(ValueError):
        tree_verify_attention(**x, parent=np.array([[-2, 0]]), prefix_len=[2])


def test_config1_shapes_and_generator():
    cfg = CONFIGS["c1_tiny"]
    par = tree_for_config(cfg)
    assert par.shape == (1, 10) and (par[0] < np.arange(10)).all() and par.min() == -1
    x = attention_inputs(cfg)
    out = tree_verify_attention(**x, parent=par, prefix_len=[cfg.prefix_len])
    assert out.shape == (1, 10, 4, 64) and np.isfinite(out).all()


def test_golden_c1_regression():
    """Stored oracle results for the tiny config (written by tests/golden/make_golden.py,
    which calls only the oracle): guards against drift, not a pin."""
    import json, os
    from oracle import accept_path
    from workloads import accept_inputs
    with open(os.path.join(os.path.dirname(__file__), "golden", "c1_oracle.json")) as f:
        g = json.load(f)
    cfg = CONFIGS["c1_tiny"]
    par = tree_for_config(cfg)
    assert par[0].tolist() == g["parent"]
    out = tree_verify_attention(**attention_inputs(cfg), parent=par, prefix_len=[cfg.prefix_len])
    assert float(out.sum()) == pytest.approx(g["out_sum"], rel=1e-12)
    for key, val in g["out_samples"].items():
        i, h, d = map(int, key.split(","))
        assert out[0, i, h, d] == pytest.approx(val, rel=1e-12, abs=1e-15)
    a = accept_inputs(cfg, par)
    r = accept_path(a["tokens"][0], par[0], a["logits"][0], "greedy")
    assert (r.path, r.accept_len, r.bonus_token) == (g["greedy_path"], g["greedy_accept_len"], g["greedy_bonus"])
