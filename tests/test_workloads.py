"""Host-side checks of the seeded generators (tree structure, reproducibility)."""
import numpy as np

from workloads import (CONFIGS, accept_inputs, attention_inputs, bf16_bits, bf16_bits_to_f32,
                       config_rng, round_to_bf16, tree_depths, tree_for_config, two_expert_tree)


def test_two_expert_tree_structure():
    for seed in range(5):
        rng = np.random.Generator(np.random.PCG64(seed))
        t = two_expert_tree(rng, depth=6, topk=5, frontier=5, budget=60)
        par = t["parent"]
        assert len(par) == 60
        assert (par < np.arange(60)).all() and par.min() == -1
        d = tree_depths(par)
        assert (d == t["depth"]).all() and d.max() == 6
        assert (np.diff(d) >= 0).all()                       # BFS order
        # children of one parent are contiguous, experts left (0) then right (1), ranks ascending
        for c in range(-1, 60):
            kids = np.nonzero(par == c)[0]
            if len(kids) == 0:
                continue
            assert (np.diff(kids) == 1).all()
            key = list(zip(t["expert"][kids], t["rank"][kids]))
            assert key == sorted(key)
            assert len(kids) <= 10


def test_tree_for_config_reproducible_and_sized():
    for name, cfg in CONFIGS.items():
        a = tree_for_config(cfg); b = tree_for_config(cfg)
        assert (a == b).all() and a.shape == (cfg.batch, cfg.n_tree)
        for row in a:
            assert tree_depths(row).max() == cfg.depth
    c4 = tree_for_config(CONFIGS["c4_llama2_13b"])
    assert any((c4[0] != c4[b]).any() for b in range(1, 4))  # per-sequence trees differ


def test_bf16_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.140625, 1e-3, 65504.0], dtype=np.float32)
    r = round_to_bf16(x)
    assert (bf16_bits_to_f32(bf16_bits(r)) == r).all()
    assert r[0] == 1.0
    assert r[1] == 1.0           # 1 + 2^-8 is a tie -> even mantissa (1.0)
    assert r[2] == np.float32(1.015625)   # 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert np.abs(r - x).max() <= np.abs(x).max() * 2.0 ** -8


def test_attention_inputs_bf16_representable():
    cfg = CONFIGS["c2_vicuna7b"].with_(prefix_len=33)
    x = attention_inputs(cfg)
    for v in x.values():
        assert (round_to_bf16(v) == v).all()
    assert x["k_cache"].shape == (1, 33, 32, 128)
    assert abs(float(x["q"].std()) * np.sqrt(128.0) - 1.0) < 0.05


def test_greedy_tokens_hit_protocol():
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=500)
    par = tree_for_config(cfg)
    a = accept_inputs(cfg, par)
    top, tok, lg = a["top_token"], a["tokens"], a["logits"]
    assert (lg.argmax(axis=2) == top).all()                  # planted entry is the row maximum
    hits = 0
    for c in range(-1, cfg.n_tree):
        kids = np.nonzero(par[0] == c)[0]
        if len(kids) == 0:
            continue
        t = tok[0, kids]
        assert len(set(t.tolist())) == len(kids)             # siblings distinct
        assert (t == top[0, c + 1]).sum() <= 1
    hits = sum(int(tok[0, k] == top[0, par[0, k] + 1]) for k in range(cfg.n_tree))
    assert 5 <= hits <= 40


def test_sample_inputs():
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=2000, n_tree=12, depth=3)
    par = tree_for_config(cfg)
    a = accept_inputs(cfg, par)
    q = a["draft_probs"]
    assert q.dtype == np.float32 and q.shape == (1, 12, 2000)
    np.testing.assert_allclose(q.sum(axis=2, dtype=np.float64), 1.0, atol=1e-5)
    assert (q[0, np.arange(12), a["tokens"][0]] > 0).all()
    u = a["uniforms"]
    assert u.shape == (1, 13) and (u >= 0).all() and (u < 1).all()


def test_chain_and_static_trees():
    from workloads import chain_tree, static_tree, tree_depths
    c = chain_tree(5)
    assert c.tolist() == [-1, 0, 1, 2, 3]
    t = static_tree()
    assert len(t) == 28 and all(-1 <= p < i for i, p in enumerate(t)) and tree_depths(t).max() == 5
    # children of one parent are consecutive (BFS) and the first child of every node has the most children
    kids = {}
    for i, p in enumerate(t):
        kids.setdefault(int(p), []).append(i)
    assert len(kids[-1]) == 4 and [len(kids.get(k, [])) for k in kids[-1]] == [3, 2, 1, 0]
    for name, T in (("c6_chain_sps", 5), ("c7_static_tree", 28)):
        par = tree_for_config(CONFIGS[name])
        assert par.shape == (CONFIGS[name].batch, T) and (par == par[0]).all()
