"""GPU parity: jk_commit_path (through the C ABI) against the oracle, bit for bit (a copy), and a
two-round decode in which the committed cache feeds the next verification."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import accept_path as oracle_accept, commit_path as oracle_commit, tree_verify_attention as oracle_attention
from workloads import CONFIGS, accept_inputs, attention_inputs, round_to_bf16, tree_for_config

pytestmark = pytest.mark.gpu


def _dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def _run(x, path, alen, plen, dtype, advance=True, cache_view=None):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    kt, vt = _dev(x["k_tree"], tdt), _dev(x["v_tree"], tdt)
    kc, vc = _dev(x["k_cache"], tdt), _dev(x["v_cache"], tdt)
    if cache_view is not None:
        kc, vc = cache_view(kc), cache_view(vc)
    p = torch.from_numpy(np.ascontiguousarray(path, dtype=np.int32)).cuda()
    al = torch.tensor(list(alen), dtype=torch.int32).cuda()
    pl = torch.tensor(list(plen), dtype=torch.int32).cuda()
    jk.commit_path(kt, vt, kc, vc, p, al, pl, advance=advance)
    torch.cuda.synchronize()
    return kc.float().cpu().numpy(), vc.float().cpu().numpy(), pl.cpu().numpy()


def _random_paths(rng, B, T, depth):
    path = np.full((B, depth), -1, dtype=np.int32)
    alen = []
    for b in range(B):
        n = int(rng.integers(0, depth + 1))
        path[b, :n] = rng.choice(T, size=n, replace=False)
        alen.append(n)
    return path, alen


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("name", ["c1_tiny", "c3_llama3_8b"])
def test_commit_matches_oracle_bitwise(name, dtype):
    cfg = CONFIGS[name].with_(batch=3, prefix_len=200)
    rng = np.random.default_rng(5)
    x = attention_inputs(cfg)
    if dtype == "bf16":
        x = {k: round_to_bf16(v) for k, v in x.items()}
    path, alen = _random_paths(rng, cfg.batch, cfg.n_tree, cfg.depth)
    alen[0] = cfg.depth  # a full-depth path
    path[0] = rng.choice(cfg.n_tree, size=cfg.depth, replace=False)
    plen = [200 - cfg.depth, 17, 0]
    rk, rv, rl = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, alen, plen)
    gk, gv, gl = _run(x, path, alen, plen, dtype)
    np.testing.assert_array_equal(gk, rk.astype(np.float32))
    np.testing.assert_array_equal(gv, rv.astype(np.float32))
    np.testing.assert_array_equal(gl, rl)


def test_commit_edge_cases_and_no_advance():
    cfg = CONFIGS["c2_vicuna7b"].with_(batch=4, prefix_len=64, n_q_heads=4, n_kv_heads=4)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg).items()}
    path = np.array([[3, 9, 11, -1, -1, -1], [5, 60, 7, 8, -1, -1], [1, 2, 3, 4, 5, 6], [0, -1, -1, -1, -1, -1]],
                    dtype=np.int32)
    alen = [-1, 4, 6, 0]        # gave up; node 60 does not exist (T = 60); runs into the end; nothing accepted
    plen = [10, 20, 61, 64]     # capacity 64
    for adv in (True, False):
        rk, rv, rl = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, alen, plen, advance=adv)
        gk, gv, gl = _run(x, path, alen, plen, "bf16", advance=adv)
        np.testing.assert_array_equal(gk, rk.astype(np.float32))
        np.testing.assert_array_equal(gv, rv.astype(np.float32))
        np.testing.assert_array_equal(gl, rl)
    assert list(rl) == [10, 20, 61, 64] and list(oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"],
                                                               path, alen, plen)[2]) == [10, 21, 64, 64]


def test_commit_into_strided_cache():
    """Head-major cache [B, Hkv, Lcap, D] viewed as [B, Lcap, Hkv, D]."""
    cfg = CONFIGS["c2_vicuna7b"].with_(batch=2, prefix_len=96, n_q_heads=8, n_kv_heads=8)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg).items()}
    rng = np.random.default_rng(11)
    path, alen = _random_paths(rng, 2, cfg.n_tree, cfg.depth)
    alen[1] = max(alen[1], 3)
    path[1, :3] = [4, 8, 15]
    plen = [40, 90]
    view = lambda t: t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)  # noqa: E731
    rk, rv, rl = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, alen, plen)
    gk, gv, gl = _run(x, path, alen, plen, "bf16", cache_view=view)
    np.testing.assert_array_equal(gk, rk.astype(np.float32))
    np.testing.assert_array_equal(gv, rv.astype(np.float32))
    np.testing.assert_array_equal(gl, rl)


def test_two_rounds_on_device():
    """verify -> accept (greedy) -> commit -> verify again, all through the library with lengths and
    paths staying on the device, against the same pipeline of oracles."""
    cfg = CONFIGS["c2_vicuna7b"].with_(batch=2, prefix_len=300, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    acc = accept_inputs(cfg, par)
    x1 = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=1, scale_mult=np.sqrt(128.0)).items()}
    x2 = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=2, scale_mult=np.sqrt(128.0)).items()}
    bf = torch.bfloat16
    plen0 = [280, 151]
    # ---- device pipeline
    kc, vc = _dev(x1["k_cache"], bf), _dev(x1["v_cache"], bf)
    parent = torch.from_numpy(par).cuda()
    pl = torch.tensor(plen0, dtype=torch.int32).cuda()
    out1 = jk.tree_verify_attention(_dev(x1["q"], bf), kc, vc, _dev(x1["k_tree"], bf), _dev(x1["v_tree"], bf), parent, pl)
    path, alen, bonus = jk.accept_path(torch.from_numpy(acc["tokens"]).cuda(), parent, torch.from_numpy(acc["logits"]).cuda(),
                                       mode=jk.JK_GREEDY, max_depth=cfg.depth)
    jk.commit_path(_dev(x1["k_tree"], bf), _dev(x1["v_tree"], bf), kc, vc, path, alen, pl)
    out2 = jk.tree_verify_attention(_dev(x2["q"], bf), kc, vc, _dev(x2["k_tree"], bf), _dev(x2["v_tree"], bf), parent, pl,
                                    max_prefix_len=cfg.prefix_len)
    torch.cuda.synchronize()
    # ---- oracle pipeline
    ref1 = oracle_attention(**x1, parent=par, prefix_len=plen0)
    rp, rl = [], []
    for b in range(cfg.batch):
        r = oracle_accept(acc["tokens"][b], par[b], acc["logits"][b], "greedy")
        rp.append((list(r.path) + [-1] * cfg.depth)[:cfg.depth])
        rl.append(min(r.accept_len, cfg.depth))
    rk, rv, new_len = oracle_commit(x1["k_cache"], x1["v_cache"], x1["k_tree"], x1["v_tree"], np.array(rp), rl, plen0)
    ref2 = oracle_attention(q=x2["q"], k_cache=rk, v_cache=rv, k_tree=x2["k_tree"], v_tree=x2["v_tree"], parent=par,
                            prefix_len=list(new_len))
    assert max(rl) >= 1
    np.testing.assert_array_equal(path.cpu().numpy(), np.array(rp))
    np.testing.assert_array_equal(pl.cpu().numpy(), new_len)
    assert np.abs(out1.float().cpu().numpy() - ref1).max() <= 2e-2
    assert np.abs(out2.float().cpu().numpy() - ref2).max() <= 2e-2


def test_commit_all_layers_in_one_call():
    """jk_commit_path_layers over 5 layers == the oracle applied to each layer; the length advances once."""
    cfg = CONFIGS["c2_vicuna7b"].with_(batch=2, prefix_len=128, n_q_heads=4, n_kv_heads=4)
    rng = np.random.default_rng(2)
    xs = [{k: round_to_bf16(v) for k, v in attention_inputs(cfg, layer=l).items()} for l in range(5)]
    path, alen = _random_paths(rng, cfg.batch, cfg.n_tree, cfg.depth)
    alen[0] = max(alen[0], 2)
    path[0, :2] = [7, 30]
    plen = [100, 125]
    bf = torch.bfloat16
    kts, vts = [_dev(x["k_tree"], bf) for x in xs], [_dev(x["v_tree"], bf) for x in xs]
    kcs, vcs = [_dev(x["k_cache"], bf) for x in xs], [_dev(x["v_cache"], bf) for x in xs]
    p = torch.from_numpy(path).cuda()
    al = torch.tensor(alen, dtype=torch.int32).cuda()
    pl = torch.tensor(plen, dtype=torch.int32).cuda()
    call = jk.prepare_commit_path_layers(kts, vts, kcs, vcs, p, al, pl, advance=True)
    call.launch()
    torch.cuda.synchronize()
    for l, x in enumerate(xs):
        rk, rv, rl = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, alen, plen)
        np.testing.assert_array_equal(kcs[l].float().cpu().numpy(), rk.astype(np.float32))
        np.testing.assert_array_equal(vcs[l].float().cpu().numpy(), rv.astype(np.float32))
    np.testing.assert_array_equal(pl.cpu().numpy(), rl)


@pytest.mark.parametrize("name", ["c6_chain_sps", "c7_static_tree"])
def test_chain_and_static_tree_rounds(name):
    """The second workload family (a chain of gamma draft tokens; a predefined static tree) through
    the same three calls, ragged prefix lengths in the batch, against the oracles."""
    cfg = CONFIGS[name].with_(batch=3, prefix_len=700, n_q_heads=8, n_kv_heads=4, vocab=3000)
    par = tree_for_config(cfg)
    acc = accept_inputs(cfg, par)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, scale_mult=np.sqrt(128.0)).items()}
    bf = torch.bfloat16
    plen0 = [690, 333, 5]
    kc, vc = _dev(x["k_cache"], bf), _dev(x["v_cache"], bf)
    kt, vt = _dev(x["k_tree"], bf), _dev(x["v_tree"], bf)
    parent = torch.from_numpy(par).cuda()
    pl = torch.tensor(plen0, dtype=torch.int32).cuda()
    out = jk.tree_verify_attention(_dev(x["q"], bf), kc, vc, kt, vt, parent, pl)
    sample = cfg.mode == "sample"
    path, alen, bonus = jk.accept_path(
        torch.from_numpy(acc["tokens"]).cuda(), parent, torch.from_numpy(acc["logits"]).cuda(),
        mode=jk.JK_SAMPLE if sample else jk.JK_GREEDY,
        draft_probs=torch.from_numpy(acc["draft_probs"]).cuda() if sample else None,
        uniforms=torch.from_numpy(acc["uniforms"]).cuda() if sample else None, max_depth=cfg.depth)
    jk.commit_path(kt, vt, kc, vc, path, alen, pl)
    torch.cuda.synchronize()
    ref = oracle_attention(**x, parent=par, prefix_len=plen0)
    assert np.abs(out.float().cpu().numpy() - ref).max() <= 2e-2
    rp, rl = [], []
    for b in range(cfg.batch):
        r = oracle_accept(acc["tokens"][b], par[b], acc["logits"][b], cfg.mode,
                          draft_probs=acc["draft_probs"][b] if sample else None,
                          uniforms=acc["uniforms"][b] if sample else None)
        assert r.min_margin is None or r.min_margin > 1e-9
        rp.append((list(r.path) + [-1] * cfg.depth)[:cfg.depth])
        rl.append(min(r.accept_len, cfg.depth))
        assert int(bonus[b]) == r.bonus_token
    np.testing.assert_array_equal(path.cpu().numpy(), np.array(rp))
    rk, rv, new_len = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], np.array(rp), rl, plen0)
    np.testing.assert_array_equal(kc.float().cpu().numpy(), rk.astype(np.float32))
    np.testing.assert_array_equal(vc.float().cpu().numpy(), rv.astype(np.float32))
    np.testing.assert_array_equal(pl.cpu().numpy(), new_len)


def test_commit_argument_errors():
    cfg = CONFIGS["c1_tiny"]
    x = attention_inputs(cfg)
    f = torch.float32
    kt, vt, kc, vc = (_dev(x[k], f) for k in ("k_tree", "v_tree", "k_cache", "v_cache"))
    path = torch.zeros((1, 3), dtype=torch.int32).cuda()
    one = torch.ones((1,), dtype=torch.int32).cuda()
    with pytest.raises(ValueError):
        jk.commit_path(kt, vt, kc, vc.transpose(1, 2), path, one, one)        # K and V strides differ
    with pytest.raises(jk.JakiroError):
        jk.commit_path(kt[..., 1:], vt[..., 1:], kc[..., 1:], vc[..., 1:], path, one, one)  # rows are not whole 16-byte chunks
