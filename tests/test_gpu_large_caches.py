"""GPU parity where the KV cache lies beyond the reach of 32-bit byte offsets: page pools and cache views of
more than 4 GiB, as a GPU with 288 GB holds them.  The data are those of small cases (the oracle sees them as
contiguous caches); only the addresses are far apart.  Attention must equal the compact call bit for bit,
the commit must write the same rows."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from gpu_util import tune
from oracle import commit_path as oracle_commit, tree_verify_attention as oracle_attention
from workloads import CONFIGS, attention_inputs, paged_layout, round_to_bf16, tree_for_config

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def _dev(a, dtype=BF):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def _bits(t):
    return t.contiguous().view(torch.int16)


@pytest.mark.parametrize("wm,wn,splits", [(4, 1, 3), (2, 2, 1)], ids=["4x1_3splits", "2x2_unsplit"])
def test_paged_pools_beyond_4_gib(wm, wn, splits):
    tune("attn_wm", wm); tune("attn_wn", wn); tune("attn_splits", splits)
    cfg = CONFIGS["c3_llama3_8b"].with_(batch=2, prefix_len=1000, n_q_heads=8, n_kv_heads=2)
    page, L = 128, 1000
    par = tree_for_config(cfg, seed=21)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=21, prefix_len=L, scale_mult=np.sqrt(128.0)).items()}
    (kp, vp), table = paged_layout(x["k_cache"], x["v_cache"], page, seed=21)
    n_small = kp.shape[0]
    page_bytes = page * cfg.n_kv_heads * cfg.head_dim * 2
    n_big = 70000                                       # 70 000 pages of 64 KiB: 4.6 GB per pool
    assert n_big * page_bytes > 2 ** 32 + 2 ** 28
    # small page i moves to the far end (even i) or stays near the start (odd i) of the big pool
    where = np.array([n_big - 1 - 531 * i if i % 2 == 0 else 17 + 3 * i for i in range(n_small)], dtype=np.int64)
    assert len(set(where.tolist())) == n_small and where.min() >= 0 and (where * page_bytes).max() > 2 ** 32
    big_table = where[table].astype(np.int32)
    kp_d, vp_d = _dev(kp), _dev(vp)
    kbig = torch.empty((n_big, page, cfg.n_kv_heads, cfg.head_dim), dtype=BF, device="cuda")
    vbig = torch.empty_like(kbig)
    idx = torch.from_numpy(where).cuda()
    kbig[idx] = kp_d
    vbig[idx] = vp_d
    plen = [L, 333]
    parent = torch.from_numpy(par).cuda()
    pl = torch.tensor(plen, dtype=torch.int32).cuda()
    q, kt, vt = _dev(x["q"]), _dev(x["k_tree"]), _dev(x["v_tree"])
    ws = torch.zeros(jk.tree_verify_attention_workspace(q, _dev(x["k_cache"]), kt, L), dtype=torch.uint8, device="cuda")
    far = jk.tree_verify_attention_paged(q, kbig, vbig, torch.from_numpy(big_table).cuda(), kt, vt, parent, pl,
                                         max_prefix_len=L, workspace=ws)
    near = jk.tree_verify_attention_paged(q, kp_d, vp_d, torch.from_numpy(table).cuda(), kt, vt, parent, pl, max_prefix_len=L)
    torch.cuda.synchronize()
    assert jk.last_device_error(ws) == 0
    assert torch.equal(far, near)
    ref = oracle_attention(**x, parent=par, prefix_len=plen)
    assert np.abs(far.float().cpu().numpy() - ref).max() <= 2e-2

    # commit of an accepted path into the far pages: the same rows as into the small pool, which the oracle checks
    path = np.full((2, cfg.depth), -1, dtype=np.int32)
    path[0, :3] = [1, 8, 30]
    path[1, :2] = [0, 5]
    alen, plen_c = [3, 2], [900, 382]                    # sequence 1 crosses a page boundary (384)
    p = torch.from_numpy(path).cuda()
    al = torch.tensor(alen, dtype=torch.int32).cuda()
    pl_far = torch.tensor(plen_c, dtype=torch.int32).cuda()
    pl_near = pl_far.clone()
    jk.prepare_commit_path_layers_paged([kt], [vt], [kbig], [vbig], torch.from_numpy(big_table).cuda(), p, al, pl_far).launch()
    jk.prepare_commit_path_layers_paged([kt], [vt], [kp_d], [vp_d], torch.from_numpy(table).cuda(), p, al, pl_near).launch()
    torch.cuda.synchronize()
    assert torch.equal(pl_far, pl_near)
    assert torch.equal(_bits(kbig[idx]), _bits(kp_d)) and torch.equal(_bits(vbig[idx]), _bits(vp_d))
    rk, rv, rl = oracle_commit(x["k_cache"], x["v_cache"], x["k_tree"], x["v_tree"], path, alen, plen_c)
    np.testing.assert_array_equal(pl_far.cpu().numpy(), rl)
    for b in range(2):
        for t in range(plen_c[b], plen_c[b] + alen[b]):
            got = kbig[int(big_table[b, t // page]), t % page].float().cpu().numpy()
            np.testing.assert_array_equal(got, rk[b, t].astype(np.float32))


def test_cache_views_with_a_batch_stride_beyond_4_gib():
    """Contiguous-call caches as views into one large allocation: sequence 1 starts 4.6 GB behind sequence 0."""
    cfg = CONFIGS["c3_llama3_8b"].with_(batch=2, prefix_len=700, n_q_heads=8, n_kv_heads=2)
    L = 700
    par = tree_for_config(cfg, seed=22)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=22, prefix_len=L, scale_mult=np.sqrt(128.0)).items()}
    row = cfg.n_kv_heads * cfg.head_dim
    cap = L + 8                                          # room for a commit behind the prefix
    sb = 2_300_000_256                                   # elements between the sequences: 4.6 GB
    assert sb * 2 > 2 ** 32 and sb % 256 == 0
    flat_k = torch.empty(sb + cap * row, dtype=BF, device="cuda")
    flat_v = torch.empty_like(flat_k)
    kview = flat_k.as_strided((2, cap, cfg.n_kv_heads, cfg.head_dim), (sb, row, cfg.head_dim, 1))
    vview = flat_v.as_strided((2, cap, cfg.n_kv_heads, cfg.head_dim), (sb, row, cfg.head_dim, 1))
    kc = torch.zeros((2, cap, cfg.n_kv_heads, cfg.head_dim), dtype=BF, device="cuda")
    vc = torch.zeros_like(kc)
    kc[:, :L] = _dev(x["k_cache"]); vc[:, :L] = _dev(x["v_cache"])
    kview.copy_(kc); vview.copy_(vc)
    plen = [L, 251]
    parent = torch.from_numpy(par).cuda()
    pl = torch.tensor(plen, dtype=torch.int32).cuda()
    q, kt, vt = _dev(x["q"]), _dev(x["k_tree"]), _dev(x["v_tree"])
    for splits in (1, 4):
        tune("attn_splits", splits)
        far = jk.tree_verify_attention(q, kview, vview, kt, vt, parent, pl, max_prefix_len=L)
        near = jk.tree_verify_attention(q, kc, vc, kt, vt, parent, pl, max_prefix_len=L)
        torch.cuda.synchronize()
        assert torch.equal(far, near)
    ref = oracle_attention(**x, parent=par, prefix_len=plen)
    assert np.abs(far.float().cpu().numpy() - ref).max() <= 2e-2
    path = np.full((2, cfg.depth), -1, dtype=np.int32)
    path[0, :2] = [2, 9]
    path[1, :4] = [0, 3, 11, 40]
    p = torch.from_numpy(path).cuda()
    al = torch.tensor([2, 4], dtype=torch.int32).cuda()
    pl_far, pl_near = pl.clone(), pl.clone()
    jk.commit_path(kt, vt, kview, vview, p, al, pl_far)
    jk.commit_path(kt, vt, kc, vc, p, al, pl_near)
    torch.cuda.synchronize()
    assert torch.equal(pl_far, pl_near) and pl_far.tolist() == [L + 2, 255]
    assert torch.equal(_bits(kview), _bits(kc)) and torch.equal(_bits(vview), _bits(vc))


@pytest.mark.parametrize("fused", [-1, 0], ids=["planned", "merge_kernel"])
def test_bf16_million_token_prefix(fused):
    """One sequence with a prefix of 2^20 + 17 tokens (a ragged last tile, more tiles than one split may hold, so the
    plan must split at least 33 ways), every element against the oracle; then the same call with a device-side
    length 70 001 tokens short of the bound (the first transfers were asked for on the bound: everything is redone)."""
    tune("attn_fused", fused)
    L = (1 << 20) + 17
    cfg = CONFIGS["c3_llama3_8b"].with_(batch=1, prefix_len=L, n_q_heads=2, n_kv_heads=1, n_tree=40)
    par = tree_for_config(cfg, seed=23)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=23, prefix_len=L, scale_mult=np.sqrt(128.0)).items()}
    # a few keys that single rows care about, so that outputs are not all averages over a million values
    for i, (t, h, pos) in enumerate([(0, 0, 5), (7, 1, L - 1), (20, 0, 777777), (39, 1, 1 << 19)]):
        x["k_cache"][0, pos, 0] = round_to_bf16(6.0 * x["q"][0, t, h])
    parent = torch.from_numpy(par).cuda()
    d = {k: _dev(v) for k, v in x.items()}
    plan = jk.tree_verify_attention_plan(d["q"], d["k_cache"], d["k_tree"], L)
    assert plan["splits"] >= 33
    for plen in ([L], [L - 70001]):
        pl = torch.tensor(plen, dtype=torch.int32).cuda()
        got = jk.tree_verify_attention(d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent, pl, max_prefix_len=L)
        torch.cuda.synchronize()
        ref = oracle_attention(**x, parent=par, prefix_len=plen)
        err = np.abs(got.float().cpu().numpy() - ref)
        assert np.isfinite(err).all()
        assert err.max() <= 2e-2 and err.max() <= 1.5e-2 * np.abs(ref).max(), (plen, err.max(), np.abs(ref).max())


@pytest.mark.parametrize("splits,fused", [(0, -1), (3, 1), (1, -1)], ids=["planned", "3_splits", "unsplit"])
def test_bf16_many_sequences_and_heads(splits, fused):
    """768 (sequence, KV head) units with ragged prefix lengths from 0 to the bound: more row-tile groups than the
    merge inside the kernel has synchronisation words for, so split calls take the merge kernel whatever is asked
    for; every element against the oracle."""
    from gpu_util import check_attention
    tune("attn_splits", splits); tune("attn_fused", fused)
    B, Hkv, G, D, T, L = 48, 16, 2, 64, 40, 300
    cfg = CONFIGS["c3_llama3_8b"].with_(batch=B, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D, prefix_len=L, n_tree=T)
    par = tree_for_config(cfg, seed=31)
    x = attention_inputs(cfg, seed=31, scale_mult=np.sqrt(float(D)))
    rng = np.random.default_rng(31)
    lens = [int(v) for v in rng.integers(0, L + 1, size=B)]
    lens[0], lens[1], lens[-1] = L, 0, L
    if splits:
        d = {k: _dev(v) for k, v in x.items()}
        assert jk.tree_verify_attention_plan(d["q"], d["k_cache"], d["k_tree"], L)["fused"] == 0
    check_attention(x, par, lens, "bf16", 2e-2, rel_tol=1.5e-2)


@pytest.mark.parametrize("wm,wn", [(4, 1), (2, 2)], ids=["4x1", "2x2"])
def test_paged_long_prefix_of_small_pages(wm, wn):
    """70 013 tokens in pages of 32: 2188 pages for the one sequence, more than a workgroup keeps page ids for
    (1024), so the plan has to split at least three ways.  Bitwise equal to the contiguous call, and against the
    oracle."""
    tune("attn_wm", wm); tune("attn_wn", wn)
    L, page = 70013, 32
    cfg = CONFIGS["c3_llama3_8b"].with_(batch=1, prefix_len=L, n_q_heads=2, n_kv_heads=1, n_tree=20)
    par = tree_for_config(cfg, seed=41)
    x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=41, prefix_len=L, scale_mult=np.sqrt(128.0)).items()}
    x["k_cache"][0, 69999, 0] = round_to_bf16(6.0 * x["q"][0, 3, 1])
    (kp, vp), table = paged_layout(x["k_cache"], x["v_cache"], page, seed=41)
    assert table.shape[1] == 2188
    parent = torch.from_numpy(par).cuda()
    pl = torch.tensor([L], dtype=torch.int32).cuda()
    q, kt, vt = _dev(x["q"]), _dev(x["k_tree"]), _dev(x["v_tree"])
    kc, vc = _dev(x["k_cache"]), _dev(x["v_cache"])
    assert jk.tree_verify_attention_plan(q, kc, kt, L)["splits"] >= 3
    got = jk.tree_verify_attention_paged(q, _dev(kp), _dev(vp), torch.from_numpy(table).cuda(), kt, vt, parent, pl, max_prefix_len=L)
    cont = jk.tree_verify_attention(q, kc, vc, kt, vt, parent, pl, max_prefix_len=L)
    torch.cuda.synchronize()
    assert torch.equal(got, cont)
    ref = oracle_attention(**x, parent=par, prefix_len=[L])
    err = np.abs(got.float().cpu().numpy() - ref).max()
    assert err <= 2e-2 and err <= 1.5e-2 * np.abs(ref).max()
