"""GPU parity: jk_tree_verify_attention (through the C ABI) against the fp64 oracle,
element by element on the same seeded inputs.  Tolerances: 2e-2 max-abs for bf16
inputs, 1e-5 for fp32 inputs; bf16 cases with O(1) outputs also bound the error
relative to max|out| (bf16 output rounding, unit roundoff 2^-8, plus bf16 softmax weights)."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, attention_inputs, coin_tree, round_to_bf16, tree_for_config, two_expert_tree

pytestmark = pytest.mark.gpu

from gpu_util import check_attention, gpu_attention, oracle_attention, reset_tuning, tune  # noqa: E402

BF16_TOL, F32_TOL = 2e-2, 1e-5


def _cfg(base, **kw):
    return CONFIGS[base].with_(**kw)


def test_c1_tiny_fp32():
    cfg = CONFIGS["c1_tiny"]
    par = tree_for_config(cfg)
    check_attention(attention_inputs(cfg), par, [cfg.prefix_len], "f32", F32_TOL)


@pytest.mark.parametrize("L", [0, 1, 7, 128, 1000, 1025, 2500])
def test_fp32_prefix_lengths(L):
    cfg = _cfg("c1_tiny", prefix_len=L, n_q_heads=4, n_kv_heads=2)
    par = tree_for_config(cfg, seed=L)
    check_attention(attention_inputs(cfg, seed=L), par, [L], "f32", F32_TOL)


def test_fp32_batched_ragged_and_wide_tree():
    cfg = _cfg("c5_llama2_70b", batch=3, n_q_heads=4, n_kv_heads=2, head_dim=32, prefix_len=300, dtype="f32",
               input_scale=1.0)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg)
    check_attention(x, par, [300, 17, 0], "f32", F32_TOL)


# (name, Hq, Hkv, D, L, T-config, unscaled?)
BF16_CASES = [
    ("mha_small", 4, 4, 128, 100, "c2_vicuna7b", True),
    ("mha_ragged", 2, 2, 128, 1021, "c2_vicuna7b", True),
    ("gqa2", 4, 2, 128, 333, "c2_vicuna7b", True),
    ("gqa4", 8, 2, 128, 515, "c3_llama3_8b", True),
    ("gqa8_t100", 8, 1, 128, 700, "c5_llama2_70b", True),
    ("d64_mha", 4, 4, 64, 257, "c2_vicuna7b", True),
    ("d64_gqa4", 8, 2, 64, 96, "c2_vicuna7b", True),
    ("scaled_inputs", 8, 2, 128, 515, "c3_llama3_8b", False),
]


@pytest.mark.parametrize("name,Hq,Hkv,D,L,base,unscaled", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_bf16_shapes(name, Hq, Hkv, D, L, base, unscaled):
    cfg = _cfg(base, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, prefix_len=L)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=(np.sqrt(128.0) if unscaled else 1.0))
    check_attention(x, par, [L, max(0, L - 3)], "bf16", BF16_TOL, rel_tol=1.5e-2)


@pytest.mark.parametrize("L", [0, 1, 7, 31, 32, 33])
def test_bf16_tiny_prefixes_tree_dominates(L):
    cfg = _cfg("c3_llama3_8b", prefix_len=L, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg, seed=10 + L)
    x = attention_inputs(cfg, seed=10 + L, scale_mult=np.sqrt(128.0))
    check_attention(x, par, [L], "bf16", BF16_TOL, rel_tol=1.5e-2)


@pytest.mark.parametrize("T", [1, 2, 31, 32, 33, 64, 65, 127, 128])
def test_bf16_tree_sizes(T):
    rng = np.random.default_rng(T)
    # random topological tree of T nodes, bushy near the root
    par = np.array([-1] + [int(rng.integers(-1, i)) for i in range(1, T)], dtype=np.int32)[None]
    cfg = _cfg("c3_llama3_8b", n_tree=T, prefix_len=70, n_q_heads=4, n_kv_heads=2)
    x = attention_inputs(cfg, seed=T, scale_mult=np.sqrt(128.0))
    check_attention(x, par, [70], "bf16", BF16_TOL, rel_tol=1.5e-2)


def test_bf16_chain_and_star_trees():
    cfg = _cfg("c3_llama3_8b", n_tree=40, prefix_len=50, n_q_heads=4, n_kv_heads=2, batch=2)
    par = np.stack([np.arange(-1, 39), np.full(40, -1)]).astype(np.int32)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    check_attention(x, par, [50, 50], "bf16", BF16_TOL, rel_tol=1.5e-2)


def test_bf16_peaked_softmax():
    # Q x8: softmax nearly one-hot, exercises the running-max rescale
    cfg = _cfg("c3_llama3_8b", prefix_len=600, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    x["q"] = round_to_bf16(x["q"] * 8.0)
    # near one-hot rows return single V rows (entries up to about 4.5): three bf16 roundings on the way
    # (probability, split partial, result; unit roundoff 2^-8 each) allow 3 * 2^-8 * 4.5 = 5.3e-2 absolute
    vmax = float(max(np.abs(x["v_cache"]).max(), np.abs(x["v_tree"]).max()))
    assert 4.0 < vmax < 5.5
    got, ref = check_attention(x, par, [600], "bf16", 3 * 2.0 ** -8 * vmax, rel_tol=2e-2)
    # The split partial's rounding is one of the three and is this library's own: with one split it is gone, and
    # the bound is two roundings (probability, result).  The measured worst cases are printed.
    tune("attn_splits", 1)
    got1, _ = check_attention(x, par, [600], "bf16", 2 * 2.0 ** -8 * vmax, rel_tol=2e-2)
    print(f"near one-hot rows: worst error {np.abs(got - ref).max():.4f} split, {np.abs(got1 - ref).max():.4f} unsplit, "
          f"bounds {3 * 2.0 ** -8 * vmax:.4f} / {2 * 2.0 ** -8 * vmax:.4f}")


@pytest.mark.parametrize("where", [40, 1500, 2999])
@pytest.mark.parametrize("splits", ["1", "3", ""])
def test_bf16_outlier_key_far_above_everything_before_it(monkeypatch, where, splits):
    """One key whose score for one query row lies about 130 binary orders of magnitude above the
    rest (a multiple of that row's own query vector).  The two-tile fast path of the 4x1 arrangement
    keeps a fixed reference per row and cannot hold such a jump when the key comes late: the
    workgroup has to notice and repeat its split on the general path.  Early (first tile), in the
    middle and in the last full tile of the prefix; one split, three, and the planner's choice."""
    if splits:
        tune("attn_splits", splits)
    tune("attn_wm", "4")
    tune("attn_wn", "1")
    cfg = _cfg("c3_llama3_8b", prefix_len=3008, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, seed=where, scale_mult=np.sqrt(128.0))
    node, head = 7, 5                                   # query row of KV head 1
    x["k_cache"][0, where, 1] = round_to_bf16(8.0 * x["q"][0, node, head])
    # (rows with a near one-hot softmax return single V rows, entries up to about 4.5: the bf16 roundings
    # of the probability, the split partial and the result, unit roundoff 2^-8 each, exceed the absolute
    # bound of the averaged rows, so the absolute bound here is 3 * 2^-8 of that magnitude = 5.3e-2;
    # the relative bound stays)
    got, ref = check_attention(x, par, [3008], "bf16", 3 * 2.0 ** -8 * 4.5, rel_tol=1.5e-2)
    # that row's softmax is one-hot on the planted key
    v = x["v_cache"][0, where, 1].astype(np.float64)
    assert np.abs(got[0, node, head] - v).max() <= 2.0 ** -7 * np.abs(v).max() + 1e-6


def test_bf16_outlier_key_head_dim_64(monkeypatch):
    """The same repeat on the general path with 64-wide heads (half as many MFMAs per phase)."""
    tune("attn_wm", "4")
    tune("attn_wn", "1")
    cfg = _cfg("c3_llama3_8b", prefix_len=1100, n_q_heads=8, n_kv_heads=2, head_dim=64)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, seed=5, scale_mult=np.sqrt(64.0))
    node, head = 3, 1
    x["k_cache"][0, 900, 0] = round_to_bf16(12.0 * x["q"][0, node, head])
    got, ref = check_attention(x, par, [1100], "bf16", 3 * 2.0 ** -8 * 4.5, rel_tol=1.5e-2)
    v = x["v_cache"][0, 900, 0].astype(np.float64)
    assert np.abs(got[0, node, head] - v).max() <= 2.0 ** -7 * np.abs(v).max() + 1e-6


def test_bf16_custom_scale_and_strided_cache():
    import paper_2502_06282_amd as jk
    from oracle import tree_verify_attention as oracle_attention
    cfg = _cfg("c3_llama3_8b", prefix_len=200, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    ref = oracle_attention(**x, parent=par, prefix_len=[150], scale=0.05)
    # cache stored head-major with spare capacity: [B, Hkv, Lcap, D] viewed as [B, Lcap, Hkv, D]
    dev = torch.device("cuda")
    kc = torch.zeros(1, 2, 256, 128, dtype=torch.bfloat16, device=dev)
    vc = torch.zeros_like(kc)
    kc[:, :, :200] = torch.from_numpy(x["k_cache"]).to(dev).to(torch.bfloat16).permute(0, 2, 1, 3)
    vc[:, :, :200] = torch.from_numpy(x["v_cache"]).to(dev).to(torch.bfloat16).permute(0, 2, 1, 3)
    f = lambda n: torch.from_numpy(x[n]).to(dev).to(torch.bfloat16)
    out = jk.tree_verify_attention(f("q"), kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), f("k_tree"), f("v_tree"),
                                   torch.from_numpy(par).to(dev), torch.tensor([150], dtype=torch.int32, device=dev),
                                   scale=0.05)
    torch.cuda.synchronize()
    err = np.abs(out.float().cpu().numpy() - ref).max()
    assert err <= BF16_TOL and err / np.abs(ref).max() <= 1.5e-2


@pytest.mark.parametrize("big", [False, True], ids=["tree60_planned", "tree128_three_splits"])
def test_bf16_sibling_independence_bitwise(big):
    """Nodes outside a query's ancestor set cannot change its output: their K rows
    may hold anything (NaN), their V rows anything finite (a reading of this library: a masked score is
    -inf before the softmax, so its weight is an exact zero, and 0 x finite = 0 in the value product);
    results stay bit-identical.  Also with the largest tree (four tree tiles) over three key splits."""
    if big:
        tune("attn_wm", 4); tune("attn_wn", 1); tune("attn_splits", 3)
        rng = np.random.default_rng(128)
        par = np.array([-1] + [int(rng.integers(max(-1, i - 9), i)) for i in range(1, 128)], dtype=np.int32)[None]
        cfg = _cfg("c3_llama3_8b", n_tree=128, prefix_len=90, n_q_heads=8, n_kv_heads=2)
    else:
        cfg = _cfg("c3_llama3_8b", prefix_len=90, n_q_heads=8, n_kv_heads=2)
        par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    base = gpu_attention(x, par, [90], "bf16")
    from oracle import ancestor_sets
    anc = ancestor_sets(par[0])
    T = cfg.n_tree
    for i in [T - 1, T // 2, 3] + ([70, 33] if big else []):
        y = {k: v.copy() for k, v in x.items()}
        others = [j for j in range(T) if j not in anc[i]]
        y["k_tree"][0, others] = np.nan
        y["v_tree"][0, others] = 3.0e38
        got = gpu_attention(y, par, [90], "bf16")
        np.testing.assert_array_equal(got[0, i], base[0, i])
    # beyond prefix_len the cache is never read
    y = {k: v.copy() for k, v in x.items()}
    y["k_cache"][0, 60:] = np.nan
    y["v_cache"][0, 60:] = np.nan
    a = gpu_attention(y, par, [60], "bf16")
    z = {k: v.copy() for k, v in x.items()}
    b = gpu_attention(z, par, [60], "bf16")
    np.testing.assert_array_equal(a, b)


def test_bf16_split_invariance(monkeypatch):
    """The number of KV splits changes only fp32 rounding."""
    cfg = _cfg("c3_llama3_8b", prefix_len=2000, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    outs = []
    for s in ("1", "3", "8", "31"):
        tune("attn_splits", s)
        outs.append(gpu_attention(x, par, [2000], "bf16"))
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() <= 2.0 ** -7 * np.abs(outs[0]).max()


@pytest.mark.parametrize("wm,wn", [(2, 2), (4, 1)], ids=["2x2", "4x1"])
@pytest.mark.parametrize("L", [0, 31, 64, 97, 130, 257, 1000])
def test_bf16_wave_arrangements(monkeypatch, wm, wn, L):
    """Both workgroup arrangements (the 4x1 one takes its tiles in hand-pipelined pairs) over prefix
    lengths that leave full pairs, a lone tile, a ragged tile and tree tiles in every position of a
    round, unsplit and with three splits."""
    tune("attn_wm", str(wm))
    tune("attn_wn", str(wn))
    cfg = _cfg("c3_llama3_8b", batch=2, prefix_len=L, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg, seed=L)
    x = attention_inputs(cfg, seed=L, scale_mult=np.sqrt(128.0))
    for s in ("1", "3"):
        tune("attn_splits", s)
        check_attention(x, par, [L, L // 2], "bf16", BF16_TOL, rel_tol=2e-2)


@pytest.mark.parametrize("wm,wn", [(2, 2), (4, 1)], ids=["2x2", "4x1"])
def test_bf16_prefix_shorter_than_bound(monkeypatch, wm, wn):
    """The first K/V transfers go out on the assumption prefix_len == max_prefix_len; here it is
    not, for one sequence by a lot and for the other by one key."""
    tune("attn_wm", str(wm))
    tune("attn_wn", str(wn))
    cfg = _cfg("c3_llama3_8b", batch=2, prefix_len=1500, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    ref = oracle_attention(**x, parent=par, prefix_len=[200, 1499])
    got = gpu_attention(x, par, [200, 1499], "bf16", max_prefix_len=1500)
    assert np.abs(got - ref).max() <= BF16_TOL


def _every_element(cfg, x, par, got):
    """The whole result against the oracle, element by element (the oracle needs well under a second per layer
    at these sizes): absolute bound of the graded metric, and relative to the layer's largest output."""
    ref = oracle_attention(**x, parent=par, prefix_len=[cfg.prefix_len] * cfg.batch)
    err = np.abs(got - ref)
    assert err.max() <= BF16_TOL
    assert err.max() <= 1.5e-2 * np.abs(ref).max(), (err.max(), np.abs(ref).max())
    return float(err.max() / np.abs(ref).max())


@pytest.mark.parametrize("scaled", [True, False], ids=["as_configured", "unit_variance"])
def test_c2_full_size_every_element(scaled):
    """Config 2 (Vicuna-7B shape) at full size: inputs as the config states them (all of Q, K, V times
    1/sqrt(128): outputs near 1e-3, where the 2e-2 bound says little) and at unit variance."""
    cfg = CONFIGS["c2_vicuna7b"]
    par = tree_for_config(cfg)
    x = attention_inputs(cfg) if scaled else attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    got = gpu_attention(x, par, [cfg.prefix_len], "bf16")
    _every_element(cfg, x, par, got)


@pytest.mark.parametrize("scaled", [True, False], ids=["as_configured", "unit_variance"])
@pytest.mark.parametrize("fused", [1, 0], ids=["merged_in_kernel", "merge_kernel"])
def test_c3_full_size_every_element(scaled, fused):
    """Config 3 (the benchmarked one) at full size, every element, in the plan bench.py times and with the
    stand-alone merge kernel."""
    tune("attn_fused", fused)
    cfg = CONFIGS["c3_llama3_8b"]
    par = tree_for_config(cfg)
    x = attention_inputs(cfg) if scaled else attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    got = gpu_attention(x, par, [cfg.prefix_len], "bf16")
    _every_element(cfg, x, par, got)


def _sampled_unit_check(cfg, x, par, got, n_samples, seed):
    """Oracle on sampled (sequence, KV head) units of a full-size result."""
    from oracle import tree_verify_attention as oracle_attention
    rng = np.random.default_rng(seed)
    G = cfg.group
    for _ in range(n_samples):
        b = int(rng.integers(cfg.batch)); kv = int(rng.integers(cfg.n_kv_heads))
        hs = slice(kv * G, kv * G + G)
        sub = {"q": x["q"][b:b + 1, :, hs], "k_cache": x["k_cache"][b:b + 1, :, kv:kv + 1],
               "v_cache": x["v_cache"][b:b + 1, :, kv:kv + 1], "k_tree": x["k_tree"][b:b + 1, :, kv:kv + 1],
               "v_tree": x["v_tree"][b:b + 1, :, kv:kv + 1]}
        ref = oracle_attention(**sub, parent=par[b:b + 1], prefix_len=[cfg.prefix_len])
        err = np.abs(got[b, :, hs] - ref[0]).max()
        assert err <= BF16_TOL and err <= 1.5e-2 * np.abs(ref).max(), (b, kv, err)


@pytest.mark.parametrize("fused", [1, 0])
def test_c3_full_size_graph_replay_as_benchmarked(fused):
    """The launch configuration bench.py times: prepared calls of several full-size c3 layers sharing
    one workspace, captured in a HIP graph and replayed, with eager work between the replays; every
    replay must reproduce the eager result bit for bit, and the result is checked against the oracle
    on sampled KV heads.  Both ways of merging the key splits: inside the attention kernel (the
    workspace's header is zero-filled once and must stay consistent from call to call) and with the
    second kernel; the partials behind the header are filled with noise before every replay."""
    import paper_2502_06282_amd as jk
    tune("attn_fused", fused)
    cfg = CONFIGS["c3_llama3_8b"]
    par = tree_for_config(cfg)
    dev = torch.device("cuda")
    n_layers = 3
    xs = [attention_inputs(cfg, layer=l, scale_mult=np.sqrt(128.0)) for l in range(n_layers)]
    lys = [{k: torch.from_numpy(v).to(dev).to(torch.bfloat16) for k, v in x.items()} for x in xs]
    parent = torch.from_numpy(par).to(dev)
    plen = torch.full((cfg.batch,), cfg.prefix_len, dtype=torch.int32, device=dev)
    outs = [torch.empty_like(l["q"]) for l in lys]
    ws = torch.empty(jk.tree_verify_attention_workspace(lys[0]["q"], lys[0]["k_cache"], lys[0]["k_tree"], cfg.prefix_len),
                     dtype=torch.uint8, device=dev)
    jk.workspace_init(ws)
    calls = [jk.prepare_tree_verify_attention(l["q"], l["k_cache"], l["v_cache"], l["k_tree"], l["v_tree"], parent, plen,
                                              o, ws, max_prefix_len=cfg.prefix_len) for l, o in zip(lys, outs)]
    for c in calls:
        c.launch()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        for c in calls:
            c.launch()
    for rep in range(3):
        for o in outs:
            o.fill_(float("nan"))
        ws[jk.JK_WORKSPACE_HEADER_BYTES:].random_(0, 255)   # stale partials must not matter
        junk = torch.randn(1 << 20, device=dev).sum()   # the program's own eager work between replays
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), f"replay {rep} differs from the eager result"
        assert torch.isfinite(junk)
    for l in (0, n_layers - 1):
        got = outs[l].float().cpu().numpy().astype(np.float64)
        _sampled_unit_check(cfg, xs[l], par, got, 3, 10 + l)
    assert jk.last_device_error(ws) == 0


def _attn_with_ws(x, par, plens, fused, ws=None, max_prefix_len=None):
    """One bf16 call with an explicit workspace; returns (out as float64, workspace, plan)."""
    import paper_2502_06282_amd as jk
    from gpu_util import to_dev
    tune("attn_fused", fused)
    dv = to_dev(x, "bf16")
    parent = torch.from_numpy(np.ascontiguousarray(par, dtype=np.int32)).cuda()
    pl = torch.tensor(list(plens), dtype=torch.int32).cuda()
    L = max_prefix_len if max_prefix_len is not None else dv["k_cache"].shape[1]
    plan = jk.tree_verify_attention_plan(dv["q"], dv["k_cache"], dv["k_tree"], L)
    if ws is None:
        ws = torch.empty(jk.tree_verify_attention_workspace(dv["q"], dv["k_cache"], dv["k_tree"], L), dtype=torch.uint8,
                         device="cuda")
        ws.random_(0, 255)
        jk.workspace_init(ws[: jk.JK_WORKSPACE_HEADER_BYTES])   # only the header needs to start at zero
    out = jk.tree_verify_attention(dv["q"], dv["k_cache"], dv["v_cache"], dv["k_tree"], dv["v_tree"], parent, pl,
                                   max_prefix_len=L, workspace=ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), ws, plan


@pytest.mark.parametrize("name,kw,arr,splits", [
    ("c3_llama3_8b", {}, None, 0),                                            # the benchmarked plan
    ("c3_llama3_8b", {"prefix_len": 1000}, (4, 1), 5),                        # rows per slice do not divide the tile
    ("c3_llama3_8b", {"prefix_len": 4093, "n_tree": 128}, (4, 1), 16),        # ragged prefix, four tree tiles
    ("c2_vicuna7b", {}, None, 0),                                             # 2x2 waves, 60 rows
    ("c2_vicuna7b", {"prefix_len": 777, "n_q_heads": 16, "n_kv_heads": 16}, (2, 2), 7),
    ("c3_llama3_8b", {"head_dim": 64, "prefix_len": 2048}, (4, 1), 8),
    ("c3_llama3_8b", {"batch": 2, "n_q_heads": 16, "n_kv_heads": 4, "prefix_len": 3000}, None, 0),
])
def test_bf16_merge_inside_the_kernel_agrees_with_the_merge_kernel(name, kw, arr, splits):
    """The key splits of a row tile are merged either by a second kernel or, when the grid allows it, by the
    attention kernel's own workgroups meeting in their XCD's L2.  Both merge the same bf16 partials in fp32 (in a
    different order of operations): the bf16 outputs may differ in the last place of an element, no more, and both
    are within tolerance of the oracle."""
    cfg = _cfg(name, **kw)
    if arr:
        tune("attn_wm", arr[0]); tune("attn_wn", arr[1])
    if splits:
        tune("attn_splits", splits)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(float(cfg.head_dim)))
    plens = [cfg.prefix_len] * cfg.batch
    a, ws_a, plan_a = _attn_with_ws(x, par, plens, 1)
    tune("attn_splits", plan_a["splits"])   # (left to itself the plan may cut the keys differently for the second kernel)
    tune("attn_wm", plan_a["wm"]); tune("attn_wn", plan_a["wn"])
    b, ws_b, plan_b = _attn_with_ws(x, par, plens, 0)
    assert plan_a["fused"] == 1 and plan_b["fused"] == 0 and plan_a["splits"] == plan_b["splits"] > 1, (plan_a, plan_b)
    assert np.isfinite(a).all()
    # one bf16 ulp (at most 2^-7 relative), plus the fp32 rounding of the weighted sums where they cancel
    assert (np.abs(a - b) <= 1.01 * 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 1e-6 * np.abs(a).max()).all()
    assert (a != b).mean() < 0.02
    import paper_2502_06282_amd as jk
    assert jk.last_device_error(ws_a) == 0 and jk.last_device_error(ws_b) == 0
    if cfg.prefix_len <= 1000:
        ref = oracle_attention(**x, parent=par, prefix_len=plens)
        assert np.abs(a - ref).max() <= BF16_TOL


def test_bf16_merge_inside_the_kernel_when_the_wait_expires():
    """spin_limit 0: no workgroup waits for its partners.  Every workgroup but a group's last arriver records its
    slice and leaves, the last arriver merges them all: same bits as the normal run, the workspace's error word
    says that waits expired, and the workspace serves the next (normal) call unchanged."""
    import paper_2502_06282_amd as jk
    cfg = _cfg("c3_llama3_8b", prefix_len=2048)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    ref, ws0, plan = _attn_with_ws(x, par, [2048], 1)
    assert plan["fused"] == 1 and jk.last_device_error(ws0) == 0
    tune("spin_limit", 0)
    got, ws, _ = _attn_with_ws(x, par, [2048], 1)
    np.testing.assert_array_equal(got, ref)
    assert jk.last_device_error(ws) & jk.JK_DEVERR_MERGE_WAIT
    # the same workspace, normal waits again: header words were left consistent
    tune("spin_limit", -1)
    for _ in range(3):
        again, _, _ = _attn_with_ws(x, par, [2048], 1, ws=ws)
        np.testing.assert_array_equal(again, ref)
    jk.workspace_init(ws[: jk.JK_WORKSPACE_HEADER_BYTES])
    again, _, _ = _attn_with_ws(x, par, [2048], 1, ws=ws)
    np.testing.assert_array_equal(again, ref)
    assert jk.last_device_error(ws) == 0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_bad_tree_is_repaired_and_reported(dtype):
    """A parent entry outside [-1, i-1] lives in device memory where the host cannot check it: the kernels treat
    the node as a child of the prefix and set JK_DEVERR_BAD_TREE in the workspace; a good tree leaves it clear."""
    import paper_2502_06282_amd as jk
    from gpu_util import to_dev
    cfg = _cfg("c1_tiny") if dtype == "f32" else _cfg("c3_llama3_8b", prefix_len=300, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=1.0 if dtype == "f32" else np.sqrt(128.0))
    bad = par.copy()
    bad[0, 5] = 7          # a parent that comes later
    bad[0, 3] = -4         # and one below -1
    fixed = par.copy()
    fixed[0, 5] = fixed[0, 3] = -1
    dv = to_dev(x, dtype)
    pl = torch.tensor([cfg.prefix_len], dtype=torch.int32).cuda()
    outs, errs = [], []
    for p_ in (bad, fixed):
        ws = torch.zeros(jk.tree_verify_attention_workspace(dv["q"], dv["k_cache"], dv["k_tree"], cfg.prefix_len),
                         dtype=torch.uint8, device="cuda")
        outs.append(jk.tree_verify_attention(dv["q"], dv["k_cache"], dv["v_cache"], dv["k_tree"], dv["v_tree"],
                                             torch.from_numpy(p_).cuda(), pl, workspace=ws))
        torch.cuda.synchronize()
        errs.append(jk.last_device_error(ws))
    assert torch.equal(outs[0], outs[1])
    assert errs == [jk.JK_DEVERR_BAD_TREE, 0]
    assert jk.validate_tree(bad[0]) == 2 and jk.validate_tree(fixed[0]) == 0


def test_c4_full_size_every_element():
    """Config 4 (LLaMA2-13B shape, batch 4 with a tree per sequence), one layer at full size, every element
    (the oracle takes a few seconds for the layer's 160 units)."""
    cfg = CONFIGS["c4_llama2_13b"]
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    got = gpu_attention(x, par, [cfg.prefix_len] * cfg.batch, "bf16")
    _every_element(cfg, x, par, got)


def test_c5_full_size_sampled_units():
    """Config 5 (LLaMA2-70B shape: batch 8, 16384-token prefix, 100-node trees, group 8) at full size."""
    cfg = CONFIGS["c5_llama2_70b"]
    par = tree_for_config(cfg)
    x = attention_inputs(cfg, scale_mult=np.sqrt(128.0))
    got = gpu_attention(x, par, [cfg.prefix_len] * cfg.batch, "bf16")
    assert np.isfinite(got).all()
    _sampled_unit_check(cfg, x, par, got, 6, 5)


def test_argument_errors():
    import paper_2502_06282_amd as jk
    dev = torch.device("cuda")
    q = torch.zeros(1, 4, 2, 128, dtype=torch.bfloat16, device=dev)
    kc = torch.zeros(1, 8, 2, 128, dtype=torch.bfloat16, device=dev)
    kt = torch.zeros(1, 4, 2, 128, dtype=torch.bfloat16, device=dev)
    par = torch.tensor([[-1, 0, 0, 1]], dtype=torch.int32, device=dev)
    pl = torch.tensor([8], dtype=torch.int32, device=dev)
    with pytest.raises(jk.JakiroError) as e:
        jk.tree_verify_attention(q, kc, kc, kt, kt, par, pl, scale=-1.0)
    assert e.value.status in (1, 3)
    ws = torch.empty(256, dtype=torch.uint8, device=dev)
    with pytest.raises(jk.JakiroError) as e:
        jk.tree_verify_attention(q, kc, kc, kt, kt, par, pl, workspace=ws[1:])
    assert e.value.status == 4
    q96 = torch.zeros(1, 4, 2, 96, dtype=torch.bfloat16, device=dev)
    with pytest.raises(jk.JakiroError) as e:
        jk.tree_verify_attention(q96, q96, q96, q96, q96, par, pl)
    assert e.value.status == 3


def _depths(par):
    d = np.zeros(len(par), dtype=np.int64)
    for i, p in enumerate(par):
        d[i] = 0 if p < 0 else d[p] + 1
    return d


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("f32", 32)])
@pytest.mark.parametrize("arr,splits", [((2, 2), 1), ((4, 1), 3), (None, 0)], ids=["2x2_unsplit", "4x1_3splits", "planned"])
def test_closed_forms_without_the_oracle(dtype, D, arr, splits):
    """What the definition fixes whatever computes it (no oracle in this test): equal value rows come back
    unchanged; equal key rows give the mean of the value rows a node sees, prefix_len + depth + 1 of them; a root over
    an empty prefix returns its own value row; and with scale = ln 2 and keys 0, e_0, 2 e_0 against q = e_0 the weights
    are 1 : 2 : 4, so a root over one prefix key gives 2/3 of its value, its child (1 * 0 + 2 * 1 + 4 * 2) / 7 and a
    sibling in the child's place (1 * 0 + 4 * 2) / 5."""
    if arr is not None:
        tune("attn_wm", arr[0]); tune("attn_wn", arr[1])
    tune("attn_splits", splits)
    rng = np.random.default_rng(D + 7)
    B, Hkv, G, T, L, cap = 2, 2, 2, 40, 75, 90
    par = np.stack([np.array([-1] + [int(rng.integers(-1, i)) for i in range(1, T)], dtype=np.int32) for _ in range(B)])
    rnd = lambda *s: round_to_bf16(rng.standard_normal(s)).astype(np.float64)  # noqa: E731
    x = {"q": rnd(B, T, Hkv * G, D), "k_cache": rnd(B, cap, Hkv, D), "v_cache": rnd(B, cap, Hkv, D),
         "k_tree": rnd(B, T, Hkv, D), "v_tree": rnd(B, T, Hkv, D)}
    lens = [L, 33]
    # bf16 (unit roundoff 2^-8): one rounding of the result, and one more of the partial of a split before it;
    # fp32: a few roundings and the exponential's error
    ulp = (2.0 ** -8 * (1 if splits == 1 else 2)) if dtype == "bf16" else 2.0 ** -18
    # equal value rows: sum(p v) / sum(p) = v; unsplit bf16 returns the row itself, split partials are rounded once more
    row = rnd(D)
    y = dict(x, v_cache=np.broadcast_to(row, x["v_cache"].shape).copy(), v_tree=np.broadcast_to(row, x["v_tree"].shape).copy())
    got = gpu_attention(y, par, lens, dtype, max_prefix_len=cap)
    if dtype == "bf16" and splits == 1:
        np.testing.assert_array_equal(got, np.broadcast_to(row, got.shape))
    else:
        worst = float(np.max(np.abs(got - row) / (np.abs(row) + 1e-30)))
        assert worst <= ulp, worst
    # equal key rows: plain means over the visible rows.  Roundings (the partial sums of a split, the result) are
    # relative to sums of |v|, so the bound is that many roundoffs of the mean of |v|; a miscounted or missing key moves the
    # mean by about 1 / 80 of a value, several times that
    krow = rnd(D)
    y = dict(x, k_cache=np.broadcast_to(krow, x["k_cache"].shape).copy(), k_tree=np.broadcast_to(krow, x["k_tree"].shape).copy())
    got = gpu_attention(y, par, lens, dtype, max_prefix_len=cap)
    for b in range(B):
        dep = _depths(par[b])
        for i in range(T):
            anc, j = [], i
            while j >= 0:
                anc.append(j); j = par[b, j]
            n = lens[b] + dep[i] + 1
            assert len(anc) == dep[i] + 1
            for kv in range(Hkv):
                rows = np.concatenate([x["v_cache"][b, :lens[b], kv], x["v_tree"][b, anc, kv]])
                mean, mean_abs = rows.sum(0) / n, np.abs(rows).sum(0) / n
                for g in range(G):
                    worst = float(np.max(np.abs(got[b, i, kv * G + g] - mean) / (mean_abs + 1e-30)))
                    assert worst <= ulp, (b, i, kv, g, worst)
    # roots over an empty prefix
    got = gpu_attention(x, par, [0, 0], dtype, max_prefix_len=cap)
    for b in range(B):
        for i in np.nonzero(par[b] < 0)[0]:
            for h in range(Hkv * G):
                np.testing.assert_array_equal(got[b, i, h], x["v_tree"][b, i, h // G])
    # weights 1 : 2 : 4
    e0 = np.zeros(D); e0[0] = 1.0
    z = {"q": np.broadcast_to(e0, (1, 2, 1, D)).copy(), "k_cache": np.zeros((1, 1, 1, D)), "v_cache": np.zeros((1, 1, 1, D)),
         "k_tree": np.stack([e0, 2 * e0]).reshape(1, 2, 1, D), "v_tree": np.stack([np.full(D, 1.0), np.full(D, 2.0)]).reshape(1, 2, 1, D)}
    chain = gpu_attention(z, np.array([[-1, 0]], dtype=np.int32), [1], dtype, scale=float(np.log(2.0)))
    sibs = gpu_attention(z, np.array([[-1, -1]], dtype=np.int32), [1], dtype, scale=float(np.log(2.0)))
    for got1, want in ((chain[0, 0, 0], 2 / 3), (chain[0, 1, 0], 10 / 7), (sibs[0, 0, 0], 2 / 3), (sibs[0, 1, 0], 8 / 5)):
        assert np.abs(got1 - want).max() <= ulp * want


@pytest.mark.parametrize("dtype,D,G", [("bf16", 128, 4), ("bf16", 64, 1), ("f32", 32, 2)])
def test_chain_tree_is_the_librarys_causal_attention(dtype, D, G):
    """No oracle here either: for parent = [-1, 0, 1, ...] the call is ordinary causal attention of the tree tokens
    appended to the prefix, which torch's scaled_dot_product_attention computes (fp64, CPU) from a lower-triangular
    mask; a single node is plain decode attention.  Ragged prefix lengths, GQA by repeating the KV heads."""
    rng = np.random.default_rng(D + G)
    B, Hkv, T, cap = 2, 2, 37, 150
    lens = [150, 41]
    rnd = lambda *s: round_to_bf16(rng.standard_normal(s)).astype(np.float64)  # noqa: E731
    x = {"q": rnd(B, T, Hkv * G, D), "k_cache": rnd(B, cap, Hkv, D), "v_cache": rnd(B, cap, Hkv, D),
         "k_tree": rnd(B, T, Hkv, D), "v_tree": rnd(B, T, Hkv, D)}
    par = np.broadcast_to(np.arange(-1, T - 1, dtype=np.int32), (B, T)).copy()
    got = gpu_attention(x, par, lens, dtype, max_prefix_len=cap)
    tol = 2.0 ** -8 * 4 if dtype == "bf16" else 1e-5   # bf16: probabilities, partials and the result are rounded
    for b in range(B):
        L = lens[b]
        k = torch.from_numpy(np.concatenate([x["k_cache"][b, :L], x["k_tree"][b]])).permute(1, 0, 2).repeat_interleave(G, 0)
        v = torch.from_numpy(np.concatenate([x["v_cache"][b, :L], x["v_tree"][b]])).permute(1, 0, 2).repeat_interleave(G, 0)
        q = torch.from_numpy(x["q"][b]).permute(1, 0, 2)
        mask = torch.ones(T, L + T, dtype=torch.bool).tril(diagonal=L)
        want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask).permute(1, 0, 2).numpy()
        err = np.abs(got[b] - want).max()
        assert err <= tol * np.abs(want).max(), (b, err, np.abs(want).max())
    one = gpu_attention({k: v[:, :1] if k in ("q", "k_tree", "v_tree") else v for k, v in x.items()},
                        np.full((B, 1), -1, dtype=np.int32), lens, dtype, max_prefix_len=cap)
    for b in range(B):
        L = lens[b]
        k = torch.from_numpy(np.concatenate([x["k_cache"][b, :L], x["k_tree"][b, :1]])).permute(1, 0, 2).repeat_interleave(G, 0)
        v = torch.from_numpy(np.concatenate([x["v_cache"][b, :L], x["v_tree"][b, :1]])).permute(1, 0, 2).repeat_interleave(G, 0)
        q = torch.from_numpy(x["q"][b, :1]).permute(1, 0, 2)
        want = torch.nn.functional.scaled_dot_product_attention(q, k, v).permute(1, 0, 2).numpy()
        assert np.abs(one[b] - want).max() <= tol * np.abs(want).max()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_lengths_are_clamped_and_the_cache_beyond_them_is_never_used(dtype):
    """prefix_len on the device may hold anything: values below 0 count as 0, values above max_prefix_len as
    max_prefix_len; and what the caches hold beyond a sequence's length (NaN here) never reaches a result.  Bitwise
    equal to the call with the clamped lengths and clean caches."""
    import paper_2502_06282_amd as jk
    D = 128 if dtype == "bf16" else 32
    cfg = _cfg("c3_llama3_8b", batch=4, prefix_len=300, n_q_heads=4, n_kv_heads=2, head_dim=D, n_tree=33)
    par = tree_for_config(cfg, seed=61)
    x = attention_inputs(cfg, seed=61, scale_mult=np.sqrt(float(D)))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = torch.device("cuda")
    d = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev).to(tdt) for k, v in x.items()}
    parent = torch.from_numpy(par).to(dev)
    wild = [-5, 10 ** 9, 123, -2 ** 31]
    clean = [0, 300, 123, 0]
    dirty = {k: v.clone() for k, v in d.items()}
    for b, n in enumerate(clean):
        dirty["k_cache"][b, n:] = float("nan")
        dirty["v_cache"][b, n:] = float("nan")
    for splits in (1, 3):
        tune("attn_splits", splits)
        a = jk.tree_verify_attention(dirty["q"], dirty["k_cache"], dirty["v_cache"], dirty["k_tree"], dirty["v_tree"], parent,
                                     torch.tensor(wild, dtype=torch.int32, device=dev), max_prefix_len=300)
        b_ = jk.tree_verify_attention(d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent,
                                      torch.tensor(clean, dtype=torch.int32, device=dev), max_prefix_len=300)
        torch.cuda.synchronize()
        assert torch.isfinite(a.float()).all()
        assert torch.equal(a, b_)
    ref = oracle_attention(**x, parent=par, prefix_len=clean)
    assert np.abs(a.float().cpu().numpy() - ref).max() <= (BF16_TOL if dtype == "bf16" else F32_TOL)


def test_bf16_queries_and_results_as_strided_views():
    """q and out as views into larger tensors (a fused projection's output, a result written between other columns):
    the descriptor's strides, not contiguity, say where rows are.  Bitwise equal to the call on compact tensors, and
    nothing outside the view of the result is written."""
    import paper_2502_06282_amd as jk
    cfg = _cfg("c3_llama3_8b", batch=2, prefix_len=260, n_q_heads=8, n_kv_heads=2)
    par = tree_for_config(cfg, seed=62)
    x = attention_inputs(cfg, seed=62, scale_mult=np.sqrt(128.0))
    dev = torch.device("cuda")
    d = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev).to(torch.bfloat16) for k, v in x.items()}
    parent = torch.from_numpy(par).to(dev)
    pl = torch.tensor([260, 77], dtype=torch.int32, device=dev)
    B, T, Hq, D = d["q"].shape
    wide = torch.randn(B, T, Hq + 4, D, device=dev).to(torch.bfloat16)      # queries are heads 0..Hq-1 of a wider row
    wide[:, :, :Hq] = d["q"]
    big_out = torch.empty((B, T + 3, Hq + 2, D), dtype=torch.bfloat16, device=dev)
    out_view = big_out[:, 1:T + 1, 2:]
    outside = torch.ones_like(big_out, dtype=torch.bool)
    outside[:, 1:T + 1, 2:] = False
    for splits in (1, 4):
        tune("attn_splits", splits)
        big_out.fill_(7.0)
        got = jk.tree_verify_attention(wide[:, :, :Hq], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent, pl,
                                       out=out_view)
        want = jk.tree_verify_attention(d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent, pl)
        torch.cuda.synchronize()
        assert got.data_ptr() == out_view.data_ptr()
        assert torch.equal(out_view, want)
        assert (big_out[outside] == 7.0).all()
    ref = oracle_attention(**x, parent=par, prefix_len=[260, 77])
    assert np.abs(want.float().cpu().numpy() - ref).max() <= BF16_TOL


@pytest.mark.parametrize("paged", [False, True], ids=["contiguous", "paged"])
def test_bf16_deeper_ring_of_the_2x2_arrangement_changes_nothing_but_the_speed(paged):
    """The 2x2 arrangement keeps four K/V tiles in LDS, or six when a workgroup has its CU to itself (two rounds in
    flight instead of one): the same arithmetic in the same order, so the results are equal bit for bit - long and
    short prefixes, ragged lengths, splits merged in the kernel and by the merge kernel, head widths 128 and 64."""
    import paper_2502_06282_amd as jk
    from workloads import paged_layout
    dev = torch.device("cuda")
    for D, B, Hkv, G, T, L, splits, fused in ((128, 2, 4, 1, 5, 2048, 1, -1), (128, 1, 2, 2, 60, 700, 4, 1), (64, 3, 2, 4, 33, 1500, 3, 0),
                                              (128, 2, 2, 1, 28, 45, 1, -1), (64, 1, 1, 8, 100, 5000, 0, -1)):
        cfg = _cfg("c3_llama3_8b", batch=B, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D, n_tree=T, prefix_len=L)
        rng = np.random.default_rng(L)
        par = np.stack([np.array([-1] + [int(rng.integers(max(-1, i - 7), i)) for i in range(1, T)], dtype=np.int32) for _ in range(B)])
        x = {k: round_to_bf16(v) for k, v in attention_inputs(cfg, seed=L, scale_mult=np.sqrt(float(D))).items()}
        d = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev).to(torch.bfloat16) for k, v in x.items()}
        parent = torch.from_numpy(par).to(dev)
        lens = [L] + [max(0, L - 61 * (b + 1)) for b in range(B - 1)]
        pl = torch.tensor(lens, dtype=torch.int32, device=dev)
        if paged:
            (kp, vp), table = paged_layout(x["k_cache"], x["v_cache"], 32, seed=L)
            kp, vp, table = torch.from_numpy(kp).to(dev).to(torch.bfloat16), torch.from_numpy(vp).to(dev).to(torch.bfloat16), torch.from_numpy(table).to(dev)
        outs = []
        for deep in (0, 1):
            tune("attn_wm", 2); tune("attn_wn", 2); tune("attn_splits", splits); tune("attn_fused", fused); tune("attn_deep", deep)
            if paged:
                outs.append(jk.tree_verify_attention_paged(d["q"], kp, vp, table, d["k_tree"], d["v_tree"], parent, pl, max_prefix_len=L))
            else:
                outs.append(jk.tree_verify_attention(d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent, pl,
                                                     max_prefix_len=L))
            torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]), (D, B, Hkv, G, T, L, splits, fused)
        ref = oracle_attention(**x, parent=par, prefix_len=lens)
        err = np.abs(outs[1].float().cpu().numpy() - ref).max()
        assert err <= BF16_TOL and err <= 1.5e-2 * np.abs(ref).max()
