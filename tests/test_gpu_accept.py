"""GPU parity: jk_accept_path (through the C ABI) against the oracle: accepted path,
accepted length and bonus token must be bit-exact on identical logits / uniforms.
Sampling decisions are thresholds on rounded sums.  The kernels do all sampling
arithmetic in fp64 like the oracle, so the two sides differ by summation order
only (~1e-13 relative); a seed is compared when every decision on the oracle's
walk has a relative margin above 1e-9, which the inverse-CDF draw (steps of
~1/vocab) still leaves to practically every seed.  Seeds below the margin are
counted and reported, never silently dropped."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from gpu_util import reset_tuning, tune
from oracle import accept_path as oracle_accept
from workloads import CONFIGS, accept_inputs, tree_for_config

pytestmark = pytest.mark.gpu
MARGIN = 1e-9


def _gpu_accept(a, par, mode, temperature=1.0, max_depth=None):
    dev = torch.device("cuda")
    t = lambda v: None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(dev)
    path, alen, bonus = jk.accept_path(t(a["tokens"]), t(par.astype(np.int32)), t(a["logits"]),
                                       jk.JK_GREEDY if mode == "greedy" else jk.JK_SAMPLE, temperature,
                                       t(a["draft_probs"]), t(a["uniforms"]), max_depth=max_depth)
    torch.cuda.synchronize()
    return path.cpu().numpy(), alen.cpu().numpy(), bonus.cpu().numpy()


def _compare(a, par, mode, temperature=1.0, max_depth=None):
    path, alen, bonus = _gpu_accept(a, par, mode, temperature, max_depth)
    skipped = 0
    for b in range(par.shape[0]):
        r = oracle_accept(a["tokens"][b], par[b], a["logits"][b], mode,
                          None if a["draft_probs"] is None else a["draft_probs"][b],
                          None if a["uniforms"] is None else a["uniforms"][b], temperature, max_depth=max_depth)
        if mode == "sample" and r.min_margin <= MARGIN:
            skipped += 1
            continue
        assert alen[b] == r.accept_len
        assert path[b, : alen[b]].tolist() == r.path
        assert (path[b, alen[b]:] == -1).all()
        assert bonus[b] == r.bonus_token
    return skipped


def test_c1_greedy():
    cfg = CONFIGS["c1_tiny"]
    par = tree_for_config(cfg)
    _compare(accept_inputs(cfg, par), par, "greedy")


@pytest.mark.parametrize("seed", range(4))
def test_c2_greedy_full_vocab(seed):
    cfg = CONFIGS["c2_vicuna7b"]
    par = tree_for_config(cfg, seed=seed)
    a = accept_inputs(cfg, par, seed=seed)
    _compare(a, par, "greedy")
    path, alen, bonus = _gpu_accept(a, par, "greedy")
    stop = path[0, alen[0] - 1] if alen[0] else -1
    assert bonus[0] == a["top_token"][0, stop + 1]          # the planted top-1, known without an argmax


def test_c4_greedy_batched():
    cfg = CONFIGS["c4_llama2_13b"]
    par = tree_for_config(cfg)
    _compare(accept_inputs(cfg, par), par, "greedy")


@pytest.mark.parametrize("V", [1, 3, 4095, 4096, 4097, 10001])
def test_greedy_odd_vocab_sizes(V):
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=V, batch=2, hit_prob=0.7 if V > 20 else 0.0)
    par = tree_for_config(cfg)
    _compare(accept_inputs(cfg, par), par, "greedy")


def test_greedy_ties_and_minus_inf():
    N, V = 5, 9000
    par = np.array([[-1, 0, 0, 1, 3]], dtype=np.int32)
    logits = np.full((1, N + 1, V), -np.inf, dtype=np.float32)
    logits[0, 0, [7000, 4100, 8999]] = 2.0         # tie -> 4100
    logits[0, 1, [5, 4096]] = 1.0                   # tie -> 5
    logits[0, 2, 8191] = 0.0
    logits[0, 4, 1] = -1e30
    tokens = np.array([[4100, 4096, 5, 8191, 0]], dtype=np.int32)
    a = {"tokens": tokens, "logits": logits, "draft_probs": None, "uniforms": None}
    _compare(a, par, "greedy")
    path, alen, bonus = _gpu_accept(a, par, "greedy")
    assert path[0, :alen[0]].tolist() == [0, 2] and bonus[0] == 0    # row 3 is all -inf -> id 0


def test_greedy_first_child_chain_and_max_depth_cap():
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=2000, hit_prob=1.0)
    par = tree_for_config(cfg)
    a = accept_inputs(cfg, par)
    _compare(a, par, "greedy")
    path, alen, bonus = _gpu_accept(a, par, "greedy")
    # with a hit at every first child the walk follows first children down to a leaf
    c, expect = -1, []
    while True:
        kids = np.nonzero(par[0] == c)[0]
        if len(kids) == 0:
            break
        c = int(kids[0]); expect.append(c)
    assert path[0, :alen[0]].tolist() == expect and len(expect) >= 2
    # a depth cap stops the walk: the token after the last kept node is that node's own top-1,
    # not the one found further down (path[:len] + bonus must stay a sequence of the target's)
    for cap in (1, 2):
        _compare(a, par, "greedy", max_depth=cap)
        path2, alen2, bonus2 = _gpu_accept(a, par, "greedy", max_depth=cap)
        assert alen2[0] == cap and path2.shape == (1, cap) and path2[0].tolist() == expect[:cap]
        assert bonus2[0] == int(np.argmax(a["logits"][0, expect[cap - 1] + 1]))


@pytest.mark.parametrize("single", [False, True])
def test_sample_max_depth_cap(single, monkeypatch):
    """Sampling walks that go deep (draft distributions close to the target's), cut at every depth:
    cooperative and single-workgroup walks against the oracle's capped walk."""
    if single:
        tune("accept_single", "1")
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=3001, batch=4)
    par = tree_for_config(cfg, seed=7)
    a = accept_inputs(cfg, par, seed=7)
    lg = a["logits"].astype(np.float64)
    for b in range(cfg.batch):
        for k in range(cfg.n_tree):
            row = lg[b, par[b, k] + 1]
            e = np.exp(row - row.max())
            a["draft_probs"][b, k] = (0.97 * e / e.sum() + 0.03 * a["draft_probs"][b, k]).astype(np.float32)
            if k == int(np.nonzero(par[b] == par[b, k])[0][0]):
                a["tokens"][b, k] = int(np.argmax(row))  # first children carry the likeliest token
    full = [oracle_accept(a["tokens"][b], par[b], a["logits"][b], "sample", a["draft_probs"][b], a["uniforms"][b]).accept_len
            for b in range(cfg.batch)]
    assert max(full) >= 3
    for cap in (1, 2, 3):
        assert _compare(a, par, "sample", max_depth=cap) == 0


@pytest.mark.parametrize("seed", range(6))
def test_sample_small_vocab(seed):
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=5000, batch=3)
    par = tree_for_config(cfg, seed=seed)
    a = accept_inputs(cfg, par, seed=seed)
    skipped = _compare(a, par, "sample")
    assert skipped == 0


def test_sample_q_close_to_p_walks_deep():
    """Draft distributions near the target's: many accepts, residual passes in between."""
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=3001, batch=4)
    rng = np.random.default_rng(5)
    par = tree_for_config(cfg, seed=5)
    a = accept_inputs(cfg, par, seed=5)
    lg = a["logits"]
    q = a["draft_probs"]
    for b in range(4):
        for k in range(cfg.n_tree):
            z = lg[b, par[b, k] + 1].astype(np.float64) + rng.standard_normal(cfg.vocab) * 0.7
            e = np.exp(z - z.max())
            qq = (e / e.sum()).astype(np.float32)
            q[b, k] = qq
            cdf = np.cumsum(qq, dtype=np.float64)
            a["tokens"][b, k] = min(int(np.searchsorted(cdf, rng.random() * cdf[-1], side="right")), cfg.vocab - 1)
    skipped = _compare(a, par, "sample")
    _, alen, _ = _gpu_accept(a, par, "sample")
    assert alen.max() >= 2 and skipped == 0


def test_sample_temperature():
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=4000, batch=2)
    par = tree_for_config(cfg, seed=9)
    a = accept_inputs(cfg, par, seed=9)
    for temp in (0.5, 2.0):
        _compare(a, par, "sample", temperature=temp)


def test_c3_sample_full_vocab():
    cfg = CONFIGS["c3_llama3_8b"]
    par = tree_for_config(cfg)
    a = accept_inputs(cfg, par)
    assert _compare(a, par, "sample") == 0, "default seed must be admissible (margin > 1e-9)"


def test_c5_sample_batched_full_vocab():
    cfg = CONFIGS["c5_llama2_70b"]
    par = tree_for_config(cfg)
    a = accept_inputs(cfg, par)
    assert _compare(a, par, "sample") == 0


def test_argument_errors():
    dev = torch.device("cuda")
    tok = torch.zeros(1, 4, dtype=torch.int32, device=dev)
    lg = torch.zeros(1, 5, 100, dtype=torch.float32, device=dev)
    with pytest.raises(jk.JakiroError) as e:
        jk.accept_path(tok, tok, lg, jk.JK_SAMPLE)            # no draft_probs
    assert e.value.status == 1
    with pytest.raises(jk.JakiroError) as e:
        jk.accept_path(tok, tok, lg, jk.JK_SAMPLE, 0.0, lg[:, :4].contiguous(), lg[:, :, 0].contiguous())
    assert e.value.status == 1
    with pytest.raises(jk.JakiroError) as e:
        jk.accept_path(tok, tok, lg, jk.JK_GREEDY, workspace=torch.zeros(16, dtype=torch.uint8, device=dev))
    assert e.value.status == 4


def test_sample_single_workgroup_walk_agrees(monkeypatch):
    """The one-workgroup walk (used when the cooperative one does not fit) gives the same answers."""
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=6000, batch=2)
    par = tree_for_config(cfg, seed=3)
    a = accept_inputs(cfg, par, seed=3)
    coop = _gpu_accept(a, par, "sample")
    tune("accept_single", "1")
    single = _gpu_accept(a, par, "sample")
    for x, y in zip(coop, single):
        assert (x == y).all()
    _compare(a, par, "sample")


def test_sample_workspace_reuse_across_shapes_and_graph_replay():
    """One zero-initialised workspace serves calls of different shapes, and a captured HIP
    graph of the call replays correctly (every replay checked against the eager result)."""
    dev = torch.device("cuda")
    big = CONFIGS["c3_llama3_8b"].with_(vocab=9000, batch=3)
    small = CONFIGS["c5_llama2_70b"].with_(vocab=2500, batch=1, n_tree=40, depth=5)
    ws = torch.empty(jk.accept_path_workspace(3, 60, 9000, jk.JK_SAMPLE), dtype=torch.uint8, device=dev)
    jk.workspace_init(ws)
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(dev)
    results = {}
    for name, cfg in (("big", big), ("small", small), ("big2", big)):
        par = tree_for_config(cfg, seed=11)
        a = accept_inputs(cfg, par, seed=11)
        path, alen, bonus = jk.accept_path(t(a["tokens"]), t(par), t(a["logits"]), jk.JK_SAMPLE, 1.0,
                                           t(a["draft_probs"]), t(a["uniforms"]), workspace=ws)
        torch.cuda.synchronize()
        results[name] = (path.cpu().numpy(), alen.cpu().numpy(), bonus.cpu().numpy())
        for b in range(par.shape[0]):
            r = oracle_accept(a["tokens"][b], par[b], a["logits"][b], "sample", a["draft_probs"][b], a["uniforms"][b])
            if r.min_margin > MARGIN:
                assert alen.cpu()[b] == r.accept_len and bonus.cpu()[b] == r.bonus_token
    assert all((x == y).all() for x, y in zip(results["big"], results["big2"]))
    # graph replay of the last configuration
    cfg = big
    par = tree_for_config(cfg, seed=11)
    a = accept_inputs(cfg, par, seed=11)
    o_path = torch.empty((3, 60), dtype=torch.int32, device=dev)
    o_len = torch.empty(3, dtype=torch.int32, device=dev)
    o_bonus = torch.empty(3, dtype=torch.int32, device=dev)
    call = jk.prepare_accept_path(t(a["tokens"]), t(par), t(a["logits"]), jk.JK_SAMPLE, 1.0, t(a["draft_probs"]),
                                  t(a["uniforms"]), o_path, o_len, o_bonus, ws)
    call.launch()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        call.launch()
    for _ in range(3):
        o_len.fill_(-7); o_bonus.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert (o_len.cpu().numpy() == results["big"][1]).all() and (o_bonus.cpu().numpy() == results["big"][2]).all()
        call.launch()                      # eager work between replays
        torch.cuda.synchronize()


def test_sample_walk_gives_up_cleanly_and_the_workspace_survives():
    """spin_limit 0: a workgroup of the cooperative walk that does not find its partners' words at once gives
    up (every kernel still ends normally).  A tree then reports accept_len = bonus = -1 and the workspace's
    error word says so; a tree that got through must be right.  The calls that follow on the same workspace,
    with normal waits, must be bit-exact again: words of the failed call can never be taken for theirs."""
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=20011, batch=3)
    par = tree_for_config(cfg, seed=11)
    a = accept_inputs(cfg, par, seed=11)
    dev = torch.device("cuda")
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(dev)
    args = (t(a["tokens"]), t(par.astype(np.int32)), t(a["logits"]), jk.JK_SAMPLE, 1.0, t(a["draft_probs"]), t(a["uniforms"]))
    ws = torch.empty(jk.accept_path_workspace(cfg.batch, cfg.n_tree, cfg.vocab, jk.JK_SAMPLE), dtype=torch.uint8, device=dev)
    jk.workspace_init(ws)
    ref = [oracle_accept(a["tokens"][b], par[b], a["logits"][b], "sample", a["draft_probs"][b], a["uniforms"][b])
           for b in range(cfg.batch)]
    assert all(r.min_margin > MARGIN for r in ref)

    def check(path, alen, bonus, allow_fail):
        failed = 0
        for b, r in enumerate(ref):
            if allow_fail and int(alen[b]) == -1:
                assert int(bonus[b]) == -1
                failed += 1
                continue
            assert int(alen[b]) == r.accept_len and int(bonus[b]) == r.bonus_token
            assert path[b, : r.accept_len].cpu().tolist() == r.path
        return failed

    tune("spin_limit", 0)
    failed = 0
    for _ in range(3):
        path, alen, bonus = jk.accept_path(*args, workspace=ws)
        torch.cuda.synchronize()
        failed += check(path, alen, bonus, True)
    assert failed > 0, "no walk gave up: the test exercised nothing"
    assert jk.last_device_error(ws) & jk.JK_DEVERR_WALK_WAIT
    tune("spin_limit", -1)
    for _ in range(3):
        path, alen, bonus = jk.accept_path(*args, workspace=ws)
        torch.cuda.synchronize()
        assert check(path, alen, bonus, False) == 0


def test_sample_calls_of_different_batch_sizes_share_a_workspace():
    """Calls with different numbers of trees alternate on one workspace (a tree's words must keep their place
    whatever the batch size of a call is): every call is bit-exact and the error word stays clear."""
    dev = torch.device("cuda")
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(dev)
    ws = torch.empty(jk.accept_path_workspace(11, 60, 7001, jk.JK_SAMPLE), dtype=torch.uint8, device=dev)
    jk.workspace_init(ws)
    for i, batch in enumerate([11, 3, 11, 1, 9, 5, 11]):
        cfg = CONFIGS["c3_llama3_8b"].with_(vocab=7001, batch=batch)
        par = tree_for_config(cfg, seed=20 + i)
        a = accept_inputs(cfg, par, seed=20 + i)
        path, alen, bonus = jk.accept_path(t(a["tokens"]), t(par), t(a["logits"]), jk.JK_SAMPLE, 1.0,
                                           t(a["draft_probs"]), t(a["uniforms"]), workspace=ws)
        torch.cuda.synchronize()
        for b in range(batch):
            r = oracle_accept(a["tokens"][b], par[b], a["logits"][b], "sample", a["draft_probs"][b], a["uniforms"][b])
            if r.min_margin > MARGIN:
                assert int(alen[b]) == r.accept_len and int(bonus[b]) == r.bonus_token, (i, batch, b)
                assert path[b, : r.accept_len].cpu().tolist() == r.path
    assert jk.last_device_error(ws) == 0


@pytest.mark.parametrize("B,V", [(20, 5001), (64, 1000), (100, 4097), (300, 257), (300, 4097), (600, 1000)])
def test_sample_large_batches(B, V):
    """The workgroups that share a tree get fewer as the batch grows (two per CU over the batch, at most 64): 25, 8, 5
    and 1 of them here; a slice of more than 4096 tokens (300 trees of 4097) and more trees than resident workgroups
    (600) go to the one-workgroup walk."""
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=V, batch=B, n_tree=12)
    par = tree_for_config(cfg, seed=B)
    a = accept_inputs(cfg, par, seed=B + V)
    skipped = _compare(a, par, "sample")
    assert skipped <= B // 20


def test_greedy_at_the_row_limit():
    """batch * (n_tree + 1) = 65 532 logits rows, just inside the limit of 65 535; one tree more is refused."""
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=300, batch=508, n_tree=128)
    par = tree_for_config(cfg, seed=1)
    a = accept_inputs(cfg, par, seed=1)
    _compare(a, par, "greedy")
    _, alen, _ = _gpu_accept(a, par, "greedy")
    assert alen.max() >= 4
    cfg = cfg.with_(batch=509)
    par = tree_for_config(cfg, seed=2)
    a = accept_inputs(cfg, par, seed=2)
    with pytest.raises(jk.JakiroError) as e:
        _gpu_accept(a, par, "greedy")
    assert e.value.status == 3


@pytest.mark.parametrize("single", [0, 1], ids=["cooperative", "one_workgroup"])
def test_sample_hand_worked_and_degenerate_cases(single):
    """Section 2.1's rule on cases small enough to work by hand, through both walks: a draft probability of zero
    (always accepted if the target's is not; rejected if that is zero too: 0 < 0 is false, and the residual of p = q
    is empty, so p is kept), a uniform of exactly zero, and the residual between siblings."""
    tune("accept_single", single)
    ninf = -np.inf
    f32 = np.float32
    cases = [
        # q[x] = 0 < p[x]: accepted at any u; the next token is drawn from the accepted node's row
        dict(tokens=[0], parent=[-1], logits=[[0, 1, 2, 3], [0, 0, 0, 0]], q=[[0, .5, .25, .25]], u=[0.999999, 0.1],
             path=[0], bonus=0),
        # p[x] = q[x] = 0: rejected, nothing to subtract; the sibling is judged against the unchanged p
        dict(tokens=[2, 0], parent=[-1, -1], logits=[[0, 0, ninf, ninf], [0] * 4, [0] * 4], q=[[.5, .5, 0, 0]] * 2,
             u=[0.3, 0.9, 0.6], path=[1], bonus=2),
        # u = 0: accepted because p[x] > 0; the draw at u = 0.999999 takes the last token
        dict(tokens=[1], parent=[-1], logits=[[0, 1, 2, 3], [0, 0, 0, 0]], q=[[.25] * 4], u=[0.0, 0.999999], path=[0], bonus=3),
        # child 0 (token 0, p/q = 0.556) is rejected at u = 0.9; the residual is (0, .625, .375): child 1 (token 1,
        # q = 0.8) is accepted iff u < 0.78125
        dict(tokens=[0, 1], parent=[-1, -1], logits=np.log([[.5, .3, .2], [1 / 3] * 3, [1 / 3] * 3]).tolist(),
             q=[[.9, .05, .05], [.1, .8, .1]], u=[0.9, 0.70, 0.5], path=[1], bonus=1),
        # ... and rejected at u = 0.8; what is left after both is (0, 0, 1)
        dict(tokens=[0, 1], parent=[-1, -1], logits=np.log([[.5, .3, .2], [1 / 3] * 3, [1 / 3] * 3]).tolist(),
             q=[[.9, .05, .05], [.1, .8, .1]], u=[0.9, 0.80, 0.999], path=[], bonus=2),
    ]
    for i, c in enumerate(cases):
        par = np.array([c["parent"]], dtype=np.int32)
        a = {"tokens": np.array([c["tokens"]], dtype=np.int32), "logits": np.array([c["logits"]], dtype=f32),
             "draft_probs": np.array([c["q"]], dtype=f32), "uniforms": np.array([c["u"]], dtype=f32)}
        path, alen, bonus = _gpu_accept(a, par, "sample")
        r = oracle_accept(a["tokens"][0], par[0], a["logits"][0], "sample", a["draft_probs"][0], a["uniforms"][0], 1.0)
        assert r.path == c["path"] and r.bonus_token == c["bonus"], (i, r.path, r.bonus_token)
        assert path[0, : alen[0]].tolist() == c["path"] and bonus[0] == c["bonus"], (i, path, alen, bonus)
        assert (path[0, alen[0]:] == -1).all()


@pytest.mark.parametrize("B,calls", [(256, 240), (4096, 15)], ids=["cooperative_256_trees", "one_workgroup_4096_trees"])
def test_sampling_is_lossless_on_the_device(B, calls):
    """Section 2.1's claim, measured on the library's own output with no oracle in between: over many trees with the
    same logits and draft distributions, draft tokens drawn from those distributions and fresh uniforms, the first
    emitted token follows softmax(row 0), and the token after a first-level node k, given that k was accepted, follows
    softmax(row k + 1).  61 440 trees of the same two-level shape as the oracle's Monte-Carlo pin, through the
    cooperative walk (256 trees a call, two workgroups each) and the one-workgroup walk (4096 trees a call)."""
    rng = np.random.default_rng(7)
    V = 4
    par1 = np.array([-1, -1, 0, 0, 1], dtype=np.int32)
    N = len(par1)
    logits1 = (rng.standard_normal((N + 1, V)) * 1.5).astype(np.float32)
    q1 = rng.dirichlet(np.ones(V) * 0.7, size=N).astype(np.float32)
    q1 /= q1.sum(1, keepdims=True)
    cdf = np.cumsum(q1.astype(np.float64), axis=1)
    dev = torch.device("cuda")
    par = torch.from_numpy(np.broadcast_to(par1, (B, N)).copy()).to(dev)
    logits = torch.from_numpy(np.broadcast_to(logits1, (B, N + 1, V)).copy()).to(dev)
    q = torch.from_numpy(np.broadcast_to(q1, (B, N, V)).copy()).to(dev)
    first = np.zeros(V)
    second = {0: np.zeros(V), 1: np.zeros(V)}
    for _ in range(calls):
        draws = rng.random((B, N))
        tokens = np.stack([np.minimum((cdf[k][None, :] <= draws[:, k:k + 1] * cdf[k][-1]).sum(1), V - 1) for k in range(N)], 1)
        uni = rng.random((B, N + 1)).astype(np.float32)
        path, alen, bonus = jk.accept_path(torch.from_numpy(tokens.astype(np.int32)).to(dev), par, logits, jk.JK_SAMPLE, 1.0,
                                           q, torch.from_numpy(uni).to(dev))
        torch.cuda.synchronize()
        path, alen, bonus = path.cpu().numpy(), alen.cpu().numpy(), bonus.cpu().numpy()
        assert (alen >= 0).all() and (alen <= 2).all()
        for b in range(B):
            seq = [int(tokens[b, k]) for k in path[b, : alen[b]]] + [int(bonus[b])]
            first[seq[0]] += 1
            if alen[b] >= 1:
                second[int(path[b, 0])][seq[1]] += 1
    trials = B * calls
    z = logits1.astype(np.float64)
    soft = lambda r: np.exp(r - r.max()) / np.exp(r - r.max()).sum()  # noqa: E731
    p0 = soft(z[0])
    assert (np.abs(first / trials - p0) < 4.5 * np.sqrt(p0 * (1 - p0) / trials)).all(), (first / trials, p0)
    for k in (0, 1):
        n = second[k].sum()
        assert n > 2000
        pk = soft(z[k + 1])
        assert (np.abs(second[k] / n - pk) < 4.5 * np.sqrt(pk * (1 - pk) / n)).all(), (k, second[k] / n, pk)
    # and the test can tell: the draft distributions themselves are far from these frequencies
    assert np.abs(first / trials - q1[0]).max() > 20 * np.sqrt(0.25 / trials)


def test_greedy_and_sampling_calls_of_any_shape_take_turns_on_one_workspace():
    """One workspace, zero-filled once, then calls of both modes, several batch sizes and vocabularies in turn (the
    cooperative walk for some, the one-workgroup walk for others): every call writes all of its outputs (they are
    filled with a sentinel first) and they equal those of the same call on a fresh workspace."""
    dev = torch.device("cuda")
    t = lambda v: None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(dev)  # noqa: E731
    calls = [("sample", 3, 5000), ("greedy", 3, 5000), ("sample", 3, 5000), ("greedy", 40, 1000), ("sample", 11, 7001),
             ("sample", 300, 4097), ("sample", 5, 300), ("greedy", 2, 32000), ("sample", 1, 32000), ("sample", 40, 1000)]
    need = max(jk.accept_path_workspace(B, 24, V, jk.JK_SAMPLE) for _, B, V in calls)
    shared = torch.zeros(need, dtype=torch.uint8, device=dev)

    def run(a, par, mode, ws):
        B = par.shape[0]
        out = [torch.full((B, 24), -77, dtype=torch.int32, device=dev), torch.full((B,), -77, dtype=torch.int32, device=dev),
               torch.full((B,), -77, dtype=torch.int32, device=dev)]
        jk.prepare_accept_path(t(a["tokens"]), t(par), t(a["logits"]), jk.JK_GREEDY if mode == "greedy" else jk.JK_SAMPLE, 1.0,
                               t(a["draft_probs"]), t(a["uniforms"]), out[0], out[1], out[2], ws).launch()
        torch.cuda.synchronize()
        return [o.cpu().numpy() for o in out]

    for i, (mode, B, V) in enumerate(calls):
        cfg = CONFIGS["c3_llama3_8b" if mode == "sample" else "c2_vicuna7b"].with_(vocab=V, batch=B, n_tree=24)
        par = tree_for_config(cfg, seed=100 + i)
        a = accept_inputs(cfg, par, seed=100 + i)
        got = run(a, par, mode, shared)
        want = run(a, par, mode, torch.zeros(need, dtype=torch.uint8, device=dev))
        assert (want[1] >= 0).all() and (want[2] >= 0).all(), (i, mode, B, V)
        for g, w in zip(got, want):
            np.testing.assert_array_equal(g, w, err_msg=f"call {i}: {mode} B{B} V{V}")
        assert jk.last_device_error(shared) == 0


@pytest.mark.parametrize("mode,single", [("greedy", 0), ("sample", 0), ("sample", 1)], ids=["greedy", "cooperative", "one_workgroup"])
def test_bad_tokens_and_parents_are_repaired_and_reported(mode, single):
    """A token id outside [0, vocab) is clamped into it, a parent entry outside [-1, k) counts as -1: the results are
    those of the repaired inputs, and the workspace's error word says which repair happened; clean inputs leave it clear."""
    tune("accept_single", single)
    dev = torch.device("cuda")
    t = lambda v: None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(dev)  # noqa: E731
    V = 3000
    cfg = CONFIGS["c3_llama3_8b" if mode == "sample" else "c2_vicuna7b"].with_(vocab=V, batch=3, n_tree=30)
    par = tree_for_config(cfg, seed=9)
    a = accept_inputs(cfg, par, seed=9)
    m = jk.JK_GREEDY if mode == "greedy" else jk.JK_SAMPLE

    def run(tokens, parent):
        ws = torch.zeros(jk.accept_path_workspace(3, 30, V, m), dtype=torch.uint8, device=dev)
        out = jk.accept_path(t(tokens), t(parent), t(a["logits"]), m, 1.0, t(a["draft_probs"]), t(a["uniforms"]), workspace=ws)
        torch.cuda.synchronize()
        return [o.cpu().numpy() for o in out], jk.last_device_error(ws)

    clean, err = run(a["tokens"], par)
    assert err == 0
    # tokens: the first-level nodes of tree 0 get wild ids (they are examined whatever happens)
    bad_tok = a["tokens"].copy()
    roots = np.nonzero(par[0] < 0)[0]
    bad_tok[0, roots[0]] = -3
    bad_tok[0, roots[-1]] = V + 5
    fixed_tok = np.clip(bad_tok, 0, V - 1)
    got, err = run(bad_tok, par)
    want, err_fixed = run(fixed_tok, par)
    assert err == jk.JK_DEVERR_BAD_TOKEN and err_fixed == 0
    for g, w in zip(got, want):
        np.testing.assert_array_equal(g, w)
    # parents: a forward reference and a value below -1 in tree 1
    bad_par = par.copy()
    bad_par[1, 4] = 17
    bad_par[1, 9] = -6
    fixed_par = bad_par.copy()
    fixed_par[1, 4] = -1
    fixed_par[1, 9] = -1
    got, err = run(a["tokens"], bad_par)
    want, err_fixed = run(a["tokens"], fixed_par)
    assert err == jk.JK_DEVERR_BAD_TREE and err_fixed == 0
    for g, w in zip(got, want):
        np.testing.assert_array_equal(g, w)
