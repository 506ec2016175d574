"""Pins for the acceptance oracle (Section 2.1 steps 2-3; Section 3.2 "strict
top-1 verification"): closed forms, special cases, exact enumeration and
Monte-Carlo of the emitted-token distribution.  Nothing here re-types the
oracle's formulae: expectations come from the target distribution itself."""
import itertools

import numpy as np
import pytest

from oracle import accept_path
from workloads import CONFIGS, accept_inputs, tree_depths, tree_for_config, two_expert_tree


def _softmax(x):
    e = np.exp(x - x.max())
    return e / e.sum()


# ------------------------------------------------------------------ greedy
def test_greedy_full_accept_along_planted_chain():
    """Q1: tokens along one root-to-leaf chain equal the successive target argmaxes."""
    rng = np.random.default_rng(0)
    par = two_expert_tree(rng, depth=5, topk=3, frontier=2, budget=30)["parent"]
    N, V = len(par), 97
    d = tree_depths(par)
    leaf = int(np.nonzero(d == 5)[0][-1])
    chain = []
    a = leaf
    while a >= 0:
        chain.append(a); a = par[a]
    chain = chain[::-1]
    logits = rng.standard_normal((N + 1, V)).astype(np.float32)
    amax = logits.argmax(axis=1)
    tokens = np.empty(N, dtype=np.int32)
    for k in range(N):                       # everything else misses on purpose
        tokens[k] = (amax[par[k] + 1] + 1 + k) % V
        if tokens[k] == amax[par[k] + 1]:
            tokens[k] = (tokens[k] + 1) % V
    for k in chain:
        tokens[k] = amax[par[k] + 1]
    r = accept_path(tokens, par, logits, "greedy")
    assert r.path == chain and r.accept_len == 5
    assert r.bonus_token == amax[leaf + 1]


def test_greedy_zero_accept():
    """Q2: no depth-1 token equals argmax(row 0) -> plain autoregressive step."""
    rng = np.random.default_rng(1)
    par = np.array([-1, -1, 0, 1])
    logits = rng.standard_normal((5, 11)).astype(np.float32)
    t0 = int(logits[0].argmax())
    tokens = np.array([(t0 + 1) % 11, (t0 + 2) % 11, int(logits[1].argmax()), int(logits[2].argmax())])
    r = accept_path(tokens, par, logits, "greedy")
    assert r.path == [] and r.accept_len == 0 and r.bonus_token == t0


def test_greedy_ties_and_duplicates():
    # argmax tie -> lowest id; duplicate sibling tokens -> first sibling
    logits = np.zeros((4, 5), dtype=np.float32)
    logits[0, [2, 4]] = 3.0
    logits[1, 1] = 1.0
    logits[2, 3] = 1.0
    par = np.array([-1, -1, 0])
    r = accept_path(np.array([2, 2, 1]), par, logits, "greedy")
    assert r.path == [0, 2] and r.bonus_token == 0          # row 3 is all zeros -> id 0
    r = accept_path(np.array([4, 2, 1]), par, logits, "greedy")
    assert r.path == [1] and r.bonus_token == 3


def test_greedy_row_of_parent_not_own_row():
    # node 0's own row has argmax 7; its child must match THAT, node 0 must match row 0
    logits = np.full((3, 9), -1.0, dtype=np.float32)
    logits[0, 5] = 1.0; logits[1, 7] = 1.0; logits[2, 2] = 1.0
    r = accept_path(np.array([5, 7]), np.array([-1, 0]), logits, "greedy")
    assert r.path == [0, 1] and r.bonus_token == 2
    r = accept_path(np.array([7, 5]), np.array([-1, 0]), logits, "greedy")
    assert r.path == [] and r.bonus_token == 5


def _node_parallel_greedy(tokens, par, logits):
    """Independent formulation: mark every node whose token equals its parent's
    row argmax, then take the deepest chain of marked nodes from the root."""
    amax = logits.argmax(axis=1)
    ok = [tokens[k] == amax[par[k] + 1] for k in range(len(par))]
    c, path = -1, []
    while True:
        kids = [k for k in range(len(par)) if par[k] == c and ok[k]]
        if not kids:
            return path, int(amax[c + 1])
        c = kids[0]; path.append(c)


@pytest.mark.parametrize("seed", range(6))
def test_greedy_node_parallel_equals_sequential(seed):
    """Q6 on the config-2 generator (70 % planted hits)."""
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=300)
    par = tree_for_config(cfg, seed=seed)
    a = accept_inputs(cfg, par, seed=seed)
    r = accept_path(a["tokens"][0], par[0], a["logits"][0], "greedy")
    path, bonus = _node_parallel_greedy(a["tokens"][0], par[0], a["logits"][0])
    assert r.path == path and r.bonus_token == bonus
    # planted top-1 of the stop row is the bonus token (generator knows it without an argmax)
    stop = r.path[-1] if r.path else -1
    assert r.bonus_token == a["top_token"][0, stop + 1]
    for k in r.path:
        assert a["tokens"][0, k] == a["top_token"][0, par[0, k] + 1]


def test_generator_expectation_band():
    """Q7: with a 0.7 hit rate per expanded node the mean accepted length over
    seeds sits in a broad band (sanity, not a bit-exact pin)."""
    cfg = CONFIGS["c2_vicuna7b"].with_(vocab=300)
    lens = []
    for seed in range(40):
        par = tree_for_config(cfg, seed=seed)
        a = accept_inputs(cfg, par, seed=seed)
        lens.append(accept_path(a["tokens"][0], par[0], a["logits"][0], "greedy").accept_len)
    assert 1.0 < np.mean(lens) < 5.5


# ------------------------------------------------------------------ sampling
def _threshold(fn, lo=0.0, hi=1.0, iters=60):
    """Largest u in [lo,hi] for which fn(u) is True (fn monotone: True then False)."""
    if not fn(lo):
        return lo
    if fn(np.nextafter(hi, 0)):
        return hi
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if fn(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def test_single_node_is_textbook_speculative_sampling():
    """Q3: 1-node tree.  By bisection on the uniforms (oracle as a black box):
    P(accept | x) = min(1, p_x/q_x), so P(accept) = sum_x min(p_x, q_x) = 1 - TV(p, q),
    and the emitted token is distributed exactly as p."""
    rng = np.random.default_rng(3)
    V = 5
    logits = rng.standard_normal((2, V)) * 2
    p = _softmax(logits[0])
    q = rng.dirichlet(np.ones(V))[None]
    par = np.array([-1])
    emitted = np.zeros(V)
    p_acc_total = 0.0
    for x in range(V):
        acc_u = _threshold(lambda u: accept_path(np.array([x]), par, logits, "sample", q,
                                                 np.array([u, 0.5])).accept_len == 1)
        assert acc_u == pytest.approx(min(1.0, p[x] / q[0, x]), abs=1e-12)
        p_acc_total += q[0, x] * acc_u
        emitted[x] += q[0, x] * acc_u
        # rejected: distribution of the replacement over the second uniform
        u_rej = 0.5 * (acc_u + 1.0)
        if acc_u < 1.0:
            prev = 0.0
            for v in range(V):
                hi = _threshold(lambda u2: accept_path(np.array([x]), par, logits, "sample", q,
                                                       np.array([u_rej, u2])).bonus_token <= v)
                emitted[v] += q[0, x] * (1.0 - acc_u) * (hi - prev)
                prev = hi
    assert p_acc_total == pytest.approx(np.minimum(p, q[0]).sum(), abs=1e-11)
    assert p_acc_total == pytest.approx(1.0 - 0.5 * np.abs(p - q[0]).sum(), abs=1e-11)
    np.testing.assert_allclose(emitted, p, atol=1e-10)


def _exact_first_token(par, logits, q, V):
    """Exact distribution of the first emitted token on a tree whose root has
    the children listed in par (all depth 1): enumerate sibling tokens weighted
    by their draft probabilities; accept probabilities and bonus distributions
    are read off the oracle's decision trace by driving the uniforms into each
    region (accept: u = 0, reject: u just below 1)."""
    N = len(par)
    kids = [k for k in range(N) if par[k] == -1]
    dist = np.zeros(V)
    for toks in itertools.product(range(V), repeat=len(kids)):
        tokens = np.zeros(N, dtype=np.int64)
        w = 1.0
        for k, x in zip(kids, toks):
            tokens[k] = x; w *= q[k, x]
        if w == 0:
            continue
        reach = 1.0                               # P(all earlier siblings rejected)
        for j, k in enumerate(kids):
            u = np.full(N + 1, 0.5)
            u[kids[:j]] = np.nextafter(1.0, 0)    # force rejections (only possible if p < q)
            u[k] = 0.0
            r = accept_path(tokens, par, logits, "sample", q, u)
            dec = [d for d in r.decisions if d[1] == k][0]
            # reconstruct a_k = min(1, p~[x]/q_k[x]) from the trace at u = 1-eps of a probe run
            u2 = u.copy(); u2[k] = np.nextafter(1.0, 0)
            r2 = accept_path(tokens, par, logits, "sample", q, u2)
            d2 = [d for d in r2.decisions if d[1] == k][0]
            lhs_full, rhs = d2[2], d2[3]          # ~ q_k[x], p~[x]
            a = 1.0 if lhs_full <= 0 else min(1.0, rhs / (lhs_full / np.nextafter(1.0, 0)))
            if dec[0] == "accept":
                dist[toks[j]] += w * reach * a
            reach *= (1.0 - a)
            if reach == 0:
                break
        if reach > 0:
            # all rejected: bonus from the final residual; integrate over its uniform by bisection
            u = np.full(N + 1, 0.5)
            u[kids] = np.nextafter(1.0, 0)
            prev = 0.0
            for v in range(V):
                def le(u_b, v=v):
                    uu = u.copy(); uu[N] = u_b
                    rr = accept_path(tokens, par, logits, "sample", q, uu)
                    assert rr.accept_len == 0
                    return rr.bonus_token <= v
                hi = _threshold(le)
                dist[v] += w * reach * (hi - prev)
                prev = hi
    return dist


@pytest.mark.parametrize("nkids", [1, 2, 3])
def test_losslessness_exact_enumeration_siblings(nkids):
    """Q4 (exact): root with 1-3 children, each with its own draft distribution
    (two experts give different q's): the first emitted token follows softmax(row 0)."""
    rng = np.random.default_rng(20 + nkids)
    V = 3
    par = np.full(nkids, -1)
    logits = rng.standard_normal((nkids + 1, V)) * 1.5
    q = rng.dirichlet(np.ones(V), size=nkids)
    dist = _exact_first_token(par, logits, q, V)
    np.testing.assert_allclose(dist, _softmax(logits[0]), atol=1e-9)


def test_losslessness_monte_carlo_two_levels():
    """Q4 (Monte-Carlo): 2-level tree, tiny vocabulary; first emitted token ~
    softmax(row 0); second emitted token given that node k was accepted first ~ softmax(row k+1)."""
    rng = np.random.default_rng(7)
    V = 4
    par = np.array([-1, -1, 0, 0, 1])
    N = len(par)
    logits = rng.standard_normal((N + 1, V)) * 1.5
    q = rng.dirichlet(np.ones(V) * 0.7, size=N)
    cdf = np.cumsum(q, axis=1)
    trials = 60000
    first = np.zeros(V)
    second = {0: np.zeros(V), 1: np.zeros(V)}
    for _ in range(trials):
        tokens = np.array([min(int(np.searchsorted(cdf[k], rng.random(), side="right")), V - 1)
                           for k in range(N)])
        r = accept_path(tokens, par, logits, "sample", q, rng.random(N + 1))
        seq = [int(tokens[k]) for k in r.path] + [r.bonus_token]
        first[seq[0]] += 1
        if r.path:
            second[r.path[0]][seq[1]] += 1
    p0 = _softmax(logits[0])
    sigma = np.sqrt(p0 * (1 - p0) / trials)
    assert (np.abs(first / trials - p0) < 4.5 * sigma).all()
    for k in (0, 1):
        n = second[k].sum()
        assert n > 2000
        pk = _softmax(logits[k + 1])
        assert (np.abs(second[k] / n - pk) < 4.5 * np.sqrt(pk * (1 - pk) / n)).all()


def test_q_equals_p_accepts_first_children_to_a_leaf():
    """Q5: draft distribution identical to the target's -> u*q < p always."""
    rng = np.random.default_rng(8)
    par = two_expert_tree(rng, depth=4, topk=2, frontier=2, budget=14)["parent"]
    N, V = len(par), 50
    logits = rng.standard_normal((N + 1, V))
    q = np.stack([_softmax(logits[par[k] + 1]) for k in range(N)])
    tokens = rng.integers(0, V, N)
    r = accept_path(tokens, par, logits, "sample", q, rng.random(N + 1))
    c, expect = -1, []
    while True:
        kids = [k for k in range(N) if par[k] == c]
        if not kids:
            break
        c = kids[0]; expect.append(c)
    assert r.path == expect


def test_temperature_and_strictness():
    # temperature divides the logits: T -> large makes p uniform
    V = 4
    logits = np.array([[0.0, 1.0, 2.0, 3.0], [0, 0, 0, 0]])
    q = np.full((1, V), 0.25)
    # p uniform (=q) at huge temperature: accepted for any u < 1
    r = accept_path(np.array([0]), np.array([-1]), logits, "sample", q, np.array([0.999, 0.1]),
                    temperature=1e9)
    assert r.accept_len == 1
    # at T=1, p[0] = 0.032 < q: accepted iff u*0.25 < p[0] strictly
    p0 = _softmax(logits[0])[0]
    u_edge = p0 / 0.25
    assert accept_path(np.array([0]), np.array([-1]), logits, "sample", q,
                       np.array([u_edge * 0.999, 0.1])).accept_len == 1
    assert accept_path(np.array([0]), np.array([-1]), logits, "sample", q,
                       np.array([u_edge * 1.001, 0.1])).accept_len == 0
    # q[x] = 0 and p[x] > 0: accepted even at u ~ 1
    q0 = np.array([[0.0, 0.5, 0.25, 0.25]])
    assert accept_path(np.array([0]), np.array([-1]), logits, "sample", q0,
                       np.array([0.999999, 0.1])).accept_len == 1


def test_residual_is_applied_between_siblings():
    """Second sibling is judged against norm(max(0, p - q_1)), not against p."""
    V = 3
    logits = np.log(np.array([[0.5, 0.3, 0.2], [1 / 3] * 3, [1 / 3] * 3]))
    q = np.array([[0.9, 0.05, 0.05], [0.1, 0.8, 0.1]])
    # child 0 proposes token 0 (p/q = 0.556) and is rejected with u = 0.9
    # residual = norm(max(0, [-.4, .25, .15])) = [0, .625, .375]
    # child 1 proposes token 1: accept iff u*0.8 < 0.625  <=>  u < 0.78125 (0.375 against raw p)
    par = np.array([-1, -1])
    r = accept_path(np.array([0, 1]), par, logits, "sample", q, np.array([0.9, 0.70, 0.5]))
    assert r.path == [1]
    r = accept_path(np.array([0, 1]), par, logits, "sample", q, np.array([0.9, 0.80, 0.5]))
    assert r.path == []
    # after both rejections the residual is norm(max(0, [0, .625, .375] - [.1, .8, .1])) = [0, 0, 1]
    assert r.bonus_token == 2
    assert accept_path(np.array([0, 1]), par, logits, "sample", q,
                       np.array([0.9, 0.80, 0.999])).bonus_token == 2


def test_bonus_inverse_cdf():
    V = 4
    logits = np.log(np.array([[0.1, 0.2, 0.3, 0.4], [0.25] * 4]))
    q = np.array([[0.0, 0.0, 0.0, 1.0]])
    # leaf stop: accept node 0 (token 3: u*1 < 0.4), bonus drawn from row 1 (uniform)
    for u_b, v in [(0.0, 0), (0.2499, 0), (0.2501, 1), (0.74, 2), (0.76, 3), (0.9999, 3)]:
        r = accept_path(np.array([3]), np.array([-1]), logits, "sample", q, np.array([0.3, u_b]))
        assert r.path == [0] and r.bonus_token == v
    # reject (u = 0.5): residual = norm([.1,.2,.3,0]) = [1/6, 1/3, 1/2, 0]
    for u_b, v in [(0.16, 0), (0.17, 1), (0.49, 1), (0.51, 2), (0.9999, 2)]:
        r = accept_path(np.array([3]), np.array([-1]), logits, "sample", q, np.array([0.5, u_b]))
        assert r.path == [] and r.bonus_token == v


def test_margins_and_fp32_variant_agree():
    cfg = CONFIGS["c3_llama3_8b"].with_(vocab=3000)
    agree = 0
    for seed in range(8):
        par = tree_for_config(cfg, seed=seed)
        a = accept_inputs(cfg, par, seed=seed)
        r64 = accept_path(a["tokens"][0], par[0], a["logits"][0], "sample", a["draft_probs"][0],
                          a["uniforms"][0])
        r32 = accept_path(a["tokens"][0], par[0], a["logits"][0], "sample", a["draft_probs"][0],
                          a["uniforms"][0], ftype=np.float32)
        assert r64.decisions and r64.decisions[-1][0] == "bonus"
        if r64.min_margin > 1e-4:
            assert (r64.path, r64.bonus_token) == (r32.path, r32.bonus_token)
            agree += 1
    assert agree >= 6


def test_argument_errors():
    with pytest.raises(ValueError):
        accept_path(np.array([1]), np.array([0]), np.zeros((2, 3)), "greedy")
    with pytest.raises(ValueError):
        accept_path(np.array([1]), np.array([-1]), np.zeros((2, 3)), "sample")
    with pytest.raises(ValueError):
        accept_path(np.array([1]), np.array([-1]), np.zeros((2, 3)), "sample",
                    np.ones((1, 3)) / 3, np.zeros(2), temperature=0.0)


def _cut_tree(par, depth_cap):
    """Nodes of depth <= depth_cap, in their old order, with parents renumbered; returns (new parent, kept old ids)."""
    depth = tree_depths(par)
    keep = [i for i in range(len(par)) if depth[i] <= depth_cap]
    new_id = {old: new for new, old in enumerate(keep)}
    return np.array([new_id.get(int(par[i]), -1) for i in keep], dtype=np.int32), keep


@pytest.mark.parametrize("mode", ["greedy", "sample"])
@pytest.mark.parametrize("cap", [1, 2, 3])
def test_max_depth_equals_the_tree_cut_below_that_depth(mode, cap):
    """Pin of the depth cap: stopping after `cap` accepted nodes must give what the same walk gives on
    the tree with every deeper node removed (path, and the token that follows it).  Section 2.1 step 3:
    the emitted sequence is accepted tokens + one token of the target's own distribution at the stop."""
    hits = 0
    for seed in range(12):
        if mode == "greedy":
            cfg = CONFIGS["c2_vicuna7b"].with_(vocab=300, hit_prob=0.9)
        else:
            cfg = CONFIGS["c3_llama3_8b"].with_(vocab=40)
        par = tree_for_config(cfg, seed=seed)[0]
        a = accept_inputs(cfg, par[None], seed=seed)
        q = None if a["draft_probs"] is None else a["draft_probs"][0]
        u = None if a["uniforms"] is None else a["uniforms"][0]
        if mode == "sample":  # draft distributions close to the target's, so that the walk goes deep
            q = np.stack([0.97 * _softmax(a["logits"][0][par[k] + 1].astype(np.float64)) + 0.03 * q[k] for k in range(len(par))])
            for k in range(len(par)):  # first children carry their parent row's likeliest token: accepted almost surely
                if k == min(j for j in range(len(par)) if par[j] == par[k]) and seed % 3:
                    a["tokens"][0][k] = int(np.argmax(a["logits"][0][par[k] + 1]))
        full = accept_path(a["tokens"][0], par, a["logits"][0], mode, q, u)
        capped = accept_path(a["tokens"][0], par, a["logits"][0], mode, q, u, max_depth=cap)
        par_c, keep = _cut_tree(par, cap)
        rows = [0] + [k + 1 for k in keep]
        cut = accept_path(a["tokens"][0][keep], par_c, a["logits"][0][rows], mode,
                          None if q is None else q[keep], None if u is None else np.concatenate([u[keep], u[-1:]]))
        assert capped.path == [keep[k] for k in cut.path]
        assert capped.accept_len == cut.accept_len <= cap
        assert capped.bonus_token == cut.bonus_token
        assert capped.path == full.path[:cap]
        if full.accept_len > cap:
            hits += 1
            # the cap must not skip tokens: the token after the last kept node is drawn from that node's row
            if mode == "greedy":
                assert capped.bonus_token == int(np.argmax(a["logits"][0][capped.path[-1] + 1]))
        elif full.accept_len < cap:  # (at exactly `cap` the uncapped walk still tried the last node's children)
            assert capped.bonus_token == full.bonus_token
    assert hits >= 1, "the cap never cut a walk: the test would prove nothing"
