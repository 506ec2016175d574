"""Pins for the draft-head oracle (Section 3.1.2 Eq. 2-5, Section 3.2 Eq. 6-8): library routines on
special cases, identities the equations imply, hand-worked numbers, brute force."""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import draft_head as dh
from workloads import draft_head_inputs, moe_inputs


def test_router_matches_library_softmax_and_ignores_common_offset():
    x = moe_inputs(6, 32, 48, 5, seed=1)
    s = dh.router_scores(x["u"], x["centroids"])
    ref = scipy.special.softmax(x["u"].astype(np.float64) @ x["centroids"].astype(np.float64).T, axis=1)
    np.testing.assert_allclose(s, ref, rtol=1e-13)
    np.testing.assert_allclose(s.sum(1), 1.0, rtol=1e-13)
    t = np.linspace(-1, 1, 32)
    np.testing.assert_allclose(dh.router_scores(x["u"], x["centroids"].astype(np.float64) + t), s, rtol=1e-10)
    # a centroid aligned with u gets the largest score
    e = np.array(x["centroids"], np.float64)
    e[3] = 4.0 * x["u"][2] / np.linalg.norm(x["u"][2])
    assert int(np.argmax(dh.router_scores(x["u"], e)[2])) == 3


def test_gate_keeps_the_k_largest_scores_ties_to_lower_index():
    s = np.array([[0.1, 0.4, 0.2, 0.3], [0.25, 0.25, 0.25, 0.25], [0.05, 0.05, 0.6, 0.3]])
    g, idx = dh.gate(s, 2)
    assert idx.tolist() == [[1, 3], [0, 1], [2, 3]]
    assert ((g != 0).sum(1) == 2).all()
    np.testing.assert_array_equal(g[0], [0, 0.4, 0, 0.3])
    rng = np.random.default_rng(0)
    s = rng.dirichlet(np.ones(8), size=20)
    g, idx = dh.gate(s, 2)
    np.testing.assert_allclose(np.sort(g, axis=1)[:, -2:], np.sort(s, axis=1)[:, -2:])
    assert (s[np.arange(20), idx[:, 0]] >= s[np.arange(20), idx[:, 1]]).all()


def test_expert_is_the_gated_mlp_of_the_library():
    x = moe_inputs(3, 32, 48, 2, seed=2)
    u = torch.tensor(x["u"], dtype=torch.float64)
    wg, wu, wd = (torch.tensor(x[k][1], dtype=torch.float64) for k in ("w_gate", "w_up", "w_down"))
    ref = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(u, wg))
                                     * torch.nn.functional.linear(u, wu), wd).numpy()
    for r in range(3):
        np.testing.assert_allclose(dh.expert_mlp(x["u"][r], x["w_gate"][1], x["w_up"][1], x["w_down"][1]), ref[r],
                                   rtol=1e-11, atol=1e-13)


def test_single_expert_is_a_dense_residual_mlp():
    x = moe_inputs(4, 32, 48, 1, seed=3)
    f, f_top, s_top, idx = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], x["w_down"], K=1)
    np.testing.assert_allclose(s_top, 1.0)
    assert (idx == 0).all()
    np.testing.assert_allclose(f, f_top[:, 0], rtol=1e-13)
    for r in range(4):
        np.testing.assert_allclose(f[r], dh.expert_mlp(x["u"][r], x["w_gate"][0], x["w_up"][0], x["w_down"][0])
                                   + x["u"][r], rtol=1e-13)


def test_mixture_identity_sparsity_and_expert_relabelling():
    x = moe_inputs(5, 32, 48, 6, seed=4)
    f, f_top, s_top, idx = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], x["w_down"])
    u = x["u"].astype(np.float64)
    # Eq. 3 written with the per-expert features: f = sum_k s_k (f_k - u) + u
    np.testing.assert_allclose(f, (s_top[:, :, None] * (f_top - u[:, None])).sum(1) + u, rtol=1e-12, atol=1e-13)
    assert (s_top[:, 0] >= s_top[:, 1]).all() and (s_top.sum(1) < 1.0).all()
    # experts that are not selected do not matter: poison them
    wd = np.array(x["w_down"], np.float64)
    for j in range(6):
        if j not in idx:
            wd[j] = np.nan
    f2, _, _, _ = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], wd)
    np.testing.assert_array_equal(f2, f)
    # relabelling the experts relabels idx and changes nothing else
    perm = np.array([3, 5, 0, 1, 4, 2])
    fp, ftp, stp, idp = dh.moe_features(x["u"], x["centroids"][perm], x["w_gate"][perm], x["w_up"][perm],
                                        x["w_down"][perm])
    np.testing.assert_allclose(fp, f, rtol=1e-12)
    np.testing.assert_allclose(ftp, f_top, rtol=1e-12)
    np.testing.assert_allclose(stp, s_top, rtol=1e-12)
    np.testing.assert_array_equal(perm[idp], idx)
    # an expert whose output projection is zero contributes the residual only
    wd0 = np.zeros_like(wd)
    _, ft0, _, _ = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], wd0)
    np.testing.assert_array_equal(ft0, np.broadcast_to(u[:, None], ft0.shape))


def test_head_hand_worked_example():
    # d = 2, V = 3; one hidden state
    f_top = np.array([[[1.0, 2.0], [3.0, -1.0]]])
    s_top = np.array([[0.5, 0.25]])
    w = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    lg = dh.dual_head_logits(f_top, s_top, w, dh.DECOUPLED)
    np.testing.assert_allclose(lg[0, 0], [0.5, 1.0, 1.5])
    np.testing.assert_allclose(lg[0, 1], [0.75, -0.25, 0.5])
    lg = dh.dual_head_logits(f_top, s_top, w, dh.CONTRASTIVE, alpha=0.5, beta=2.0)
    np.testing.assert_allclose(lg[0, 0], [1.25, 0.75, 2.0])          # 0.5 f1 + 0.25 f2 = (1.25, 0.75)
    np.testing.assert_allclose(lg[0, 1], [0.5, 4.5, 5.0])            # 2 f1 - 0.5 f2 = (0.5, 4.5)


def test_head_is_a_linear_layer_and_the_two_modes_agree_where_they_must():
    x = draft_head_inputs(5, 64, 300, seed=5)
    f, s, w = x["f_top"], x["s_top"], x["w_head"]
    ones = np.ones_like(s)
    ref = torch.nn.functional.linear(torch.tensor(f, dtype=torch.float64), torch.tensor(w, dtype=torch.float64)).numpy()
    np.testing.assert_allclose(dh.dual_head_logits(f, ones, w, dh.DECOUPLED), ref, rtol=1e-12, atol=1e-12)
    dec = dh.dual_head_logits(f, s, w, dh.DECOUPLED)
    np.testing.assert_allclose(dec, s.astype(np.float64)[:, :, None] * ref, rtol=1e-12, atol=1e-12)
    con = dh.dual_head_logits(f, s, w, dh.CONTRASTIVE, alpha=0.3, beta=1.1)
    # left + right = Head(f^moe) by linearity
    np.testing.assert_allclose(dec[:, 0] + dec[:, 1], con[:, 0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(con[:, 1], 1.1 * ref[:, 0] - 0.3 * ref[:, 1], rtol=1e-11, atol=1e-12)
    # beta = 1, alpha = 0: the second head sees the top-1 expert alone
    np.testing.assert_allclose(dh.dual_head_logits(f, s, w, dh.CONTRASTIVE, 0.0, 1.0)[:, 1], ref[:, 0],
                               rtol=1e-12, atol=1e-12)
    # identical experts and beta = alpha: nothing to contrast, uniform distribution, ties to low ids
    f_same = np.array(f)
    f_same[:, 1] = f_same[:, 0]
    lg, q, ids, qs = dh.draft_heads(f_same, s, w, dh.CONTRASTIVE, 1.0, 4, alpha=0.7, beta=0.7)
    np.testing.assert_array_equal(lg[:, 1], 0.0)
    np.testing.assert_allclose(q[:, 1], 1.0 / 300)
    assert (ids[:, 1] == np.arange(4)).all()


def test_identity_head_returns_the_scaled_features():
    x = draft_head_inputs(3, 16, 16, seed=6)
    lg = dh.dual_head_logits(x["f_top"], x["s_top"], np.eye(16), dh.DECOUPLED)
    np.testing.assert_allclose(lg, x["s_top"].astype(np.float64)[:, :, None] * x["f_top"], rtol=1e-13)


def test_distribution_matches_library_and_limits():
    rng = np.random.default_rng(7)
    lg = rng.normal(size=(3, 2, 50)) * 3
    q = dh.draft_distribution(lg, 0.7)
    np.testing.assert_allclose(q, scipy.special.softmax(lg / 0.7, axis=-1), rtol=1e-12)
    np.testing.assert_allclose(q.sum(-1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(dh.draft_distribution(lg + 5.0, 0.7), q, rtol=1e-10)
    np.testing.assert_allclose(dh.draft_distribution(lg, 1e9), 1.0 / 50, rtol=1e-6)
    cold = dh.draft_distribution(lg, 1e-3)
    assert (np.argmax(cold, -1) == np.argmax(lg, -1)).all() and np.allclose(cold.max(-1), 1.0)


def test_top_candidates_brute_force_and_ties():
    rng = np.random.default_rng(8)
    lg = np.round(rng.normal(size=(4, 2, 40)) * 2) / 2       # many ties
    ids = dh.top_candidates(lg, 6)
    for r in range(4):
        for h in range(2):
            row = lg[r, h].copy()
            for i in range(6):
                best = 0
                for v in range(40):          # first maximum
                    if row[v] > row[best]:
                        best = v
                assert ids[r, h, i] == best
                row[best] = -np.inf
    # the order of the logits is the order of the probabilities
    lg2 = rng.normal(size=(2, 2, 30))
    q = dh.draft_distribution(lg2, 1.3)
    np.testing.assert_array_equal(dh.top_candidates(lg2, 5), dh.top_candidates(q, 5))
    assert dh.top_k_desc([1.0, 3.0, 3.0, 2.0], 3).tolist() == [1, 2, 3]


@pytest.mark.parametrize("plant", ["dropped residual", "swapped scores"])
def test_planted_mistakes_are_caught(plant):
    x = moe_inputs(3, 32, 48, 4, seed=9)
    f, f_top, s_top, idx = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], x["w_down"])
    u = x["u"].astype(np.float64)
    if plant == "dropped residual":
        bad = (s_top[:, :, None] * (f_top - u[:, None])).sum(1)
        assert not np.allclose(bad, f)
    else:
        w = draft_head_inputs(3, 32, 100, seed=9)["w_head"]
        good = dh.dual_head_logits(f_top, s_top, w, dh.DECOUPLED)
        bad = dh.dual_head_logits(f_top, s_top[:, ::-1], w, dh.DECOUPLED)
        assert not np.allclose(good, bad)


def test_linear_and_attention_block_against_library_routines():
    rng = np.random.default_rng(11)
    x, w, r = rng.normal(size=(5, 16)), rng.normal(size=(7, 16)), rng.normal(size=(5, 7))
    ref = torch.nn.functional.linear(torch.tensor(x), torch.tensor(w)).numpy() + r
    np.testing.assert_allclose(dh.linear(x, w, r), ref, rtol=1e-13)
    # Eq. 1 on a chain of T nodes after L cached rows = causal attention of a decoder layer + residual
    T, L, H, D = 6, 9, 4, 8
    d = H * D
    h = rng.normal(size=(T, d))
    wq, wk, wv, wo = (rng.normal(size=(d, d)) / np.sqrt(d) for _ in range(4))
    kc, vc = rng.normal(size=(L, H, D)), rng.normal(size=(L, H, D))
    u = dh.draft_attention_block(h, wq, wk, wv, wo, kc, vc, np.arange(-1, T - 1), H, H)
    th = torch.tensor(h)
    q = torch.nn.functional.linear(th, torch.tensor(wq)).reshape(T, H, D).transpose(0, 1)
    k = torch.cat([torch.tensor(kc), torch.nn.functional.linear(th, torch.tensor(wk)).reshape(T, H, D)]).transpose(0, 1)
    v = torch.cat([torch.tensor(vc), torch.nn.functional.linear(th, torch.tensor(wv)).reshape(T, H, D)]).transpose(0, 1)
    mask = torch.ones(T, L + T, dtype=torch.bool).tril(diagonal=L)
    att = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask).transpose(0, 1).reshape(T, d)
    ref = torch.nn.functional.linear(att, torch.tensor(wo)).numpy() + h
    np.testing.assert_allclose(u, ref, rtol=1e-10, atol=1e-12)
