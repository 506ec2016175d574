"""GPU parity: jk_draft_heads (through the C ABI) against the draft-head oracle.

Logits: the library rounds the two head inputs to bf16 once (8 significant bits, round to nearest:
relative error at most 2^-8 per element) and accumulates products in fp32, so
|logit - oracle| <= (2^-8 + K 2^-23) * sum_k |x_k w_k| element by element.  The rounding errors are
independent and uniform within half a unit in the last place, i.e. of standard deviation at most
2^-7 / sqrt(12) relative to the element, so the root mean square of the logit errors must stay
below 2^-7 / sqrt(12) times the root mean square of sqrt(sum_k (x_k w_k)^2): a bound that a
systematic mistake sqrt(K) times smaller than the first one allows would still break.
Inputs whose products and sums are exact in fp32 must give the oracle's logits bit for bit.
Candidates are an integer decision taken on the library's own fp32 logits: they must equal the
oracle's selection applied to those logits exactly.  Probabilities: fp32 exp and a double
normaliser against the oracle's softmax of the same logits, relative 3e-5.
"""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import draft_head as dh
from workloads import draft_head_inputs

pytestmark = pytest.mark.gpu


def _call(x, mode=jk.JK_HEADS_DECOUPLED, temperature=1.0, top_k=5, alpha=0.0, beta=0.0, want_probs=True):
    f = torch.from_numpy(x["f_top"]).cuda().to(torch.bfloat16)
    s = torch.from_numpy(x["s_top"]).cuda()
    w = torch.from_numpy(x["w_head"]).cuda().to(torch.bfloat16)
    lg, q, tk, tp = jk.draft_heads(f, s, w, mode, temperature, top_k, alpha, beta, want_probs)
    torch.cuda.synchronize()
    return (lg.cpu().numpy(), None if q is None else q.cpu().numpy(), tk.cpu().numpy(), tp.cpu().numpy())


def _check(x, mode=jk.JK_HEADS_DECOUPLED, temperature=1.0, top_k=5, alpha=0.0, beta=0.0, exact=False):
    lg, q, tk, tp = _call(x, mode, temperature, top_k, alpha, beta)
    xin = dh.head_inputs(x["f_top"], x["s_top"], mode, alpha, beta)
    w = x["w_head"].astype(np.float64)
    ref = xin @ w.T
    K = w.shape[1]
    if exact:
        np.testing.assert_array_equal(lg.astype(np.float64), ref)
    else:
        bound = (2.0 ** -8 + K * 2.0 ** -23) * (np.abs(xin) @ np.abs(w).T) + 1e-30
        err = np.abs(lg - ref)
        assert (err <= bound).all(), f"worst ratio {np.max(err / bound):.3f}"
        spread = np.sqrt((xin * xin) @ (w * w).T)
        assert np.sqrt(np.mean(err ** 2)) <= 2.0 ** -7 / np.sqrt(12.0) * np.sqrt(np.mean(spread ** 2)) + 1e-30
    # decisions and probabilities from the library's own logits
    np.testing.assert_array_equal(tk, dh.top_candidates(lg, top_k))
    qref = dh.draft_distribution(lg, temperature)
    np.testing.assert_allclose(q, qref, rtol=3e-5, atol=1e-30)
    np.testing.assert_allclose(tp, np.take_along_axis(qref, tk.astype(np.int64), axis=-1), rtol=3e-5, atol=1e-30)
    return lg, q, tk, tp


def _exact_inputs(rows, d, vocab, seed):
    rng = np.random.default_rng(seed)
    return {"f_top": rng.integers(-2, 3, size=(rows, 2, d)).astype(np.float32),
            "s_top": np.stack([np.full(rows, 0.5), np.full(rows, 0.25)], 1).astype(np.float32),
            "w_head": (rng.integers(-1, 2, size=(vocab, d)) * 0.125).astype(np.float32)}


@pytest.mark.parametrize("rows,d,vocab", [(3, 256, 1000), (16, 128, 130), (17, 384, 4099), (128, 256, 513),
                                            (5, 1024, 3000), (40, 2048, 700), (90, 256, 600)])   # two of them split k
def test_exact_arithmetic_inputs_are_bit_exact(rows, d, vocab):
    _check(_exact_inputs(rows, d, vocab, rows), exact=True)
    _check(_exact_inputs(rows, d, vocab, rows + 1), mode=jk.JK_HEADS_CONTRASTIVE, alpha=0.5, beta=2.0, exact=True)


@pytest.mark.parametrize("rows", [1, 5, 16, 33, 40, 64, 80, 90, 100, 128])   # 1..8 row blocks of 32
def test_random_inputs_every_row_block_count(rows):
    _check(draft_head_inputs(rows, 512, 4096 + 37 * (rows % 4), seed=rows), top_k=10)


def test_widest_model_and_longest_candidate_lists():
    """d_model 16 384 and top-16, the largest the call takes (a small vocabulary keeps the oracle quick)."""
    _check(draft_head_inputs(3, 16384, 300, seed=5), top_k=16)
    _check(_exact_inputs(2, 16384, 257, 6), top_k=16, exact=True)


@pytest.mark.parametrize("mode,alpha,beta", [(jk.JK_HEADS_DECOUPLED, 0, 0), (jk.JK_HEADS_CONTRASTIVE, 0.3, 1.1),
                                             (jk.JK_HEADS_CONTRASTIVE, -0.25, 0.5)])
@pytest.mark.parametrize("temperature", [1.0, 0.6, 2.5])
def test_modes_and_temperatures(mode, alpha, beta, temperature):
    _check(draft_head_inputs(24, 1024, 32000, seed=11), mode, temperature, 10, alpha, beta)


def test_left_plus_right_is_the_mixture_head():
    x = _exact_inputs(8, 256, 777, 3)
    dec = _call(x)[0]
    con = _call(x, jk.JK_HEADS_CONTRASTIVE, alpha=1.0, beta=1.0)[0]
    np.testing.assert_array_equal(dec[:, 0] + dec[:, 1], con[:, 0])


def test_all_equal_logits_take_the_lowest_ids_and_a_uniform_distribution():
    x = draft_head_inputs(4, 256, 9000, seed=5)      # more ties than the candidate list holds
    x["f_top"][:, 1] = x["f_top"][:, 0]
    lg, q, tk, tp = _check(x, jk.JK_HEADS_CONTRASTIVE, alpha=0.75, beta=0.75, top_k=16)
    assert (lg[:, 1] == 0).all() and (tk[:, 1] == np.arange(16)).all()
    np.testing.assert_allclose(q[:, 1], 1.0 / 9000, rtol=1e-6)


def test_duplicated_embedding_rows_tie_towards_the_lower_id():
    # exact-arithmetic inputs: workgroups sum over k in different orders, so only sums without
    # rounding are guaranteed to agree bit for bit between the two copies of a row
    x = _exact_inputs(6, 256, 2048, 6)
    x["w_head"][1024:] = x["w_head"][:1024]
    lg, q, tk, tp = _check(x, top_k=8, exact=True)
    assert (lg[:, :, 1024:] == lg[:, :, :1024]).all()
    best = tk[:, :, 0]
    assert (best < 1024).all()        # of two equal logits the lower id comes first


def test_decoupled_heads_do_not_see_the_other_expert():
    x = draft_head_inputs(5, 256, 1500, seed=7)
    ref = _call(x)[0]
    x["f_top"][2, 1] = np.nan
    got = _call(x)[0]
    np.testing.assert_array_equal(got[:, 0], ref[:, 0])
    assert np.isnan(got[2, 1]).all() and np.isfinite(np.delete(got[:, 1], 2, axis=0)).all()


def test_probabilities_are_optional_and_rows_are_independent():
    x = draft_head_inputs(9, 256, 3000, seed=8)
    a = _call(x, top_k=4)
    b = _call(x, top_k=4, want_probs=False)
    assert b[1] is None
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[2], b[2])
    np.testing.assert_array_equal(a[3], b[3])
    sub = {"f_top": x["f_top"][3:4], "s_top": x["s_top"][3:4], "w_head": x["w_head"]}
    np.testing.assert_array_equal(_call(sub, top_k=4)[0][0], a[0][3])


def test_argument_errors():
    x = draft_head_inputs(2, 256, 300, seed=9)
    f = torch.from_numpy(x["f_top"]).cuda().to(torch.bfloat16)
    s = torch.from_numpy(x["s_top"]).cuda()
    w = torch.from_numpy(x["w_head"]).cuda().to(torch.bfloat16)
    for kw, status in [(dict(temperature=0.0), 1), (dict(top_k=17), 3), (dict(top_k=0), 1), (dict(top_k=301), 1),
                       (dict(mode=2), 1), (dict(mode=1, alpha=float("nan")), 1)]:
        with pytest.raises(jk.JakiroError) as e:
            jk.draft_heads(f, s, w, **kw)
        assert e.value.status == status, kw
    with pytest.raises(jk.JakiroError) as e:       # d_model not a multiple of 128
        jk.draft_heads(f[:, :, :192].contiguous(), s, w[:, :192].contiguous())
    assert e.value.status == 3
    f129 = torch.zeros((129, 2, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(jk.JakiroError) as e:
        jk.draft_heads(f129, torch.zeros((129, 2), device="cuda"), w)
    assert e.value.status == 3
    # workspace too small / missing
    R, d, V = 2, 256, 300
    lg = torch.empty((R, 2, V), device="cuda")
    tk = torch.empty((R, 2, 3), dtype=torch.int32, device="cuda")
    tp = torch.empty((R, 2, 3), device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(jk.JakiroError) as e:
        jk.prepare_draft_heads(f, s, w, 0, 1.0, 3, 0.0, 0.0, lg, None, tk, tp, small).launch()
    assert e.value.status == 4
    torch.cuda.synchronize()


def test_full_size_llama3_shape_sampled_against_the_oracle():
    """The shape the benchmark times: 80 hidden states (8 sequences x 10 expanded nodes), d = 4096, the
    128 256-token vocabulary.  Logits against the oracle on sampled vocabulary rows (including both
    ends of the last, ragged 128-row strip); candidates and probabilities on every row."""
    R, d, V, k = 80, 4096, 128256, 10
    x = draft_head_inputs(R, d, V, seed=12)
    lg, q, tk, tp = _call(x, temperature=1.0, top_k=k)
    rng = np.random.default_rng(0)
    ids = np.unique(np.concatenate([rng.integers(0, V, 1500), np.arange(0, 130), np.arange(V - 130, V)]))
    xin = dh.head_inputs(x["f_top"], x["s_top"], dh.DECOUPLED)
    w = x["w_head"][ids].astype(np.float64)
    ref = xin @ w.T
    bound = (2.0 ** -8 + d * 2.0 ** -23) * (np.abs(xin) @ np.abs(w).T)
    err = np.abs(lg[:, :, ids] - ref)
    assert (err <= bound).all()
    spread = np.sqrt((xin * xin) @ (w * w).T)
    assert np.sqrt(np.mean(err ** 2)) <= 2.0 ** -7 / np.sqrt(12.0) * np.sqrt(np.mean(spread ** 2))
    np.testing.assert_array_equal(tk, dh.top_candidates(lg, k))
    qref = dh.draft_distribution(lg, 1.0)
    np.testing.assert_allclose(q, qref, rtol=3e-5, atol=1e-30)
    np.testing.assert_allclose(tp, np.take_along_axis(qref, tk.astype(np.int64), axis=-1), rtol=3e-5)


def test_rows_with_fewer_finite_logits_than_candidates():
    """Only three tokens of the vocabulary have logits above -inf (the other embedding rows carry -inf against a
    positive feature): they come first, best first, with probabilities that sum to one; the remaining places of the
    candidate lists report token 0 with probability 0, and every other draft probability is an exact zero."""
    rows, d, V, k = 3, 256, 1500, 6
    x = draft_head_inputs(rows, d, V, seed=21)
    x["f_top"] = np.abs(x["f_top"]).astype(np.float32) + 0.5       # positive features
    x["s_top"] = np.full((rows, 2), 0.5, dtype=np.float32)
    w = x["w_head"].copy()
    alive = [7, 900, 1499]
    for v in range(V):
        if v not in alive:
            w[v] = 0.0
            w[v, 0] = -np.inf
    x["w_head"] = w
    lg, q, tk, tp = _call(x, top_k=k)
    dead = np.setdiff1d(np.arange(V), alive)
    assert np.isneginf(lg[:, :, dead]).all() and np.isfinite(lg[:, :, alive]).all()
    assert (q[:, :, dead] == 0).all()
    np.testing.assert_allclose(q[:, :, alive].sum(-1), 1.0, rtol=1e-6)
    for r in range(rows):
        for h in range(2):
            order = sorted(alive, key=lambda v: (-lg[r, h, v], v))
            assert tk[r, h, :3].tolist() == order
            np.testing.assert_allclose(tp[r, h, :3], q[r, h, order], rtol=1e-6)
            assert (tk[r, h, 3:] == 0).all() and (tp[r, h, 3:] == 0).all()
