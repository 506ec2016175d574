"""GPU parity: jk_moe_experts (through the C ABI) against the draft-head oracle (Eq. 2, 3, 5).

Tolerances, derived from the arithmetic of the library (bf16 operands, fp32 accumulation, the hidden
activation h = silu(gate)*up and the outputs rounded to bf16 once each, unit roundoff 2^-8):
  gate/up projections   dg, du = K 2^-23 sum_k |x_k w_k|                       (fp32 accumulation only)
  hidden activation     dh = 2^-8 |h| + 1.1 |up| dg + |silu(g)| du + 2^-22 |h| (rounding + propagated + expf)
  expert output         dy = dh . |w_down| + F 2^-23 sum |h w_down|
  f_top = y + u         df = dy + 2^-8 |f_top|
and the root mean square of the errors must stay near what independent roundings give.
The router's choice is an integer decided by fp32 dot products: it is compared with the oracle's on
rows whose decisive score gaps exceed 1e-4 (all rows of the seeds used here, asserted).
"""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import draft_head as dh
from workloads import draft_head_inputs, moe_inputs

pytestmark = pytest.mark.gpu

U = 2.0 ** -8


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(torch.bfloat16)


def _call(x, want_mix=True):
    f_top, s_top, idx, f_mix = jk.moe_experts(_dev(x["u"]), _dev(x["centroids"]), _dev(x["w_gate"]), _dev(x["w_up"]),
                                              _dev(x["w_down"]), want_mix)
    torch.cuda.synchronize()
    return (f_top.float().cpu().numpy().astype(np.float64), s_top.cpu().numpy().astype(np.float64), idx.cpu().numpy(),
            None if f_mix is None else f_mix.float().cpu().numpy().astype(np.float64))


def _expert_with_bounds(u, wg, wu, wd):
    """Oracle expert output for one row and the error bound dy of the library's arithmetic."""
    K, F = u.shape[0], wg.shape[0]
    g, up = wg @ u, wu @ u
    dg, du = K * 2.0 ** -23 * (np.abs(wg) @ np.abs(u)), K * 2.0 ** -23 * (np.abs(wu) @ np.abs(u))
    sg = g / (1.0 + np.exp(-g))
    h = sg * up
    d_h = U * np.abs(h) + 1.1 * np.abs(up) * dg + np.abs(sg) * du + 2.0 ** -22 * np.abs(h)
    y = wd @ h
    dy = np.abs(wd) @ d_h + F * 2.0 ** -23 * (np.abs(wd) @ np.abs(h))
    spread = np.sqrt((wd * wd) @ (h * h))          # rms scale of the bf16 rounding of h seen through w_down
    return y, dy, spread


def _check(x, min_gap=1e-4):
    f_top, s_top, idx, f_mix = _call(x)
    u = x["u"].astype(np.float64)
    wg, wu, wd = (x[k].astype(np.float64) for k in ("w_gate", "w_up", "w_down"))
    s = dh.router_scores(x["u"], x["centroids"])
    _, ref_idx = dh.gate(s, 2)
    srt = -np.sort(-s, axis=1)
    gaps = np.minimum(srt[:, 0] - srt[:, 1], srt[:, 1] - srt[:, 2] if s.shape[1] > 2 else np.inf)
    assert (gaps > min_gap).all(), "seed with an undecidable router row: pick another"
    np.testing.assert_array_equal(idx, ref_idx)
    np.testing.assert_allclose(s_top, np.take_along_axis(s, ref_idx, axis=1), rtol=2e-5, atol=1e-7)
    errs, scales = [], []
    for r in range(u.shape[0]):
        ys, dys = [], []
        for k in range(2):
            j = int(ref_idx[r, k])
            y, dy, spread = _expert_with_bounds(u[r], wg[j], wu[j], wd[j])
            f_ref = y + u[r]
            err = np.abs(f_top[r, k] - f_ref)
            assert (err <= dy + U * np.abs(f_ref) + 1e-30).all(), (r, k, float(np.max(err / (dy + U * np.abs(f_ref)))))
            errs.append(err)
            scales.append(np.sqrt(spread ** 2 + f_ref ** 2))
            ys.append(y)
            dys.append(dy)
        mix_ref = s_top[r, 0] * ys[0] + s_top[r, 1] * ys[1] + u[r]
        tol = s_top[r, 0] * dys[0] + s_top[r, 1] * dys[1] + U * np.abs(mix_ref) + 1e-6 * (np.abs(ys[0]) + np.abs(ys[1]))
        assert (np.abs(f_mix[r] - mix_ref) <= tol + 1e-30).all()
    rms_err = np.sqrt(np.mean(np.square(errs)))
    rms_scale = np.sqrt(np.mean(np.square(scales)))
    assert rms_err <= 2.0 ** -7 / np.sqrt(12.0) * rms_scale * 1.05
    return f_top, s_top, idx, f_mix


@pytest.mark.parametrize("rows,d,f,n", [(1, 256, 384, 8), (7, 256, 384, 4), (33, 128, 256, 2), (80, 256, 512, 8),
                                        (128, 384, 128, 5)])
def test_against_the_oracle(rows, d, f, n):
    _check(moe_inputs(rows, d, f, n, seed=rows))


def test_sixty_four_experts():
    """The largest expert count the call takes: most experts are chosen by nobody and are skipped."""
    _check(moe_inputs(6, 256, 256, 64, seed=6))


def test_model_like_widths():
    _check(moe_inputs(40, 1024, 2816, 8, seed=2))


def test_experts_nobody_selected_are_not_evaluated():
    x = moe_inputs(2, 256, 384, 8, seed=3)
    ref = _call(x)
    used = set(ref[2].reshape(-1).tolist())
    assert len(used) < 8
    for j in range(8):
        if j not in used:
            x["w_down"][j] = np.nan
            x["w_gate"][j] = np.nan
    got = _call(x)
    for a, b in zip(ref, got):
        np.testing.assert_array_equal(a, b)
    assert np.isfinite(got[0]).all()


def test_mixture_is_optional_and_rows_are_independent():
    x = moe_inputs(9, 256, 384, 4, seed=4)
    a = _call(x)
    b = _call(x, want_mix=False)
    assert b[3] is None
    for i in range(3):
        np.testing.assert_array_equal(a[i], b[i])
    sub = dict(x, u=x["u"][4:5])
    c = _call(sub)
    np.testing.assert_array_equal(c[0][0], a[0][4])
    np.testing.assert_array_equal(c[2][0], a[2][4])


def test_zero_output_projection_leaves_the_residual():
    x = moe_inputs(6, 256, 384, 4, seed=5)
    x["w_down"][:] = 0
    f_top, s_top, idx, f_mix = _call(x)
    np.testing.assert_array_equal(f_top, np.broadcast_to(x["u"].astype(np.float64)[:, None], f_top.shape))
    np.testing.assert_array_equal(f_mix, x["u"].astype(np.float64))


def test_experts_feed_the_heads_on_the_device():
    """u -> experts -> both heads without leaving the GPU; the first candidate of every head equals the fp64
    oracle's on rows where the oracle's best two logits are further apart than the bf16 error can bridge."""
    x = moe_inputs(12, 256, 512, 4, seed=6)
    w_head = draft_head_inputs(1, 256, 3000, seed=6)["w_head"]
    f_top, s_top, idx, _ = jk.moe_experts(_dev(x["u"]), _dev(x["centroids"]), _dev(x["w_gate"]), _dev(x["w_up"]),
                                          _dev(x["w_down"]), False)
    lg, q, tk, tp = jk.draft_heads(f_top, s_top, _dev(w_head), jk.JK_HEADS_DECOUPLED, 1.0, 5)
    torch.cuda.synchronize()
    _, f_ref, s_ref, _ = dh.moe_features(x["u"], x["centroids"], x["w_gate"], x["w_up"], x["w_down"])
    ref = dh.dual_head_logits(f_ref, s_ref, w_head, dh.DECOUPLED)
    got = lg.cpu().numpy()
    err = np.abs(got - ref).max()
    assert err <= 0.05 * np.abs(ref).max()
    srt = -np.sort(-ref, axis=-1)
    sure = (srt[..., 0] - srt[..., 1]) > 3.0 * err
    assert sure.sum() >= 4
    assert (tk.cpu().numpy()[..., 0][sure] == np.argmax(ref, axis=-1)[sure]).all()


def test_argument_errors():
    x = moe_inputs(2, 256, 384, 4, seed=7)
    a = [_dev(x[k]) for k in ("u", "centroids", "w_gate", "w_up", "w_down")]
    with pytest.raises(jk.JakiroError) as e:      # one expert only: no top-2
        jk.moe_experts(a[0], a[1][:1].contiguous(), a[2][:1].contiguous(), a[3][:1].contiguous(), a[4][:1].contiguous())
    assert e.value.status in (1, 3)
    with pytest.raises(jk.JakiroError) as e:      # d_ff not a multiple of 128
        jk.moe_experts(a[0], a[1], a[2][:, :320].contiguous(), a[3][:, :320].contiguous(), a[4][:, :, :320].contiguous())
    assert e.value.status == 3
    f_top = torch.empty((2, 2, 256), dtype=torch.bfloat16, device="cuda")
    s_top = torch.empty((2, 2), device="cuda")
    idx = torch.empty((2, 2), dtype=torch.int32, device="cuda")
    small = torch.empty(512, dtype=torch.uint8, device="cuda")
    with pytest.raises(jk.JakiroError) as e:
        jk.prepare_moe_experts(*a, f_top, s_top, idx, None, small).launch()
    assert e.value.status == 4
    torch.cuda.synchronize()


def test_draft_step_captured_in_a_hip_graph_replays_bit_for_bit():
    """Experts -> heads as prepared calls sharing their workspaces, captured in a HIP graph and replayed with
    eager work between the replays: every replay reproduces the eager results bit for bit (stale workspace
    contents must not matter: partial sums and candidate lists are rewritten by every call)."""
    R, d, F, N, V, k = 24, 512, 1024, 4, 9000, 8
    x = moe_inputs(R, d, F, N, seed=8)
    w_head = _dev(draft_head_inputs(1, d, V, seed=8)["w_head"])
    a = [_dev(x[key]) for key in ("u", "centroids", "w_gate", "w_up", "w_down")]
    dev = "cuda"
    f_top = torch.empty((R, 2, d), dtype=torch.bfloat16, device=dev)
    s_top = torch.empty((R, 2), device=dev)
    idx = torch.empty((R, 2), dtype=torch.int32, device=dev)
    lg = torch.empty((R, 2, V), device=dev)
    q = torch.empty((R, 2, V), device=dev)
    tk = torch.empty((R, 2, k), dtype=torch.int32, device=dev)
    tp = torch.empty((R, 2, k), device=dev)
    ws1 = torch.empty(jk.moe_experts_workspace(R, d, F, N), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(jk.draft_heads_workspace(R, d, V), dtype=torch.uint8, device=dev)
    c1 = jk.prepare_moe_experts(*a, f_top, s_top, idx, None, ws1)
    c2 = jk.prepare_draft_heads(f_top, s_top, w_head, jk.JK_HEADS_CONTRASTIVE, 0.8, k, 0.3, 1.1, lg, q, tk, tp, ws2)
    c1.launch()
    c2.launch()
    torch.cuda.synchronize()
    outs = (f_top, s_top, idx, lg, q, tk, tp)
    eager = [o.clone() for o in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        c1.launch()
        c2.launch()
    for rep in range(3):
        for o in outs:
            o.zero_()
        ws1.random_(0, 255)
        ws2.random_(0, 255)
        junk = torch.randn(1 << 20, device=dev).sum()
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), f"replay {rep} differs from the eager result"
        assert torch.isfinite(junk)
