"""GPU parity on seeded random shapes: jk_tree_verify_attention (bf16), jk_accept_path and the draft-side
calls against the oracles, over batch sizes, head groupings, head widths, tree sizes and shapes, ragged prefix lengths,
cache capacities above the lengths, both wave arrangements and forced split counts (including more splits
than tiles), with an occasional key far above every other score of one query row (the fast path of the
4x1 arrangement then has to repeat its split on the general path).  Same bounds as the fixed cases: 2e-2
absolute for bf16 attention (3 * 2^-8 max|v| where that is larger: inputs here are not scaled down like the
workloads') and 2e-2 relative to max|out|; acceptance bit-exact on seeds whose decisions have a margin above 1e-9."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import accept_path as oracle_accept
from workloads import CONFIGS, accept_inputs, attention_inputs, round_to_bf16

pytestmark = pytest.mark.gpu

from gpu_util import gpu_attention, oracle_attention, reset_tuning, tune  # noqa: E402


def _random_parents(rng, B, T, reach):
    return np.stack([np.array([-1] + [int(rng.integers(max(-1, i - 1 - int(rng.integers(0, reach))), i))
                                      for i in range(1, T)], dtype=np.int32) for _ in range(B)])


@pytest.mark.parametrize("block", range(8))
def test_attention_random_shapes(monkeypatch, block):
    for case in range(block * 25, block * 25 + 25):
        rng = np.random.default_rng(991 * 100003 + case)
        B = int(rng.integers(1, 4))
        Hkv = int(rng.choice([1, 2, 3, 4]))
        G = int(rng.choice([1, 2, 4, 8]))
        D = int(rng.choice([64, 128]))
        T = int(rng.integers(1, 129))
        Lmax = int(rng.choice([0, 5, 40, 200, 700, 1500, 2600]))
        lens = [int(rng.integers(0, Lmax + 1)) for _ in range(B)]
        lens[int(rng.integers(0, B))] = Lmax
        cap = Lmax + int(rng.integers(0, 3)) * 7
        par = _random_parents(rng, B, T, 12)
        arr = [None, (2, 2), (4, 1)][int(rng.integers(0, 3))]
        splits = int(rng.choice([0, 0, 1, 2, 3, 5, 8, 16, 33]))
        reset_tuning()
        if arr is not None:
            tune("attn_wm", str(arr[0]))
            tune("attn_wn", str(arr[1]))
        if splits:
            tune("attn_splits", str(splits))
        cfg = CONFIGS["c3_llama3_8b"].with_(batch=B, n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D,
                                             prefix_len=max(cap, 1), n_tree=T)
        x = attention_inputs(cfg, seed=case, scale_mult=np.sqrt(float(D)))
        planted = bool(rng.random() < 0.25) and Lmax > 0
        if planted:
            b = int(rng.integers(0, B))
            pos = int(rng.integers(0, max(lens[b], 1)))
            kvh = int(rng.integers(0, Hkv))
            node, hq = int(rng.integers(0, T)), kvh * G + int(rng.integers(0, G))
            if lens[b] > 0:
                x["k_cache"][b, pos, kvh] = round_to_bf16(float(rng.choice([4.0, 8.0, 16.0])) * x["q"][b, node, hq]
                                                          * (128.0 / D) ** 0.5)
        what = f"case {case}: B{B} Hkv{Hkv} G{G} D{D} T{T} lens{lens} cap{cap} arr{arr} splits{splits} planted{planted}"
        ref = oracle_attention(**x, parent=par, prefix_len=lens, scale=None)
        got = gpu_attention(x, par, lens, "bf16")
        assert np.isfinite(got).all(), what
        err = np.abs(got - ref).max()
        # Inputs here are N(0, 1), not the workloads' 0.09: rows that see few keys, or one key far above the
        # rest, return (nearly) single V rows.  An output is sum_j p_j v_j / l with the p_j rounded to bf16,
        # the split partial rounded to bf16 and the result rounded to bf16 (unit roundoff 2^-8 each), so its
        # error is at most 3 * 2^-8 * max|v| (a near one-hot row whose largest weight is not a power of two really
        # shows the first of the three: the numerator carries the rounded weight, the denominator the exact one); the relative bound is the workloads' 2e-2.
        peak_v = max(np.abs(x["v_cache"]).max() if Lmax > 0 else 0.0, np.abs(x["v_tree"]).max())
        peak = np.abs(ref).max()
        assert err <= max(2e-2, 3 * 2.0 ** -8 * peak_v) and err <= 2e-2 * max(peak, 1e-30), f"{what}: error {err:.3e}"


@pytest.mark.parametrize("block", range(4))
def test_accept_random_shapes(monkeypatch, block):
    dev = torch.device("cuda")
    compared = 0
    for case in range(block * 25, block * 25 + 25):
        rng = np.random.default_rng(577 * 100003 + case)
        B = int(rng.choice([1, 1, 2, 3, 8]))
        T = int(rng.integers(1, 129))
        V = int(rng.choice([2, 17, 257, 1000, 4096, 5001, 32000]))
        mode = "greedy" if rng.random() < 0.3 else "sample"
        temp = float(rng.choice([1.0, 1.0, 0.5, 1.7]))
        closeness = float(rng.choice([0.0, 0.3, 0.7, 2.0]))
        if V >= 32000:
            B = min(B, 2)
        reset_tuning()
        if rng.random() < 0.25:
            tune("accept_single", "1")
        par = _random_parents(rng, B, T, 10)
        cfg = CONFIGS["c3_llama3_8b"].with_(vocab=V, batch=B, n_tree=T, mode=mode, hit_prob=0.0)
        a = accept_inputs(cfg, par, seed=case)
        if mode == "greedy":       # plant hits of the parent row's top-1 so that chains form
            for b in range(B):
                for k in range(T):
                    if rng.random() < 0.6:
                        a["tokens"][b, k] = int(np.argmax(a["logits"][b, par[b, k] + 1]))
        elif closeness > 0:        # draft distributions near the target's: the walk goes deep
            for b in range(B):
                for k in range(T):
                    z = a["logits"][b, par[b, k] + 1].astype(np.float64) / temp + rng.standard_normal(V) * closeness
                    e = np.exp(z - z.max())
                    qq = (e / e.sum()).astype(np.float32)
                    a["draft_probs"][b, k] = qq
                    cdf = np.cumsum(qq, dtype=np.float64)
                    a["tokens"][b, k] = min(int(np.searchsorted(cdf, rng.random() * cdf[-1], side="right")), V - 1)
        t = lambda v: None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(dev)  # noqa: E731
        path, alen, bonus = jk.accept_path(t(a["tokens"]), t(par), t(a["logits"]),
                                           jk.JK_GREEDY if mode == "greedy" else jk.JK_SAMPLE, temp,
                                           t(a["draft_probs"]), t(a["uniforms"]))
        torch.cuda.synchronize()
        path, alen, bonus = path.cpu().numpy(), alen.cpu().numpy(), bonus.cpu().numpy()
        what = f"case {case}: B{B} T{T} V{V} {mode} temp{temp} close{closeness}"
        for b in range(B):
            r = oracle_accept(a["tokens"][b], par[b], a["logits"][b], mode,
                              None if a["draft_probs"] is None else a["draft_probs"][b],
                              None if a["uniforms"] is None else a["uniforms"][b], temp)
            if mode == "sample" and r.min_margin <= 1e-9:
                continue
            compared += 1
            assert alen[b] == r.accept_len, what
            assert path[b, : alen[b]].tolist() == r.path, what
            assert (path[b, alen[b]:] == -1).all(), what
            assert bonus[b] == r.bonus_token, what
    assert compared >= 20


@pytest.mark.parametrize("seed", range(3))
def test_draft_side_random_shapes(seed):
    """The draft-side calls on random shapes within their documented limits, checked with the fixed cases'
    own helpers (bounds and decisions as described there)."""
    import test_gpu_draft_head as heads
    import test_gpu_draft_tree as tree
    import test_gpu_linear as lin
    import test_gpu_moe_experts as moe
    from oracle import draft_head as dh
    from workloads import draft_head_inputs, moe_inputs
    rng = np.random.default_rng(4242 + seed)
    for i in range(4):
        rows, d = int(rng.integers(1, 129)), 128 * int(rng.integers(1, 9))
        V, k = int(rng.integers(17, 20000)), int(rng.integers(1, 17))
        mode, temp = int(rng.integers(0, 2)), float(rng.uniform(0.3, 3.0))
        heads._check(draft_head_inputs(rows, d, V, seed=10 * seed + i), mode, temp, k, 0.4, 0.9)
        heads._check(heads._exact_inputs(rows, d, V, 10 * seed + i), exact=True, top_k=min(k, 5))
    for i in range(3):
        rows, d = int(rng.integers(1, 129)), 128 * int(rng.integers(1, 5))
        f, n = 128 * int(rng.integers(1, 9)), int(rng.integers(2, 10))
        x = moe_inputs(rows, d, f, n, seed=100 + 10 * seed + i)
        s = dh.router_scores(x["u"], x["centroids"])
        srt = -np.sort(-s, axis=1)
        gaps = np.minimum(srt[:, 0] - srt[:, 1], srt[:, 1] - srt[:, 2] if n > 2 else np.inf)
        if (gaps > 1e-4).all():       # (a row whose top-2 choice hangs on the last bits cannot be compared)
            moe._check(x)
    for i in range(3):
        B, k = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        width, depth = min(int(rng.integers(1, 9)), 2 * k), int(rng.integers(1, 6))
        if width * 2 * k > 256:
            continue
        mx = int(rng.integers(16, 1025))
        keep = int(rng.integers(1, min(mx, 128) + 1))
        tree._run_round(200 + 10 * seed + i, B, depth, k, width, mx, keep, ties=bool(i % 2))
    for i in range(3):
        lin.test_exact_arithmetic_inputs_are_bit_exact(int(rng.integers(1, 257)), int(rng.integers(1, 3000)),
                                                       128 * int(rng.integers(1, 17)))
