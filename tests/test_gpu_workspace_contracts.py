"""What the header promises of workspaces, tested as promised: an attention workspace, zero-filled once, serves
calls of any shapes, paths and plans in turn; the draft-side workspaces carry nothing from call to call (their
contents may be anything when a call starts)."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from gpu_util import tune
from workloads import CONFIGS, attention_inputs, draft_head_inputs, moe_inputs, paged_layout, round_to_bf16, tree_for_config

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def _dev(a, dtype=BF):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(dtype)


def test_attention_calls_of_any_shape_take_turns_on_one_workspace():
    """Shapes that merge their key splits inside the kernel (with different numbers of row-tile groups and splits),
    shapes that use the merge kernel, an unsplit call, a paged call and an fp32 call, in turn and twice over, on one
    workspace that was zero-filled once and whose partial area is refilled with noise before every call: each result
    equals the one on a fresh workspace bit for bit, and the error word stays clear."""
    dev = torch.device("cuda")
    # (name, batch, Hq, Hkv, D, T, L, dtype, splits forced, fused forced, paged page size)
    cases = [("c3_like", 1, 32, 8, 128, 60, 4096, "bf16", 0, -1, 0), ("c2_like", 1, 32, 32, 128, 60, 1024, "bf16", 0, -1, 0),
             ("five_splits", 2, 8, 2, 64, 33, 700, "bf16", 5, 1, 0), ("merge_kernel", 2, 8, 2, 128, 100, 900, "bf16", 3, 0, 0),
             ("unsplit", 3, 4, 4, 128, 17, 300, "bf16", 1, -1, 0), ("paged", 2, 8, 2, 128, 60, 1000, "bf16", 4, -1, 64),
             ("fp32", 2, 4, 2, 32, 24, 2500, "f32", 0, -1, 0), ("many_groups", 16, 32, 16, 64, 40, 200, "bf16", 2, 1, 0)]
    prepared = []
    need = 0
    for i, (name, B, Hq, Hkv, D, T, L, dtype, splits, fused, page) in enumerate(cases):
        cfg = CONFIGS["c3_llama3_8b"].with_(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_tree=T, prefix_len=L)
        par = tree_for_config(cfg, seed=50 + i)
        x = attention_inputs(cfg, seed=50 + i, scale_mult=np.sqrt(float(D)))
        tdt = torch.float32 if dtype == "f32" else BF
        if dtype == "bf16":
            x = {k: round_to_bf16(v) for k, v in x.items()}
        d = {k: _dev(v, tdt) for k, v in x.items()}
        extra = {}
        if page:
            (kp, vp), table = paged_layout(x["k_cache"], x["v_cache"], page, seed=i)
            extra = {"kp": _dev(kp), "vp": _dev(vp), "table": torch.from_numpy(table).to(dev)}
        lens = [L] + [max(0, L - 37 * (b + 1)) for b in range(B - 1)]
        tune("attn_splits", splits); tune("attn_fused", fused)   # (a forced split count changes the size asked for)
        need = max(need, jk.tree_verify_attention_workspace(d["q"], d["k_cache"], d["k_tree"], L))
        prepared.append((name, d, extra, torch.from_numpy(par).to(dev), torch.tensor(lens, dtype=torch.int32, device=dev), L,
                         splits, fused))
    shared = torch.zeros(need, dtype=torch.uint8, device=dev)
    gen = torch.Generator(device="cuda").manual_seed(3)

    def run(case, ws):
        name, d, extra, parent, pl, L, splits, fused = case
        tune("attn_splits", splits); tune("attn_fused", fused)
        if extra:
            out = jk.tree_verify_attention_paged(d["q"], extra["kp"], extra["vp"], extra["table"], d["k_tree"], d["v_tree"],
                                                 parent, pl, max_prefix_len=L, workspace=ws)
        else:
            out = jk.tree_verify_attention(d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], parent, pl,
                                           max_prefix_len=L, workspace=ws)
        torch.cuda.synchronize()
        return out

    for rnd in range(2):
        for case in prepared:
            shared[jk.JK_WORKSPACE_HEADER_BYTES:] = torch.randint(0, 256, (need - jk.JK_WORKSPACE_HEADER_BYTES,), dtype=torch.uint8,
                                                                  device=dev, generator=gen)
            got = run(case, shared)
            want = run(case, torch.zeros(need, dtype=torch.uint8, device=dev))
            assert torch.isfinite(want.float()).all(), case[0]
            assert torch.equal(got.view(torch.int16) if got.dtype == BF else got.view(torch.int32),
                               want.view(torch.int16) if want.dtype == BF else want.view(torch.int32)), (rnd, case[0])
            assert jk.last_device_error(shared) == 0, case[0]


def test_draft_side_workspaces_may_hold_anything():
    """jk_draft_heads and jk_moe_experts with workspaces full of 0xFF bytes (NaN patterns) against workspaces of
    zeros: the same outputs bit for bit, for two shapes in turn on the same buffers."""
    dev = torch.device("cuda")

    def heads(x, fill, top_k=8):
        R, _, d = x["f_top"].shape
        V = x["w_head"].shape[0]
        ws = torch.full((jk.draft_heads_workspace(R, d, V),), fill, dtype=torch.uint8, device=dev)
        lg = torch.empty((R, 2, V), dtype=torch.float32, device=dev)
        q = torch.empty_like(lg)
        tk = torch.empty((R, 2, top_k), dtype=torch.int32, device=dev)
        tp = torch.empty((R, 2, top_k), dtype=torch.float32, device=dev)
        call = jk.prepare_draft_heads(_dev(x["f_top"]), torch.from_numpy(x["s_top"]).to(dev), _dev(x["w_head"]),
                                      jk.JK_HEADS_DECOUPLED, 1.0, top_k, 0.0, 0.0, lg, q, tk, tp, ws)
        call.launch(); call.launch()
        torch.cuda.synchronize()
        return [lg, q, tk, tp]

    def experts(x, fill):
        R, d = x["u"].shape
        N, F = x["w_gate"].shape[0], x["w_gate"].shape[1]
        ws = torch.full((jk.moe_experts_workspace(R, d, F, N),), fill, dtype=torch.uint8, device=dev)
        f_top = torch.empty((R, 2, d), dtype=BF, device=dev)
        s_top = torch.empty((R, 2), dtype=torch.float32, device=dev)
        idx = torch.empty((R, 2), dtype=torch.int32, device=dev)
        f_mix = torch.empty((R, d), dtype=BF, device=dev)
        call = jk.prepare_moe_experts(_dev(x["u"]), _dev(x["centroids"]), _dev(x["w_gate"]), _dev(x["w_up"]), _dev(x["w_down"]),
                                      f_top, s_top, idx, f_mix, ws)
        call.launch(); call.launch()
        torch.cuda.synchronize()
        return [f_top, s_top, idx, f_mix]

    def same(a, b):
        for s, t in zip(a, b):
            assert torch.equal(s.contiguous().view(torch.uint8), t.contiguous().view(torch.uint8))

    for x in (draft_head_inputs(7, 512, 4099, seed=1), draft_head_inputs(40, 2048, 700, seed=2)):   # the second splits k
        same(heads(x, 0xFF), heads(x, 0))
    for x in (moe_inputs(5, 256, 384, 8, seed=3), moe_inputs(33, 128, 256, 4, seed=4)):
        same(experts(x, 0xFF), experts(x, 0))


def test_attention_calls_on_several_streams_at_once():
    """Calls with workspaces of their own may run on different streams at the same time.  Three streams of c3-shaped
    calls (each wants the whole chip for its 256 workgroups and merges its splits inside the kernel, waiting for
    partners that may not be resident yet: the wait is bounded and the last arriver finishes what others left) and one
    stream of sampling acceptance calls: every result equals the one computed alone, whatever the error words say
    about expired waits."""
    from workloads import accept_inputs
    dev = torch.device("cuda")
    cfg = CONFIGS["c3_llama3_8b"]
    par = tree_for_config(cfg)
    parent = torch.from_numpy(par).to(dev)
    plen = torch.tensor([cfg.prefix_len], dtype=torch.int32, device=dev)
    n_streams, n_rep = 3, 6
    layers = [{k: _dev(round_to_bf16(v)) for k, v in attention_inputs(cfg, layer=l, scale_mult=np.sqrt(128.0)).items()}
              for l in range(n_streams)]
    need = jk.tree_verify_attention_workspace(layers[0]["q"], layers[0]["k_cache"], layers[0]["k_tree"], cfg.prefix_len)
    alone = []
    for l in layers:
        alone.append(jk.tree_verify_attention(l["q"], l["k_cache"], l["v_cache"], l["k_tree"], l["v_tree"], parent, plen))
    acfg = CONFIGS["c3_llama3_8b"].with_(vocab=32000, batch=2)
    a = accept_inputs(acfg, np.broadcast_to(par, (2, par.shape[1])).copy(), seed=3)
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(dev)  # noqa: E731
    apar = t(np.broadcast_to(par, (2, par.shape[1])).copy())
    acc_in = [t(a["tokens"]), apar, t(a["logits"]), jk.JK_SAMPLE, 1.0, t(a["draft_probs"]), t(a["uniforms"])]
    acc_alone = jk.accept_path(*acc_in)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(n_streams + 1)]
    wss = [torch.zeros(need, dtype=torch.uint8, device=dev) for _ in range(n_streams)]
    outs = [[torch.empty_like(l["q"]) for _ in range(n_rep)] for l in layers]
    ws_acc = torch.zeros(jk.accept_path_workspace(2, par.shape[1], 32000, jk.JK_SAMPLE), dtype=torch.uint8, device=dev)
    acc_outs = []
    for rep in range(n_rep):
        for s, l in enumerate(layers):
            jk.tree_verify_attention(l["q"], l["k_cache"], l["v_cache"], l["k_tree"], l["v_tree"], parent, plen,
                                     out=outs[s][rep], workspace=wss[s], stream=streams[s])
        acc_outs.append(jk.accept_path(*acc_in, workspace=ws_acc, stream=streams[-1]))
    torch.cuda.synchronize()
    for s in range(n_streams):
        for rep in range(n_rep):
            assert torch.equal(outs[s][rep], alone[s]), (s, rep)
    for got in acc_outs:
        if int(got[1].min()) < 0:      # a walk that gave up says so (-1) and may simply be repeated
            assert jk.last_device_error(ws_acc) & jk.JK_DEVERR_WALK_WAIT
            continue
        for g, w in zip(got, acc_alone):
            assert torch.equal(g, w)
