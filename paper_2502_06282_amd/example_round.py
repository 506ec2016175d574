"""One speculative-decoding round (Section 2.1: draft, verify, refine) strung together from the library's
calls, with random weights and a synthetic target model: what a serving loop does per round, and in
which order.  Run on an MI355X:  python -m paper_2502_06282_amd.example_round

  draft, per depth      jk_linear (reduction layer and q/k/v/o projections of Eq. 1) + jk_tree_verify_attention over
                        the draft layer's own cache and the partial draft tree (a node attends to the committed
                        prefix and to its draft ancestors, Section 3.1.1) -> jk_moe_experts (Eq. 2, 3, 5) ->
                        jk_draft_heads (Eq. 4) -> jk_tree_grow
  after the last depth  jk_tree_finalize
  verify                jk_tree_verify_attention per target layer (the target's projections and MLPs are not
                        part of this library: q/k/v and the logits are random here)
  refine                jk_accept_path_rows (speculative sampling against the draft passes' distributions, addressed
                        through the tree's row table), jk_commit_path

The three phases allocate nothing that outlives them and read no result on the host, so each can be captured
as a HIP graph and replayed (`Round.capture`, `Round.time_phases`).  torch is used for device memory, random
numbers, row gathers and concatenations of the hidden states; every step of the method itself runs in the library.
"""
from __future__ import annotations

import argparse

import torch

import paper_2502_06282_amd as jk

SHAPES = {
    # small: runs in a blink, for tests
    "small": dict(batch=2, d_model=512, n_heads=4, n_kv_heads=4, head_dim=128, d_ff=512, n_experts=4, vocab=8000, depth=4,
                  top_k=4, width=4, n_tree=24, prefix=256, target_layers=2),
    # the shapes of an 8B model with a 128K vocabulary: the tree of Section 3.1.2 (depth 6, five candidates per head,
    # five nodes expanded per depth, 60 nodes kept), 32 target layers with grouped-query attention
    "llama3_8b": dict(batch=1, d_model=4096, n_heads=32, n_kv_heads=8, head_dim=128, d_ff=4096, n_experts=8, vocab=128256,
                      depth=6, top_k=5, width=5, n_tree=60, prefix=4096, target_layers=32),
}


class Round:
    """Weights, caches and buffers of one round; `draft()`, `verify()`, `refine()` enqueue its three phases."""

    def __init__(self, batch=2, d_model=512, n_heads=4, n_kv_heads=4, head_dim=128, d_ff=512, n_experts=4, vocab=8000,
                 depth=4, top_k=4, width=4, n_tree=24, prefix=256, target_layers=2, seed=0):
        dev = self.dev = torch.device("cuda")
        g = torch.Generator(device=dev).manual_seed(seed)
        bf = torch.bfloat16
        rn = lambda *shape, sc=1.0: (torch.randn(shape, device=dev, generator=g) * sc).to(bf)
        d = d_model
        assert n_heads * head_dim == d
        self.cfg = dict(batch=batch, d_model=d, n_heads=n_heads, n_kv_heads=n_kv_heads, head_dim=head_dim, d_ff=d_ff,
                        n_experts=n_experts, vocab=vocab, depth=depth, top_k=top_k, width=width, n_tree=n_tree,
                        prefix=prefix, target_layers=target_layers)
        dkv = n_kv_heads * head_dim
        # draft layer weights (random): reduction layer, attention projections (q, k, v stacked), router, experts;
        # output embedding shared by both heads
        self.w_red = rn(d, 2 * d, sc=(2 * d) ** -0.5)
        self.w_qkv = rn(d + 2 * dkv, d, sc=d ** -0.5)
        self.wo = rn(d, d, sc=d ** -0.5)
        self.centroids = rn(n_experts, d, sc=1.5 * d ** -0.5)
        self.w_gate, self.w_up = rn(n_experts, d_ff, d, sc=d ** -0.5), rn(n_experts, d_ff, d, sc=d ** -0.5)
        self.w_down = rn(n_experts, d, d_ff, sc=d_ff ** -0.5)
        self.w_head = rn(vocab, d, sc=4.0 * d ** -0.5)
        self.embed = rn(vocab, d)
        # draft layer KV cache of the committed prefix, and the feature / token of the last committed position
        self.dk_cache, self.dv_cache = rn(batch, prefix, n_kv_heads, head_dim), rn(batch, prefix, n_kv_heads, head_dim)
        self.plen = torch.full((batch,), prefix, dtype=torch.int32, device=dev)
        self.root_feature = rn(batch, d)
        self.root_token = torch.randint(0, vocab, (batch,), device=dev, generator=g)
        # the partial draft tree as the draft layer's attention sees it: slot 0 is the last committed token, then
        # the nodes expanded at each depth; q, k, v, outputs of all slots, parents as slot numbers
        self.t_max = 1 + width * (depth - 1)
        self.q_acc = torch.zeros((batch, self.t_max, n_heads, head_dim), dtype=bf, device=dev)
        self.k_acc = torch.zeros((batch, self.t_max, n_kv_heads, head_dim), dtype=bf, device=dev)
        self.v_acc = torch.zeros_like(self.k_acc)
        self.o_acc = torch.zeros_like(self.q_acc)
        self.state = jk.TreeState(batch, 512)
        self.n_q_rows = 2 * batch * self.t_max
        self.q_all = torch.zeros((self.n_q_rows, vocab), dtype=torch.float32, device=dev)  # the passes' distributions
        # target side: per layer q / k / v of the tree nodes and the caches (random), logits made afterwards
        sc = head_dim ** -0.5
        self.layers = [dict(q=rn(batch, n_tree, n_heads, head_dim, sc=sc),
                            k_cache=rn(batch, prefix + 64, n_kv_heads, head_dim), v_cache=rn(batch, prefix + 64, n_kv_heads, head_dim),
                            k_tree=rn(batch, n_tree, n_kv_heads, head_dim), v_tree=rn(batch, n_tree, n_kv_heads, head_dim),
                            out=torch.zeros((batch, n_tree, n_heads, head_dim), dtype=bf, device=dev))
                       for _ in range(target_layers)]
        self.base_logits = torch.randn((batch, n_tree + 1, vocab), device=dev, generator=g) * 2
        self.logits = torch.empty_like(self.base_logits)
        self.uniforms = torch.rand((batch, n_tree + 1), device=dev, generator=g)
        # workspaces, made once: the largest attention call of the round, the acceptance walk
        l0 = self.layers[0]
        need = max(jk.tree_verify_attention_workspace(l0["q"], l0["k_cache"], l0["k_tree"], prefix),
                   jk.tree_verify_attention_workspace(self.q_acc, self.dk_cache, self.k_acc, prefix))
        self.ws_attn = torch.empty(need, dtype=torch.uint8, device=dev)
        jk.workspace_init(self.ws_attn)
        self.ws_acc = torch.empty(jk.accept_path_workspace(batch, n_tree, vocab, jk.JK_SAMPLE), dtype=torch.uint8, device=dev)
        jk.workspace_init(self.ws_acc)
        self.result = {}

    # ------------------------------------------------------------------ draft
    def draft(self):
        c = self.cfg
        B, d, H, Hkv, D, V = c["batch"], c["d_model"], c["n_heads"], c["n_kv_heads"], c["head_dim"], c["vocab"]
        width, top_k = c["width"], c["top_k"]
        dkv = Hkv * D
        self.plen.fill_(c["prefix"])           # (a replayed round starts from the same prefix)
        self.state.reset()
        frontier, q_base, off = None, 0, 0
        feat_parent, tok = self.root_feature, self.root_token
        parent_acc = torch.full((B, 1), -1, dtype=torch.int32, device=self.dev)
        slot_node = [torch.full((B, 1), -1, dtype=torch.int32, device=self.dev)]   # tree node behind each slot
        for dep in range(c["depth"]):
            nf = 1 if frontier is None else frontier.shape[1]
            rows = B * nf
            t_cur = off + nf
            # reduction layer: h = W_red [emb(t); f_parent]
            h = jk.linear(torch.cat([self.embed[tok.reshape(-1).long()], feat_parent.reshape(rows, d)], 1).contiguous(), self.w_red)
            # Eq. 1: the new nodes' q, k, v join those of the earlier passes; every node attends to the draft layer's
            # cache and to its draft ancestors (slots of earlier passes), which is what the call does given the
            # partial tree.  Rows of earlier passes are recomputed along the way and not used.
            qkv = jk.linear(h, self.w_qkv)
            self.q_acc[:, off:t_cur].copy_(qkv[:, :d].reshape(B, nf, H, D))
            self.k_acc[:, off:t_cur].copy_(qkv[:, d:d + dkv].reshape(B, nf, Hkv, D))
            self.v_acc[:, off:t_cur].copy_(qkv[:, d + dkv:].reshape(B, nf, Hkv, D))
            jk.tree_verify_attention(self.q_acc[:, :t_cur], self.dk_cache, self.dv_cache, self.k_acc[:, :t_cur],
                                     self.v_acc[:, :t_cur], parent_acc, self.plen, max_prefix_len=c["prefix"],
                                     out=self.o_acc[:, :t_cur], workspace=self.ws_attn)
            u = jk.linear(self.o_acc[:, off:t_cur].reshape(rows, d).contiguous(), self.wo, residual=h)
            f_top, s_top, idx, f_mix = jk.moe_experts(u, self.centroids, self.w_gate, self.w_up, self.w_down)
            _, _, tk, tp = jk.draft_heads(f_top, s_top, self.w_head, jk.JK_HEADS_DECOUPLED, 1.0, top_k,
                                          out_probs=self.q_all[q_base:q_base + 2 * rows].view(rows, 2, V))
            frontier = jk.tree_grow(self.state, frontier, tk.reshape(rows, 2, top_k), tp.reshape(rows, 2, top_k), width, q_base)
            # next pass: the chosen nodes' tokens, their parents' mixed features (Eq. 3) and their parents' slots
            fl = frontier.long()
            tok = torch.gather(self.state.tokens, 1, fl)
            par_row = (torch.gather(self.state.q_row, 1, fl) - q_base) // 2          # row of the parent in this pass
            feat_parent = f_mix[par_row.reshape(-1).long()].reshape(B, width, d)
            in_batch = par_row - torch.arange(B, device=self.dev, dtype=par_row.dtype)[:, None] * nf
            if dep + 1 < c["depth"]:
                parent_acc = torch.cat([parent_acc, (off + in_batch).to(torch.int32)], 1).contiguous()
                slot_node.append(frontier)
            q_base += 2 * rows
            off = t_cur
        tokens, parent, q_row, old, n_valid = jk.tree_finalize(self.state, c["n_tree"])
        self.result.update(tokens=tokens, parent=parent, q_row=q_row, n_valid=n_valid, draft_parent=parent_acc,
                           draft_slot_node=torch.cat(slot_node, 1))

    # ----------------------------------------------------------------- verify
    def verify(self):
        c, r = self.cfg, self.result
        for l in self.layers:
            jk.tree_verify_attention(l["q"], l["k_cache"], l["v_cache"], l["k_tree"], l["v_tree"], r["parent"], self.plen,
                                     max_prefix_len=c["prefix"], out=l["out"], workspace=self.ws_attn)
        # the target's logits (random, with the draft tokens made likely so that something is accepted)
        self.logits.copy_(self.base_logits)
        rows_of = (r["parent"] + 1).long()
        b_idx = torch.arange(c["batch"], device=self.dev)[:, None].expand_as(rows_of)
        self.logits.index_put_((b_idx, rows_of, r["tokens"].long().clamp(min=0)),
                               torch.full(rows_of.shape, 6.0, device=self.dev), accumulate=True)

    # ----------------------------------------------------------------- refine
    def refine(self):
        c, r = self.cfg, self.result
        path, alen, bonus = jk.accept_path_rows(r["tokens"], r["parent"], self.logits, self.q_all, r["q_row"], self.uniforms,
                                                1.0, max_depth=c["depth"], workspace=self.ws_acc)
        for l in self.layers:
            jk.commit_path(l["k_tree"], l["v_tree"], l["k_cache"], l["v_cache"], path, alen, self.plen,
                           advance=l is self.layers[-1])
        r.update(path=path, accept_len=alen, bonus=bonus, prefix_len=self.plen, outs=[l["out"] for l in self.layers])

    def run(self):
        self.draft()
        self.verify()
        self.refine()
        return self.result

    # ------------------------------------------------------- graphs and timing
    def capture(self):
        """The three phases as three HIP graphs (after one eager round, which also makes every launch plan).
        Returns {"draft": graph, "verify": graph, "refine": graph}; a replayed phase leaves its results in the same
        tensors as the eager one (`self.result`)."""
        self.run()
        torch.cuda.synchronize()
        graphs = {}
        pool = None
        for name in ("draft", "verify", "refine"):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, pool=pool, stream=torch.cuda.Stream()):
                getattr(self, name)()
            pool = g.pool()
            graphs[name] = g
        return graphs

    def time_phases(self, reps=20):
        """Median microseconds of each phase over `reps` replays of the whole round (phases back to back on one
        stream, an event between them)."""
        graphs = self.capture()
        names = ("draft", "verify", "refine")
        for _ in range(3):
            for n in names:
                graphs[n].replay()
        torch.cuda.synchronize()
        samples = {n: [] for n in names}
        total = []
        for _ in range(reps):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record()
            for i, n in enumerate(names):
                graphs[n].replay()
                ev[i + 1].record()
            torch.cuda.synchronize()
            for i, n in enumerate(names):
                samples[n].append(ev[i].elapsed_time(ev[i + 1]) * 1e3)
            total.append(ev[0].elapsed_time(ev[3]) * 1e3)
        med = lambda v: sorted(v)[len(v) // 2]
        out = {f"{n}_us": round(med(samples[n]), 1) for n in names}
        out["round_us"] = round(med(total), 1)
        out["accept_len"] = self.result["accept_len"].cpu().tolist()
        out["tokens_per_round"] = [a + 1 for a in out["accept_len"]]
        return out


def run(batch=2, seed=0, verbose=True, shape="small", **overrides):
    cfg = dict(SHAPES[shape])
    cfg.update(batch=batch, **overrides)
    rd = Round(seed=seed, **cfg)
    r = rd.run()
    torch.cuda.synchronize()
    if verbose:
        print("tree nodes kept per sequence:", r["n_valid"].cpu().tolist())
        print("accepted draft tokens per sequence:", r["accept_len"].cpu().tolist(), "-> tokens per round:",
              [a + 1 for a in r["accept_len"].cpu().tolist()])
        print("bonus tokens:", r["bonus"].cpu().tolist(), " new prefix lengths:", r["prefix_len"].cpu().tolist())
    r["round"] = rd
    return r


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--shape", choices=sorted(SHAPES), default="small")
    ap.add_argument("--time", action="store_true", help="capture the three phases as HIP graphs and time them")
    a = ap.parse_args()
    batch = SHAPES[a.shape]["batch"] if a.batch is None else a.batch
    res = run(batch=batch, seed=a.seed, shape=a.shape)
    if a.time:
        print(res["round"].time_phases())
