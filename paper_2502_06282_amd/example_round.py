"""One speculative-decoding round (Section 2.1: draft, verify, refine) strung together from the library's
calls, with random weights and a synthetic target model: what a serving loop does per round, and in
which order.  Run on an MI355X:  python -m paper_2502_06282_amd.example_round

  draft, per depth      jk_linear (reduction layer and q/k/v/o projections of Eq. 1) + jk_tree_verify_attention over
                        the draft layer's own cache -> jk_moe_experts (Eq. 2, 3, 5) -> jk_draft_heads (Eq. 4) ->
                        jk_tree_grow
  after the last depth  jk_tree_finalize
  verify                jk_tree_verify_attention per target layer (the target's projections and MLPs are not
                        part of this library: q/k/v and the logits are random here)
  refine                jk_accept_path_rows (speculative sampling against the draft passes' distributions, addressed
                        through the tree's row table), jk_commit_path

torch is used for device memory, random numbers and row gathers of the hidden states; every step of the
method itself runs in the library.
"""
from __future__ import annotations

import argparse

import torch

import paper_2502_06282_amd as jk


def run(batch=2, d_model=512, n_heads=4, head_dim=128, d_ff=512, n_experts=4, vocab=8000, depth=4, top_k=4, width=4,
        n_tree=24, prefix=256, target_layers=2, seed=0, verbose=True):
    dev = torch.device("cuda")
    g = torch.Generator(device=dev).manual_seed(seed)
    bf = torch.bfloat16
    rn = lambda *shape, sc=1.0: (torch.randn(shape, device=dev, generator=g) * sc).to(bf)
    d = d_model
    assert n_heads * head_dim == d
    # draft layer weights (random): reduction layer, attention projections, router, experts; shared output embedding
    w_red = rn(d, 2 * d, sc=(2 * d) ** -0.5)
    wq, wk, wv, wo = (rn(d, d, sc=d ** -0.5) for _ in range(4))
    centroids = rn(n_experts, d, sc=1.5 * d ** -0.5)
    w_gate, w_up = rn(n_experts, d_ff, d, sc=d ** -0.5), rn(n_experts, d_ff, d, sc=d ** -0.5)
    w_down = rn(n_experts, d, d_ff, sc=d_ff ** -0.5)
    w_head = rn(vocab, d, sc=4.0 * d ** -0.5)
    embed = rn(vocab, d)
    # draft layer KV cache of the committed prefix, and the feature of the last committed token
    dk_cache, dv_cache = rn(batch, prefix, n_heads, head_dim), rn(batch, prefix, n_heads, head_dim)
    plen = torch.full((batch,), prefix, dtype=torch.int32, device=dev)
    root_feature, root_token = rn(batch, d), torch.randint(0, vocab, (batch,), device=dev, generator=g)

    state = jk.TreeState(batch, 512)
    frontier = None
    q_rows, q_base = [], 0
    feat_parent, tok = root_feature, root_token                    # inputs of the first draft pass
    for dep in range(depth):
        nf = 1 if frontier is None else frontier.shape[1]
        rows = batch * nf
        # reduction layer: h = W_red [emb(t); f_parent]
        h = jk.linear(torch.cat([embed[tok.reshape(-1).long()], feat_parent.reshape(rows, d)], 1).contiguous(), w_red)
        # Eq. 1 over the draft layer's cache (each frontier node as a one-node tree; a full implementation also
        # attends to the node's draft ancestors, which the same call does when given the partial tree)
        q = jk.linear(h, wq).reshape(batch, nf, n_heads, head_dim)
        kt = jk.linear(h, wk).reshape(batch, nf, n_heads, head_dim)
        vt = jk.linear(h, wv).reshape(batch, nf, n_heads, head_dim)
        lone = torch.full((batch, nf), -1, dtype=torch.int32, device=dev)
        attn = jk.tree_verify_attention(q, dk_cache, dv_cache, kt, vt, lone, plen)
        u = jk.linear(attn.reshape(rows, d), wo, residual=h)
        f_top, s_top, idx, f_mix = jk.moe_experts(u, centroids, w_gate, w_up, w_down)
        lg, qd, tk, tp = jk.draft_heads(f_top, s_top, w_head, jk.JK_HEADS_DECOUPLED, 1.0, top_k)
        frontier = jk.tree_grow(state, frontier, tk.reshape(rows, 2, top_k), tp.reshape(rows, 2, top_k), width, q_base)
        q_rows.append(qd.reshape(-1, vocab))
        q_base += 2 * rows
        # next pass: the chosen nodes' tokens and their parents' mixed features (Eq. 3)
        fl = frontier.long()
        tok = torch.gather(state.tokens, 1, fl)
        par_slot = (torch.gather(state.q_row, 1, fl) - (q_base - 2 * rows)) // 2      # row of the parent in this pass
        feat_parent = f_mix[par_slot.reshape(-1).long()].reshape(batch, width, d)
    tokens, parent, q_row, old, n_valid = jk.tree_finalize(state, n_tree)
    q_all = torch.cat(q_rows, 0).contiguous()      # (a serving loop writes the passes' distributions into one buffer)

    # verification: the target's attention layers over the tree (random q/k/v), then its logits (random, with
    # the draft tokens made likely so that something is accepted)
    layers = []
    for _ in range(target_layers):
        layers.append(dict(q=rn(batch, n_tree, n_heads, head_dim, sc=head_dim ** -0.5), k_cache=rn(batch, prefix + 64, n_heads, head_dim),
                           v_cache=rn(batch, prefix + 64, n_heads, head_dim), k_tree=rn(batch, n_tree, n_heads, head_dim),
                           v_tree=rn(batch, n_tree, n_heads, head_dim)))
    outs = [jk.tree_verify_attention(l["q"], l["k_cache"], l["v_cache"], l["k_tree"], l["v_tree"], parent, plen,
                                     max_prefix_len=prefix) for l in layers]
    logits = torch.randn((batch, n_tree + 1, vocab), device=dev, generator=g) * 2
    rows_of = (parent + 1).long()
    for b in range(batch):
        logits[b, rows_of[b], tokens[b].long().clamp(min=0)] += 6.0
    uniforms = torch.rand((batch, n_tree + 1), device=dev, generator=g)
    path, alen, bonus = jk.accept_path_rows(tokens, parent, logits, q_all, q_row, uniforms, 1.0, max_depth=depth)
    for l in layers:
        jk.commit_path(l["k_tree"], l["v_tree"], l["k_cache"], l["v_cache"], path, alen, plen, advance=l is layers[-1])
    torch.cuda.synchronize()
    if verbose:
        print("tree nodes kept per sequence:", n_valid.cpu().tolist())
        print("accepted draft tokens per sequence:", alen.cpu().tolist(), "-> tokens per round:",
              [a + 1 for a in alen.cpu().tolist()])
        print("bonus tokens:", bonus.cpu().tolist(), " new prefix lengths:", plen.cpu().tolist())
    return dict(tokens=tokens, parent=parent, accept_len=alen, bonus=bonus, prefix_len=plen, path=path, outs=outs)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=2)
    ap.add_argument("--seed", type=int, default=0)
    a = ap.parse_args()
    run(batch=a.batch, seed=a.seed)
