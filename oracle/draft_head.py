"""Oracle: one step of the MoE draft head and its two output distributions.

TEST INFRASTRUCTURE ONLY.  Not imported by the product path.

What is computed (Section 3.1.2, Eq. 2-5, and Section 3.2, Eq. 6-8 of the
paper), for one hidden state u (the draft decoder layer's attention output
plus residual, Eq. 1, which is an input here):

    s_j      = softmax_j(u . e_j)                          router over N centroids       (Eq. 2)
    g_j      = s_j if s_j is among the K largest, else 0   sparse gate, K = 2            (Eq. 5)
    f        = sum_j g_j Expert_j(u) + u                   mixed feature                 (Eq. 3)
    top1, top2 = the two selected experts, larger score first ("left"), smaller second ("right")
    f^top    = Expert_top(u) + u                           per-expert feature

  decoupled heads (Eq. 4; the tree takes one candidate list from each expert):
    logits^left, logits^right = Head(s^top1 f^top1), Head(s^top2 f^top2)
  contrastive heads (Eq. 6-8):
    f^moe   = s^top1 f^top1 + s^top2 f^top2,   f^const = beta f^top1 - alpha f^top2
    logits^moe, logits^const = Head(f^moe), Head(f^const)

    Head(x) = W_head x    (the target model's output embedding, shared by both heads)

and from each logits row the draft distribution q = softmax(logits / temperature)
that the acceptance test later divides by, and its top-k candidates ("top-k
construction principle", Section 3.1.2), most probable first.

Readings taken where the paper leaves a choice:
  * Eq. 4 prints the mixed feature f inside both heads, which would make the
    two logits rows multiples of each other; Eq. 6 and the description of the
    decoupled tree (one candidate list per expert) show that the per-expert
    features are meant.  Here the two heads see s^top1 f^top1 and s^top2 f^top2,
    i.e. the two addends of Eq. 6, so that left + right = Head(f^moe).
  * f^top carries the residual u of Eq. 3 (each expert is a residual MLP block
    like the decoder MLP it replaces).  With that, Eq. 6 equals Eq. 3 up to
    the factor (s^top1 + s^top2) on the residual.
  * Expert_j is a gated MLP of the LLaMA form, down(silu(gate x) * up x); the
    paper only calls it a lightweight MLP.  Normalisation layers are left out,
    as in the paper's equations.
  * Ties (equal scores, equal logits) go to the lower index.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

DECOUPLED = 0
CONTRASTIVE = 1


def router_scores(u: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """Eq. 2.  u [R,d], centroids [N,d] -> s [R,N], rows sum to 1."""
    z = np.asarray(u, np.float64) @ np.asarray(centroids, np.float64).T
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def top_k_desc(x: Sequence[float], k: int) -> np.ndarray:
    """Indices of the k largest entries of a vector, largest first, ties to the lower index."""
    x = np.asarray(x)
    order = sorted(range(x.shape[0]), key=lambda i: (-float(x[i]), i))
    return np.asarray(order[:k], dtype=np.int64)


def gate(s: np.ndarray, K: int = 2) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 5.  s [R,N] -> (g [R,N] with K non-zeros per row, idx [R,K] selected experts, larger score first)."""
    s = np.asarray(s, np.float64)
    g = np.zeros_like(s)
    idx = np.zeros((s.shape[0], K), dtype=np.int64)
    for r in range(s.shape[0]):
        idx[r] = top_k_desc(s[r], K)
        g[r, idx[r]] = s[r, idx[r]]
    return g, idx


def expert_mlp(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """Gated MLP.  x [d]; w_gate, w_up [d_ff,d]; w_down [d,d_ff]."""
    x = np.asarray(x, np.float64)
    a = np.asarray(w_gate, np.float64) @ x
    b = np.asarray(w_up, np.float64) @ x
    h = a / (1.0 + np.exp(-a)) * b
    return np.asarray(w_down, np.float64) @ h


def moe_features(u: np.ndarray, centroids: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray,
                 K: int = 2):
    """Eq. 2, 3, 5 for R hidden states.

    u [R,d]; centroids [N,d]; w_gate, w_up [N,d_ff,d]; w_down [N,d,d_ff].
    Returns (f [R,d] of Eq. 3, f_top [R,K,d], s_top [R,K], idx [R,K])."""
    u = np.asarray(u, np.float64)
    s = router_scores(u, centroids)
    g, idx = gate(s, K)
    R, d = u.shape
    f = np.array(u, copy=True)
    f_top = np.zeros((R, K, d))
    s_top = np.zeros((R, K))
    for r in range(R):
        for k in range(K):
            j = int(idx[r, k])
            y = expert_mlp(u[r], w_gate[j], w_up[j], w_down[j])
            f[r] += g[r, j] * y
            f_top[r, k] = y + u[r]
            s_top[r, k] = s[r, j]
    return f, f_top, s_top, idx


def head_inputs(f_top: np.ndarray, s_top: np.ndarray, mode: int, alpha: float = 0.0, beta: float = 0.0) -> np.ndarray:
    """The two feature rows the shared head sees.  f_top [R,2,d], s_top [R,2] -> x [R,2,d]."""
    f_top = np.asarray(f_top, np.float64)
    s_top = np.asarray(s_top, np.float64)
    x = np.zeros_like(f_top)
    if mode == DECOUPLED:          # Eq. 4
        x[:, 0] = s_top[:, 0:1] * f_top[:, 0]
        x[:, 1] = s_top[:, 1:2] * f_top[:, 1]
    elif mode == CONTRASTIVE:      # Eq. 6, 7
        x[:, 0] = s_top[:, 0:1] * f_top[:, 0] + s_top[:, 1:2] * f_top[:, 1]
        x[:, 1] = beta * f_top[:, 0] - alpha * f_top[:, 1]
    else:
        raise ValueError("mode")
    return x


def dual_head_logits(f_top: np.ndarray, s_top: np.ndarray, w_head: np.ndarray, mode: int,
                     alpha: float = 0.0, beta: float = 0.0) -> np.ndarray:
    """Eq. 4 / Eq. 8.  w_head [V,d] -> logits [R,2,V]."""
    x = head_inputs(f_top, s_top, mode, alpha, beta)
    return x @ np.asarray(w_head, np.float64).T


def draft_distribution(logits: np.ndarray, temperature: float) -> np.ndarray:
    """q = softmax(logits / temperature) over the last axis."""
    z = np.asarray(logits, np.float64) / float(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def top_candidates(logits: np.ndarray, k: int) -> np.ndarray:
    """Top-k token ids of every logits row, best first, ties to the lower id.  logits [...,V] -> [...,k]."""
    logits = np.asarray(logits)
    flat = logits.reshape(-1, logits.shape[-1])
    out = np.zeros((flat.shape[0], k), dtype=np.int64)
    for r in range(flat.shape[0]):
        # a full stable sort of the negated row is the definition; partial selection is only faster
        out[r] = np.argsort(-flat[r], kind="stable")[:k]
    return out.reshape(logits.shape[:-1] + (k,))


def draft_heads(f_top: np.ndarray, s_top: np.ndarray, w_head: np.ndarray, mode: int, temperature: float, k: int,
                alpha: float = 0.0, beta: float = 0.0):
    """The whole head step: (logits [R,2,V], q [R,2,V], top-k ids [R,2,k], their q values [R,2,k])."""
    logits = dual_head_logits(f_top, s_top, w_head, mode, alpha, beta)
    q = draft_distribution(logits, temperature)
    ids = top_candidates(logits, k)
    return logits, q, ids, np.take_along_axis(q, ids, axis=-1)


def linear(x: np.ndarray, w: np.ndarray, residual=None) -> np.ndarray:
    """x [m,k], w [n,k] -> x w^T (+ residual)."""
    y = np.asarray(x, np.float64) @ np.asarray(w, np.float64).T
    return y if residual is None else y + np.asarray(residual, np.float64)


def draft_attention_block(h: np.ndarray, wq: np.ndarray, wk: np.ndarray, wv: np.ndarray, wo: np.ndarray,
                          k_cache: np.ndarray, v_cache: np.ndarray, parent: np.ndarray, n_heads: int,
                          n_kv_heads: int) -> np.ndarray:
    """Eq. 1 for the tree nodes of one sequence: u = Attn(h) + h with the attention of one decoder layer
    over the draft layer's own key/value cache plus the nodes' tree ancestors (the draft model sees the
    same tree the target will verify).  h [T,d]; wq, wo [d,d]; wk, wv [n_kv_heads*D, d];
    k_cache, v_cache [L, n_kv_heads, D].  Position encodings are outside (applied to q and k by the caller,
    here: none)."""
    from .tree_attention import tree_verify_attention
    T, d = h.shape
    D = d // n_heads
    q = linear(h, wq).reshape(1, T, n_heads, D)
    kt = linear(h, wk).reshape(1, T, n_kv_heads, D)
    vt = linear(h, wv).reshape(1, T, n_kv_heads, D)
    L = k_cache.shape[0]
    attn = tree_verify_attention(q, np.asarray(k_cache, np.float64)[None], np.asarray(v_cache, np.float64)[None], kt, vt,
                                 parent=np.asarray(parent)[None], prefix_len=[L])
    return linear(attn.reshape(T, d), wo, residual=h)
