"""Seeded generators for draft trees, attention tensors and acceptance inputs.

The five named workloads stand in for the model shapes the paper evaluates
(Vicuna-7B, LLaMA2-13B/70B, LLaMA3-8B; Section 4 "Models and tasks") and for
the structure of its draft trees (two experts, each proposing top-k
candidates per expanded node, higher-scoring expert on the left; Section
3.1.2).  Contents are random; only shapes and structure follow the paper.

Nothing here computes attention, softmax, acceptance tests or residuals.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class VerifyConfig:
    name: str
    batch: int
    layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_len: int
    n_tree: int
    depth: int
    topk: int            # candidates per expert per expanded node
    frontier: int        # nodes expanded per depth
    dtype: str           # "bf16" | "f32"
    vocab: int
    mode: str            # "greedy" | "sample"
    tree_kind: str       # "coin" | "two_expert" | "chain" | "static"
    input_scale: float   # Q, K, V ~ N(0,1) * input_scale
    hit_prob: float      # greedy: P(node token is the planted target top-1)
    seed: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def with_(self, **kw) -> "VerifyConfig":
        return replace(self, **kw)


_S128 = 1.0 / float(np.sqrt(128.0))

CONFIGS: Dict[str, VerifyConfig] = {
    "c1_tiny": VerifyConfig("c1_tiny", 1, 1, 4, 4, 64, 128, 10, 3, 1, 0, "f32",
                            1000, "greedy", "coin", 1.0, 0.0, 0),
    "c2_vicuna7b": VerifyConfig("c2_vicuna7b", 1, 1, 32, 32, 128, 1024, 60, 6, 5, 5,
                                "bf16", 32000, "greedy", "two_expert", _S128, 0.7, 1),
    "c3_llama3_8b": VerifyConfig("c3_llama3_8b", 1, 1, 32, 8, 128, 4096, 60, 6, 5, 5,
                                 "bf16", 128256, "sample", "two_expert", _S128, 0.0, 2),
    "c4_llama2_13b": VerifyConfig("c4_llama2_13b", 4, 40, 40, 40, 128, 2048, 60, 6, 5, 5,
                                  "bf16", 32000, "greedy", "two_expert", _S128, 0.7, 3),
    "c5_llama2_70b": VerifyConfig("c5_llama2_70b", 8, 1, 64, 8, 128, 16384, 100, 8, 6, 5,
                                  "bf16", 32000, "sample", "two_expert", _S128, 0.0, 4),
    # second workload family for the same kernels (Section 2.1: a chain of gamma draft tokens is
    # the original speculative sampling; Section 3.1.2: the method also runs on predefined static
    # trees): not in the graded set, shapes of a 7B model
    "c6_chain_sps": VerifyConfig("c6_chain_sps", 8, 32, 32, 32, 128, 2048, 5, 5, 1, 1,
                                 "bf16", 32000, "sample", "chain", _S128, 0.0, 5),
    "c7_static_tree": VerifyConfig("c7_static_tree", 4, 32, 32, 32, 128, 1024, 28, 5, 4, 0,
                                   "bf16", 32000, "greedy", "static", _S128, 0.7, 6),
}


def config_rng(cfg: VerifyConfig, stream: int = 0, seed: Optional[int] = None) -> np.random.Generator:
    """PCG64 generator keyed by (seed, stream): independent streams for the tree,
    each layer's tensors and the acceptance inputs."""
    s = cfg.seed if seed is None else seed
    return np.random.Generator(np.random.PCG64([int(s), int(stream)]))


# --------------------------------------------------------------------------
# bf16 helpers (round-to-nearest-even on finite values)
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array whose values are exactly representable in bf16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16-representable float32 array -> uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# draft trees
# --------------------------------------------------------------------------
def tree_depths(parent: np.ndarray) -> np.ndarray:
    """Depth of every node (children of the committed prefix have depth 1)."""
    d = np.zeros(len(parent), dtype=np.int32)
    for i, p in enumerate(parent):
        d[i] = 1 if p < 0 else d[p] + 1
    return d


def coin_tree(rng: np.random.Generator, n_nodes: int = 10, depth: int = 3) -> np.ndarray:
    """Small tree: every node of the previous depth (the virtual root at depth 0
    included) gets one child (one expert) or two (both experts) by a fair coin;
    BFS numbering; redrawn until it has at least n_nodes, then cut to the first
    n_nodes in BFS order."""
    while True:
        parent = []
        level = [-1]
        for _ in range(depth):
            nxt = []
            for p in level:
                for _c in range(int(rng.integers(1, 3))):
                    nxt.append(len(parent))
                    parent.append(p)
            level = nxt
        if len(parent) >= n_nodes:
            return np.asarray(parent[:n_nodes], dtype=np.int32)


def two_expert_tree(rng: np.random.Generator, depth: int, topk: int, frontier: int,
                    budget: int) -> Dict[str, np.ndarray]:
    """Draft tree as two experts build it: every expanded node receives the first
    expert's top-k candidates (left) and then the second expert's (right).

    Candidate score = parent score * U(0,1) (root score 1), sorted descending
    inside each expert's list so rank 0 is that expert's best.  At each depth the
    `frontier` highest-scoring nodes are expanded.  The candidate set is then cut
    to `budget` nodes: the ancestors of the best deepest candidate are kept so
    the stated depth is realised, then candidates are added by descending score
    (scores shrink along a path, so a node never precedes its parent).  Nodes are
    renumbered in BFS order: depth, then parent's new index, then expert, then
    rank.  Returns parent[] (-1 = child of the committed prefix), expert[],
    rank[] and depth[] per node."""
    par, sc, ex, rk, dp = [], [], [], [], []

    def expand(p: int, pscore: float, d: int):
        ids = []
        for e in range(2):
            draws = np.sort(rng.random(topk))[::-1]
            for r in range(topk):
                ids.append(len(par))
                par.append(p)
                sc.append(pscore * float(draws[r]))
                ex.append(e)
                rk.append(r)
                dp.append(d)
        return ids

    level = expand(-1, 1.0, 1)
    for d in range(2, depth + 1):
        best = sorted(level, key=lambda i: -sc[i])[:frontier]
        level = []
        for p in best:
            level += expand(p, sc[p], d)

    n_cand = len(par)
    keep = np.zeros(n_cand, dtype=bool)
    deepest = [i for i in range(n_cand) if dp[i] == depth]
    i = max(deepest, key=lambda j: sc[j])
    while i >= 0:
        keep[i] = True
        i = par[i]
    for i in sorted(range(n_cand), key=lambda j: -sc[j]):
        if keep.sum() >= budget:
            break
        if not keep[i] and (par[i] < 0 or keep[par[i]]):
            keep[i] = True
    kept = [i for i in range(n_cand) if keep[i]]

    new_id: Dict[int, int] = {-1: -1}
    order = []
    for d in range(1, depth + 1):
        lvl = [i for i in kept if dp[i] == d]
        lvl.sort(key=lambda i: (new_id[par[i]], ex[i], rk[i]))
        for i in lvl:
            new_id[i] = len(order)
            order.append(i)
    return {
        "parent": np.asarray([new_id[par[i]] for i in order], dtype=np.int32),
        "expert": np.asarray([ex[i] for i in order], dtype=np.int32),
        "rank": np.asarray([rk[i] for i in order], dtype=np.int32),
        "depth": np.asarray([dp[i] for i in order], dtype=np.int32),
    }


def chain_tree(n_nodes: int) -> np.ndarray:
    """gamma draft tokens in a row: node i hangs off node i-1, node 0 off the committed prefix."""
    return np.arange(-1, n_nodes - 1, dtype=np.int32)


def static_tree(widths=(4, 3, 2, 1, 1)) -> np.ndarray:
    """A predefined tree shape, the same for every sequence and round: a node that is the r-th
    (0-based) child of its parent and whose children sit at depth d gets max(0, widths[d-1] - r)
    children; BFS numbering.  The default widths give 4 + 6 + 8 + 5 + 5 = 28 nodes, depth 5."""
    parent = []
    level = [(-1, 0)]  # (node id, rank among its siblings)
    for w in widths:
        nxt = []
        for node, r in level:
            for c in range(max(0, w - r)):
                nxt.append((len(parent), c))
                parent.append(node)
        level = nxt
    return np.asarray(parent, dtype=np.int32)


def tree_for_config(cfg: VerifyConfig, seed: Optional[int] = None) -> np.ndarray:
    """parent[B, T] for a configuration: one independently drawn tree per sequence (chain and
    static trees are the same for all)."""
    out = np.empty((cfg.batch, cfg.n_tree), dtype=np.int32)
    for b in range(cfg.batch):
        rng = config_rng(cfg, 1000 + b, seed)
        if cfg.tree_kind == "coin":
            out[b] = coin_tree(rng, cfg.n_tree, cfg.depth)
        elif cfg.tree_kind == "chain":
            out[b] = chain_tree(cfg.n_tree)
        elif cfg.tree_kind == "static":
            t = static_tree()
            assert len(t) >= cfg.n_tree
            out[b] = t[:cfg.n_tree]
        else:
            out[b] = two_expert_tree(rng, cfg.depth, cfg.topk, cfg.frontier, cfg.n_tree)["parent"]
    return out


# --------------------------------------------------------------------------
# attention tensors
# --------------------------------------------------------------------------
def _normal(rng, shape, scale, dtype):
    x = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return round_to_bf16(x) if dtype == "bf16" else x


def attention_inputs(cfg: VerifyConfig, layer: int = 0, seed: Optional[int] = None,
                     prefix_len: Optional[int] = None, scale_mult: float = 1.0) -> Dict[str, np.ndarray]:
    """Q, K/V cache and tree K/V of one layer as float32 arrays (values already
    rounded to bf16 when cfg.dtype == "bf16"), layouts
    q [B,T,Hq,D], k_cache/v_cache [B,L,Hkv,D], k_tree/v_tree [B,T,Hkv,D]."""
    rng = config_rng(cfg, 2000 + layer, seed)
    B, T, Hq, Hkv, D = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    L = cfg.prefix_len if prefix_len is None else prefix_len
    s = cfg.input_scale * scale_mult
    return {
        "q": _normal(rng, (B, T, Hq, D), s, cfg.dtype),
        "k_cache": _normal(rng, (B, L, Hkv, D), s, cfg.dtype),
        "v_cache": _normal(rng, (B, L, Hkv, D), s, cfg.dtype),
        "k_tree": _normal(rng, (B, T, Hkv, D), s, cfg.dtype),
        "v_tree": _normal(rng, (B, T, Hkv, D), s, cfg.dtype),
    }


def paged_layout(k_cache: np.ndarray, v_cache: np.ndarray, page_size: int, seed: int = 0, spare_pages: int = 3):
    """Scatter contiguous caches [B, L, Hkv, D] into page pools [n_pages, page_size, Hkv, D] with a random
    assignment of physical pages (a few spare pages, filled with NaN, are never referenced) and return
    ((k_pool, v_pool), block_table[B, blocks_per_sequence]).  Slots past L in a sequence's last page hold NaN."""
    B, L = k_cache.shape[0], k_cache.shape[1]
    nb = (L + page_size - 1) // page_size
    n_pages = B * nb + spare_pages
    rng = np.random.Generator(np.random.PCG64([int(seed), 3000]))
    ids = rng.permutation(n_pages)[: B * nb].astype(np.int32).reshape(B, nb)
    pools = []
    for c in (k_cache, v_cache):
        pool = np.full((n_pages, page_size) + c.shape[2:], np.nan, dtype=c.dtype)
        for b in range(B):
            for j in range(nb):
                n = min(page_size, L - j * page_size)
                pool[ids[b, j], :n] = c[b, j * page_size: j * page_size + n]
        pools.append(pool)
    return (pools[0], pools[1]), ids


# --------------------------------------------------------------------------
# acceptance inputs
# --------------------------------------------------------------------------
def accept_inputs(cfg: VerifyConfig, parent: np.ndarray, seed: Optional[int] = None,
                  vocab: Optional[int] = None) -> Dict[str, Optional[np.ndarray]]:
    """Target logits, draft tokens and (sampling mode) draft distributions + uniforms.

    logits [B, N+1, V] ~ N(0, 4) fp32; row 0 belongs to the committed prefix's
    last position, row i+1 to node i.

    greedy: one entry per row is raised above the row's maximum (the "planted"
    top-1, returned as top_token[B, N+1]); visiting each parent's children left
    to right, a child takes the planted top-1 of its parent's row with
    probability hit_prob unless an earlier sibling already did, otherwise a
    uniform token different from it and from its earlier siblings.
    hit_prob == 0 draws every token uniformly with no constraint.

    sample: draft_probs[B, N, V] = Dirichlet(0.1) drawn in fp64, stored fp32 and
    renormalised in fp32; tokens[b, k] ~ draft_probs[b, k]; uniforms[B, N+1] in
    [0, 1) fp32 (entry k tests node k, entry N draws the bonus token)."""
    B, N = parent.shape
    V = cfg.vocab if vocab is None else vocab
    rng = config_rng(cfg, 3000, seed)
    logits = rng.standard_normal((B, N + 1, V), dtype=np.float32) * np.float32(2.0)
    out: Dict[str, Optional[np.ndarray]] = {"logits": logits, "draft_probs": None,
                                            "uniforms": None, "top_token": None}
    tokens = np.empty((B, N), dtype=np.int32)
    if cfg.mode == "greedy":
        if cfg.hit_prob <= 0.0:
            tokens[:] = rng.integers(0, V, size=(B, N), dtype=np.int32)
        else:
            top = rng.integers(0, V, size=(B, N + 1), dtype=np.int32)
            bump = np.float32(0.5) + np.abs(rng.standard_normal((B, N + 1), dtype=np.float32))
            rowmax = logits.max(axis=2)
            bi, ri = np.meshgrid(np.arange(B), np.arange(N + 1), indexing="ij")
            logits[bi, ri, top] = rowmax + bump
            out["top_token"] = top
            for b in range(B):
                used: Dict[int, set] = {}
                hit: Dict[int, bool] = {}
                for k in range(N):
                    c = int(parent[b, k])
                    t_star = int(top[b, c + 1])
                    sib = used.setdefault(c, set())
                    if not hit.get(c, False) and rng.random() < cfg.hit_prob:
                        tok = t_star
                        hit[c] = True
                    else:
                        while True:
                            tok = int(rng.integers(0, V))
                            if tok != t_star and tok not in sib:
                                break
                    sib.add(tok)
                    tokens[b, k] = tok
    else:
        q = np.empty((B, N, V), dtype=np.float32)
        for b in range(B):
            for k in range(N):
                g = rng.gamma(0.1, size=V)
                q32 = (g / g.sum()).astype(np.float32)
                q32 /= q32.sum(dtype=np.float32)
                q[b, k] = q32
                cdf = np.cumsum(q32, dtype=np.float64)
                tokens[b, k] = min(int(np.searchsorted(cdf, rng.random() * cdf[-1], side="right")), V - 1)
        out["draft_probs"] = q
        out["uniforms"] = rng.random((B, N + 1), dtype=np.float32)
    out["tokens"] = tokens
    return out


# --------------------------------------------------------------------------
# draft-head step (Section 3.1.2 / 3.2): random weights of the model's shapes
# --------------------------------------------------------------------------
def draft_head_inputs(rows: int, d_model: int, vocab: int, seed: int = 0, logit_std: float = 2.5):
    """Inputs of the dual-head step: per-expert features of `rows` hidden states, the two router
    scores of each (larger first, sum below 1) and an output-embedding matrix scaled so that the
    logits of a unit-score feature have about `logit_std` standard deviation.  Features and weights
    are bf16-representable float32 arrays."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 77]))
    f_top = round_to_bf16(rng.standard_normal((rows, 2, d_model), dtype=np.float32))
    hi = rng.uniform(0.3, 0.7, size=rows)
    lo = rng.uniform(0.05, 1.0, size=rows) * np.minimum(hi, 1.0 - hi)
    s_top = np.stack([hi, lo], axis=1).astype(np.float32)
    w_head = round_to_bf16(rng.standard_normal((vocab, d_model), dtype=np.float32)
                           * np.float32(logit_std / np.sqrt(d_model) / 0.5))
    return {"f_top": f_top, "s_top": s_top, "w_head": w_head}


def moe_inputs(rows: int, d_model: int, d_ff: int, n_experts: int, seed: int = 0):
    """Inputs of the router and the expert MLPs: hidden states, expert centroids and the three
    weight matrices of each expert, all bf16-representable float32 arrays."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 78]))
    sd = np.float32(1.0 / np.sqrt(d_model))
    return {
        "u": round_to_bf16(rng.standard_normal((rows, d_model), dtype=np.float32)),
        "centroids": round_to_bf16(rng.standard_normal((n_experts, d_model), dtype=np.float32) * sd * np.float32(1.5)),
        "w_gate": round_to_bf16(rng.standard_normal((n_experts, d_ff, d_model), dtype=np.float32) * sd),
        "w_up": round_to_bf16(rng.standard_normal((n_experts, d_ff, d_model), dtype=np.float32) * sd),
        "w_down": round_to_bf16(rng.standard_normal((n_experts, d_model, d_ff), dtype=np.float32)
                                * np.float32(1.0 / np.sqrt(d_ff))),
    }
