"""CPU oracle for the Token Recycling decode step.  TEST INFRASTRUCTURE ONLY.

Plain, slow numpy written from the paper; it shares no code with the HIP path and
imports nothing from it.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may call it; the product path never does.

What follows the paper, function by function
  build_tree      Section 3.2 worked example and Algorithm 1 (static-tree BFS)
  topk_ids        Section 2.1, argtopk with x^0 = argmax; ties to the smallest
                  index (Appendix A.1)
  accept          Section 2.2 "Guess and Verify" (chain rule) applied to every
                  root-to-node path; the longest correct sequence wins (Section 3.3)
  update_matrix   Section 3.3, M[x_i] = argtopk(p_{i+1}) for every node of S,
                  duplicates resolved as in Appendix A.5 ("Last" by default)
  forward_nodes   Section 2.2 equations: node i sees P(x | s, its ancestors), i.e.
                  tree attention (Section 2.2 "Tree Attention")
  prefill_then_forward   the same two passes with the layer loop outermost (large models
                  whose weights are produced one layer at a time); pinned to them by equality
  tr_step / tr_generate / ar_generate   the decode loop of Sections 2.1 and 3
  sample_tokens   Section 5.3 "Temperature Sampling": the model's token at a node is
                  drawn from softmax(logits / T) instead of taken as the argmax

The paper runs unmodified HuggingFace Llama-family models and does not restate the
architecture.  The transformer here is the public Llama description: pre-RMSNorm
(eps 1e-5), rotary embedding with base 10000 and half-split pairing (i, i+hd/2),
grouped-query attention scaled by 1/sqrt(hd), SwiGLU down(silu(gate)*up), final
RMSNorm, untied LM head, no biases.  Masked positions are excluded exactly (the
paper's additive-mask leakage, Appendix A.1, is an artefact and is not reproduced).

Readings taken where the paper is silent or garbled
  * Algorithm 1 never advances d and gathers once more than needed: d is advanced
    and the last gather skipped.
  * depth = number of tree layers including the root; a step confirms 1..depth tokens.
  * duplicates in S update M last-wins (one of the outcomes the paper allows).
  * duplicate tokens among siblings both "match"; winner = deepest fully matched
    node, then smallest breadth-first index.
  * prefill covers prompt[0..P-2]; the last prompt token is the first root; prefill
    does not touch M.
  * tree node n sits at position L + depth(n).
  * temperature sampling (the paper reports results but gives no rule): the token
    "the model outputs" at a node is drawn from softmax(logits / T); a draft is
    correct when it equals the token drawn at its parent (the chain rule of Section
    2.2 unchanged); the matrix still stores the top-k of the logits, as the paper
    says it does.  The draw is the Gumbel-max form argmax_j(logits_j / T + g_j) with
    noise g supplied by the caller per sequence position, so that the same noise
    gives the same token whether the position is reached by a tree node or by plain
    one-token decoding: TR under sampling then reproduces plain sampling token for
    token.

Precision: `dtype` is float64 by default (weights are float32 / bf16-representable
values, converted on use); float32 is available for large shapes.

Pins (tests/test_oracle_*.py): worked examples of Sections 2.2, 3.2 and Appendix A.5,
brute force over explicit paths, per-path causal attention, an independent Llama
forward (HuggingFace `LlamaForCausalLM`) on a chain, full sort for top-k, and
losslessness against plain greedy decoding.  MAT / speed-up values are parity
unpinned (they need the paper's datasets and trained weights).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np


# ----------------------------------------------------------------------------
# tree template (Section 3.2; Appendix A.2)
# ----------------------------------------------------------------------------
@dataclass
class Tree:
    parent: np.ndarray          # [N] int, parent[0] = -1
    rank: np.ndarray            # [N] int, column of M[token(parent)], rank[0] = -1
    depth: np.ndarray           # [N] int, root = 0
    paths: List[List[int]]      # paths[n] = node indices root..n
    n_layers: int               # number of layers including the root layer

    @property
    def n_nodes(self) -> int:
        return len(self.parent)


def make_tree(parent: Sequence[int], rank: Sequence[int], k: int) -> Tree:
    """Derive depths and root-to-node paths; check breadth-first order."""
    parent = np.asarray(parent, dtype=np.int64)
    rank = np.asarray(rank, dtype=np.int64)
    n = len(parent)
    if n < 1 or parent[0] != -1:
        raise ValueError("node 0 must be the root")
    depth = np.zeros(n, dtype=np.int64)
    paths: List[List[int]] = [[0]]
    seen = set()
    for i in range(1, n):
        p = int(parent[i])
        if not (0 <= p < i):
            raise ValueError("parent must precede child")
        if not (0 <= rank[i] < k):
            raise ValueError("rank out of range")
        if (p, int(rank[i])) in seen:
            raise ValueError("duplicate (parent, rank)")
        seen.add((p, int(rank[i])))
        depth[i] = depth[p] + 1
        if depth[i] < depth[i - 1]:
            raise ValueError("nodes must be in layer order")
        paths.append(paths[p] + [i])
    return Tree(parent, rank, depth, paths, int(depth.max()) + 1)


def build_tree(M: np.ndarray, tree: Tree, root: int) -> np.ndarray:
    """Merged sequence S of the static draft tree (Algorithm 1).  The root holds the last
    token; every other node holds the candidate its template entry names: column rank[n]
    of the matrix row of its parent's token.  Nodes are numbered layer by layer, so a
    parent is always filled before its children and one pass in index order visits the
    layers in the order the algorithm expands them."""
    S = np.zeros(tree.n_nodes, dtype=np.int64)
    S[0] = root
    for n in range(1, tree.n_nodes):
        S[n] = M[S[tree.parent[n]], tree.rank[n]]
    return S


# ----------------------------------------------------------------------------
# candidates, acceptance, update (Sections 2.1, 2.2, 3.3; Appendix A.5)
# ----------------------------------------------------------------------------
def topk_ids(p: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, most probable first; equal values keep the
    smaller index first (so column 0 is argmax with the smallest-index tie rule)."""
    return np.argsort(-np.asarray(p), kind="stable")[:k].astype(np.int64)


@dataclass
class Accept:
    n_accepted: int            # a: matched draft tokens (0..depth-1)
    winner: int                # node whose output is the bonus token
    path: List[int]            # node indices root..winner (a + 1 entries)
    emitted: List[int]         # a matched draft tokens followed by the bonus token
    bonus: int


def accept(S: np.ndarray, out: np.ndarray, tree: Tree) -> Accept:
    """Guess-and-verify on every root-to-node path: node n is correct when each draft
    token on its path equals the model output at that token's parent."""
    best = 0
    for n in range(tree.n_nodes):
        path = tree.paths[n]
        good = all(S[path[i]] == out[path[i - 1]] for i in range(1, len(path)))
        if good and tree.depth[n] > tree.depth[best]:
            best = n                                     # deepest, then smallest index
    path = tree.paths[best]
    emitted = [int(S[i]) for i in path[1:]] + [int(out[best])]
    return Accept(len(path) - 1, best, list(path), emitted, int(out[best]))


def update_matrix(M: np.ndarray, S: np.ndarray, topk: np.ndarray, mode: str = "last",
                  nodes: Optional[Sequence[int]] = None) -> None:
    """M[S[n]] = topk[n] for every node (accepted, rejected and the root).
    mode "last": a token that occurs several times keeps its last occurrence's
    candidates; "first": its first occurrence's.  `nodes` restricts the update
    (e.g. to the accepted path, the ablation of Section 5.2)."""
    order = list(range(len(S))) if nodes is None else list(nodes)
    if mode == "last":
        for n in order:
            M[S[n]] = topk[n]
    elif mode == "first":
        done = set()
        for n in order:
            if int(S[n]) not in done:
                M[S[n]] = topk[n]
                done.add(int(S[n]))
    else:
        raise ValueError(mode)


# ----------------------------------------------------------------------------
# transformer (public Llama architecture; see module docstring)
# ----------------------------------------------------------------------------
@dataclass
class Config:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0


class KVCache:
    """k[l], v[l]: [capacity, n_kv_heads, head_dim]; rows 0..len-1 are committed."""

    def __init__(self, cfg: Config, capacity: int, dtype=np.float64):
        self.k = [np.zeros((capacity, cfg.n_kv_heads, cfg.head_dim), dtype) for _ in range(cfg.n_layers)]
        self.v = [np.zeros((capacity, cfg.n_kv_heads, cfg.head_dim), dtype) for _ in range(cfg.n_layers)]
        self.len = 0
        self.capacity = capacity


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def rope(x: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """x: [heads, hd].  Pair (i, i + hd/2) is rotated by pos * theta**(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    ang = pos * theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    c, s = np.cos(ang).astype(x.dtype), np.sin(ang).astype(x.dtype)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, group: int) -> np.ndarray:
    """q: [H, hd]; K, V: [T, Hkv, hd] — the keys this query may see, nothing else.
    Softmax over exactly those T keys, scale 1/sqrt(hd); query head h uses KV head
    h // group."""
    H, hd = q.shape
    qg = q.reshape(H // group, group, hd)
    s = np.einsum("tkd,kgd->kgt", K, qg) / np.sqrt(hd)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("kgt,tkd->kgd", p, V).reshape(H, hd)


def _attend_batched(Q: np.ndarray, Kp: np.ndarray, Vp: np.ndarray, K: np.ndarray, V: np.ndarray,
                    paths: Sequence[Sequence[int]], group: int) -> np.ndarray:
    """Same result as `_attend` per node, with the prefix part done as matrix products
    for all nodes at once.  Q: [N, H, hd]; Kp, Vp: [L, Hkv, hd]; K, V: [N, Hkv, hd]."""
    N, H, hd = Q.shape
    Hkv = H // group
    L = Kp.shape[0]
    Qg = Q.reshape(N, Hkv, group, hd)
    Qm = Qg.transpose(1, 0, 2, 3).reshape(Hkv, N * group, hd)
    sp = np.matmul(Qm, np.ascontiguousarray(Kp.transpose(1, 2, 0)))        # [Hkv, N*g, L]
    sp = sp.reshape(Hkv, N, group, L).transpose(1, 0, 2, 3) / np.sqrt(hd)  # [N, Hkv, g, L]
    Pp = np.empty((N, Hkv, group, L), Q.dtype)
    out = np.empty((N, Hkv, group, hd), Q.dtype)
    for n in range(N):
        idx = list(paths[n])
        st = np.einsum("tkd,kgd->kgt", K[idx], Qg[n]) / np.sqrt(hd)        # [Hkv, g, |path|]
        m = np.maximum(sp[n].max(axis=-1), st.max(axis=-1))[..., None] if L else st.max(axis=-1)[..., None]
        ep, et = np.exp(sp[n] - m), np.exp(st - m)
        z = ep.sum(axis=-1, keepdims=True) + et.sum(axis=-1, keepdims=True)
        Pp[n] = ep / z
        out[n] = np.einsum("kgt,tkd->kgd", et / z, V[idx])
    Pm = Pp.transpose(1, 0, 2, 3).reshape(Hkv, N * group, L)
    op = np.matmul(Pm, np.ascontiguousarray(Vp.transpose(1, 0, 2)))        # [Hkv, N*g, hd]
    out += op.reshape(Hkv, N, group, hd).transpose(1, 0, 2, 3)
    return out.reshape(N, H, hd)


def _lin(Wm: np.ndarray, A: np.ndarray, dtype, row_independent: bool) -> np.ndarray:
    """A W^T for W stored [out, in]; row by row when results must not depend on the batch."""
    Wd = Wm.astype(dtype, copy=False)
    if row_independent:
        return np.stack([Wd @ A[n] for n in range(A.shape[0])])
    return A @ Wd.T


def _layer_forward(cfg: Config, lw: dict, Kp: np.ndarray, Vp: np.ndarray, X: np.ndarray,
                   pos: Sequence[int], paths: Sequence[Sequence[int]], dtype, row_independent: bool):
    """One decoder layer over N nodes that follow the prefix keys/values Kp, Vp [L, Hkv, hd].
    Returns (X after the layer, the nodes' rotated keys [N, Hkv, hd], their values)."""
    N = X.shape[0]
    H, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    group = H // Hkv
    Hn = rmsnorm(X, lw["attn_norm"].astype(dtype), cfg.rms_eps)
    Q = _lin(lw["wq"], Hn, dtype, row_independent).reshape(N, H, hd)
    K = _lin(lw["wk"], Hn, dtype, row_independent).reshape(N, Hkv, hd)
    V = _lin(lw["wv"], Hn, dtype, row_independent).reshape(N, Hkv, hd)
    for n in range(N):
        Q[n] = rope(Q[n], pos[n], cfg.rope_theta)
        K[n] = rope(K[n], pos[n], cfg.rope_theta)
    if row_independent:
        A = np.empty((N, H, hd), dtype)
        for n in range(N):
            idx = list(paths[n])
            A[n] = _attend(Q[n], np.concatenate([Kp, K[idx]], axis=0),
                           np.concatenate([Vp, V[idx]], axis=0), group)
    else:
        A = _attend_batched(Q, Kp, Vp, K, V, paths, group)
    X = X + _lin(lw["wo"], A.reshape(N, H * hd), dtype, row_independent)
    Hn = rmsnorm(X, lw["ffn_norm"].astype(dtype), cfg.rms_eps)
    X = X + _lin(lw["w_down"], silu(_lin(lw["w_gate"], Hn, dtype, row_independent)) *
                 _lin(lw["w_up"], Hn, dtype, row_independent), dtype, row_independent)
    return X, K, V


def forward_nodes(cfg: Config, w: dict, kv: KVCache, tokens: Sequence[int], pos: Sequence[int],
                  paths: Sequence[Sequence[int]], dtype=np.float64, row_independent: bool = False,
                  want_logits: bool = True):
    """One forward over N nodes that all follow the committed prefix kv[0..len-1].

    Node n is at position pos[n] and attends to the whole prefix plus the nodes listed
    in paths[n] (its ancestors and itself, root first).  Returns (logits [N, V],
    node_k, node_v) with node_k[l], node_v[l]: [N, Hkv, hd]; the cache is not modified.

    row_independent=True computes every node with vector operations only, so a node's
    result does not depend on which other nodes share the pass (same operation shapes
    as decoding that token alone)."""
    L = kv.len
    X = np.stack([w["embed"][t].astype(dtype) for t in tokens])          # [N, d]
    node_k, node_v = [], []
    for l in range(cfg.n_layers):
        X, K, V = _layer_forward(cfg, w["layers"][l], kv.k[l][:L].astype(dtype, copy=False),
                                 kv.v[l][:L].astype(dtype, copy=False), X, pos, paths, dtype, row_independent)
        node_k.append(K)
        node_v.append(V)
    logits = None
    if want_logits:
        logits = _lin(w["lm_head"], rmsnorm(X, w["final_norm"].astype(dtype), cfg.rms_eps), dtype,
                      row_independent)
    return logits, node_k, node_v


def prefill_then_forward(cfg: Config, w: dict, kv: KVCache, prompt_tokens: Sequence[int],
                         tokens: Sequence[int], depth: Sequence[int], paths: Sequence[Sequence[int]],
                         dtype=np.float64, chunk: int = 128):
    """`prefill(prompt_tokens)` followed by `forward_nodes(tokens at kv.len + depth)`, with the
    loops exchanged: layer l of a pass needs the cache of layer l only, so every pass (the
    prompt chunks in order, then the nodes) is taken through layer l before anything enters
    layer l + 1.  Each layer's weights are then used in one place, and w["layers"] may be any
    object whose [l] builds layer l on demand (a model too large to hold in host memory).
    Same arithmetic as the two calls; returns what forward_nodes returns, with the prompt
    committed to the cache."""
    prompt_tokens = list(prompt_tokens)
    L0 = kv.len
    if L0 + len(prompt_tokens) > kv.capacity:
        raise ValueError("KV capacity exceeded")
    chunks = [(lo, prompt_tokens[lo:lo + chunk]) for lo in range(0, len(prompt_tokens), chunk)]
    Xs = [np.stack([w["embed"][t].astype(dtype) for t in part]) for _, part in chunks]
    Xn = np.stack([w["embed"][t].astype(dtype) for t in tokens])
    Ln = L0 + len(prompt_tokens)
    node_k, node_v = [], []
    for l in range(cfg.n_layers):
        lw = w["layers"][l]
        for c, (lo, part) in enumerate(chunks):
            n, L = len(part), L0 + lo
            Xs[c], K, V = _layer_forward(cfg, lw, kv.k[l][:L].astype(dtype, copy=False),
                                         kv.v[l][:L].astype(dtype, copy=False), Xs[c],
                                         [L + i for i in range(n)], [list(range(i + 1)) for i in range(n)],
                                         dtype, False)
            kv.k[l][L:L + n] = K
            kv.v[l][L:L + n] = V
        Xn, K, V = _layer_forward(cfg, lw, kv.k[l][:Ln].astype(dtype, copy=False),
                                  kv.v[l][:Ln].astype(dtype, copy=False), Xn,
                                  [Ln + int(d) for d in depth], paths, dtype, False)
        node_k.append(K)
        node_v.append(V)
    kv.len = Ln
    logits = _lin(w["lm_head"], rmsnorm(Xn, w["final_norm"].astype(dtype), cfg.rms_eps), dtype, False)
    return logits, node_k, node_v


def commit(kv: KVCache, node_k, node_v, nodes: Sequence[int]) -> None:
    """Append the listed nodes' keys/values, in order, after the committed prefix."""
    L = kv.len
    if L + len(nodes) > kv.capacity:
        raise ValueError("KV capacity exceeded")
    for l in range(len(kv.k)):
        for i, n in enumerate(nodes):
            kv.k[l][L + i] = node_k[l][n]
            kv.v[l][L + i] = node_v[l][n]
    kv.len = L + len(nodes)


def prefill(cfg: Config, w: dict, kv: KVCache, tokens: Sequence[int], dtype=np.float64,
            row_independent: bool = False, chunk: int = 64) -> None:
    """Run `tokens` causally after the committed prefix and commit their keys/values."""
    tokens = list(tokens)
    for lo in range(0, len(tokens), chunk):
        part = tokens[lo:lo + chunk]
        n = len(part)
        pos = [kv.len + i for i in range(n)]
        paths = [list(range(i + 1)) for i in range(n)]                    # chain
        _, nk, nv = forward_nodes(cfg, w, kv, part, pos, paths, dtype, row_independent,
                                  want_logits=False)
        commit(kv, nk, nv, list(range(n)))


# ----------------------------------------------------------------------------
# temperature sampling (Section 5.3)
# ----------------------------------------------------------------------------
def sample_tokens(logits: np.ndarray, pos: Sequence[int], inv_temperature: float,
                  noise: np.ndarray) -> np.ndarray:
    """Token drawn at each row: argmax_j (logits[r, j] * (1/T) + noise[pos[r], j]), ties to the
    smallest index.  With g ~ Gumbel(0, 1) this is a draw from softmax(logits / T) (Gumbel-max).
    The arithmetic is fixed to float32 (one rounded multiply, one rounded add), because it decides
    an integer: whoever repeats it in float32 gets the same tokens."""
    y = (logits.astype(np.float32) * np.float32(inv_temperature)).astype(np.float32)
    y = (y + noise[np.asarray(pos, dtype=np.int64)].astype(np.float32)).astype(np.float32)
    return np.argmax(y, axis=1).astype(np.int64)            # first occurrence of the maximum


# ----------------------------------------------------------------------------
# decode loops
# ----------------------------------------------------------------------------
@dataclass
class StepResult:
    S: np.ndarray
    logits: np.ndarray
    topk: np.ndarray
    acc: Accept


def integer_pipeline(M: np.ndarray, tree: Tree, S: np.ndarray, logits: np.ndarray, k: int,
                     update_mode: str = "last", update_accepted_only: bool = False, out=None):
    """Top-k, accept and matrix update from given logits (in place on M).  `out` = the model's token
    per node when it is not the argmax (temperature sampling)."""
    topk = np.stack([topk_ids(logits[n], k) for n in range(tree.n_nodes)])
    acc = accept(S, topk[:, 0] if out is None else out, tree)
    update_matrix(M, S, topk, update_mode, acc.path if update_accepted_only else None)
    return topk, acc


def tr_step(cfg: Config, w: dict, kv: KVCache, M: np.ndarray, tree: Tree, root: int, k: int,
            dtype=np.float64, row_independent: bool = False, update_mode: str = "last",
            update_accepted_only: bool = False, sampler=None) -> StepResult:
    """Draft (build_tree), verify (one forward), accept, update M, commit accepted K/V.
    sampler = (1/T, noise[position, vocab]) switches the model's tokens from argmax to draws."""
    S = build_tree(M, tree, root)
    L = kv.len
    pos = [L + int(d) for d in tree.depth]
    logits, nk, nv = forward_nodes(cfg, w, kv, S, pos, tree.paths, dtype, row_independent)
    out = None if sampler is None else sample_tokens(logits, pos, sampler[0], sampler[1])
    topk, acc = integer_pipeline(M, tree, S, logits, k, update_mode, update_accepted_only, out)
    commit(kv, nk, nv, acc.path)
    return StepResult(S, logits, topk, acc)


def tr_generate(cfg: Config, w: dict, M: np.ndarray, tree: Tree, prompt: Sequence[int],
                n_new: int, k: int, capacity: Optional[int] = None, dtype=np.float64,
                row_independent: bool = False, on_step=None, sampler=None):
    """Prefill prompt[:-1], then repeat tr_step from root = prompt[-1] until n_new tokens
    exist (overshoot truncated).  Returns (tokens, accepted_lengths, kv)."""
    capacity = capacity or (len(prompt) + n_new + tree.n_nodes + tree.n_layers)
    kv = KVCache(cfg, capacity, dtype)
    prefill(cfg, w, kv, prompt[:-1], dtype, row_independent)
    root, out, lens = int(prompt[-1]), [], []
    while len(out) < n_new:
        r = tr_step(cfg, w, kv, M, tree, root, k, dtype, row_independent, sampler=sampler)
        out.extend(r.acc.emitted)
        lens.append(r.acc.n_accepted + 1)
        root = r.acc.bonus
        if on_step is not None:
            on_step(r)
    return out[:n_new], lens, kv


def ar_generate(cfg: Config, w: dict, prompt: Sequence[int], n_new: int,
                capacity: Optional[int] = None, dtype=np.float64, row_independent: bool = False,
                sampler=None):
    """Plain decoding (Section 2.1): one token per forward, x = argmax p, or a draw from
    softmax(logits / T) when sampler = (1/T, noise[position, vocab]) is given."""
    capacity = capacity or (len(prompt) + n_new + 1)
    kv = KVCache(cfg, capacity, dtype)
    prefill(cfg, w, kv, prompt[:-1], dtype, row_independent)
    tok, out, all_logits = int(prompt[-1]), [], []
    for _ in range(n_new):
        logits, nk, nv = forward_nodes(cfg, w, kv, [tok], [kv.len], [[0]], dtype, row_independent)
        pos = kv.len
        commit(kv, nk, nv, [0])
        tok = int(topk_ids(logits[0], 1)[0]) if sampler is None else \
            int(sample_tokens(logits, [pos], sampler[0], sampler[1])[0])
        out.append(tok)
        all_logits.append(logits[0])
    return out, all_logits, kv
