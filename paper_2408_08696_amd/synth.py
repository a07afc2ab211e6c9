"""Seeded synthetic inputs for the Token Recycling decode step.

This module only *produces data*: model shapes, random-init weights, prompts,
the initial adjacency matrix and static tree templates.  It holds none of the
method's arithmetic (no forward pass, no tree gather, no accept rule) and it
imports neither the HIP binding nor the CPU oracle; tests and the benchmark
hand its outputs to both sides.

Stand-ins: the paper measures trained Vicuna / Code Llama checkpoints on
SpecBench / MBPP prompts (Section 4.1).  Neither weights nor prompts are
available offline, so weights are random-init at the same shapes and prompts
are Zipf-distributed token ids with planted repeated n-grams (the redundancy
the paper attributes to its workloads, Section 4.2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch


# ----------------------------------------------------------------------------
# model shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "f32" | "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def weight_params(self) -> int:
        """Projection + LM-head parameters streamed once per step (no embedding)."""
        d, hq, hk = self.d_model, self.n_heads * self.head_dim, self.n_kv_heads * self.head_dim
        per_layer = d * hq + 2 * d * hk + hq * d + 3 * d * self.d_ffn
        return self.n_layers * per_layer + self.vocab * d


SHAPES: Dict[str, ModelShape] = {
    # tiny fp32 config the CPU oracle finishes in seconds
    "tiny": ModelShape("tiny", 2, 128, 4, 4, 32, 344, 1024, "f32"),
    # tiny bf16 config with head_dim 128 (exercises the MFMA kernels at toy size)
    "tiny_bf16": ModelShape("tiny_bf16", 2, 256, 2, 2, 128, 672, 2048, "bf16"),
    "tiny_gqa_bf16": ModelShape("tiny_gqa_bf16", 2, 512, 4, 2, 128, 1376, 4096, "bf16"),
    # bf16 shape the packed layout does not cover (d_ffn not a multiple of 32): generic kernels
    "tiny_odd_bf16": ModelShape("tiny_odd_bf16", 2, 192, 3, 3, 64, 500, 1000, "bf16"),
    # packed projections with a head width the matrix-core attention does not take (generic attention, plain KV)
    "tiny_hd64_bf16": ModelShape("tiny_hd64_bf16", 2, 256, 4, 2, 64, 672, 2048, "bf16"),
    # one-layer shapes with a narrow model but a wide FFN / many heads / a large vocabulary: they make the
    # launch planner pick the projection-kernel variants the full-size models use (2, 3, 4 gate/up tile
    # pairs, 3 and 4 Q/K/V tiles, 8 LM-head tiles per workgroup) at a size the CPU oracle runs in seconds
    "zoo_ffn5504": ModelShape("zoo_ffn5504", 1, 256, 2, 2, 128, 5504, 2048, "bf16"),
    "zoo_ffn11008": ModelShape("zoo_ffn11008", 1, 256, 2, 2, 128, 11008, 2048, "bf16"),
    "zoo_ffn13824": ModelShape("zoo_ffn13824", 1, 256, 2, 2, 128, 13824, 2048, "bf16"),
    "zoo_heads32": ModelShape("zoo_heads32", 1, 256, 32, 32, 128, 672, 32000, "bf16"),
    "zoo_heads40": ModelShape("zoo_heads40", 1, 256, 40, 40, 128, 672, 2048, "bf16"),
    "7b": ModelShape("7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16"),
    "13b": ModelShape("13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16"),
    "70b": ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 128256, "bf16"),
}


def with_layers(shape: ModelShape, n_layers: int) -> ModelShape:
    """Same widths, fewer layers (full-width parity cases the oracle can afford)."""
    return ModelShape(f"{shape.name}_l{n_layers}", n_layers, shape.d_model, shape.n_heads,
                      shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab, shape.dtype,
                      shape.rms_eps, shape.rope_theta)


# ----------------------------------------------------------------------------
# counter-based uniform generator (identical on CPU and GPU: integer ops only
# until the final scale, which is one exactly-rounded fp32 multiply)
# ----------------------------------------------------------------------------
_C1, _C2, _C3 = 0x1E3779B1, 0x05EBCA77, 0x42B2AE3D  # odd, < 2**31
_M1, _M2 = 0x7FEB352D, 0x046CA68B                   # odd, < 2**31
_MASK = 0xFFFFFFFF


def _hash_u32(idx: torch.Tensor, seed: int, tensor_id: int) -> torch.Tensor:
    """32-bit mix of (seed, tensor_id, flat index) in int64 arithmetic without overflow."""
    x = (idx * _C1 + ((seed * _C2 + tensor_id * _C3) & _MASK)) & _MASK
    x = x ^ (x >> 16)
    x = (x * _M1) & _MASK
    x = x ^ (x >> 15)
    x = (x * _M2) & _MASK
    x = x ^ (x >> 16)
    return x


def uniform_tensor(shape: Sequence[int], scale: float, seed: int, tensor_id: int,
                   dtype: torch.dtype, device: str | torch.device = "cpu",
                   chunk: int = 1 << 25) -> torch.Tensor:
    """Values (2u-1)*scale with u = top 24 hash bits / 2**24, rounded to `dtype` (RNE)."""
    n = int(np.prod(shape))
    assert n < (1 << 31), "flat index must stay below 2**31"
    out = torch.empty(n, dtype=dtype, device=device)
    s = torch.tensor(scale, dtype=torch.float32, device=device)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = _hash_u32(idx, seed, tensor_id)
        u = (h >> 8).to(torch.float32) * (1.0 / (1 << 24))          # exact in fp32
        out[lo:hi] = ((u * 2.0 - 1.0) * s).to(dtype)
    return out.view(*shape)


def gumbel_noise(n_positions: int, vocab: int, seed: int = 0) -> torch.Tensor:
    """Standard Gumbel noise g = -log(-log(u)), float32 [n_positions, vocab], u from the counter hash
    (strictly inside (0, 1)): the random numbers a temperature-sampling run draws, one row per
    sequence position, handed to both the oracle and the GPU path as an input."""
    n = n_positions * vocab
    idx = torch.arange(n, dtype=torch.int64)
    u = ((_hash_u32(idx, seed, 0x51) >> 8).to(torch.float64) + 0.5) * (1.0 / (1 << 24))
    return (-torch.log(-torch.log(u))).to(torch.float32).view(n_positions, vocab)


_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def head_weights(shape: ModelShape, seed: int = 0, device: str | torch.device = "cpu") -> dict:
    """Embedding table, final norm gain and LM head of make_weights (same values)."""
    dt = _TORCH_DTYPE[shape.dtype]
    d = shape.d_model
    return {
        "embed": uniform_tensor((shape.vocab, d), float(np.sqrt(3.0)), seed, 1, dt, device),
        "final_norm": torch.ones(d, dtype=dt, device=device),
        "lm_head": uniform_tensor((shape.vocab, d), float(np.sqrt(3.0 / d)), seed, 2, dt, device),
    }


def layer_weights(shape: ModelShape, l: int, seed: int = 0, device: str | torch.device = "cpu") -> dict:
    """Layer l of make_weights (same values), so that a large model can be built one layer at a time."""
    dt = _TORCH_DTYPE[shape.dtype]
    d, hd = shape.d_model, shape.head_dim
    hq, hk, f = shape.n_heads * hd, shape.n_kv_heads * hd, shape.d_ffn

    def mat(out_f: int, in_f: int, tid: int) -> torch.Tensor:
        return uniform_tensor((out_f, in_f), float(np.sqrt(3.0 / in_f)), seed, tid, dt, device)

    base = 16 * (l + 1)
    return {
        "attn_norm": torch.ones(d, dtype=dt, device=device),
        "wq": mat(hq, d, base + 0), "wk": mat(hk, d, base + 1), "wv": mat(hk, d, base + 2),
        "wo": mat(d, hq, base + 3),
        "ffn_norm": torch.ones(d, dtype=dt, device=device),
        "w_gate": mat(f, d, base + 4), "w_up": mat(f, d, base + 5), "w_down": mat(d, f, base + 6),
    }


def make_weights(shape: ModelShape, seed: int = 0, device: str | torch.device = "cpu") -> dict:
    """Random-init Llama-style weights, all matrices stored [out, in] row-major.

    Uniform(-s, s) with s = sqrt(3 / fan_in) (unit-variance-preserving), embedding
    s = sqrt(3); norm gains are 1.  Returns
    {"embed", "final_norm", "lm_head", "layers": [{"attn_norm","wq","wk","wv","wo",
    "ffn_norm","w_gate","w_up","w_down"}, ...]} as torch tensors on `device`.
    """
    w = head_weights(shape, seed, device)
    w["layers"] = [layer_weights(shape, l, seed, device) for l in range(shape.n_layers)]
    return w


def weights_to_numpy(w: dict) -> dict:
    """Host float32 numpy copy of `make_weights` output (bf16 values are exact in fp32)."""
    def cv(t: torch.Tensor) -> np.ndarray:
        return t.detach().to("cpu").to(torch.float32).numpy()
    return {
        "embed": cv(w["embed"]), "final_norm": cv(w["final_norm"]), "lm_head": cv(w["lm_head"]),
        "layers": [{k: cv(v) for k, v in layer.items()} for layer in w["layers"]],
    }


# ----------------------------------------------------------------------------
# adjacency matrix, prompts, microbench tensors
# ----------------------------------------------------------------------------
def init_matrix(vocab: int, k: int) -> np.ndarray:
    """M[i, j] = (i + j) mod V, int32 — the initial state the small config names."""
    i = np.arange(vocab, dtype=np.int64)[:, None]
    j = np.arange(k, dtype=np.int64)[None, :]
    return ((i + j) % vocab).astype(np.int32)


def planted_matrix(M0: np.ndarray, seq: Sequence[int], plan: Sequence[int]) -> np.ndarray:
    """Hot-start matrix (the paper's Section 3.1 lets the matrix carry over from earlier text) that
    makes a decoding run accept planned numbers of drafts.  `seq` = the last prompt token followed by
    the tokens decoding will produce; `plan` = accepted drafts wanted per step.  A step that starts at
    seq[s] and is to accept a drafts gets M[seq[s+i], 0] = seq[s+i+1] for i < a, while the row of
    seq[s+a] keeps its value from M0 (the chain breaks there); the next step starts at seq[s+a+1].
    Data only: which lengths a run really accepts is for the caller to observe."""
    M = np.array(M0, copy=True)
    s = 0
    for a in plan:
        if s + a + 1 >= len(seq):
            break
        for i in range(a):
            M[seq[s + i], 0] = seq[s + i + 1]
        s += a + 1
    return M


def zipf_prompt(vocab: int, length: int, seed: int, ngram: int = 4, n_plants: int | None = None,
                alpha: float = 1.1) -> np.ndarray:
    """Token ids with rank r drawn with p ~ r**-alpha (id = r - 1), plus planted repeats:
    `n_plants` spans of `ngram` tokens copied from earlier in the prompt to later offsets."""
    rng = np.random.Generator(np.random.PCG64(seed))
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-alpha)
    p /= p.sum()
    toks = rng.choice(vocab, size=length, p=p).astype(np.int32)
    if n_plants is None:
        n_plants = max(1, length // (4 * ngram))
    if length >= 3 * ngram:
        for _ in range(n_plants):
            src = int(rng.integers(0, length // 2 - ngram + 1))
            dst = int(rng.integers(length // 2, length - ngram + 1))
            toks[dst:dst + ngram] = toks[src:src + ngram]
    return toks


def normal_tensor(shape: Sequence[int], std: float, seed: int, dtype: torch.dtype,
                  device: str | torch.device = "cpu") -> torch.Tensor:
    """N(0, std) values generated on the host (seeded), rounded to `dtype`, moved to `device`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.standard_normal(size=tuple(shape), dtype=np.float32) * np.float32(std)
    return torch.from_numpy(a).to(dtype).to(device)


def random_tokens(vocab: int, n: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=n).astype(np.int32)


# ----------------------------------------------------------------------------
# static tree templates (data only: parent index and candidate rank per node,
# breadth-first / layer-major order, root first)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class TreeTemplate:
    name: str
    parent: np.ndarray  # int32 [N], parent[0] = -1
    rank: np.ndarray    # int32 [N], rank[0] = -1; column of M[token(parent)]
    n_layers: int
    layer_sizes: Tuple[int, ...] = field(default=())

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])


def template_from_child_counts(name: str, counts: List[List[int]]) -> TreeTemplate:
    """counts[d][i] = number of children of the i-th node of layer d; child j takes rank j."""
    parent, rank, sizes = [-1], [-1], [1]
    layer_start, layer_size = 0, 1
    for layer in counts:
        assert len(layer) == layer_size, (name, len(layer), layer_size)
        nxt = 0
        for i, c in enumerate(layer):
            for j in range(c):
                parent.append(layer_start + i)
                rank.append(j)
                nxt += 1
        layer_start += layer_size
        layer_size = nxt
        if nxt:
            sizes.append(nxt)
    return TreeTemplate(name, np.asarray(parent, np.int32), np.asarray(rank, np.int32),
                        len(sizes), tuple(sizes))


def _tree80_counts() -> List[List[int]]:
    # 1 + 8 + 21 + 25 + 15 + 10 = 80 rows in 6 layers; earlier nodes of a layer get more
    # children and go deeper (static + imbalanced, Section 3.2; the paper's own drawing
    # is not available, its first two layer widths 8 and 21 are kept).
    return [
        [8],
        [8, 4, 3, 2, 1, 1, 1, 1],
        [5, 3, 2, 1, 1, 1, 1, 0, 2, 1, 1, 0, 2, 1, 0, 1, 0, 1, 1, 1, 0],
        [4, 2, 1, 1, 0, 2, 1, 0, 1, 0, 1, 0, 0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0],
        [3, 1, 1, 0, 1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0],
    ]


def tree80() -> TreeTemplate:
    return template_from_child_counts("tree80", _tree80_counts())


def tree81() -> TreeTemplate:
    """The paper's row count (81 including the root, Appendix A.2): tree80 plus one leaf."""
    c = _tree80_counts()
    c[4][3] = 1
    return template_from_child_counts("tree81", c)


def tree15() -> TreeTemplate:
    """15 rows, 4 layers: 1 + 4 + 8 + 2."""
    return template_from_child_counts("tree15", [[4], [4, 2, 1, 1], [1, 1, 0, 0, 0, 0, 0, 0]])


def tree15_alt() -> TreeTemplate:
    """15 rows, 4 layers: 1 + 4 + 5 + 5."""
    return template_from_child_counts("tree15_alt", [[4], [2, 1, 1, 1], [1, 1, 1, 1, 1]])


def chain(n: int) -> TreeTemplate:
    return template_from_child_counts(f"chain{n}", [[1]] * (n - 1)) if n > 1 else single()


def single() -> TreeTemplate:
    """Root only: the step degenerates to plain autoregressive decoding."""
    return TreeTemplate("single", np.asarray([-1], np.int32), np.asarray([-1], np.int32), 1, (1,))


def star(n_children: int) -> TreeTemplate:
    return template_from_child_counts(f"star{n_children}", [[n_children]])


def wide128() -> TreeTemplate:
    """128 rows (the library maximum), 8 layers."""
    c = _tree80_counts()
    c[4] = [3, 2, 2, 1, 2, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1]          # 20
    c.append([2, 2, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1])  # 22
    c.append([1] * 16 + [0] * 6)                                   # 16
    t = template_from_child_counts("wide128", c)
    assert t.n_nodes == 128, t.n_nodes
    return t


def prefix_template(n: int) -> TreeTemplate:
    """The first n nodes (breadth-first order) of wide128: a breadth-first prefix of a tree is a tree.
    Used for the step-time-versus-tree-size sweep (the paper's Figure 3a varies breadth the same way)."""
    base = wide128()
    assert 1 <= n <= base.n_nodes
    parent, rank = base.parent[:n].copy(), base.rank[:n].copy()
    depth = np.zeros(n, np.int64)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    sizes = tuple(int(c) for c in np.bincount(depth))
    return TreeTemplate(f"prefix{n}", parent, rank, len(sizes), sizes)


# 80-row templates of 4..8 layers for the depth sweep (the paper's Figure 3b fixes the node count at 80
# and varies the depth; its trees are not given, so these keep 8 children at the root, layer widths that
# fall off with depth, and more children for the earlier nodes of a layer, like tree80)
_DEPTH_LAYER_SIZES = {
    4: (1, 8, 28, 43),
    5: (1, 8, 24, 28, 19),
    6: (1, 8, 21, 25, 15, 10),
    7: (1, 8, 18, 20, 15, 10, 8),
    8: (1, 8, 16, 18, 13, 10, 8, 6),
}


def _spread_children(n_parents: int, n_children: int, k: int) -> List[int]:
    """Child counts for one layer: dealt one at a time to the parent with the largest share still owed,
    shares proportional to 1/(i+1) (earlier parents first on ties), at most k per parent."""
    assert n_children <= n_parents * k
    w = np.array([1.0 / (i + 1) for i in range(n_parents)])
    w = w / w.sum() * n_children
    c = [0] * n_parents
    for _ in range(n_children):
        owed = [(w[i] - c[i]) if c[i] < k else -1e9 for i in range(n_parents)]
        i = int(np.argmax(owed))
        c[i] += 1
    return c


def depth_template(n_layers: int, k: int = 8) -> TreeTemplate:
    """80 rows in n_layers layers (4..8); the 6-layer one is tree80 itself."""
    if n_layers == 6:
        t = tree80()
        return TreeTemplate("depth6", t.parent, t.rank, t.n_layers, t.layer_sizes)
    sizes = _DEPTH_LAYER_SIZES[n_layers]
    counts = [_spread_children(sizes[d], sizes[d + 1], k) for d in range(n_layers - 1)]
    t = template_from_child_counts(f"depth{n_layers}", counts)
    assert t.n_nodes == 80 and t.n_layers == n_layers, (t.n_nodes, t.n_layers)
    return t


TEMPLATES = {
    "tree80": tree80, "tree81": tree81, "tree15": tree15, "tree15_alt": tree15_alt,
    "single": single, "wide128": wide128,
    "depth4": lambda: depth_template(4), "depth5": lambda: depth_template(5), "depth7": lambda: depth_template(7),
    "depth8": lambda: depth_template(8),
}
