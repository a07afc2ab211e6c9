"""Pins for the oracle's transformer forward and tree attention: an independent library
implementation (HuggingFace LlamaForCausalLM in float64) run on every root-to-node
sequence, closed forms, and textbook special cases."""
import numpy as np
import pytest
import torch

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth


def _cfg(sh):
    return O.Config(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn,
                    sh.vocab, sh.rms_eps, sh.rope_theta)


def _hf_model(sh, w):
    tr = pytest.importorskip("transformers")
    kw = dict(vocab_size=sh.vocab, hidden_size=sh.d_model, intermediate_size=sh.d_ffn,
              num_hidden_layers=sh.n_layers, num_attention_heads=sh.n_heads,
              num_key_value_heads=sh.n_kv_heads, head_dim=sh.head_dim, rms_norm_eps=sh.rms_eps,
              hidden_act="silu", attention_bias=False, mlp_bias=False, tie_word_embeddings=False,
              max_position_embeddings=4096, attn_implementation="eager")
    try:
        cfg = tr.LlamaConfig(rope_theta=sh.rope_theta, **kw)
    except TypeError:
        cfg = tr.LlamaConfig(**kw)
    model = tr.LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["final_norm"],
          "lm_head.weight": w["lm_head"]}
    names = {"attn_norm": "input_layernorm", "wq": "self_attn.q_proj", "wk": "self_attn.k_proj",
             "wv": "self_attn.v_proj", "wo": "self_attn.o_proj", "ffn_norm": "post_attention_layernorm",
             "w_gate": "mlp.gate_proj", "w_up": "mlp.up_proj", "w_down": "mlp.down_proj"}
    for l, lw in enumerate(w["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{l}.{names[k]}.weight"] = v
    sd = {k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in sd.items()}
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    return model


def _rand_gains(w, seed):
    """Non-trivial norm gains so that a dropped gain would show."""
    rng = np.random.default_rng(seed)
    w["final_norm"] = (1 + 0.3 * rng.standard_normal(w["final_norm"].shape)).astype(np.float32)
    for lw in w["layers"]:
        for k in ("attn_norm", "ffn_norm"):
            lw[k] = (1 + 0.3 * rng.standard_normal(lw[k].shape)).astype(np.float32)
    return w


@pytest.mark.parametrize("shape_name,row_independent", [("tiny", True), ("tiny", False),
                                                        ("gqa", False), ("gqa", True)])
def test_tree_forward_equals_library_llama_on_every_path(shape_name, row_independent):
    """Section 2.2: node i's distribution is P(x | s, ancestors of i).  Each root-to-node
    sequence is run through an independent causal Llama; its last-row logits must equal
    the oracle's logits for that node in the single tree pass."""
    if shape_name == "tiny":
        sh = synth.SHAPES["tiny"]
    else:
        sh = synth.ModelShape("gqa", 2, 96, 6, 2, 16, 200, 300, "f32")
    w = _rand_gains(synth.weights_to_numpy(synth.make_weights(sh, seed=3)), 0)
    hf = _hf_model(sh, w)
    cfg = _cfg(sh)
    t = synth.tree15()
    tree = O.make_tree(t.parent, t.rank, 8)
    prompt = synth.zipf_prompt(sh.vocab, 21, seed=5).tolist()
    S = synth.random_tokens(sh.vocab, t.n_nodes, seed=9).tolist()
    kv = O.KVCache(cfg, 64)
    O.prefill(cfg, w, kv, prompt, row_independent=row_independent, chunk=8)
    assert kv.len == 21
    pos = [kv.len + int(d) for d in tree.depth]
    logits, _, _ = O.forward_nodes(cfg, w, kv, S, pos, tree.paths, row_independent=row_independent)
    with torch.no_grad():
        for n in range(t.n_nodes):
            seq = prompt + [S[i] for i in tree.paths[n]]
            ref = hf(torch.tensor([seq])).logits[0, -1].numpy()
            # the library computes its rotary tables in float32 whatever the model dtype:
            # agreement is to ~1e-7, structural mistakes are O(0.1)
            assert np.abs(ref - logits[n]).max() < 5e-6 * max(1.0, np.abs(ref).max()), n


def test_batched_and_row_independent_modes_agree():
    sh = synth.SHAPES["tiny"]
    w = synth.weights_to_numpy(synth.make_weights(sh, seed=1))
    cfg = _cfg(sh)
    t = synth.tree15_alt()
    tree = O.make_tree(t.parent, t.rank, 8)
    prompt = synth.zipf_prompt(sh.vocab, 17, seed=2).tolist()
    S = synth.random_tokens(sh.vocab, t.n_nodes, seed=4).tolist()
    res = []
    for ri in (True, False):
        kv = O.KVCache(cfg, 64)
        O.prefill(cfg, w, kv, prompt, row_independent=ri)
        res.append(O.forward_nodes(cfg, w, kv, S, [kv.len + int(d) for d in tree.depth], tree.paths,
                                   row_independent=ri))
    assert np.abs(res[0][0] - res[1][0]).max() < 1e-10
    assert np.abs(res[0][1][1] - res[1][1][1]).max() < 1e-10


def test_attention_special_cases():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((4, 8))
    K = rng.standard_normal((5, 2, 8))
    V = rng.standard_normal((5, 2, 8))
    # one visible key: the output is that key's value, whatever the score
    o = O._attend(q, K[:1], V[:1], 2)
    assert np.allclose(o, V[0][[0, 0, 1, 1]], atol=1e-15)
    # identical keys: uniform weights, output = mean of values
    Ks = np.repeat(K[:1], 5, axis=0)
    o = O._attend(q, Ks, V, 2)
    assert np.allclose(o, V.mean(axis=0)[[0, 0, 1, 1]], atol=1e-14)
    # library softmax attention, head by head
    o = O._attend(q, K, V, 2)
    for h in range(4):
        s = torch.from_numpy(K[:, h // 2] @ q[h] / np.sqrt(8.0))
        ref = (torch.softmax(s, 0)[:, None] * torch.from_numpy(V[:, h // 2])).sum(0).numpy()
        assert np.allclose(o[h], ref, atol=1e-14)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    x, y = rng.standard_normal((3, 16)), rng.standard_normal((3, 16))
    assert np.array_equal(O.rope(x, 0, 10000.0), x)                       # position 0 = identity
    for m in (1, 17, 1000):
        r = O.rope(x, m, 10000.0)
        # pairs (i, i + hd/2) are rotated: pair norms are preserved
        assert np.allclose(r[:, :8] ** 2 + r[:, 8:] ** 2, x[:, :8] ** 2 + x[:, 8:] ** 2)
        # first pair turns by m radians (frequency theta**0 = 1), last pair by m * theta**(-14/16)
        z = (x[:, 0] + 1j * x[:, 8]) * np.exp(1j * m)
        assert np.allclose(r[:, 0] + 1j * r[:, 8], z)
        z = (x[:, 7] + 1j * x[:, 15]) * np.exp(1j * m * 10000.0 ** (-14 / 16))
        assert np.allclose(r[:, 7] + 1j * r[:, 15], z)
    # scores depend on the position difference only
    a = (O.rope(x, 40, 10000.0) * O.rope(y, 33, 10000.0)).sum()
    b = (O.rope(x, 107, 10000.0) * O.rope(y, 100, 10000.0)).sum()
    assert abs(a - b) < 1e-12


def test_rmsnorm_and_silu_closed_forms():
    x = np.full((2, 10), 3.0)
    g = np.arange(10, dtype=np.float64)
    assert np.allclose(O.rmsnorm(x, g, 0.0), np.tile(g, (2, 1)))           # x / |x| * g
    assert np.allclose(O.rmsnorm(x, g, 7.0), np.tile(g, (2, 1)) * 3 / 4)   # 3 / sqrt(9 + 7)
    v = np.linspace(-6, 6, 25)
    assert np.allclose(O.silu(v), torch.nn.functional.silu(torch.from_numpy(v)).numpy())
    assert O.silu(np.zeros(1))[0] == 0.0


class _LazyLayers:
    """w["layers"] stand-in that hands a layer out on access and counts the accesses."""

    def __init__(self, layers):
        self.layers, self.hits = layers, []

    def __getitem__(self, l):
        self.hits.append(l)
        return self.layers[l]


@pytest.mark.parametrize("shape", ["tiny", "tiny_gqa_bf16"])
def test_layer_major_sweep_equals_prefill_then_forward(shape):
    """prefill_then_forward is prefill + forward_nodes with the loops exchanged: same cache, same
    logits, bit for bit, and every layer's weights are fetched exactly once."""
    sh = synth.SHAPES[shape]
    w = synth.weights_to_numpy(synth.make_weights(sh, seed=5))
    cfg = O.Config(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn, sh.vocab)
    t = synth.tree15()
    tree = O.make_tree(t.parent, t.rank, 8)
    prompt = synth.zipf_prompt(sh.vocab, 45, seed=5).tolist()
    S = synth.random_tokens(sh.vocab, tree.n_nodes, seed=6).tolist()
    kv_a, kv_b = O.KVCache(cfg, 96), O.KVCache(cfg, 96)
    pre = synth.zipf_prompt(sh.vocab, 7, seed=8).tolist()     # both start from a non-empty cache
    O.prefill(cfg, w, kv_a, pre)
    O.prefill(cfg, w, kv_b, pre)
    O.prefill(cfg, w, kv_a, prompt, chunk=16)
    lo_a, k_a, v_a = O.forward_nodes(cfg, w, kv_a, S, [kv_a.len + int(d) for d in tree.depth], tree.paths)
    lazy = dict(w, layers=_LazyLayers(w["layers"]))
    lo_b, k_b, v_b = O.prefill_then_forward(cfg, lazy, kv_b, prompt, S, tree.depth, tree.paths, chunk=16)
    assert lazy["layers"].hits == list(range(cfg.n_layers))
    assert kv_a.len == kv_b.len == 7 + 45
    assert np.array_equal(lo_a, lo_b)
    for l in range(cfg.n_layers):
        assert np.array_equal(kv_a.k[l], kv_b.k[l]) and np.array_equal(kv_a.v[l], kv_b.v[l])
        assert np.array_equal(k_a[l], k_b[l]) and np.array_equal(v_a[l], v_b[l])
