"""Pins for the oracle's temperature sampling (Section 5.3): the draw is a draw from
softmax(logits / T), it degenerates to the greedy rule, its float32 arithmetic is the stated one,
and Token Recycling under sampling reproduces plain sampling token for token."""
import numpy as np
import pytest

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth

K = 8


def test_zero_noise_is_the_greedy_rule_with_ties_to_the_smallest_index():
    rng = np.random.default_rng(0)
    logits = rng.normal(0, 3, size=(7, 50)).astype(np.float32)
    logits[2, 11] = logits[2, 40] = logits[2].max() + 1.0          # planted tie
    logits[5, 0] = logits[5, 49] = logits[5].max() + 2.0
    noise = np.zeros((3, 50), np.float32)
    got = O.sample_tokens(logits, [0, 1, 2, 0, 1, 2, 0], 1.0 / 0.7, noise)
    assert got.tolist() == [int(O.topk_ids(logits[r], 1)[0]) for r in range(7)]
    assert got[2] == 11 and got[5] == 0


def test_float32_arithmetic_is_one_rounded_multiply_and_one_rounded_add():
    rng = np.random.default_rng(1)
    logits = rng.normal(0, 3, size=(4, 33)).astype(np.float32)
    noise = synth.gumbel_noise(9, 33, seed=3).numpy()
    pos = [8, 0, 3, 3]
    inv_t = np.float32(1.0 / 0.3)
    want = []
    for r in range(4):
        best, arg = None, -1
        for j in range(33):
            y = np.float32(np.float32(logits[r, j] * inv_t) + noise[pos[r], j])
            if best is None or y > best:
                best, arg = y, j
        want.append(arg)
    assert O.sample_tokens(logits, pos, float(inv_t), noise).tolist() == want


@pytest.mark.parametrize("temperature", [0.5, 1.0])
def test_draws_follow_softmax_of_scaled_logits(temperature):
    """Gumbel-max: over many positions the drawn tokens have the frequencies softmax(logits / T)."""
    logits = np.array([1.5, 0.2, -0.7, 2.1, 0.0, 1.0], np.float32)
    n = 40000
    noise = synth.gumbel_noise(n, 6, seed=5).numpy()
    got = O.sample_tokens(np.tile(logits, (n, 1)), list(range(n)), 1.0 / temperature, noise)
    freq = np.bincount(got, minlength=6) / n
    p = np.exp(logits.astype(np.float64) / temperature)
    p /= p.sum()
    assert np.abs(freq - p).max() < 4 * np.sqrt(0.25 / n)          # 4 sigma of a proportion


def test_low_temperature_is_greedy():
    rng = np.random.default_rng(2)
    logits = rng.normal(0, 3, size=(30, 200)).astype(np.float32)
    noise = synth.gumbel_noise(30, 200, seed=1).numpy()
    got = O.sample_tokens(logits, list(range(30)), 1.0 / 1e-3, noise)
    assert got.tolist() == logits.argmax(axis=1).tolist()


@pytest.mark.parametrize("tmpl", ["tree15", "chain5"])
def test_recycling_under_sampling_reproduces_plain_sampling(tmpl):
    """With the noise tied to the sequence position, a tree node and a one-token decoding step that sit
    at the same position after the same prefix draw the same token, so the speculative run emits exactly
    the sampled sequence of plain decoding (the lossless property of Section 2.2 carried over)."""
    sh = synth.SHAPES["tiny"]
    w = synth.weights_to_numpy(synth.make_weights(sh, seed=0))
    cfg = O.Config(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn, sh.vocab)
    prompt = synth.zipf_prompt(sh.vocab, 40, seed=0, ngram=4).tolist()
    t = synth.chain(5) if tmpl == "chain5" else synth.tree15()
    tree = O.make_tree(t.parent, t.rank, K)
    n_new = 32
    noise = synth.gumbel_noise(len(prompt) + n_new + tree.n_layers + 1, sh.vocab, seed=7).numpy()
    sampler = (1.0 / 0.8, noise)
    M = synth.init_matrix(sh.vocab, K).astype(np.int64)
    toks, lens, _ = O.tr_generate(cfg, w, M, tree, prompt, n_new, K, row_independent=True, sampler=sampler)
    ar, _, _ = O.ar_generate(cfg, w, prompt, n_new, row_independent=True, sampler=sampler)
    assert toks == ar
    greedy, _, _ = O.ar_generate(cfg, w, prompt, n_new, row_independent=True)
    assert toks != greedy                                          # the noise did change the sequence
    assert all(1 <= x <= tree.n_layers for x in lens)
