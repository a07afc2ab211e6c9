"""GPU parity at the benchmark's full sizes (bf16): teacher-forced lockstep of whole decode steps
against the float32 oracle, in the launch configuration bench.py times (packed weights, tiled KV,
80-node tree).

Two tiers.  Fast: the 7B workload itself with a hot-started matrix (drafts are accepted and compacted),
and the 13B / 70B-GQA widths with a reduced layer count.  Full depth: all 40 layers of the 13B shape
after its 2048-token prompt, and all 80 layers of the 70B-GQA shape at a committed length of 4096; the
oracle then receives its weights one layer at a time (generated on the GPU from the seeded recipe,
copied to the host as float32, dropped) and takes prompt and step through each layer together."""
import time

import numpy as np
import pytest
import torch

from paper_2408_08696_amd import synth, tr
from gpu_util import kv_fill_prefix, lockstep, lockstep_streamed, require_gpu, say

pytestmark = pytest.mark.gpu
K = 8


def _run(sh, prompt_len, n_steps, seed=0, hot_plan=None):
    tmpl = synth.tree80()
    w = synth.make_weights(sh, seed=seed, device="cuda")
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, prompt_len, seed=seed, ngram=8).tolist()
    eng = tr.Engine(sh, w, tmpl, k=K, capacity=prompt_len + n_steps * tmpl.n_layers + tmpl.n_nodes + 32)
    assert eng.model.packed and eng.kv.tiled
    del w
    stats, _ = lockstep(eng, sh, wn, tmpl, prompt, n_steps, synth.init_matrix(sh.vocab, K), dtype=np.float32,
                        label=sh.name, hot_plan=hot_plan)
    say(stats)
    return stats


@pytest.mark.timeout(900)
def test_7b_shape_lockstep():
    """The benchmark workload itself: 32 layers, d 4096, 32 heads, FFN 11008, vocab 32000, prompt 512,
    with the oracle's continuation planted in the matrix (Section 3.1 hot start) so that the steps accept
    1, 5 and 0 drafts: accepted rows are compacted in the tiled cache and the next step attends over them."""
    require_gpu()
    plan = [1, 5, 0, 2]
    stats = _run(synth.SHAPES["7b"], 512, len(plan), hot_plan=plan)
    assert max(s["max_rel"] for s in stats) <= 2e-2
    seen = {s["n_emitted"] - 1 for s in stats}
    assert {0, 1, 5} <= seen, seen


@pytest.mark.timeout(600)
def test_13b_width_lockstep():
    require_gpu()
    _run(synth.with_layers(synth.SHAPES["13b"], 3), 700, 3, seed=1)


@pytest.mark.timeout(600)
def test_70b_gqa_width_lockstep():
    """64 query heads on 8 KV heads, d 8192, FFN 28672, vocab 128256."""
    require_gpu()
    _run(synth.with_layers(synth.SHAPES["70b"], 2), 400, 2, seed=2)


def _packed_model(sh, seed):
    """The model as bench.py builds the large shapes: generated and packed one layer at a time."""
    packed = synth.head_weights(sh, seed=seed, device="cuda")
    packed["lm_head"] = tr.pack_weight(packed["lm_head"])
    packed["layers"] = []
    for l in range(sh.n_layers):
        lw = synth.layer_weights(sh, l, seed=seed, device="cuda")
        packed["layers"].append(tr.pack_layer(sh, lw))
        del lw
        if l % 16 == 15:
            torch.cuda.synchronize()
            say(f"  model layer {l + 1}/{sh.n_layers} generated and packed")
    return tr.ModelDesc(sh, packed, pack=True, prepacked=True)


@pytest.mark.timeout(900)
def test_13b_full_depth_lockstep():
    """All 40 layers of the 13B shape after its 2048-token prompt (2047 committed by the GPU prefill and by
    the oracle's causal prefill), one whole step; prints the largest relative logit error and the flips."""
    require_gpu()
    sh, seed, tmpl = synth.SHAPES["13b"], 1, synth.tree80()
    t0 = time.time()
    prompt = synth.zipf_prompt(sh.vocab, 2048, seed=seed, ngram=8).tolist()
    eng = tr.Engine(sh, None, tmpl, k=K, capacity=2048 + tmpl.n_layers + tmpl.n_nodes + 32,
                    model=_packed_model(sh, seed))
    assert eng.model.packed and eng.kv.tiled
    stats, _ = lockstep_streamed(eng, sh, seed, tmpl, prompt, 1, synth.init_matrix(sh.vocab, K), label="13b full depth")
    say(stats, f"{time.time() - t0:.0f} s")
    assert max(s["max_rel"] for s in stats) <= 2e-2


@pytest.mark.timeout(900)
def test_70b_full_depth_lockstep():
    """All 80 layers of the 70B-GQA shape at the committed length of its workload (4096): the cache starts
    with 3840 positions of seeded N(0,1) bf16 keys / values on both sides (the oracle cannot afford the
    causal prefill of 4095 tokens through 80 layers: about 137 Gflop per token), then a 257-token Zipf prompt
    goes through the GPU prefill and the oracle's, then one whole step.  Prints the largest relative logit
    error and the flips."""
    require_gpu()
    sh, seed, tmpl = synth.SHAPES["70b"], 2, synth.tree80()
    t0 = time.time()
    P0, plen = 3840, 257
    prompt = synth.zipf_prompt(sh.vocab, plen, seed=seed, ngram=8).tolist()
    eng = tr.Engine(sh, None, tmpl, k=K, capacity=P0 + plen + tmpl.n_layers + tmpl.n_nodes + 32,
                    model=_packed_model(sh, seed))
    assert eng.model.packed and eng.kv.tiled
    Hkv, hd = sh.n_kv_heads, sh.head_dim
    pk = np.empty((sh.n_layers, P0, Hkv, hd), np.float32)
    pv = np.empty((sh.n_layers, P0, Hkv, hd), np.float32)
    for l in range(sh.n_layers):
        kt = synth.normal_tensor((Hkv, P0, hd), 1.0, seed=1000 + 2 * l, dtype=torch.bfloat16)
        vt = synth.normal_tensor((Hkv, P0, hd), 1.0, seed=1001 + 2 * l, dtype=torch.bfloat16)
        kv_fill_prefix(eng.kv, l, kt.cuda(), vt.cuda(), k_interleaved=True)
        pk[l] = kt.float().numpy().transpose(1, 0, 2)
        pv[l] = vt.float().numpy().transpose(1, 0, 2)
    eng.kv.reset(P0)
    say(f"70b: model and cache prefix ready, {time.time() - t0:.0f} s")
    stats, _ = lockstep_streamed(eng, sh, seed, tmpl, prompt, 1, synth.init_matrix(sh.vocab, K),
                                 prefix_kv=(pk, pv), label="70b full depth")
    say(stats, f"{time.time() - t0:.0f} s")
    assert max(s["max_rel"] for s in stats) <= 2e-2
