"""GPU parity at the benchmark's full sizes (bf16): teacher-forced lockstep of whole decode steps
against the float32 oracle, in the launch configuration bench.py times (packed weights, tiled KV,
80-node tree).  The 13B / 70B-GQA widths run with a reduced layer count so that the CPU oracle
stays within a minute; every kernel still sees its real shape."""
import numpy as np
import pytest
import torch

from paper_2408_08696_amd import synth, tr
from gpu_util import lockstep, require_gpu, say

pytestmark = pytest.mark.gpu
K = 8


def _run(sh, prompt_len, n_steps, seed=0):
    tmpl = synth.tree80()
    w = synth.make_weights(sh, seed=seed, device="cuda")
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, prompt_len, seed=seed, ngram=8).tolist()
    eng = tr.Engine(sh, w, tmpl, k=K, capacity=prompt_len + n_steps * tmpl.n_layers + tmpl.n_nodes + 32)
    assert eng.model.packed and eng.kv.tiled
    del w
    stats, _ = lockstep(eng, sh, wn, tmpl, prompt, n_steps, synth.init_matrix(sh.vocab, K), dtype=np.float32,
                        label=sh.name)
    say(stats)
    return stats


@pytest.mark.timeout(900)
def test_7b_shape_lockstep():
    """The benchmark workload itself: 32 layers, d 4096, 32 heads, FFN 11008, vocab 32000, prompt 512."""
    require_gpu()
    stats = _run(synth.SHAPES["7b"], 512, 3)
    assert max(s["max_rel"] for s in stats) <= 2e-2


@pytest.mark.timeout(600)
def test_13b_width_lockstep():
    require_gpu()
    _run(synth.with_layers(synth.SHAPES["13b"], 3), 700, 3, seed=1)


@pytest.mark.timeout(600)
def test_70b_gqa_width_lockstep():
    """64 query heads on 8 KV heads, d 8192, FFN 28672, vocab 128256."""
    require_gpu()
    _run(synth.with_layers(synth.SHAPES["70b"], 2), 400, 2, seed=2)
