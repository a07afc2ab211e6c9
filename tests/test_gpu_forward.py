"""GPU parity of the verification forward and of whole decode steps against the oracle."""
import numpy as np
import pytest
import torch

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth, tr
from gpu_util import kv_fill, kv_plain_views, lockstep, oracle_cfg, require_gpu, say, to_gpu
from test_oracle_loop import FIXTURE_MIN_GAP, fixture_min_gap

pytestmark = pytest.mark.gpu
K = 8


@pytest.mark.parametrize("tmpl_name", ["tree15", "tree15_alt", "single"])
def test_tiny_fp32_free_running(tmpl_name):
    """The small fp32 config end to end, free running: 64 new tokens; emitted tokens, trees,
    accepted lengths and M bit-exact, logits within 1e-4 absolute — and within a quarter of the
    smallest top-k gap of the run, so no decision could have flipped."""
    require_gpu()
    sh = synth.SHAPES["tiny"]
    tmpl = synth.TEMPLATES[tmpl_name]()
    w = synth.make_weights(sh, seed=0)
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, 64, seed=0, ngram=4).tolist()
    M0 = synth.init_matrix(sh.vocab, K)
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=64 + 64 + tmpl.n_nodes + 8)
    eng.ctx.matrix_load(M0)
    eng.prefill(prompt)

    cfg = oracle_cfg(sh)
    tree = O.make_tree(tmpl.parent, tmpl.rank, K)
    M = M0.astype(np.int64)
    steps = []
    toks, lens, kv = O.tr_generate(cfg, wn, M, tree, prompt, 64, K, on_step=steps.append)
    M_run = M0.astype(np.int64)
    got, max_err = [], 0.0
    for i, r in enumerate(steps):
        say("tiny fp32", tmpl_name, "step", i)
        h = eng.step(sync=True)
        assert eng.S.cpu().tolist() == r.S.tolist(), f"step {i}: tree"
        max_err = max(max_err, float(np.abs(eng.logits.cpu().numpy() - r.logits).max()))
        assert np.array_equal(eng.topk.cpu().numpy(), r.topk), f"step {i}: top-k"
        assert h.n_accepted == r.acc.n_accepted and list(h.path[:h.n_emitted]) == r.acc.path
        assert list(h.emitted[:h.n_emitted]) == r.acc.emitted
        got.extend(h.emitted[:h.n_emitted])
        O.update_matrix(M_run, r.S, r.topk)
        assert np.array_equal(eng.ctx.matrix_store().astype(np.int64), M_run), f"step {i}: matrix"
    assert got[:64] == toks
    ar, _, _ = O.ar_generate(cfg, wn, prompt, 64)
    assert got[:64] == ar                                     # lossless on the GPU too
    say("max |logit error|", max_err)
    assert max_err < 1e-4
    if tmpl_name == "tree15":
        assert 4 * max_err < FIXTURE_MIN_GAP <= fixture_min_gap(0)
    # committed KV equals the oracle's cache (K as stored, V transposed)
    L = kv.len
    kp, vp = kv_plain_views(eng.kv)
    kg = kp[:, :, :L, :].permute(0, 2, 1, 3).cpu().numpy()
    vg = vp[:, :, :L, :].permute(0, 2, 1, 3).cpu().numpy()
    for l in range(sh.n_layers):
        assert np.abs(kg[l] - kv.k[l][:L]).max() < 1e-4 and np.abs(vg[l] - kv.v[l][:L]).max() < 1e-4


@pytest.mark.parametrize("shape_name,tmpl_name", [("tiny_bf16", "tree80"), ("tiny_gqa_bf16", "tree80"),
                                                  ("tiny_bf16", "tree81"), ("tiny_bf16", "wide128"),
                                                  ("tiny_bf16", "single"), ("tiny", "tree80"),
                                                  ("tiny_odd_bf16", "tree80"), ("tiny_bf16:rowmajor", "tree15"),
                                                  ("tiny_bf16", "prefix48"), ("tiny_gqa_bf16", "prefix97"),
                                                  # the depth sweep's 80-node templates of 4, 5, 7 and 8 layers
                                                  ("tiny_bf16", "depth4"), ("tiny_bf16", "depth5"),
                                                  ("tiny_gqa_bf16", "depth7"), ("tiny_bf16", "depth8"),
                                                  ("tiny_hd64_bf16", "tree80"), ("tiny_gqa_bf16:plainkv", "tree80"),
                                                  # projection-kernel variants of the full-size models
                                                  ("zoo_ffn5504", "tree80"), ("zoo_ffn5504", "tree81"),
                                                  ("zoo_ffn11008", "tree80"), ("zoo_ffn11008", "wide128"),
                                                  ("zoo_ffn11008", "single"), ("zoo_ffn13824", "tree80"),
                                                  ("zoo_ffn13824", "prefix64"), ("zoo_heads32", "tree80"),
                                                  ("zoo_heads40", "tree80"), ("zoo_heads32", "wide128")])
def test_small_shapes_lockstep(shape_name, tmpl_name):
    require_gpu()
    pack, kv_tiled = None, None
    if shape_name.endswith(":rowmajor"):
        shape_name, pack = shape_name.split(":")[0], False    # bf16 through the generic kernels
    if shape_name.endswith(":plainkv"):
        shape_name, kv_tiled = shape_name.split(":")[0], False  # packed projections, position-major cache
    sh = synth.SHAPES[shape_name]
    tmpl = (synth.prefix_template(int(tmpl_name[6:])) if tmpl_name.startswith("prefix")
            else synth.TEMPLATES[tmpl_name]())
    w = synth.make_weights(sh, seed=1)
    prompt = synth.zipf_prompt(sh.vocab, 150, seed=3, ngram=8).tolist()
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=512, pack=pack, kv_tiled=kv_tiled)
    assert eng.model.packed == (tr.can_pack(sh) if pack is None else pack)
    assert eng.kv.tiled == ((sh.dtype == "bf16" and sh.head_dim == 128) if kv_tiled is None else kv_tiled)
    abs_tol = 1e-4 if sh.dtype == "f32" else None
    stats, _ = lockstep(eng, sh, synth.weights_to_numpy(w), tmpl, prompt, 6, synth.init_matrix(sh.vocab, K),
                        abs_tol=abs_tol, label=f"{shape_name}/{tmpl_name}")
    say(stats)


HOT_PLAN = [5, 1, 0, 5, 2, 0, 1, 3]


@pytest.mark.parametrize("shape_name,tmpl_name", [("tiny_bf16", "tree80"), ("tiny_gqa_bf16", "tree80"),
                                                  ("zoo_heads32", "tree80"), ("tiny_gqa_bf16:plainkv", "tree80"),
                                                  ("tiny_bf16", "wide128"), ("tiny", "tree15")])
def test_hot_started_lockstep_accepts_drafts(shape_name, tmpl_name):
    """Whole steps on the packed / matrix-core / tiled-cache path with drafts really accepted
    (Section 2.2 chain rule, Section 3.3): the matrix starts with the oracle's continuation of the
    prompt planted (Section 3.1 hot start), so steps accept 0, 1, ... depth-1 drafts, the accepted
    rows are compacted, and the next step attends over the compacted rows.  Every step is compared
    with the oracle, and so are the cache rows each step commits."""
    require_gpu()
    kv_tiled = None
    if shape_name.endswith(":plainkv"):
        shape_name, kv_tiled = shape_name.split(":")[0], False
    sh = synth.SHAPES[shape_name]
    tmpl = synth.TEMPLATES[tmpl_name]()
    plan = [tmpl.n_layers - 1 if a == 5 else min(a, tmpl.n_layers - 1) for a in HOT_PLAN]
    w = synth.make_weights(sh, seed=1)
    prompt = synth.zipf_prompt(sh.vocab, 150, seed=3, ngram=8).tolist()
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=512, kv_tiled=kv_tiled)
    stats, _ = lockstep(eng, sh, synth.weights_to_numpy(w), tmpl, prompt, len(plan), synth.init_matrix(sh.vocab, K),
                        abs_tol=1e-4 if sh.dtype == "f32" else None, label=f"hot {shape_name}/{tmpl_name}",
                        hot_plan=plan, check_cache=True)
    say(stats)
    seen = {s["n_emitted"] - 1 for s in stats}
    assert {0, 1, tmpl.n_layers - 1} <= seen, seen


def test_hot_started_sampling_lockstep():
    """The same under temperature sampling (Section 5.3): the planted continuation is the oracle's
    sampled one (same per-position noise), so sampled drafts are accepted and compacted."""
    require_gpu()
    sh = synth.SHAPES["tiny_gqa_bf16"]
    tmpl = synth.tree80()
    w = synth.make_weights(sh, seed=4)
    prompt = synth.zipf_prompt(sh.vocab, 70, seed=4).tolist()
    noise = synth.gumbel_noise(70 + (len(HOT_PLAN) + 1) * tmpl.n_layers, sh.vocab, seed=9).numpy()
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=70 + len(HOT_PLAN) * tmpl.n_layers + tmpl.n_nodes + 32)
    stats, _ = lockstep(eng, sh, synth.weights_to_numpy(w), tmpl, prompt, len(HOT_PLAN),
                        synth.init_matrix(sh.vocab, K), label="hot sampling", sampler=(1.0, noise),
                        hot_plan=HOT_PLAN, check_cache=True)
    say(stats)
    seen = {s["n_emitted"] - 1 for s in stats}
    assert {0, 1, tmpl.n_layers - 1} <= seen, seen


@pytest.mark.parametrize("shape_name,temperature", [("tiny", 0.8), ("tiny_bf16", 0.5), ("tiny_gqa_bf16", 1.0)])
def test_temperature_sampling_lockstep(shape_name, temperature):
    """Whole steps under temperature sampling (Section 5.3): drawn tokens, accept lengths, emitted
    tokens, the matrix and the cache length must follow the oracle's rule applied to the GPU's logits."""
    require_gpu()
    sh = synth.SHAPES[shape_name]
    tmpl = synth.tree80()
    w = synth.make_weights(sh, seed=4)
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, 70, seed=4).tolist()
    n_steps = 6
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=70 + n_steps * tmpl.n_layers + tmpl.n_nodes + 32)
    noise = synth.gumbel_noise(70 + (n_steps + 1) * tmpl.n_layers, sh.vocab, seed=9).numpy()
    stats, _ = lockstep(eng, sh, wn, tmpl, prompt, n_steps, synth.init_matrix(sh.vocab, K),
                        abs_tol=1e-4 if sh.dtype == "f32" else None, label=f"{shape_name} T={temperature}",
                        sampler=(1.0 / temperature, noise))
    say(stats)


def test_prefill_crosses_chunk_boundaries():
    """A 300-token prompt goes through three chain chunks (128 + 128 + 43); the cache must equal
    the oracle's causal prefill."""
    require_gpu()
    sh = synth.SHAPES["tiny"]
    w = synth.make_weights(sh, seed=2)
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, 300, seed=1).tolist()
    eng = tr.Engine(sh, to_gpu(w), synth.tree15(), k=K, capacity=400)
    eng.prefill(prompt)
    torch.cuda.synchronize()
    assert int(eng.kv.d_len.item()) == 299 and eng.kv.c.len_bound == 299
    cfg = oracle_cfg(sh)
    kv = O.KVCache(cfg, 400)
    O.prefill(cfg, wn, kv, prompt[:-1])
    kp, vp = kv_plain_views(eng.kv)
    kg = kp[:, :, :299, :].permute(0, 2, 1, 3).cpu().numpy()
    vg = vp[:, :, :299, :].permute(0, 2, 1, 3).cpu().numpy()
    for l in range(sh.n_layers):
        assert np.abs(kg[l] - kv.k[l][:299]).max() < 1e-4
        assert np.abs(vg[l] - kv.v[l][:299]).max() < 1e-4


@pytest.mark.parametrize("shape_name,plen", [("tiny_bf16", 100), ("tiny_bf16", 150), ("tiny_gqa_bf16", 150),
                                             ("tiny_bf16", 513), ("tiny_gqa_bf16", 600), ("tiny_bf16", 700),
                                             ("zoo_heads32", 300), ("tiny_gqa_bf16", 1100), ("tiny_bf16", 2049)])
def test_packed_prefill_cache_matches_oracle(shape_name, plen):
    """Packed bf16 models rotate and store queries, keys and values in the epilogue of the fused Q/K/V
    projection; the committed cache must hold the oracle's keys (read back through the interleaved feature
    order of such models) and values, to bf16 accuracy.  With a tiled cache, prompts beyond 128 tokens go
    through the wide projection kernel in passes of up to 512 rows with attention per block of 128: the
    lengths cover one decode-path pass (99 rows), a ragged second block (149), exactly one full pass (512), a
    full pass plus a decode-path remainder (599 = 512 + 87), plus a ragged wide pass (699 = 512 + 187), a
    single-layer model (only the Q/K/V projection runs), two full passes (1099 = 512 + 512 + 75) and four (2048)."""
    require_gpu()
    say("packed prefill cache", shape_name, plen)
    sh = synth.SHAPES[shape_name]
    w = synth.make_weights(sh, seed=2)
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, plen, seed=2).tolist()
    eng = tr.Engine(sh, to_gpu(w), synth.tree15(), k=K, capacity=plen + 106)
    assert eng.model.packed and eng.kv.tiled
    eng.prefill(prompt)
    torch.cuda.synchronize()
    n = plen - 1
    assert int(eng.kv.d_len.item()) == n and eng.kv.c.len_bound == n
    cfg = oracle_cfg(sh)
    kv = O.KVCache(cfg, plen + 106)
    O.prefill(cfg, wn, kv, prompt[:-1])
    kp, vp = kv_plain_views(eng.kv, k_interleaved=True)
    kg = kp[:, :, :n, :].permute(0, 2, 1, 3).float().cpu().numpy()
    vg = vp[:, :, :n, :].permute(0, 2, 1, 3).float().cpu().numpy()
    for l in range(sh.n_layers):
        # per row, so that a wrong row in one block cannot hide behind the largest entry of the whole cache
        dk = np.abs(kg[l] - kv.k[l][:n]).max(axis=(1, 2)) / np.abs(kv.k[l][:n]).max(axis=(1, 2))
        dv = np.abs(vg[l] - kv.v[l][:n]).max(axis=(1, 2)) / np.abs(kv.v[l][:n]).max(axis=(1, 2))
        say("layer", l, "relative K error", dk.max(), "at row", int(dk.argmax()), "V error", dv.max(), "at row",
            int(dv.argmax()))
        assert dk.max() < 2e-2 and dv.max() < 2e-2


def test_packed_prefill_appends_after_a_committed_prefix():
    """Two calls: 201 tokens, then 400 more on top (keep_cache).  The second call's wide pass starts at a
    non-zero committed length, so its rotary positions, cache rows and attention prefixes are all offset;
    the cache must equal the oracle's single causal prefill of all 600 tokens."""
    require_gpu()
    sh = synth.SHAPES["tiny_gqa_bf16"]
    w = synth.make_weights(sh, seed=4)
    wn = synth.weights_to_numpy(w)
    prompt = synth.zipf_prompt(sh.vocab, 601, seed=4).tolist()
    eng = tr.Engine(sh, to_gpu(w), synth.tree15(), k=K, capacity=720)
    assert eng.model.packed and eng.kv.tiled
    eng.prefill(prompt[:201])                      # commits 200, the 201st becomes the root and is dropped here
    eng.prefill(prompt[200:], keep_cache=True)     # commits tokens 200 .. 599
    torch.cuda.synchronize()
    n = 600
    assert int(eng.kv.d_len.item()) == n and eng.kv.c.len_bound == n
    cfg = oracle_cfg(sh)
    kv = O.KVCache(cfg, 720)
    O.prefill(cfg, wn, kv, prompt[:n])
    kp, vp = kv_plain_views(eng.kv, k_interleaved=True)
    kg = kp[:, :, :n, :].permute(0, 2, 1, 3).float().cpu().numpy()
    vg = vp[:, :, :n, :].permute(0, 2, 1, 3).float().cpu().numpy()
    for l in range(sh.n_layers):
        dk = np.abs(kg[l] - kv.k[l][:n]).max(axis=(1, 2)) / np.abs(kv.k[l][:n]).max(axis=(1, 2))
        dv = np.abs(vg[l] - kv.v[l][:n]).max(axis=(1, 2)) / np.abs(kv.v[l][:n]).max(axis=(1, 2))
        say("layer", l, "relative K error", dk.max(), "V error", dv.max())
        assert dk.max() < 2e-2 and dv.max() < 2e-2


def test_pack_weight_rope_interleaves_rows():
    """y = x W^T through a matrix packed with tr_pack_weight_rope comes out with output feature
    h*hd + 2j + b holding what feature h*hd + j + b*hd/2 holds with the plain packing."""
    require_gpu()
    n, K_, O_, hd = 33, 256, 512, 128
    x = synth.normal_tensor((n, K_), 1.0, seed=4, dtype=torch.bfloat16)
    wt = synth.uniform_tensor((O_, K_), float(np.sqrt(3.0 / K_)), seed=6, tensor_id=3, dtype=torch.bfloat16)
    ctx = tr.Context(16, 8, [-1], [-1], 1)
    ws = torch.empty(((n + 15) // 16 * 16 * K_ * 2 + 512 + n * O_ * 4 + 512), dtype=torch.uint8, device="cuda")
    y0 = torch.zeros(n, O_, dtype=torch.float32, device="cuda")
    y1 = torch.zeros_like(y0)
    ctx.op_linear(x.cuda(), tr.pack_weight(wt.cuda()), y0, ws, packed=True, splits=1)
    ctx.op_linear(x.cuda(), tr.pack_weight(wt.cuda(), rope_head_dim=hd), y1, ws, packed=True, splits=1)
    o = np.arange(O_)
    src = (o // hd) * hd + (o % hd) // 2 + ((o % hd) % 2) * (hd // 2)
    assert np.array_equal(y1.cpu().numpy(), y0.cpu().numpy()[:, src])
    with pytest.raises(tr.TRError):
        tr.pack_weight(wt.cuda(), rope_head_dim=96)            # 512 is not a multiple of 96


def test_capacity_is_checked_on_the_host():
    require_gpu()
    sh = synth.SHAPES["tiny"]
    w = synth.make_weights(sh, seed=2)
    tmpl = synth.tree15()
    eng = tr.Engine(sh, to_gpu(w), tmpl, k=K, capacity=64)
    assert eng.kv.capacity == 64
    with pytest.raises(tr.TRError) as e:
        eng.prefill(list(range(80)))
    assert e.value.status == tr.TR_ECAPACITY
    eng.prefill(list(range(55)))
    with pytest.raises(tr.TRError) as e:
        eng.step()                                            # 54 + 15 > 64
    assert e.value.status == tr.TR_ECAPACITY


@pytest.mark.parametrize("tmpl_name,H,Hkv,L,tiled", [("tree80", 32, 32, 1024, True), ("tree80", 8, 2, 1000, True),
                                                     ("tree81", 4, 4, 37, True), ("wide128", 4, 1, 300, True),
                                                     ("single", 8, 8, 513, True), ("tree15", 4, 4, 0, True),
                                                     ("tree80", 4, 2, 200, False),
                                                     # grouped-query shapes: the 70B head layout at its prompt
                                                     # length (two heads per workgroup), an odd group (one head
                                                     # per workgroup), six node tiles with shared heads, one node
                                                     ("tree80", 64, 8, 4096, True), ("tree80", 6, 2, 150, True),
                                                     ("prefix96", 8, 4, 70, True), ("single", 16, 2, 777, True)])
def test_tree_attention_matches_per_path_attention(tmpl_name, H, Hkv, L, tiled):
    """One layer of tree attention at the microbenchmark shape (32 heads x 128, prefix 1024, 80
    nodes, N(0,1) values) and smaller ones: every node must equal plain softmax attention over
    (prefix, its root-to-node path) computed by the oracle in float64."""
    require_gpu()
    say("tree attention", tmpl_name, H, Hkv, L, tiled)
    t = synth.prefix_template(int(tmpl_name[6:])) if tmpl_name.startswith("prefix") else synth.TEMPLATES[tmpl_name]()
    tree = O.make_tree(t.parent, t.rank, K)
    n, hd = t.n_nodes, 128
    sh = synth.ModelShape("att", 1, H * hd, H, Hkv, hd, 64, 64, "bf16")
    kv = tr.KVDesc(sh, capacity=L + n + 5, tiled=tiled)
    kv.reset(L)
    q = synth.normal_tensor((n, H, hd), 1.0, seed=1, dtype=torch.bfloat16)
    kp = synth.normal_tensor((1, Hkv, kv.capacity, hd), 1.0, seed=2, dtype=torch.bfloat16)
    vp = synth.normal_tensor((1, Hkv, kv.capacity, hd), 1.0, seed=3, dtype=torch.bfloat16)
    kv_fill(kv, kp.cuda(), vp.cuda())
    ctx = tr.Context(64, K, t.parent, t.rank, t.n_layers)
    out = torch.zeros(n, H, hd, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(16 * 128 * H * (2 + hd) * 4 + 4096, dtype=torch.uint8, device="cuda")
    ctx.op_tree_attention(kv, 0, H, q.cuda(), out, ws)
    got = out.float().cpu().numpy()
    qn = q.double().numpy()
    kn = kp[0].double().numpy().transpose(1, 0, 2)             # [cap, Hkv, hd]
    vn = vp[0].double().numpy().transpose(1, 0, 2)
    worst = 0.0
    for i in range(n):
        idx = list(range(L)) + [L + j for j in tree.paths[i]]
        ref = O._attend(qn[i], kn[idx], vn[idx], H // Hkv)
        err = np.abs(got[i] - ref).max()
        worst = max(worst, err / np.abs(ref).max())
        assert err <= 2e-2 * np.abs(ref).max(), (i, err)
    say("worst relative error", worst)


@pytest.mark.parametrize("n,K_,O_,splits", [(80, 4096, 4096, 2), (80, 11008, 4096, 2), (81, 4096, 1024, 4),
                                            (1, 4096, 512, 1), (128, 512, 2048, 1), (16, 256, 64, 1),
                                            (80, 1024, 32000, 1), (80, 4096, 12288, 1), (37, 96, 32, 3),
                                            # above 128 rows: the prompt-ingestion kernel in each of its shapes
                                            (129, 64, 32, 1), (250, 4096, 4096, 4), (256, 736, 2080, 1),
                                            (300, 256, 18432, 1), (511, 4096, 4608, 4), (512, 11008, 4096, 4),
                                            (401, 4096, 1024, 4), (300, 2240, 96, 3)])
def test_linear_bf16_packed_matches_oracle_matmul(n, K_, O_, splits):
    """The projection kernel alone (packed weights, MFMA) against a float64 matrix product of the
    same bf16 values; also checks the repack kernel, since a misplaced element would show here.
    Row counts above 128 reach the prompt-ingestion kernel, whose launcher picks the workgroup shape (12 out-tiles
    x 2 row tiles per wave, 6 x 4 with one workgroup over all rows, or 6 x 2) and the K-splits from a cost model:
    the cases cover one and two row blocks, ragged out-tile groups (2080 features), an odd number of k-steps
    (736), the 6 x 4 shape (18432 features), and K-split shares that are rounded to whole stages and leave a
    shorter last share (11008, 2240 in-features)."""
    require_gpu()
    say("linear packed", n, K_, O_, splits)
    x = synth.normal_tensor((n, K_), 1.0, seed=n + K_, dtype=torch.bfloat16)
    w = synth.uniform_tensor((O_, K_), float(np.sqrt(3.0 / K_)), seed=5, tensor_id=O_, dtype=torch.bfloat16)
    ctx = tr.Context(16, 8, [-1], [-1], 1)
    y = torch.zeros(n, O_, dtype=torch.float32, device="cuda")
    ws = torch.empty(((n + 15) // 16 * 16 * K_ * 2 + 512 + splits * n * O_ * 4 + 512), dtype=torch.uint8, device="cuda")
    wp = tr.pack_weight(w.cuda())
    ctx.op_linear(x.cuda(), wp, y, ws, packed=True, splits=splits)
    ref = x.double().numpy() @ w.double().numpy().T
    err = np.abs(y.cpu().numpy() - ref).max()
    say("max err", err)
    assert err < 2e-5 * np.sqrt(K_)                           # fp32 accumulation of K products of O(1/sqrt(K))


def test_linear_row_limits():
    """Packed weights take up to TR_PREFILL_ROWS rows (the prompt-ingestion kernel above TR_MAX_NODES), row-major
    ones TR_MAX_NODES; one more is TR_EINVAL, on the host, before any launch."""
    require_gpu()
    ctx = tr.Context(16, 8, [-1], [-1], 1)
    K_, O_ = 64, 32
    w = synth.uniform_tensor((O_, K_), 0.1, seed=1, tensor_id=0, dtype=torch.bfloat16).cuda()
    wp = tr.pack_weight(w)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    for n, packed, ok in ((512, True, True), (513, True, False), (128, False, True), (129, False, False)):
        x = torch.zeros(n, K_, dtype=torch.bfloat16, device="cuda")
        y = torch.zeros(n, O_, dtype=torch.float32, device="cuda")
        if ok:
            ctx.op_linear(x, wp if packed else w, y, ws, packed=packed, splits=1)
        else:
            with pytest.raises(tr.TRError) as e:
                ctx.op_linear(x, wp if packed else w, y, ws, packed=packed, splits=1)
            assert e.value.status == tr.TR_EINVAL
    torch.cuda.synchronize()


def test_linear_packed_every_planned_variant():
    """Every (row tiles, weight tiles per workgroup) pair the launch planner can choose over a grid of shapes,
    with 1, 2 and 4 K-splits, is run once at the cheapest shape that selects it, against a float64 matrix
    product."""
    require_gpu()
    chosen = {}
    for n in (1, 5, 16, 17, 33, 48, 64, 65, 80, 96, 97, 112, 128):
        for K_ in (256, 1024, 2048, 4096, 8192, 11008):
            for O_ in (64, 256, 1024, 2048, 4096, 8192, 12288, 32000):
                if K_ * O_ > 140e6:
                    continue
                for ms in (1, 2, 4):
                    p, _, _ = tr.plan_projection(n, K_, O_, False, ms)
                    key, cost = ((n + 15) // 16, p, ms), n * K_ * O_   # the op runs exactly ms K-splits
                    if key not in chosen or cost < chosen[key][0]:
                        chosen[key] = (cost, (n, K_, O_, ms))
    assert len(chosen) >= 70, len(chosen)
    ctx = tr.Context(16, 8, [-1], [-1], 1)
    for key, (_, (n, K_, O_, ms)) in sorted(chosen.items()):
        say("linear variant", key, "shape", n, K_, O_, "max splits", ms)
        x = synth.normal_tensor((n, K_), 1.0, seed=n + K_, dtype=torch.bfloat16)
        w = synth.uniform_tensor((O_, K_), float(np.sqrt(3.0 / K_)), seed=7, tensor_id=O_, dtype=torch.bfloat16)
        y = torch.zeros(n, O_, dtype=torch.float32, device="cuda")
        ws = torch.empty(((n + 15) // 16 * 16 * K_ * 2 + 512 + ms * n * O_ * 4 + 512), dtype=torch.uint8, device="cuda")
        ctx.op_linear(x.cuda(), tr.pack_weight(w.cuda()), y, ws, packed=True, splits=ms)
        ref = x.double().numpy() @ w.double().numpy().T
        err = np.abs(y.cpu().numpy() - ref).max()
        assert err < 2e-5 * np.sqrt(K_), (key, n, K_, O_, ms, err)
    ctx.close()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_linear_generic_matches_oracle_matmul(dtype):
    require_gpu()
    n, K_, O_ = 45, 344, 130
    x = synth.normal_tensor((n, K_), 1.0, seed=1, dtype=dtype)
    w = synth.uniform_tensor((O_, K_), float(np.sqrt(3.0 / K_)), seed=5, tensor_id=3, dtype=dtype)
    ctx = tr.Context(16, 8, [-1], [-1], 1)
    y = torch.zeros(n, O_, dtype=torch.float32, device="cuda")
    ctx.op_linear(x.cuda(), w.cuda(), y)
    ref = x.double().numpy() @ w.double().numpy().T
    assert np.abs(y.cpu().numpy() - ref).max() < 2e-5 * np.sqrt(K_)


def test_pack_rejects_bad_sizes():
    require_gpu()
    w = torch.zeros(48, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(tr.TRError) as e:
        tr.pack_weight(w)                                      # 48 is not a multiple of 32
    assert e.value.status == tr.TR_EINVAL
