"""GPU parity, integer kernels: tree gather, top-k, accept, matrix update — bit-exact against the
oracle on the same seeded inputs, through the C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth, tr
from gpu_util import kv_fill, kv_plain_views, require_gpu, say

pytestmark = pytest.mark.gpu
K = 8


def _ctx(t, V, k=K):
    return tr.Context(V, k, t.parent, t.rank, t.n_layers)


@pytest.mark.parametrize("name", ["tree80", "tree81", "tree15", "tree15_alt", "wide128", "single"])
def test_build_tree_matches_oracle(name):
    require_gpu()
    t = synth.TEMPLATES[name]()
    V = 32000
    rng = np.random.default_rng(11)
    M = rng.integers(0, V, size=(V, K)).astype(np.int32)
    ctx = _ctx(t, V)
    ctx.matrix_load(M)
    assert np.array_equal(ctx.matrix_store(), M)
    tree = O.make_tree(t.parent, t.rank, K)
    d_S = torch.zeros(t.n_nodes, dtype=torch.int32, device="cuda")
    for root in (0, 17, V - 1):
        say("build_tree", name, "root", root)
        d_root = torch.tensor([root], dtype=torch.int32, device="cuda")
        ctx.build_tree(d_root, d_S)
        assert d_S.cpu().tolist() == O.build_tree(M.astype(np.int64), tree, root).tolist()
    ctx.close()


def test_worked_example_on_gpu(golden):
    require_gpu()
    g = golden("bfs_worked_example.txt")
    M = np.zeros((32, 3), np.int32)
    for key, val in g.items():
        if key.startswith("row"):
            M[int(key.split()[1])] = [int(x) for x in val[0]]
    pr = [tuple(int(x) for x in s.split(",")) for s in g["nodes"][0]]
    ctx = tr.Context(32, 3, [p for p, _ in pr], [r for _, r in pr], 3)
    ctx.matrix_load(M)
    d_S = torch.zeros(len(pr), dtype=torch.int32, device="cuda")
    ctx.build_tree(torch.tensor([int(g["root"][0][0])], dtype=torch.int32, device="cuda"), d_S)
    assert d_S.cpu().tolist() == [int(x) for x in g["expect"][0]]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [1024, 32000, 128256])
def test_topk_matches_oracle(dtype, V):
    """Rows ~ N(0,3) (the microbench distribution; bf16 rounding makes ties at the top common),
    plus planted exact ties, signed zeros and constant rows."""
    require_gpu()
    rows = 80
    say("topk", dtype, V)
    x = synth.normal_tensor((rows, V), 3.0, seed=V, dtype=dtype)
    x[3, :] = 0.0
    x[3, 5] = -0.0
    x[4, :] = x[4, 0]
    x[5, V - 9:] = x[5].max() + 1
    x[6, ::7] = x[6].max()
    ctx = _ctx(synth.single(), V)
    d_topk = torch.zeros(rows, K, dtype=torch.int32, device="cuda")
    ctx.op_topk(x.cuda(), d_topk)
    got = d_topk.cpu().numpy()
    xn = x.float().numpy()
    for r in range(rows):
        assert got[r].tolist() == O.topk_ids(xn[r], K).tolist(), r
    ctx.close()


def test_topk_other_k():
    require_gpu()
    V = 5000
    x = synth.normal_tensor((7, V), 1.0, seed=1, dtype=torch.float32)
    for k in (1, 3, 32):
        ctx = _ctx(synth.single(), V, k)
        d_topk = torch.zeros(7, k, dtype=torch.int32, device="cuda")
        ctx.op_topk(x.cuda(), d_topk)
        for r in range(7):
            assert d_topk[r].cpu().tolist() == O.topk_ids(x[r].numpy(), k).tolist()
        ctx.close()


@pytest.mark.parametrize("V", [8, 9, 1023, 1025, 2049, 131072, 131073, 152064])
def test_topk_vocabulary_edges(V):
    """Vocabularies around the kernel's units: below and above one wave's 1024 elements, the largest row
    the two-stage path takes (128 waves) and the first sizes beyond it (one-kernel path); ties included."""
    require_gpu()
    rows = 5
    say("topk edges", V)
    x = synth.normal_tensor((rows, V), 3.0, seed=V, dtype=torch.float32)
    x[1, :] = 1.5
    x[2, V - 8:] = x[2].max() + 1
    x[3, ::3] = x[3].max()
    x[4, 0] = -0.0
    ctx = _ctx(synth.single(), V)
    d_topk = torch.zeros(rows, K, dtype=torch.int32, device="cuda")
    ctx.op_topk(x.cuda(), d_topk)
    got = d_topk.cpu().numpy()
    for r in range(rows):
        assert got[r].tolist() == O.topk_ids(x[r].numpy(), K).tolist(), (V, r)
    ctx.close()


@pytest.mark.parametrize("name", ["tree80", "wide128", "tree15"])
def test_matrix_update_last_wins(name):
    require_gpu()
    t = synth.TEMPLATES[name]()
    V = 32000
    rng = np.random.default_rng(5)
    for vocab_used in (V, 40):                    # 40: heavy duplication among the node tokens
        M = synth.init_matrix(V, K)
        S = rng.integers(0, vocab_used, size=t.n_nodes).astype(np.int32)
        topk = rng.integers(0, V, size=(t.n_nodes, K)).astype(np.int32)
        ctx = _ctx(t, V)
        ctx.matrix_load(M)
        ctx.op_matrix_update(torch.from_numpy(S).cuda(), torch.from_numpy(topk).cuda())
        want = M.astype(np.int64)
        O.update_matrix(want, S.astype(np.int64), topk.astype(np.int64), "last")
        assert np.array_equal(ctx.matrix_store().astype(np.int64), want)
        ctx.close()


def test_update_example_on_gpu(golden):
    require_gpu()
    g = golden("update_strategies_example.txt")
    S = np.array([int(x) for x in g["sequence"][0]], np.int32)
    topk = np.array([[int(x) for x in g[f"out {i}"][0]] for i in range(5)], np.int32)
    ctx = tr.Context(500, 4, [-1, 0, 1, 2, 3], [-1, 0, 0, 0, 0], 5)
    ctx.op_matrix_update(torch.from_numpy(S).cuda(), torch.from_numpy(topk).cuda())
    M = ctx.matrix_store()
    assert M[1].tolist() == [int(x) for x in g["expect_last 1"][0]]
    for tok in (2, 3, 4):
        assert M[tok].tolist() == [int(x) for x in g[f"expect_both {tok}"][0]]


def _run_accept(t, S, topk, V=64, L=10, hd=32, layers=2, heads=2, dtype="f32", mode=0):
    """Calls tr_accept_and_update on a small cache whose tree rows are tagged with their node
    index, returns (StepOut, M, k-cache, v-cache) with the caches in natural [.., pos, hd] order."""
    sh = synth.ModelShape("acc", layers, 64, heads, heads, hd, 64, V, dtype)
    ctx = tr.Context(V, topk.shape[1], t.parent, t.rank, t.n_layers)
    ctx.set_update_mode(mode)
    kv = tr.KVDesc(sh, capacity=L + t.n_nodes + 4)
    kv.reset(L)
    n = t.n_nodes
    tag = torch.arange(n, dtype=torch.float32, device="cuda") + 100.0
    kp = torch.zeros(layers, heads, kv.capacity, hd, dtype=kv.k.dtype, device="cuda")
    vp = torch.zeros_like(kp)
    kp[:, :, L:L + n, :] = tag[None, None, :, None].to(kp.dtype)
    vp[:, :, L:L + n, :] = -tag[None, None, :, None].to(kp.dtype)
    kv_fill(kv, kp, vp)
    d_out = torch.zeros(tr.STEP_OUT_INTS, dtype=torch.int32, device="cuda")
    h = ctx.accept_and_update(kv, torch.from_numpy(S.astype(np.int32)).cuda(),
                              torch.from_numpy(topk.astype(np.int32)).cuda(), d_out, sync=True)
    assert int(kv.d_len.item()) == h.kv_len == kv.c.len_bound
    kc, vc = kv_plain_views(kv)
    return h, ctx.matrix_store(), kc.float().cpu().numpy(), vc.float().cpu().numpy(), ctx


def test_chain_accept_example_on_gpu(golden):
    require_gpu()
    g = golden("chain_accept_example.txt")
    S = np.array([int(x) for x in g["sequence"][0]])
    out = np.array([int(x) for x in g["outputs"][0]])
    t = synth.chain(5)
    topk = np.stack([out, (out + 1) % 64], axis=1)
    h, M, _, _, _ = _run_accept(t, S, topk)
    assert list(h.emitted[:h.n_emitted]) == [int(x) for x in g["expect_confirmed"][0]]
    assert h.n_accepted == int(g["expect_matched"][0][0]) and h.next_root == 5


@pytest.mark.parametrize("name,kvmode", [("tree80", "plain"), ("tree81", "plain"), ("tree15", "plain"),
                                         ("wide128", "plain"), ("single", "plain"), ("tree80", "tiled"),
                                         ("wide128", "tiled")])
def test_accept_update_compact_matches_oracle(name, kvmode):
    require_gpu()
    kw = dict(hd=128, dtype="bf16") if kvmode == "tiled" else {}
    t = synth.TEMPLATES[name]()
    tree = O.make_tree(t.parent, t.rank, K)
    rng = np.random.default_rng(23)
    L = 10
    depths = set()
    for trial in range(40):
        V = int(rng.choice([3, 5, 64]))
        S = rng.integers(0, V, size=t.n_nodes)
        topk = np.stack([rng.permutation(64)[:K] % max(V, K) for _ in range(t.n_nodes)])
        if V < K:
            topk = rng.integers(0, V, size=(t.n_nodes, K))
        if trial % 2 == 0:
            n = int(rng.integers(0, t.n_nodes))
            for i in range(1, len(tree.paths[n])):
                topk[tree.paths[n][i - 1], 0] = S[tree.paths[n][i]]
        say("accept", name, "trial", trial)
        h, M, kc, vc, ctx = _run_accept(t, S, topk, **kw)
        acc = O.accept(S, topk[:, 0], tree)
        assert h.n_accepted == acc.n_accepted and h.winner == acc.winner
        assert list(h.path[:h.n_emitted]) == acc.path
        assert list(h.emitted[:h.n_emitted]) == acc.emitted
        assert h.next_root == acc.bonus and h.kv_len == L + acc.n_accepted + 1
        want = np.zeros((64, K), np.int64)
        O.update_matrix(want, S, topk, "last")
        assert np.array_equal(M.astype(np.int64), want)
        # compaction: cache position L+i holds the row the forward wrote for node path[i]
        for i, node in enumerate(acc.path):
            assert (kc[:, :, L + i, :] == 100.0 + node).all()
            assert (vc[:, :, L + i, :] == -(100.0 + node)).all()
        assert (kc[:, :, :L, :] == 0).all() and (vc[:, :, :L, :] == 0).all()
        depths.add(acc.n_accepted)
        ctx.close()
    if name != "single":
        assert len(depths) >= min(3, tree.n_layers)


@pytest.mark.parametrize("mode", [tr.TR_UPDATE_FIRST, tr.TR_UPDATE_ACCEPTED_ONLY,
                                  tr.TR_UPDATE_FIRST | tr.TR_UPDATE_ACCEPTED_ONLY])
def test_update_variants_match_oracle(mode):
    """First-occurrence and accepted-only updates (Section 5.2, Appendix A.5, Table 4) against the
    oracle's update_matrix on heavily duplicated node tokens."""
    require_gpu()
    t = synth.tree80()
    tree = O.make_tree(t.parent, t.rank, K)
    rng = np.random.default_rng(31)
    for trial in range(25):
        V = int(rng.choice([3, 6, 64]))
        S = rng.integers(0, V, size=t.n_nodes)
        topk = rng.integers(0, 64, size=(t.n_nodes, K))
        n = int(rng.integers(0, t.n_nodes))
        for i in range(1, len(tree.paths[n])):
            topk[tree.paths[n][i - 1], 0] = S[tree.paths[n][i]]
        say("update variant", mode, "trial", trial)
        h, M, _, _, ctx = _run_accept(t, S, topk, mode=mode)
        acc = O.accept(S, topk[:, 0], tree)
        assert list(h.path[:h.n_emitted]) == acc.path
        want = np.zeros((64, K), np.int64)
        O.update_matrix(want, S, topk, "first" if mode & tr.TR_UPDATE_FIRST else "last",
                        acc.path if mode & tr.TR_UPDATE_ACCEPTED_ONLY else None)
        assert np.array_equal(M.astype(np.int64), want)
        ctx.close()


def test_update_example_first_on_gpu(golden):
    require_gpu()
    g = golden("update_strategies_example.txt")
    S = np.array([int(x) for x in g["sequence"][0]], np.int32)
    topk = np.array([[int(x) for x in g[f"out {i}"][0]] for i in range(5)], np.int32)
    ctx = tr.Context(500, 4, [-1, 0, 1, 2, 3], [-1, 0, 0, 0, 0], 5)
    ctx.set_update_mode(tr.TR_UPDATE_FIRST)
    ctx.op_matrix_update(torch.from_numpy(S).cuda(), torch.from_numpy(topk).cuda())
    M = ctx.matrix_store()
    assert M[1].tolist() == [int(x) for x in g["expect_first 1"][0]]
    with pytest.raises(tr.TRError):
        ctx.set_update_mode(4)


@pytest.mark.parametrize("V,L", [(1000, 0), (32000, 513), (128256, 37)])
def test_sample_tokens_match_oracle(V, L):
    """Temperature sampling draw (Section 5.3): argmax of logits / T + position-keyed noise in the stated
    float32 arithmetic, ties to the smallest index, bit-exact against the oracle."""
    require_gpu()
    say("sample", V, L)
    t = synth.tree80()
    tree = O.make_tree(t.parent, t.rank, 8)
    ctx = tr.Context(V, 8, t.parent, t.rank, t.n_layers)
    sh = synth.ModelShape("s", 1, 128, 1, 1, 128, 128, V, "bf16")
    kv = tr.KVDesc(sh, L + 128)
    kv.reset(L)
    logits = synth.normal_tensor((t.n_nodes, V), 3.0, seed=V, dtype=torch.float32)
    logits[3, 5] = logits[3, V - 1] = 50.0                       # planted tie: index 5 must win with equal noise
    noise = synth.gumbel_noise(L + t.n_layers, V, seed=L)
    noise[L + int(tree.depth[3]), 5] = noise[L + int(tree.depth[3]), V - 1] = 0.0
    tokens = torch.zeros(t.n_nodes, dtype=torch.int32, device="cuda")
    pos = [L + int(d) for d in tree.depth]
    for inv_t in (1.0 / 0.3, 1.0, 2.0):
        ctx.op_sample(kv, logits.cuda(), noise.cuda(), inv_t, tokens)
        want = O.sample_tokens(logits.numpy(), pos, inv_t, noise.numpy())
        assert tokens.cpu().tolist() == want.tolist()
        assert want[3] == 5
    with pytest.raises(tr.TRError):
        ctx.op_sample(kv, logits.cuda(), noise[:L + 2].cuda(), 1.0, tokens)     # table too short for the tree
    with pytest.raises(tr.TRError):
        ctx.op_sample(kv, logits.cuda(), noise.cuda(), 0.0, tokens)
