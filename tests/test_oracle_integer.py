"""Pins for the oracle's integer steps: the paper's worked examples, brute force on
explicit paths, and a full sort.  None of these re-types the oracle's own formula."""
import itertools

import numpy as np
import pytest

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth


def _nodes(rows):
    pr = [tuple(int(x) for x in t.split(",")) for t in rows]
    return [p for p, _ in pr], [r for _, r in pr]


# ---- Section 3.2 worked example -------------------------------------------------------
def test_bfs_worked_example(golden):
    g = golden("bfs_worked_example.txt")
    M = np.zeros((32, 3), np.int64)
    for key, val in g.items():
        if key.startswith("row"):
            M[int(key.split()[1])] = [int(x) for x in val[0]]
    parent, rank = _nodes(g["nodes"][0])
    tree = O.make_tree(parent, rank, 3)
    S = O.build_tree(M, tree, int(g["root"][0][0]))
    assert S.tolist() == [int(x) for x in g["expect"][0]]
    assert tree.n_layers == 3


def _walk(M, parent, rank, root, n):
    """Follow node n's root-to-node path through M by hand (recursion on the parent)."""
    if n == 0:
        return root
    return int(M[_walk(M, parent, rank, root, parent[n])][rank[n]])


@pytest.mark.parametrize("name", ["tree80", "tree81", "tree15", "tree15_alt", "wide128", "single", "depth4", "depth5",
                                  "depth7", "depth8"])
def test_build_tree_equals_path_walk(name):
    t = synth.TEMPLATES[name]()
    rng = np.random.default_rng(1)
    V, k = 97, 8
    M = rng.integers(0, V, size=(V, k))
    tree = O.make_tree(t.parent, t.rank, k)
    assert tree.n_layers == t.n_layers
    for root in (0, 5, 96):
        S = O.build_tree(M, tree, root)
        assert S.tolist() == [_walk(M, t.parent, t.rank, root, n) for n in range(t.n_nodes)]


def test_chain_template_follows_column_zero():
    t = synth.chain(7)
    M = synth.init_matrix(50, 8).astype(np.int64)
    S = O.build_tree(M, O.make_tree(t.parent, t.rank, 8), 48)
    assert S.tolist() == [48] * 7                          # column 0 of (i + j) mod V is i itself
    M[:, 0] = (np.arange(50) + 3) % 50
    S = O.build_tree(M, O.make_tree(t.parent, t.rank, 8), 48)
    assert S.tolist() == [48, 1, 4, 7, 10, 13, 16]


def test_default_template_sizes(golden):
    g = golden("sizes.txt")
    t81, t80 = synth.tree81(), synth.tree80()
    assert t81.n_nodes == int(g["tree_rows"][0][0]) and t81.n_layers == int(g["tree_layers"][0][0])
    assert t80.n_nodes == 80 and t80.n_layers == 6 and t80.layer_sizes[:3] == (1, 8, 21)
    k = int(g["k"][0][0])
    for t in (t80, t81):
        fan = np.bincount(t.parent[1:], minlength=t.n_nodes)
        assert fan.max() <= k
        O.make_tree(t.parent, t.rank, k)                    # well-formed
    rows = int(g["matrix_rows"][0][0])
    assert round(rows * k * 8 / 2 ** 20, 2) == float(g["matrix_mib_at_8_bytes"][0][0])


def test_depth_sweep_templates_keep_80_rows():
    """Section 5.1 varies the depth at a fixed 80 nodes: the sweep's templates have 80 rows, the asked
    number of layers, at most k children per node, and a first-child chain that reaches the last layer
    (so a step can accept depth - 1 drafts)."""
    for D in (4, 5, 6, 7, 8):
        t = synth.depth_template(D)
        tree = O.make_tree(t.parent, t.rank, 8)
        assert t.n_nodes == 80 and t.n_layers == D == tree.n_layers and sum(t.layer_sizes) == 80
        assert np.bincount(t.parent[1:], minlength=80).max() <= 8
        n, hops = 0, 0
        while True:
            kids = [c for c in range(80) if t.parent[c] == n and t.rank[c] == 0]
            if not kids:
                break
            n, hops = kids[0], hops + 1
        assert hops == D - 1


def test_make_tree_rejects_malformed():
    with pytest.raises(ValueError):
        O.make_tree([0, 0], [-1, 0], 8)                     # root must have parent -1
    with pytest.raises(ValueError):
        O.make_tree([-1, 1], [-1, 0], 8)                    # parent must precede child
    with pytest.raises(ValueError):
        O.make_tree([-1, 0], [-1, 8], 8)                    # rank < k
    with pytest.raises(ValueError):
        O.make_tree([-1, 0, 0], [-1, 1, 1], 8)              # duplicate (parent, rank)
    with pytest.raises(ValueError):
        O.make_tree([-1, 0, 1, 0], [-1, 0, 0, 1], 8)        # not in layer order


# ---- Section 2.2 chain example ----------------------------------------------------------
def test_chain_accept_example(golden):
    g = golden("chain_accept_example.txt")
    S = np.array([int(x) for x in g["sequence"][0]])
    out = np.array([int(x) for x in g["outputs"][0]])
    parent, rank = _nodes(g["nodes"][0])
    acc = O.accept(S, out, O.make_tree(parent, rank, 8))
    assert acc.emitted == [int(x) for x in g["expect_confirmed"][0]]
    assert acc.n_accepted == int(g["expect_matched"][0][0])
    assert acc.path == [0, 1, 2] and acc.bonus == 5


def _leaf_paths(parent):
    n = len(parent)
    kids = [[] for _ in range(n)]
    for i in range(1, n):
        kids[parent[i]].append(i)
    paths = []

    def rec(node, acc):
        acc = acc + [node]
        if not kids[node]:
            paths.append(acc)
        for c in kids[node]:
            rec(c, acc)
    rec(0, [])
    return paths


def _brute_accept(S, out, parent):
    """Every root-to-leaf sequence is verified as a chain (Section 2.2); the longest
    confirmed run wins.  Returns (matched count, confirmed tokens)."""
    best = (-1, None)
    for path in _leaf_paths(list(parent)):
        j = 0
        while j + 1 < len(path) and S[path[j + 1]] == out[path[j]]:
            j += 1
        conf = [int(S[p]) for p in path[1:j + 1]] + [int(out[path[j]])]
        if j > best[0]:
            best = (j, conf)
    return best


@pytest.mark.parametrize("name", ["tree80", "tree15", "tree15_alt", "wide128", "depth4", "depth8"])
def test_accept_equals_brute_force_over_leaf_paths(name):
    t = synth.TEMPLATES[name]()
    tree = O.make_tree(t.parent, t.rank, 8)
    rng = np.random.default_rng(7)
    hit_depths = set()
    for trial in range(300):
        V = int(rng.choice([3, 5, 50]))                     # small V: many matches and duplicate siblings
        S = rng.integers(0, V, size=t.n_nodes)
        out = rng.integers(0, V, size=t.n_nodes)
        if trial % 3 == 0:                                  # plant a fully correct random path
            n = int(rng.integers(0, t.n_nodes))
            for i in range(1, len(tree.paths[n])):
                out[tree.paths[n][i - 1]] = S[tree.paths[n][i]]
        acc = O.accept(S, out, tree)
        j, conf = _brute_accept(S, out, t.parent)
        assert acc.n_accepted == j
        assert acc.emitted == conf
        assert len(acc.path) == j + 1 and acc.path[0] == 0 and acc.path[-1] == acc.winner
        assert 1 <= len(acc.emitted) <= tree.n_layers
        # tie rule: no node of the same depth with a smaller index is fully matched
        for n in range(acc.winner):
            if tree.depth[n] == tree.depth[acc.winner]:
                p = tree.paths[n]
                assert not all(S[p[i]] == out[p[i - 1]] for i in range(1, len(p)))
        hit_depths.add(j)
    assert hit_depths == set(range(tree.n_layers))


# ---- Appendix A.5 update example ----------------------------------------------------------
def test_update_strategies_example(golden):
    g = golden("update_strategies_example.txt")
    S = np.array([int(x) for x in g["sequence"][0]])
    topk = np.array([[int(x) for x in g[f"out {i}"][0]] for i in range(5)])
    for mode in ("first", "last"):
        M = np.full((8, 4), -1, np.int64)
        O.update_matrix(M, S, topk, mode)
        assert M[1].tolist() == [int(x) for x in g[f"expect_{mode} 1"][0]]
        for tok in (2, 3, 4):
            assert M[tok].tolist() == [int(x) for x in g[f"expect_both {tok}"][0]]
        assert (M[[0, 5, 6, 7]] == -1).all()                 # untouched rows


def test_update_last_is_one_of_the_racing_outcomes():
    # Section 3.3: a token that appears twice with outputs [y0,y1] and [z0,z1] may end as any
    # per-element mix; "last" must be exactly [z0, z1].
    S = np.array([9, 4, 9])
    topk = np.array([[10, 11], [20, 21], [30, 31]])
    M = np.zeros((12, 2), np.int64)
    O.update_matrix(M, S, topk, "last")
    assert M[9].tolist() == [30, 31] and M[4].tolist() == [20, 21]
    allowed = {(a, b) for a in (10, 30) for b in (11, 31)}
    assert tuple(M[9]) in allowed


def test_update_accepted_only_touches_only_path_rows():
    S = np.array([1, 2, 3, 4])
    topk = np.arange(8).reshape(4, 2) + 100
    M = np.zeros((6, 2), np.int64)
    O.update_matrix(M, S, topk, "last", nodes=[0, 2])
    assert M[1].tolist() == [100, 101] and M[3].tolist() == [104, 105]
    assert (M[[0, 2, 4, 5]] == 0).all()


# ---- argtopk (Section 2.1; tie rule of Appendix A.1) -----------------------------------------
def test_topk_equals_full_sort_with_ties():
    rng = np.random.default_rng(3)
    for trial in range(50):
        n = int(rng.integers(9, 400))
        p = rng.integers(-4, 5, size=n).astype(np.float32)   # few distinct values: ties everywhere
        if trial % 2:
            p = rng.standard_normal(n).astype(np.float32)
            p[rng.integers(0, n, 5)] = p.max()               # tie at the top
        p[rng.integers(0, n)] = -0.0
        want = [i for _, i in sorted((-(float(v) + 0.0), i) for i, v in enumerate(p))][:8]
        assert O.topk_ids(p, 8).tolist() == want
        assert O.topk_ids(p, 1)[0] == int(np.argmax(p))      # argmax returns the smallest index


def test_topk_signed_zero_is_a_tie():
    p = np.array([-0.0, 0.0, -1.0, 0.0], np.float32)
    assert O.topk_ids(p, 3).tolist() == [0, 1, 3]


def test_update_first_and_last_restricted_to_path():
    # token 7 occurs at nodes 0, 2, 3; only nodes 0 and 3 are on the path
    S = np.array([7, 5, 7, 7])
    topk = np.array([[1, 1], [2, 2], [3, 3], [4, 4]])
    M = np.zeros((9, 2), np.int64)
    O.update_matrix(M, S, topk, "last", nodes=[0, 3])
    assert M[7].tolist() == [4, 4] and (M[5] == 0).all()
    M[:] = 0
    O.update_matrix(M, S, topk, "first", nodes=[0, 3])
    assert M[7].tolist() == [1, 1]
    M[:] = 0
    O.update_matrix(M, S, topk, "first")
    assert M[7].tolist() == [1, 1] and M[5].tolist() == [2, 2]
