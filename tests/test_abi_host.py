"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU (so these run without one)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_08696_amd import synth, tr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tr.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return tr.lib()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "tr.h")).read()
    declared = set(re.findall(r"\b(tr_[a-z_]+)\s*\(", hdr))
    assert declared == set(tr.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    assert C.sizeof(tr.StepOut) == 4 * (5 + 2 * tr.TR_MAX_LAYERS)
    assert C.sizeof(tr.Layer) == 9 * 8
    hdr = open(os.path.join(ROOT, "include", "tr.h")).read()
    assert f"#define TR_MAX_NODES {tr.TR_MAX_NODES}" in hdr
    assert f"#define TR_MAX_LAYERS {tr.TR_MAX_LAYERS}" in hdr
    assert f"#define TR_MAX_K {tr.TR_MAX_K}" in hdr


def test_strerror(lib):
    for s in (0, -1, -2, -3, -4, -5, -6, 7):
        assert lib.tr_strerror(s)


def _create(lib, V, k, parent, rank, n_layers):
    t, keep = tr.make_template(parent, rank, n_layers)
    h = C.c_void_p()
    return lib.tr_create(V, k, C.byref(t), C.byref(h)), h


@pytest.mark.parametrize("args,want", [
    ((0, 8, [-1], [-1], 1), tr.TR_EINVAL),
    ((10, 0, [-1], [-1], 1), tr.TR_EINVAL),
    ((10, 33, [-1], [-1], 1), tr.TR_EINVAL),
    ((10, 8, [0], [-1], 1), tr.TR_ETEMPLATE),                      # root parent must be -1
    ((10, 8, [-1, 1], [-1, 0], 2), tr.TR_ETEMPLATE),               # parent must precede child
    ((10, 8, [-1, 0], [-1, 8], 2), tr.TR_ETEMPLATE),               # rank >= k
    ((10, 8, [-1, 0, 0], [-1, 1, 1], 2), tr.TR_ETEMPLATE),         # duplicate (parent, rank)
    ((10, 8, [-1, 0, 1, 0], [-1, 0, 0, 1], 3), tr.TR_ETEMPLATE),   # not layer-major
    ((10, 8, [-1, 0], [-1, 0], 3), tr.TR_ETEMPLATE),               # n_layers disagrees
    ((10, 8, [-1] + list(range(128)), [-1] + [0] * 128, 129), tr.TR_ETEMPLATE),  # N > 128
])
def test_create_rejects_before_any_gpu_call(lib, args, want):
    st, h = _create(lib, *args)
    assert st == want and not h.value


def test_null_arguments(lib):
    assert lib.tr_create(10, 8, None, None) == tr.TR_EINVAL
    assert lib.tr_destroy(None) == tr.TR_EINVAL
    assert lib.tr_build_tree(None, None, None, None) == tr.TR_EINVAL
    assert lib.tr_matrix_load(None, None) == tr.TR_EINVAL
    assert lib.tr_verify_forward(None, None, None, None, None, None, None, 0, None) == tr.TR_EINVAL
    assert lib.tr_accept_and_update(None, None, None, None, None, None, None) == tr.TR_EINVAL
    assert lib.tr_prefill(None, None, None, None, 0, None, 0, None) == tr.TR_EINVAL
    assert lib.tr_op_topk(None, None, 0, 0, None, None) == tr.TR_EINVAL
    assert lib.tr_set_update_mode(None, 0) == tr.TR_EINVAL


def test_default_templates_are_accepted_by_the_host_check():
    # derive the same facts the library derives, from the header's rules, for all shipped templates
    for name, f in synth.TEMPLATES.items():
        t = f()
        assert t.parent[0] == -1 and t.rank[0] == -1
        assert all(0 <= t.parent[i] < i for i in range(1, t.n_nodes))
        assert t.n_nodes <= tr.TR_MAX_NODES and t.n_layers <= tr.TR_MAX_LAYERS


# ---- launch planners (host logic only) ----
def _variant_exists(nt, p, fused):
    """Kernel variants the projection source instantiates, by weight tiles per workgroup."""
    wt = 2 * p if fused else p
    if wt == 8:
        return nt in (4, 5)
    if wt == 6:
        return True
    if wt == 5:
        return not fused and nt <= 5
    return wt in ((2, 4) if fused else (1, 2, 3, 4))


@pytest.mark.parametrize("fused", [False, True])
def test_projection_plans_cover_every_tile_once(lib, fused):
    for n in (1, 15, 16, 17, 48, 64, 80, 81, 96, 112, 128):
        for in_f, out_f in ((256, 256), (4096, 4096), (4096, 12288), (4096, 11008), (11008, 4096), (5120, 13824),
                            (8192, 28672), (28672, 8192), (4096, 32000), (4096, 128256), (64, 32), (288, 96)):
            for ms in (1, 2, 4):
                p, groups, splits = tr.plan_projection(n, in_f, out_f, fused, ms)
                tiles = out_f // 16
                assert _variant_exists((n + 15) // 16, p, fused), (n, in_f, out_f, p)
                assert 1 <= groups <= tiles and groups * p >= tiles       # each tile has exactly one owner
                assert -(-tiles // groups) <= p                             # largest share fits the variant
                assert splits in (1, 2, 4) and splits <= (1 if fused else ms)
                assert splits == 1 or (in_f // 32) // splits >= 8           # every wave keeps >= 1 k-tile


def test_projection_plan_rejects_bad_shapes(lib):
    plan = (C.c_int32 * 3)()
    assert lib.tr_plan_projection(80, 4096, 4096, 0, 4, None) == tr.TR_EINVAL
    assert lib.tr_plan_projection(0, 4096, 4096, 0, 4, plan) == tr.TR_EINVAL
    assert lib.tr_plan_projection(129, 4096, 4096, 0, 4, plan) == tr.TR_EINVAL
    assert lib.tr_plan_projection(80, 4100, 4096, 0, 4, plan) == tr.TR_EINVAL
    assert lib.tr_plan_projection(80, 4096, 4100, 0, 4, plan) == tr.TR_EINVAL
    assert lib.tr_plan_projection(80, 4096, 4096, 0, 0, plan) == tr.TR_EINVAL


def test_projection_plans_of_the_7b_step_fill_the_chip(lib):
    # the five projections of a 7B layer at the 80-node tree: every plan puts work on >= 230 of 256 CUs
    for in_f, out_f, fused, ms in ((4096, 12288, False, 1), (4096, 4096, False, 4), (4096, 11008, True, 1),
                                   (11008, 4096, False, 4), (4096, 32000, False, 1)):
        p, groups, splits = tr.plan_projection(80, in_f, out_f, fused, ms)
        assert groups * splits >= 230, (in_f, out_f, p, groups, splits)


def test_attention_plan(lib):
    plan = (C.c_int32 * 2)()
    assert lib.tr_plan_attention(32, 32, 80, 600, None) == tr.TR_EINVAL
    assert lib.tr_plan_attention(0, 1, 80, 600, plan) == tr.TR_EINVAL
    assert lib.tr_plan_attention(32, 0, 80, 600, plan) == tr.TR_EINVAL
    assert lib.tr_plan_attention(32, 5, 80, 600, plan) == tr.TR_EINVAL      # not a multiple
    assert lib.tr_plan_attention(32, 32, 0, 600, plan) == tr.TR_EINVAL
    assert lib.tr_plan_attention(32, 32, 129, 600, plan) == tr.TR_EINVAL
    assert lib.tr_plan_attention(32, 32, 80, 0, plan) == tr.TR_EINVAL
    for H, Hkv in ((1, 1), (8, 8), (32, 32), (40, 40), (64, 8), (32, 8), (4, 2), (12, 4), (256, 256)):
        for n in (1, 16, 80, 128):
            prev = 1
            for L in (1, 31, 32, 33, 64, 100, 600, 2048, 8192, 65536):
                hpw, ns = tr.plan_attention(H, Hkv, n, L)
                if ns == 0:                                           # one-launch form: short sequences only
                    assert hpw == 1 and L <= 832 and H // Hkv <= 2 and prev <= 1
                    continue
                assert hpw in (1, 2) and (H // Hkv) % hpw == 0       # heads of one workgroup share a K/V head
                assert ((n + 15) // 16) * hpw <= (12 if hpw == 2 else 8)   # one wave per (head, node tile)
                groups = H // hpw
                assert 1 <= ns <= 16
                assert ns == 1 or 2 * ns <= -(-L // 32)               # at least two 32-key tiles per split
                assert ns == 1 or groups * ns <= 256                  # at most one workgroup per CU
                assert ns >= prev                                     # never fewer splits for a longer context
                prev = ns
    assert tr.plan_attention(32, 32, 80, 600) == (1, 0)
    assert tr.plan_attention(32, 32, 80, 1104) == (1, 8)
    assert tr.plan_attention(64, 8, 80, 600)[1] >= 1                      # eight query heads per K/V head: split form
    assert tr.plan_attention(40, 40, 80, 2128) == (1, 6)
    assert tr.plan_attention(64, 8, 80, 4176)[0] == 2


def test_static_topk_validates_before_touching_the_gpu(lib):
    """The entry point that allocates nothing: argument errors and its size limits are reported
    from the host, before any HIP call."""
    buf = np.zeros(64, np.int32)
    p = buf.ctypes.data
    f = lib.tr_op_topk_static
    assert f(None, tr.TR_F32, 4, 64, 8, p, None) == tr.TR_EINVAL
    assert f(p, tr.TR_F32, 4, 64, 8, None, None) == tr.TR_EINVAL
    assert f(p, 7, 4, 64, 8, p, None) == tr.TR_EINVAL
    assert f(p, tr.TR_F32, -1, 64, 8, p, None) == tr.TR_EINVAL
    assert f(p, tr.TR_F32, 4, 0, 8, p, None) == tr.TR_EINVAL
    assert f(p, tr.TR_F32, 4, 4, 8, p, None) == tr.TR_EINVAL                      # k > V
    assert f(p, tr.TR_F32, 4, 64, 9, p, None) == tr.TR_ECAPACITY                  # k beyond the two-stage kernels
    assert f(p, tr.TR_F32, tr.TR_MAX_NODES + 1, 64, 8, p, None) == tr.TR_ECAPACITY
    assert f(p, tr.TR_F32, 4, 131073, 8, p, None) == tr.TR_ECAPACITY              # beyond the static scratch
    assert f(p, tr.TR_F32, 4, 7, 7, p, None) == tr.TR_ECAPACITY                   # V below the kernels' minimum


def test_create_rejects_more_candidates_than_tokens(lib):
    st, _ = _create(lib, 4, 8, [-1], [-1], 1)
    assert st == tr.TR_EINVAL
