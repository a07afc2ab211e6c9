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
