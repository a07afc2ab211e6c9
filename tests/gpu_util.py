"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import os

import numpy as np
import pytest
import torch

from oracle import tr_oracle as O
from paper_2408_08696_amd import synth, tr


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(tr.LIB_PATH):
        pytest.fail("libtr.so is missing on a GPU box: build it before running GPU tests")
    tr.lib()


def to_gpu(w):
    return {k: (v.cuda() if not isinstance(v, list) else [{a: b.cuda() for a, b in l.items()} for l in v])
            for k, v in w.items()}


def oracle_cfg(sh):
    return O.Config(sh.n_layers, sh.d_model, sh.n_heads, sh.n_kv_heads, sh.head_dim, sh.d_ffn, sh.vocab,
                    sh.rms_eps, sh.rope_theta)


def say(*a):
    print(*a, flush=True)


def greedy_continuation(cfg, w_np, kv, root, n_new, dtype, sampler=None):
    """The oracle's own next n_new tokens after (cache, root), on a copy of the cache."""
    kc = O.KVCache(cfg, kv.len + n_new + 1, dtype)
    for l in range(cfg.n_layers):
        kc.k[l][:kv.len] = kv.k[l][:kv.len]
        kc.v[l][:kv.len] = kv.v[l][:kv.len]
    kc.len = kv.len
    tok, out = int(root), []
    for _ in range(n_new):
        logits, nk, nv = O.forward_nodes(cfg, w_np, kc, [tok], [kc.len], [[0]], dtype)
        pos = kc.len
        O.commit(kc, nk, nv, [0])
        tok = int(O.topk_ids(logits[0], 1)[0]) if sampler is None else \
            int(O.sample_tokens(logits, [pos], sampler[0], sampler[1])[0])
        out.append(tok)
    return out


def compare_step(eng, h, tree, M, S, kv_len, lo, k, rel_tol, abs_tol, step, sampler, pos):
    """One step's GPU results against the oracle's logits `lo` for the same integer state: logits
    under the tolerance, then the oracle's integer pipeline on the GPU's own logits bit for bit
    (M is updated in place).  Returns (stats, accept)."""
    lg = eng.logits.cpu().numpy().astype(np.float64)
    err = np.abs(lg - lo).max(axis=1)
    scale = np.abs(lo).max(axis=1)
    if abs_tol is not None:
        assert err.max() <= abs_tol, f"step {step}: logits differ by {err.max()}"
    else:
        assert (err <= rel_tol * scale).all(), f"step {step}: rel err {np.max(err / scale)}"
    out = None
    if sampler is not None:
        out = O.sample_tokens(eng.logits.cpu().numpy(), pos, sampler[0], sampler[1])
        assert eng.tokens.cpu().tolist() == out.tolist(), f"step {step}: drawn tokens differ"
    topk, acc = O.integer_pipeline(M, tree, S, lg, k, out=out)  # oracle integers on the GPU's logits
    assert np.array_equal(eng.topk.cpu().numpy().astype(np.int64), topk), f"step {step}: top-k differs"
    assert h.n_accepted == acc.n_accepted and h.winner == acc.winner
    assert list(h.path[:h.n_emitted]) == acc.path and list(h.emitted[:h.n_emitted]) == acc.emitted
    assert h.next_root == acc.bonus and h.kv_len == kv_len + acc.n_accepted + 1
    assert np.array_equal(eng.ctx.matrix_store().astype(np.int64), M), f"step {step}: matrix differs"
    # rows whose own-logit top-k differs from the GPU's must be near-ties within the error
    flips = 0
    for n in range(tree.n_nodes):
        mine = O.topk_ids(lo[n], k)
        if not np.array_equal(mine, topk[n]):
            flips += 1
            srt = -np.sort(-lo[n])[:k + 1]
            assert np.min(srt[:-1] - srt[1:]) <= 2 * err[n] + 1e-12, f"step {step} row {n}: flip without near-tie"
    return dict(step=step, max_err=float(err.max()), max_rel=float(np.max(err / scale)), flips=flips,
                n_emitted=acc.n_accepted + 1), acc


def compare_cache(eng, kv, lo, hi, packed, tol=2e-2):
    """Committed GPU cache rows lo..hi-1 against the oracle's, per layer, relative to the largest entry."""
    kp, vp = kv_plain_views(eng.kv, k_interleaved=packed)
    worst = 0.0
    for l in range(len(kv.k)):
        kg = kp[l, :, lo:hi, :].permute(1, 0, 2).float().cpu().numpy()
        vg = vp[l, :, lo:hi, :].permute(1, 0, 2).float().cpu().numpy()
        ek = np.abs(kg - kv.k[l][lo:hi]).max() / np.abs(kv.k[l][lo:hi]).max()
        ev = np.abs(vg - kv.v[l][lo:hi]).max() / np.abs(kv.v[l][lo:hi]).max()
        worst = max(worst, float(ek), float(ev))
    assert worst <= tol, f"committed cache rows {lo}..{hi}: relative error {worst}"
    return worst


def lockstep(eng, sh, w_np, tmpl, prompt, n_steps, M0, k=8, rel_tol=2e-2, abs_tol=None, dtype=np.float64,
             label="", sampler=None, hot_plan=None, check_cache=False):
    """Teacher-forced parity of whole steps.  Each step the oracle starts from the same integer
    state as the GPU (root, M, committed tokens), its logits are compared under the tolerance, and
    its integer pipeline (top-k, accept, matrix update) is applied to the GPU's own logits and must
    reproduce the GPU's integers bit for bit.  Returns per-step stats.
    sampler = (1/T, noise [positions, vocab] float32 numpy): temperature sampling on both sides; the
    oracle's draws from the GPU's logits must equal the GPU's draws.
    hot_plan = accepted drafts wanted per step: the matrix both sides start from is M0 with the
    oracle's own continuation of the prompt planted pair by pair (synth.planted_matrix), so that
    drafts are accepted and the compacted cache rows feed the next step's attention.
    check_cache: after every step the rows the step committed are compared with the oracle's."""
    cfg = oracle_cfg(sh)
    tree = O.make_tree(tmpl.parent, tmpl.rank, k)
    kv = O.KVCache(cfg, len(prompt) + n_steps * tree.n_layers + tree.n_nodes + 8, dtype)
    O.prefill(cfg, w_np, kv, list(prompt[:-1]), dtype)
    root = int(prompt[-1])
    if hot_plan is not None:
        y = greedy_continuation(cfg, w_np, kv, root, sum(a + 1 for a in hot_plan), dtype, sampler)
        say(f"lockstep {label}: oracle continuation {y}")
        M0 = synth.planted_matrix(M0, [root] + y, hot_plan)
    eng.ctx.matrix_load(M0)
    eng.prefill(prompt)
    M = M0.astype(np.int64).copy()
    stats = []
    gpu_sampler = None if sampler is None else (sampler[0], torch.from_numpy(sampler[1]).cuda())
    for step in range(n_steps):
        say(f"lockstep {label} step {step} L={kv.len}")
        h = eng.step(sync=True, sampler=gpu_sampler)
        S = O.build_tree(M, tree, root)
        assert eng.S.cpu().tolist() == S.tolist(), f"step {step}: tree differs"
        pos = [kv.len + int(d) for d in tree.depth]
        lo, nk, nv = O.forward_nodes(cfg, w_np, kv, S, pos, tree.paths, dtype)
        st, acc = compare_step(eng, h, tree, M, S, kv.len, lo, k, rel_tol, abs_tol, step, sampler, pos)
        L0 = kv.len
        O.commit(kv, nk, nv, acc.path)
        if check_cache:
            st["cache_err"] = compare_cache(eng, kv, L0, kv.len, eng.model.packed,
                                            tol=1e-4 if abs_tol is not None else 2e-2)
        root = acc.bonus
        stats.append(st)
    return stats, kv


class StreamedLayers:
    """w["layers"] for the oracle when the model does not fit host memory as float32: layer l is
    generated on the GPU from the seeded recipe (synth.layer_weights), copied to the host as float32
    and dropped again when the next one is asked for."""

    def __init__(self, sh, seed):
        self.sh, self.seed, self.fetches = sh, seed, 0

    def __getitem__(self, l):
        lw = synth.layer_weights(self.sh, l, seed=self.seed, device="cuda")
        out = {k: v.to(torch.float32).cpu().numpy() for k, v in lw.items()}
        del lw
        self.fetches += 1
        if l % 8 == 7:
            say(f"  oracle layer {l + 1}/{self.sh.n_layers}")
        return out


def lockstep_streamed(eng, sh, seed, tmpl, prompt, n_steps, M0, prefix_kv=None, k=8, rel_tol=2e-2, label=""):
    """lockstep for models whose float32 weights the host cannot hold: the oracle gets its layers
    one at a time (StreamedLayers) and takes prompt and first step through each layer together
    (O.prefill_then_forward), so a step costs one pass over the layers.  float32 oracle.
    prefix_kv = (k, v) float32 numpy [layers, positions, kv heads, head_dim] (bf16-representable
    values): cache contents both sides start from before the prompt; the caller has already written
    the same values into the GPU cache and set its length."""
    cfg = oracle_cfg(sh)
    tree = O.make_tree(tmpl.parent, tmpl.rank, k)
    head = synth.head_weights(sh, seed=seed, device="cuda")
    w = {n: t.to(torch.float32).cpu().numpy() for n, t in head.items()}
    del head
    w["layers"] = StreamedLayers(sh, seed)
    L0 = 0 if prefix_kv is None else prefix_kv[0].shape[1]
    kv = O.KVCache(cfg, L0 + len(prompt) + n_steps * tree.n_layers + tree.n_nodes + 8, np.float32)
    if prefix_kv is not None:
        for l in range(cfg.n_layers):
            kv.k[l][:L0] = prefix_kv[0][l]
            kv.v[l][:L0] = prefix_kv[1][l]
        kv.len = L0
    eng.ctx.matrix_load(M0)
    eng.prefill(prompt, keep_cache=prefix_kv is not None)
    M = M0.astype(np.int64).copy()
    root = int(prompt[-1])
    stats = []
    for step in range(n_steps):
        say(f"lockstep {label} step {step} L={kv.len}")
        h = eng.step(sync=True)
        S = O.build_tree(M, tree, root)
        assert eng.S.cpu().tolist() == S.tolist(), f"step {step}: tree differs"
        if step == 0:
            lo, nk, nv = O.prefill_then_forward(cfg, w, kv, list(prompt[:-1]), S, tree.depth, tree.paths,
                                                np.float32)
        else:
            lo, nk, nv = O.forward_nodes(cfg, w, kv, S, [kv.len + int(d) for d in tree.depth], tree.paths,
                                         np.float32)
        st, acc = compare_step(eng, h, tree, M, S, kv.len, lo, k, rel_tol, None, step, None, None)
        O.commit(kv, nk, nv, acc.path)
        root = acc.bonus
        stats.append(st)
    return stats, kv


# ---- tiled KV layout, restated from include/tr.h (TR_KV_TILED) for test-side encode/decode ----
def _k_index(p, d):
    return ((p // 16) * 4 + d // 32) * 512 + ((p % 16) + 16 * ((d % 32) // 8)) * 8 + d % 8


def _v_index(p, d):
    return ((p // 32) * 8 + d // 16) * 512 + ((d % 16) + 16 * ((p % 16) // 4)) * 8 + ((p // 16) % 2) * 4 + p % 4


def kv_maps(cap, hd=128):
    p, d = np.meshgrid(np.arange(cap), np.arange(hd), indexing="ij")
    return _k_index(p, d), _v_index(p, d)          # [cap, hd] -> flat offset


def kv_plain_views(kvdesc, k_interleaved=False):
    """(k, v) as torch tensors [layers, heads, cap, hd] in natural order, whatever the layout.
    k_interleaved: the cache was written by a packed model, whose keys carry the rotation-pair
    interleaved feature order (stored feature 2j + b is natural feature j + b*hd/2)."""
    L, Hk, cap, hd = kvdesc.k.shape
    if not kvdesc.tiled:
        kf, vf = kvdesc.k, kvdesc.v.permute(0, 1, 3, 2)
    else:
        ki, vi = kv_maps(cap, hd)
        ki = torch.from_numpy(ki).to(kvdesc.k.device).reshape(-1)
        vi = torch.from_numpy(vi).to(kvdesc.k.device).reshape(-1)
        kf = kvdesc.k.reshape(L, Hk, cap * hd)[:, :, ki].reshape(L, Hk, cap, hd)
        vf = kvdesc.v.reshape(L, Hk, cap * hd)[:, :, vi].reshape(L, Hk, cap, hd)
    if k_interleaved:
        nat = torch.arange(hd, device=kf.device)
        kf = kf[..., 2 * (nat % (hd // 2)) + nat // (hd // 2)]
    return kf, vf


def kv_fill(kvdesc, k_plain, v_plain, k_interleaved=False):
    """Write natural-order tensors [layers, heads, cap, hd] into the cache in its layout.
    k_interleaved: the cache belongs to a packed model, whose keys are stored with the two features
    of a rotation pair adjacent (stored feature 2j + b is natural feature j + b*hd/2)."""
    L, Hk, cap, hd = kvdesc.k.shape
    if k_interleaved:
        st = torch.arange(hd, device=k_plain.device)
        k_plain = k_plain[..., st // 2 + (st % 2) * (hd // 2)]
    if not kvdesc.tiled:
        kvdesc.k.copy_(k_plain)
        kvdesc.v.copy_(v_plain.permute(0, 1, 3, 2))
        return
    ki, vi = kv_maps(cap, hd)
    ki = torch.from_numpy(ki).to(kvdesc.k.device).reshape(-1)
    vi = torch.from_numpy(vi).to(kvdesc.k.device).reshape(-1)
    kvdesc.k.reshape(L, Hk, cap * hd)[:, :, ki] = k_plain.reshape(L, Hk, cap * hd)
    kvdesc.v.reshape(L, Hk, cap * hd)[:, :, vi] = v_plain.reshape(L, Hk, cap * hd)


def kv_fill_prefix(kvdesc, layer, k_plain, v_plain, k_interleaved=False):
    """Write positions 0..P-1 of one layer of a tiled cache from natural-order tensors [heads, P, hd]
    (the tiled offsets of a position do not depend on the capacity)."""
    assert kvdesc.tiled
    _, Hk, cap, hd = kvdesc.k.shape
    P = k_plain.shape[1]
    if k_interleaved:
        st = torch.arange(hd, device=k_plain.device)
        k_plain = k_plain[..., st // 2 + (st % 2) * (hd // 2)]
    p, d = np.meshgrid(np.arange(P), np.arange(hd), indexing="ij")
    ki = torch.from_numpy(_k_index(p, d)).to(kvdesc.k.device).reshape(-1)
    vi = torch.from_numpy(_v_index(p, d)).to(kvdesc.k.device).reshape(-1)
    kvdesc.k[layer].reshape(Hk, cap * hd)[:, ki] = k_plain.reshape(Hk, P * hd)
    kvdesc.v[layer].reshape(Hk, cap * hd)[:, vi] = v_plain.reshape(Hk, P * hd)
