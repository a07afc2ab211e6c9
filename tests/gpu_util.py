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


def lockstep(eng, sh, w_np, tmpl, prompt, n_steps, M0, k=8, rel_tol=2e-2, abs_tol=None, dtype=np.float64,
             label="", sampler=None):
    """Teacher-forced parity of whole steps.  Each step the oracle starts from the same integer
    state as the GPU (root, M, committed tokens), its logits are compared under the tolerance, and
    its integer pipeline (top-k, accept, matrix update) is applied to the GPU's own logits and must
    reproduce the GPU's integers bit for bit.  Returns per-step stats.
    sampler = (1/T, noise [positions, vocab] float32 numpy): temperature sampling on both sides; the
    oracle's draws from the GPU's logits must equal the GPU's draws."""
    cfg = oracle_cfg(sh)
    tree = O.make_tree(tmpl.parent, tmpl.rank, k)
    eng.ctx.matrix_load(M0)
    eng.prefill(prompt)
    M = M0.astype(np.int64).copy()
    kv = O.KVCache(cfg, len(prompt) + n_steps * tree.n_layers + tree.n_nodes + 8, dtype)
    O.prefill(cfg, w_np, kv, list(prompt[:-1]), dtype)
    root = int(prompt[-1])
    stats = []
    gpu_sampler = None if sampler is None else (sampler[0], torch.from_numpy(sampler[1]).cuda())
    for step in range(n_steps):
        say(f"lockstep {label} step {step} L={kv.len}")
        h = eng.step(sync=True, sampler=gpu_sampler)
        S = O.build_tree(M, tree, root)
        assert eng.S.cpu().tolist() == S.tolist(), f"step {step}: tree differs"
        pos = [kv.len + int(d) for d in tree.depth]
        lo, nk, nv = O.forward_nodes(cfg, w_np, kv, S, pos, tree.paths, dtype)
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
        assert h.next_root == acc.bonus and h.kv_len == kv.len + acc.n_accepted + 1
        assert np.array_equal(eng.ctx.matrix_store().astype(np.int64), M), f"step {step}: matrix differs"
        # rows whose own-logit top-k differs from the GPU's must be near-ties within the error
        flips = 0
        for n in range(tree.n_nodes):
            mine = O.topk_ids(lo[n], k)
            if not np.array_equal(mine, topk[n]):
                flips += 1
                srt = -np.sort(-lo[n])[:k + 1]
                assert np.min(srt[:-1] - srt[1:]) <= 2 * err[n] + 1e-12, f"step {step} row {n}: flip without near-tie"
        O.commit(kv, nk, nv, acc.path)
        root = acc.bonus
        stats.append(dict(step=step, max_err=float(err.max()), max_rel=float(np.max(err / scale)), flips=flips,
                          n_emitted=acc.n_accepted + 1))
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


def kv_fill(kvdesc, k_plain, v_plain):
    """Write natural-order tensors [layers, heads, cap, hd] into the cache in its layout."""
    L, Hk, cap, hd = kvdesc.k.shape
    if not kvdesc.tiled:
        kvdesc.k.copy_(k_plain)
        kvdesc.v.copy_(v_plain.permute(0, 1, 3, 2))
        return
    ki, vi = kv_maps(cap, hd)
    ki = torch.from_numpy(ki).to(kvdesc.k.device).reshape(-1)
    vi = torch.from_numpy(vi).to(kvdesc.k.device).reshape(-1)
    kvdesc.k.reshape(L, Hk, cap * hd)[:, :, ki] = k_plain.reshape(L, Hk, cap * hd)
    kvdesc.v.reshape(L, Hk, cap * hd)[:, :, vi] = v_plain.reshape(L, Hk, cap * hd)
