"""Thin ctypes binding over libtr (the C ABI declared in include/tr.h).

Argument marshalling only: every step of the decode path runs inside the library's HIP
kernels.  PyTorch supplies device memory and the stream.  There is no fallback: if the
shared library is missing, importing symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtr.so")

TR_MAX_NODES, TR_MAX_LAYERS, TR_MAX_K = 128, 32, 32
TR_OK, TR_EINVAL, TR_ETEMPLATE, TR_ENOMEM, TR_EHIP, TR_ECAPACITY, TR_ESTATE = 0, -1, -2, -3, -4, -5, -6
TR_F32, TR_BF16 = 0, 1
TR_ROW_MAJOR, TR_PACKED = 0, 1
TR_KV_PLAIN, TR_KV_TILED = 0, 1
TR_UPDATE_LAST, TR_UPDATE_FIRST, TR_UPDATE_ACCEPTED_ONLY = 0, 1, 2
DTYPES = {"f32": TR_F32, "bf16": TR_BF16}


class TreeTemplate(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_layers", C.c_int32),
                ("parent", C.POINTER(C.c_int32)), ("rank", C.POINTER(C.c_int32))]


class Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm",
                                          "w_gate", "w_up", "w_down")]


class Model(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("layout", C.c_int32), ("n_layers", C.c_int32), ("d_model", C.c_int32),
                ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("embed", C.c_void_p), ("layers", C.POINTER(Layer)),
                ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class KV(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("layout", C.c_int32), ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("capacity", C.c_int32), ("k", C.c_void_p),
                ("v", C.c_void_p), ("d_len", C.c_void_p), ("len_bound", C.c_int32)]


class StepOut(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("n_emitted", C.c_int32), ("winner", C.c_int32),
                ("next_root", C.c_int32), ("kv_len", C.c_int32),
                ("path", C.c_int32 * TR_MAX_LAYERS), ("emitted", C.c_int32 * TR_MAX_LAYERS)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("launches", C.c_int32), ("ms", C.c_double)]


STEP_OUT_INTS = C.sizeof(StepOut) // 4

_SIGS = {
    "tr_create": [C.c_int32, C.c_int32, C.POINTER(TreeTemplate), C.POINTER(C.c_void_p)],
    "tr_destroy": [C.c_void_p],
    "tr_set_update_mode": [C.c_void_p, C.c_int32],
    "tr_matrix_load": [C.c_void_p, C.c_void_p],
    "tr_matrix_store": [C.c_void_p, C.c_void_p],
    "tr_build_tree": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "tr_workspace_bytes": [C.c_void_p, C.POINTER(Model), C.POINTER(C.c_size_t)],
    "tr_plan_projection": [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)],
    "tr_plan_attention": [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)],
    "tr_verify_forward": [C.c_void_p, C.POINTER(Model), C.POINTER(KV), C.c_void_p, C.c_void_p,
                          C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "tr_accept_and_update": [C.c_void_p, C.POINTER(KV), C.c_void_p, C.c_void_p, C.c_void_p,
                             C.POINTER(StepOut), C.c_void_p],
    "tr_accept_and_update_sampled": [C.c_void_p, C.POINTER(KV), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.POINTER(StepOut), C.c_void_p],
    "tr_op_sample": [C.c_void_p, C.POINTER(KV), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
                     C.c_void_p, C.c_void_p],
    "tr_prefill": [C.c_void_p, C.POINTER(Model), C.POINTER(KV), C.c_void_p, C.c_int32, C.c_void_p,
                   C.c_size_t, C.c_void_p],
    "tr_op_topk": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "tr_op_topk_static": [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
    "tr_op_matrix_update": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "tr_op_tree_attention": [C.c_void_p, C.POINTER(KV), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_size_t, C.c_void_p],
    "tr_op_linear": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                     C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "tr_pack_weight": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p],
    "tr_pack_weight_rope": [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p],
    "tr_op_stream": [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p],
    "tr_profile_enable": [C.c_void_p, C.c_int32],
    "tr_profile_read": [C.c_void_p, C.POINTER(ProfileEntry), C.c_int32, C.POINTER(C.c_int32)],
}
EXPORTS = tuple(_SIGS) + ("tr_strerror",)

_lib = None


def lib() -> C.CDLL:
    """Load libtr.so (built in-tree by __graft_entry__.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        l = C.CDLL(LIB_PATH)
        for name, args in _SIGS.items():
            fn = getattr(l, name)
            fn.argtypes, fn.restype = args, C.c_int32
        l.tr_strerror.argtypes, l.tr_strerror.restype = [C.c_int32], C.c_char_p
        _lib = l
    return _lib


class TRError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().tr_strerror(status).decode()} ({status})")


def _check(status: int, where: str) -> None:
    if status != TR_OK:
        raise TRError(status, where)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_template(parent: Sequence[int], rank: Sequence[int], n_layers: int):
    p = np.ascontiguousarray(parent, dtype=np.int32)
    r = np.ascontiguousarray(rank, dtype=np.int32)
    t = TreeTemplate(len(p), n_layers, p.ctypes.data_as(C.POINTER(C.c_int32)),
                     r.ctypes.data_as(C.POINTER(C.c_int32)))
    return t, (p, r)


class Context:
    """Owns a tr_ctx: the adjacency matrix M[V, k] and the static tree."""

    def __init__(self, vocab: int, k: int, parent: Sequence[int], rank: Sequence[int], n_layers: int):
        self.vocab, self.k = vocab, k
        self.n_nodes, self.n_layers = len(parent), n_layers
        t, keep = make_template(parent, rank, n_layers)
        h = C.c_void_p()
        _check(lib().tr_create(vocab, k, C.byref(t), C.byref(h)), "tr_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().tr_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_update_mode(self, mode: int) -> None:
        _check(lib().tr_set_update_mode(self._h, mode), "tr_set_update_mode")

    def matrix_load(self, M: np.ndarray) -> None:
        M = np.ascontiguousarray(M, dtype=np.int32)
        assert M.shape == (self.vocab, self.k)
        _check(lib().tr_matrix_load(self._h, M.ctypes.data), "tr_matrix_load")

    def matrix_store(self) -> np.ndarray:
        M = np.empty((self.vocab, self.k), np.int32)
        _check(lib().tr_matrix_store(self._h, M.ctypes.data), "tr_matrix_store")
        return M

    def build_tree(self, d_root, d_S) -> None:
        _check(lib().tr_build_tree(self._h, _ptr(d_root), _ptr(d_S), _stream()), "tr_build_tree")

    def workspace_bytes(self, model: "ModelDesc") -> int:
        n = C.c_size_t()
        _check(lib().tr_workspace_bytes(self._h, C.byref(model.c), C.byref(n)), "tr_workspace_bytes")
        return n.value

    def verify_forward(self, model: "ModelDesc", kv: "KVDesc", d_S, d_logits, d_topk, ws) -> None:
        _check(lib().tr_verify_forward(self._h, C.byref(model.c), C.byref(kv.c), _ptr(d_S), _ptr(d_logits),
                                       _ptr(d_topk), _ptr(ws), ws.numel() * ws.element_size(), _stream()),
               "tr_verify_forward")

    def accept_and_update(self, kv: "KVDesc", d_S, d_topk, d_out, sync: bool = False,
                          d_tokens=None) -> Optional[StepOut]:
        """d_tokens: the model's token per node when it is a draw (temperature sampling), else the argmax."""
        h = StepOut() if sync else None
        if d_tokens is None:
            _check(lib().tr_accept_and_update(self._h, C.byref(kv.c), _ptr(d_S), _ptr(d_topk), _ptr(d_out),
                                              C.byref(h) if sync else None, _stream()), "tr_accept_and_update")
        else:
            _check(lib().tr_accept_and_update_sampled(self._h, C.byref(kv.c), _ptr(d_S), _ptr(d_topk),
                                                      _ptr(d_tokens), _ptr(d_out), C.byref(h) if sync else None,
                                                      _stream()), "tr_accept_and_update_sampled")
        return h

    def op_sample(self, kv: "KVDesc", d_logits, d_noise, inv_temperature: float, d_tokens, noise_pos0: int = 0) -> None:
        _check(lib().tr_op_sample(self._h, C.byref(kv.c), _ptr(d_logits), _ptr(d_noise), noise_pos0,
                                  d_noise.shape[0], inv_temperature, _ptr(d_tokens), _stream()), "tr_op_sample")

    def prefill(self, model: "ModelDesc", kv: "KVDesc", d_tokens, ws) -> None:
        _check(lib().tr_prefill(self._h, C.byref(model.c), C.byref(kv.c), _ptr(d_tokens), d_tokens.numel(),
                                _ptr(ws), ws.numel() * ws.element_size(), _stream()), "tr_prefill")

    def profile_enable(self, on: bool) -> None:
        _check(lib().tr_profile_enable(self._h, 1 if on else 0), "tr_profile_enable")

    def profile_read(self) -> dict:
        arr = (ProfileEntry * 32)()
        n = C.c_int32()
        _check(lib().tr_profile_read(self._h, arr, 32, C.byref(n)), "tr_profile_read")
        return {arr[i].name.decode(): (arr[i].launches, arr[i].ms) for i in range(n.value)}

    def op_topk(self, d_logits, d_topk) -> None:
        import torch
        dt = TR_BF16 if d_logits.dtype == torch.bfloat16 else TR_F32
        _check(lib().tr_op_topk(self._h, _ptr(d_logits), dt, d_logits.shape[0], _ptr(d_topk), _stream()),
               "tr_op_topk")

    def op_matrix_update(self, d_S, d_topk) -> None:
        _check(lib().tr_op_matrix_update(self._h, _ptr(d_S), _ptr(d_topk), _stream()), "tr_op_matrix_update")

    def op_tree_attention(self, kv: "KVDesc", layer: int, n_heads: int, d_q, d_out, ws) -> None:
        _check(lib().tr_op_tree_attention(self._h, C.byref(kv.c), layer, n_heads, _ptr(d_q), _ptr(d_out),
                                          _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                          _stream()), "tr_op_tree_attention")

    def op_linear(self, d_x, d_w, d_y, ws=None, packed: bool = False, splits: int = 1) -> None:
        """d_w: [out_f, in_f] row-major, or the packed buffer of the same logical shape."""
        import torch
        dt = TR_BF16 if d_x.dtype == torch.bfloat16 else TR_F32
        _check(lib().tr_op_linear(self._h, _ptr(d_x), _ptr(d_w), dt, TR_PACKED if packed else TR_ROW_MAJOR,
                                  d_x.shape[0], d_x.shape[1], d_w.shape[0], splits, _ptr(d_y), _ptr(ws),
                                  0 if ws is None else ws.numel() * ws.element_size(), _stream()), "tr_op_linear")


def plan_projection(n_rows: int, in_f: int, out_f: int, fused_pair: bool = False, max_splits: int = 4):
    """(weight tiles per workgroup, workgroups per split, splits) of one packed projection launch."""
    plan = (C.c_int32 * 3)()
    _check(lib().tr_plan_projection(n_rows, in_f, out_f, int(fused_pair), max_splits, plan), "tr_plan_projection")
    return tuple(plan)


def plan_attention(n_heads: int, n_kv_heads: int, n_nodes: int, len_bound: int):
    """(query heads per workgroup, key-axis splits) of one tree-attention launch."""
    plan = (C.c_int32 * 2)()
    _check(lib().tr_plan_attention(n_heads, n_kv_heads, n_nodes, len_bound, plan), "tr_plan_attention")
    return tuple(plan)


def op_topk_static(d_logits, d_topk) -> None:
    """argtopk of every row of d_logits [rows, V] (f32 or bf16) into d_topk [rows, k] int32 through the
    entry point that allocates nothing (no context; the library's static device scratch)."""
    import torch
    dt = TR_BF16 if d_logits.dtype == torch.bfloat16 else TR_F32
    _check(lib().tr_op_topk_static(_ptr(d_logits), dt, d_logits.shape[0], d_logits.shape[1], d_topk.shape[1],
                                   _ptr(d_topk), _stream()), "tr_op_topk_static")


def op_stream(src, dst=None) -> None:
    """Plain streaming read of `src` (or copy into `dst`) through the library's streaming kernel."""
    _check(lib().tr_op_stream(src.data_ptr(), _ptr(dst), src.numel() * src.element_size(), _stream()), "tr_op_stream")


def pack_weight(w, rope_head_dim: int = 0):
    """Packed copy of a row-major bf16 [out_f, in_f] device tensor (same shape tag, packed bytes).
    rope_head_dim > 0: a query / key projection, packed with its rows interleaved per head."""
    import torch
    assert w.dtype == torch.bfloat16 and w.is_contiguous() and w.dim() == 2
    out = torch.empty_like(w)
    if rope_head_dim > 0:
        _check(lib().tr_pack_weight_rope(w.data_ptr(), out.data_ptr(), w.shape[0], w.shape[1], rope_head_dim,
                                         _stream()), "tr_pack_weight_rope")
    else:
        _check(lib().tr_pack_weight(w.data_ptr(), out.data_ptr(), w.shape[0], w.shape[1], _stream()),
               "tr_pack_weight")
    return out


def pack_layer(shape, lw: dict) -> dict:
    """One layer of synth.make_weights with every projection matrix packed (wq, wk interleaved for RoPE)."""
    return {k: (pack_weight(v, shape.head_dim if k in ("wq", "wk") else 0) if k in ModelDesc.MATS else v)
            for k, v in lw.items()}


def can_pack(shape) -> bool:
    hq, hk = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    return shape.dtype == "bf16" and all(v % 32 == 0 for v in (shape.d_model, shape.d_ffn, hq, hk, shape.vocab))


class ModelDesc:
    """tr_model over torch tensors (kept alive here).  `weights` has the layout of
    synth.make_weights; `shape` carries the dimensions.  With pack=True (default where the shape
    allows it) every projection matrix and the LM head are repacked once into the MFMA operand
    order; the row-major originals are not referenced afterwards.  prepacked=True says the caller
    has already done that with pack_weight (a model too large to hold twice is packed layer by layer)."""

    MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")

    def __init__(self, shape, weights: dict, pack: Optional[bool] = None, prepacked: bool = False):
        if pack is None:
            pack = can_pack(shape)
        self.packed = bool(pack)
        if pack and not prepacked:
            weights = {"embed": weights["embed"], "final_norm": weights["final_norm"],
                       "lm_head": pack_weight(weights["lm_head"]),
                       "layers": [pack_layer(shape, lw) for lw in weights["layers"]]}
        self.weights = weights
        n = shape.n_layers
        self._layers = (Layer * n)()
        for l, lw in enumerate(weights["layers"]):
            for name, _ in Layer._fields_:
                setattr(self._layers[l], name, lw[name].data_ptr())
        self.c = Model(DTYPES[shape.dtype], TR_PACKED if pack else TR_ROW_MAJOR, n, shape.d_model, shape.n_heads,
                       shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_theta,
                       weights["embed"].data_ptr(), self._layers, weights["final_norm"].data_ptr(),
                       weights["lm_head"].data_ptr())


class KVDesc:
    """tr_kv plus the torch tensors behind it (zero-initialised).  Tiled layout (the fast attention
    kernel's operand order) for bf16 with head_dim 128 unless tiled=False; capacity is rounded up
    to a multiple of 32.  Plain layout: k [layers, kv_heads, capacity, head_dim],
    v [layers, kv_heads, head_dim, capacity]."""

    def __init__(self, shape, capacity: int, device="cuda", tiled: Optional[bool] = None):
        import torch
        dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        capacity = (capacity + 31) // 32 * 32
        if tiled is None:
            tiled = shape.dtype == "bf16" and shape.head_dim == 128
        self.tiled, self.capacity = bool(tiled), capacity
        self.k = torch.zeros(shape.n_layers, shape.n_kv_heads, capacity, shape.head_dim, dtype=dt, device=device)
        self.v = torch.zeros(shape.n_layers, shape.n_kv_heads, shape.head_dim, capacity, dtype=dt, device=device)
        self.d_len = torch.zeros(1, dtype=torch.int32, device=device)
        self.c = KV(DTYPES[shape.dtype], TR_KV_TILED if tiled else TR_KV_PLAIN, shape.n_layers, shape.n_kv_heads,
                    shape.head_dim, capacity, self.k.data_ptr(), self.v.data_ptr(), self.d_len.data_ptr(), 0)

    def reset(self, length: int = 0) -> None:
        self.d_len.fill_(length)
        self.c.len_bound = length


class Engine:
    """One decoding session: context + model + KV cache + the per-step device buffers.
    `step()` issues the three calls of a decode step on the current stream."""

    def __init__(self, shape, weights: dict, template, k: int = 8, capacity: int = 2048, device="cuda",
                 keep_logits: bool = True, pack: Optional[bool] = None, model: Optional[ModelDesc] = None,
                 kv_tiled: Optional[bool] = None):
        import torch
        self.shape, self.k = shape, k
        self.ctx = Context(shape.vocab, k, template.parent, template.rank, template.n_layers)
        self.model = model if model is not None else ModelDesc(shape, weights, pack)
        self.kv = KVDesc(shape, capacity, device, kv_tiled)
        n = template.n_nodes
        self.n_nodes = n
        self.ws = torch.empty(self.ctx.workspace_bytes(self.model), dtype=torch.uint8, device=device)
        self.S = torch.zeros(n, dtype=torch.int32, device=device)
        self.topk = torch.zeros(n, k, dtype=torch.int32, device=device)
        self.logits = torch.zeros(n, shape.vocab, dtype=torch.float32, device=device) if keep_logits else None
        self.out = torch.zeros(STEP_OUT_INTS, dtype=torch.int32, device=device)
        self.tokens = None                              # drawn tokens per node (temperature sampling)
        self.root = self.out[3:4]                       # next_root field of tr_step_out

    def prefill(self, prompt: Sequence[int], keep_cache: bool = False) -> None:
        """Commit prompt[:-1]; the last prompt token becomes the first root.  keep_cache: append to
        what the cache already holds instead of starting from an empty one."""
        import torch
        toks = torch.tensor(list(prompt), dtype=torch.int32, device=self.S.device)
        if not keep_cache:
            self.kv.reset(0)
        if len(prompt) > 1:
            self.ctx.prefill(self.model, self.kv, toks[:-1].contiguous(), self.ws)
        self.root.copy_(toks[-1:])

    def step(self, sync: bool = False, sampler=None) -> Optional[StepOut]:
        """sampler = (1/T, noise [positions, vocab] float32 device tensor): temperature sampling."""
        self.ctx.build_tree(self.root, self.S)
        self.ctx.verify_forward(self.model, self.kv, self.S, self.logits, self.topk, self.ws)
        if sampler is None:
            return self.ctx.accept_and_update(self.kv, self.S, self.topk, self.out, sync)
        if self.logits is None:
            raise ValueError("temperature sampling needs the logits: create the Engine with keep_logits=True")
        if self.tokens is None:
            import torch
            self.tokens = torch.zeros(self.n_nodes, dtype=torch.int32, device=self.S.device)
        self.ctx.op_sample(self.kv, self.logits, sampler[1], sampler[0], self.tokens)
        return self.ctx.accept_and_update(self.kv, self.S, self.topk, self.out, sync, self.tokens)
