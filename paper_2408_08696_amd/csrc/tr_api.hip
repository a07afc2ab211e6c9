// C ABI of the Token Recycling decode step: argument validation (always before the first HIP call
// of a function), context lifetime, and the three step calls.
#include <new>
#include <string.h>

#include "tr_internal.h"
#include "tr_kernels.h"

using namespace tr;

namespace {

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Derive depth and ancestor masks on the host; returns false if the template is malformed.
bool derive_tree(const tr_tree_template *t, int32_t k, int32_t *depth, uint64_t *anc) {
  const int n = t->n_nodes;
  if (n < 1 || n > TR_MAX_NODES || t->parent == nullptr || t->rank == nullptr) return false;
  if (t->parent[0] != -1 || t->rank[0] != -1) return false;
  depth[0] = 0;
  anc[0] = 1;
  anc[1] = 0;
  for (int i = 1; i < n; ++i) {
    const int p = t->parent[i], r = t->rank[i];
    if (p < 0 || p >= i || r < 0 || r >= k) return false;
    for (int j = 1; j < i; ++j)
      if (t->parent[j] == p && t->rank[j] == r) return false;
    depth[i] = depth[p] + 1;
    if (depth[i] < depth[i - 1]) return false; // layer-major order
    anc[2 * i] = anc[2 * p];
    anc[2 * i + 1] = anc[2 * p + 1];
    anc[2 * i + (i >> 6)] |= 1ull << (i & 63);
  }
  const int layers = depth[n - 1] + 1;
  return layers == t->n_layers && layers <= TR_MAX_LAYERS;
}

tr_status check_model(const tr_model *m) {
  if (m == nullptr) return TR_EINVAL;
  if (m->dtype != TR_F32 && m->dtype != TR_BF16) return TR_EINVAL;
  if (m->n_layers <= 0 || m->d_model <= 0 || m->n_heads <= 0 || m->n_kv_heads <= 0 || m->head_dim <= 0 ||
      m->d_ffn <= 0 || m->vocab <= 0)
    return TR_EINVAL;
  if (m->n_heads % m->n_kv_heads != 0) return TR_EINVAL;
  if (m->head_dim % 2 != 0 || m->head_dim > 256) return TR_EINVAL;
  if (m->d_model % 4 != 0 || m->d_ffn % 4 != 0) return TR_EINVAL;
  if (!(m->rms_eps >= 0.f) || !(m->rope_theta > 0.f)) return TR_EINVAL;
  if (m->layout != TR_ROW_MAJOR && m->layout != TR_PACKED) return TR_EINVAL;
  if (!model_layout_ok(*m)) return TR_EINVAL;
  if (m->embed == nullptr || m->layers == nullptr || m->final_norm == nullptr || m->lm_head == nullptr)
    return TR_EINVAL;
  for (int l = 0; l < m->n_layers; ++l) {
    const tr_layer &w = m->layers[l];
    if (!w.attn_norm || !w.wq || !w.wk || !w.wv || !w.wo || !w.ffn_norm || !w.w_gate || !w.w_up || !w.w_down)
      return TR_EINVAL;
  }
  return TR_OK;
}

tr_status check_kv(const tr_kv *kv) {
  if (kv == nullptr) return TR_EINVAL;
  if (kv->dtype != TR_F32 && kv->dtype != TR_BF16) return TR_EINVAL;
  if (kv->n_layers <= 0 || kv->n_kv_heads <= 0 || kv->head_dim <= 0 || kv->head_dim > 256 || kv->capacity <= 0)
    return TR_EINVAL;
  if (kv->k == nullptr || kv->v == nullptr || kv->d_len == nullptr) return TR_EINVAL;
  if (kv->len_bound < 0) return TR_EINVAL;
  if (kv->layout != TR_KV_PLAIN && kv->layout != TR_KV_TILED) return TR_EINVAL;
  if (kv->layout == TR_KV_TILED && (kv->dtype != TR_BF16 || kv->head_dim != 128 || kv->capacity % 32 != 0))
    return TR_EINVAL;
  return TR_OK;
}

tr_status check_model_kv(const tr_ctx *ctx, const tr_model *m, const tr_kv *kv) {
  tr_status s = check_model(m);
  if (s != TR_OK) return s;
  s = check_kv(kv);
  if (s != TR_OK) return s;
  if (kv->dtype != m->dtype || kv->n_layers != m->n_layers || kv->n_kv_heads != m->n_kv_heads ||
      kv->head_dim != m->head_dim)
    return TR_EINVAL;
  if (ctx != nullptr && m->vocab != ctx->V) return TR_EINVAL;
  return TR_OK;
}

} // namespace

extern "C" {

const char *tr_strerror(tr_status s) {
  switch (s) {
  case TR_OK: return "ok";
  case TR_EINVAL: return "invalid argument";
  case TR_ETEMPLATE: return "malformed tree template";
  case TR_ENOMEM: return "out of memory";
  case TR_EHIP: return "HIP runtime error";
  case TR_ECAPACITY: return "KV cache or workspace too small";
  case TR_ESTATE: return "call not allowed in this state";
  }
  return "unknown status";
}

tr_status tr_create(int32_t V, int32_t k, const tr_tree_template *t, tr_ctx **out) {
  if (out == nullptr || t == nullptr || V <= 0 || k <= 0 || k > TR_MAX_K || k > V) return TR_EINVAL;
  int32_t depth[TR_MAX_NODES];
  uint64_t anc[2 * TR_MAX_NODES];
  if (!derive_tree(t, k, depth, anc)) return TR_ETEMPLATE;

  tr_ctx *c = new (std::nothrow) tr_ctx();
  if (c == nullptr) return TR_ENOMEM;
  memset(c, 0, sizeof(*c));
  c->V = V;
  c->k = k;

  // host image of both trees and of the context's scratch.  The 64-bit parts come first so that every
  // section is 8-byte aligned whatever the node count: anc u64 x 2(n + cn) (tree, then chain), the top-k
  // candidate scratch (u64), then [parent | rank | depth] int32 x n of the tree and x cn of the chain, then
  // the step's committed length.
  const int n = t->n_nodes, cn = TR_MAX_NODES;
  const size_t ancs = 2 * (size_t)(n + cn) * sizeof(uint64_t);
  const size_t cand = topk_scratch_bytes();
  const size_t ints = 3 * (size_t)(n + cn) * sizeof(int32_t);
  static_assert(sizeof(uint64_t) == 8, "section offsets below assume 8-byte words");
  const size_t blob = ancs + cand + ints + sizeof(int32_t) * 64;
  unsigned char *h = new (std::nothrow) unsigned char[blob];
  if (h == nullptr) {
    delete c;
    return TR_ENOMEM;
  }
  memset(h, 0, blob);
  uint64_t *ha = reinterpret_cast<uint64_t *>(h);
  int32_t *hi = reinterpret_cast<int32_t *>(h + ancs + cand);
  memcpy(hi, t->parent, sizeof(int32_t) * n);
  memcpy(hi + n, t->rank, sizeof(int32_t) * n);
  memcpy(hi + 2 * n, depth, sizeof(int32_t) * n);
  memcpy(ha, anc, sizeof(uint64_t) * 2 * n);
  int32_t *ci = hi + 3 * n;
  uint64_t *ca = ha + 2 * n;
  for (int i = 0; i < cn; ++i) {
    ci[i] = i - 1;                   // parent
    ci[cn + i] = i == 0 ? -1 : 0;    // rank
    ci[2 * cn + i] = i;              // depth
    ca[2 * i] = i >= 63 ? ~0ull : ((1ull << (i + 1)) - 1);
    ca[2 * i + 1] = i < 64 ? 0ull : (i - 64 >= 63 ? ~0ull : ((1ull << (i - 64 + 1)) - 1));
  }

  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->d_M), (size_t)V * k * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(c->d_M, 0, (size_t)V * k * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(&c->d_tree_blob, blob);
  if (e == hipSuccess) e = hipMemcpy(c->d_tree_blob, h, blob, hipMemcpyHostToDevice);
  delete[] h;
  if (e != hipSuccess) {
    const tr_status st = e == hipErrorOutOfMemory ? TR_ENOMEM : TR_EHIP;
    if (c->d_M) (void)hipFree(c->d_M);
    if (c->d_tree_blob) (void)hipFree(c->d_tree_blob);
    delete c;
    return st;
  }
  unsigned char *d = static_cast<unsigned char *>(c->d_tree_blob); // hipMalloc: 256-byte aligned
  const uint64_t *da = reinterpret_cast<const uint64_t *>(d);
  const int32_t *di = reinterpret_cast<const int32_t *>(d + ancs + cand);
  c->tree = TreeDev{n, t->n_layers, di, di + n, di + 2 * n, da};
  c->chain = TreeDev{cn, cn, di + 3 * n, di + 3 * n + cn, di + 3 * n + 2 * cn, da + 2 * n};
  c->d_topk_cand = d + ancs;
  c->d_step_L = reinterpret_cast<int32_t *>(d + ancs + cand + ints);
  *out = c;
  return TR_OK;
}

tr_status tr_destroy(tr_ctx *c) {
  if (c == nullptr) return TR_EINVAL;
  if (c->prof.ev != nullptr) {
    for (int i = 0; i < 2 * Profiler::MAX_PAIRS; ++i) (void)hipEventDestroy(c->prof.ev[i]);
    delete[] c->prof.ev;
    delete[] c->prof.cat;
  }
  hipError_t e1 = hipFree(c->d_M), e2 = hipFree(c->d_tree_blob);
  delete c;
  return (e1 == hipSuccess && e2 == hipSuccess) ? TR_OK : TR_EHIP;
}

tr_status tr_set_update_mode(tr_ctx *c, int32_t mode) {
  if (c == nullptr || mode < 0 || mode > (TR_UPDATE_FIRST | TR_UPDATE_ACCEPTED_ONLY)) return TR_EINVAL;
  c->update_mode = mode;
  return TR_OK;
}

tr_status tr_matrix_load(tr_ctx *c, const int32_t *h_M) {
  if (c == nullptr || h_M == nullptr) return TR_EINVAL;
  const size_t cnt = (size_t)c->V * c->k;
  for (size_t i = 0; i < cnt; ++i)
    if (h_M[i] < 0 || h_M[i] >= c->V) return TR_EINVAL;
  return hipMemcpy(c->d_M, h_M, cnt * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_matrix_store(tr_ctx *c, int32_t *h_M) {
  if (c == nullptr || h_M == nullptr) return TR_EINVAL;
  const size_t cnt = (size_t)c->V * c->k;
  if (hipDeviceSynchronize() != hipSuccess) return TR_EHIP;
  return hipMemcpy(h_M, c->d_M, cnt * sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_build_tree(tr_ctx *c, const int32_t *d_root, int32_t *d_S, void *stream) {
  if (c == nullptr || d_root == nullptr || d_S == nullptr) return TR_EINVAL;
  return launch_build_tree(c, d_root, d_S, as_stream(stream)) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_plan_projection(int32_t n_rows, int32_t in_f, int32_t out_f, int32_t fused_pair, int32_t max_splits,
                             int32_t *plan) {
  if (plan == nullptr || max_splits < 1 || !gemm_mfma_supported(n_rows, in_f, out_f)) return TR_EINVAL;
  const int32_t tiles = out_f / 16;
  gemm_choose(n_rows, in_f, tiles, fused_pair != 0, fused_pair != 0 ? 1 : max_splits, &plan[0], &plan[1], &plan[2]);
  return TR_OK;
}

tr_status tr_plan_attention(int32_t n_heads, int32_t n_kv_heads, int32_t n_nodes, int32_t len_bound, int32_t *plan) {
  if (plan == nullptr || n_kv_heads < 1 || n_heads < n_kv_heads || n_heads % n_kv_heads != 0 || n_nodes < 1 ||
      n_nodes > TR_MAX_NODES || len_bound < 1)
    return TR_EINVAL;
  if (attn_one_launch(n_heads, n_kv_heads, len_bound)) { // one workgroup per (head, node tile), no key splits
    plan[0] = 1;
    plan[1] = 0;
    return TR_OK;
  }
  plan[0] = attn_heads_per_wg(n_heads, n_kv_heads, n_nodes);
  plan[1] = attn_choose_splits(n_heads / plan[0], len_bound);
  return TR_OK;
}

tr_status tr_workspace_bytes(const tr_ctx *c, const tr_model *m, size_t *bytes) {
  if (c == nullptr || bytes == nullptr) return TR_EINVAL;
  tr_status s = check_model(m);
  if (s != TR_OK) return s;
  *bytes = plan_workspace(*m).total;
  return TR_OK;
}

tr_status tr_verify_forward(tr_ctx *c, const tr_model *m, tr_kv *kv, const int32_t *d_S, float *d_logits,
                            int32_t *d_topk, void *ws, size_t ws_bytes, void *stream) {
  if (c == nullptr || d_S == nullptr || d_topk == nullptr || ws == nullptr) return TR_EINVAL;
  tr_status s = check_model_kv(c, m, kv);
  if (s != TR_OK) return s;
  const int n = c->tree.n_nodes;
  if ((int64_t)kv->len_bound + n > kv->capacity) return TR_ECAPACITY;
  const Workspace w = plan_workspace(*m);
  if (ws_bytes < w.total) return TR_ECAPACITY;
  float *logits = d_logits != nullptr ? d_logits : reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + w.logits);
  hipStream_t st = as_stream(stream);
  if (run_forward(*m, *kv, c->tree, n, d_S, logits, ws, &c->prof, st) != hipSuccess) return TR_EHIP;
  if (launch_topk(logits, TR_F32, n, m->vocab, c->k, d_topk, c->d_topk_cand, &c->prof, st) != hipSuccess) return TR_EHIP;
  return TR_OK;
}

static tr_status accept_and_update(tr_ctx *c, tr_kv *kv, const int32_t *d_S, const int32_t *d_topk,
                                   const int32_t *d_tokens, tr_step_out *d_out, tr_step_out *h_out, void *stream) {
  if (c == nullptr || d_S == nullptr || d_topk == nullptr || d_out == nullptr) return TR_EINVAL;
  tr_status s = check_kv(kv);
  if (s != TR_OK) return s;
  if ((int64_t)kv->len_bound + c->tree.n_nodes > kv->capacity) return TR_ECAPACITY;
  hipStream_t st = as_stream(stream);
  if (launch_accept_update(c, kv, d_S, d_topk, d_tokens, d_out, st) != hipSuccess) return TR_EHIP;
  if (h_out != nullptr) {
    if (hipMemcpyAsync(h_out, d_out, sizeof(tr_step_out), hipMemcpyDeviceToHost, st) != hipSuccess) return TR_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return TR_EHIP;
    kv->len_bound = h_out->kv_len;
  } else {
    kv->len_bound += c->tree.n_layers;
  }
  return TR_OK;
}

tr_status tr_accept_and_update(tr_ctx *c, tr_kv *kv, const int32_t *d_S, const int32_t *d_topk, tr_step_out *d_out,
                               tr_step_out *h_out, void *stream) {
  return accept_and_update(c, kv, d_S, d_topk, nullptr, d_out, h_out, stream);
}

tr_status tr_accept_and_update_sampled(tr_ctx *c, tr_kv *kv, const int32_t *d_S, const int32_t *d_topk,
                                       const int32_t *d_tokens, tr_step_out *d_out, tr_step_out *h_out, void *stream) {
  if (d_tokens == nullptr) return TR_EINVAL;
  return accept_and_update(c, kv, d_S, d_topk, d_tokens, d_out, h_out, stream);
}

tr_status tr_op_sample(tr_ctx *c, const tr_kv *kv, const float *d_logits, const float *d_noise, int32_t noise_pos0,
                       int32_t noise_rows, float inv_temperature, int32_t *d_tokens, void *stream) {
  if (c == nullptr || d_logits == nullptr || d_noise == nullptr || d_tokens == nullptr) return TR_EINVAL;
  tr_status s = check_kv(kv);
  if (s != TR_OK) return s;
  if (noise_pos0 < 0 || noise_rows <= 0 || !(inv_temperature > 0.0f) || !(inv_temperature < 3.0e38f)) return TR_EINVAL;
  // the deepest node sits at L + n_layers - 1 with L <= len_bound
  if ((int64_t)kv->len_bound + c->tree.n_layers > (int64_t)noise_pos0 + noise_rows) return TR_ECAPACITY;
  return launch_sample_tokens(c, kv, d_logits, d_noise, noise_pos0, noise_rows, inv_temperature, d_tokens,
                              as_stream(stream)) == hipSuccess
             ? TR_OK
             : TR_EHIP;
}

tr_status tr_prefill(tr_ctx *c, const tr_model *m, tr_kv *kv, const int32_t *d_tokens, int32_t n_tokens, void *ws,
                     size_t ws_bytes, void *stream) {
  if (c == nullptr || d_tokens == nullptr || ws == nullptr || n_tokens < 0) return TR_EINVAL;
  tr_status s = check_model_kv(c, m, kv);
  if (s != TR_OK) return s;
  if ((int64_t)kv->len_bound + n_tokens > kv->capacity) return TR_ECAPACITY;
  if (ws_bytes < plan_workspace(*m).total) return TR_ECAPACITY;
  hipStream_t st = as_stream(stream);
  const int rows = prefill_rows(*m, *kv);
  for (int lo = 0; lo < n_tokens; lo += rows) {
    const int n = n_tokens - lo < rows ? n_tokens - lo : rows;
    if (run_prefill_pass(*m, *kv, c->chain, n, d_tokens + lo, ws, st) != hipSuccess) return TR_EHIP;
    if (launch_advance_len(kv->d_len, n, st) != hipSuccess) return TR_EHIP;
    kv->len_bound += n;
  }
  return TR_OK;
}

tr_status tr_op_topk(tr_ctx *c, const void *d_logits, int32_t dtype, int32_t n_rows, int32_t *d_topk, void *stream) {
  if (c == nullptr || d_logits == nullptr || d_topk == nullptr || n_rows < 0) return TR_EINVAL;
  if (dtype != TR_F32 && dtype != TR_BF16) return TR_EINVAL;
  return launch_topk(d_logits, dtype, n_rows, c->V, c->k, d_topk, c->d_topk_cand, nullptr, as_stream(stream)) == hipSuccess
             ? TR_OK
             : TR_EHIP;
}

tr_status tr_op_topk_static(const void *d_logits, int32_t dtype, int32_t n_rows, int32_t V, int32_t k,
                            int32_t *d_topk, void *stream) {
  if (d_logits == nullptr || d_topk == nullptr || n_rows < 0) return TR_EINVAL;
  if (dtype != TR_F32 && dtype != TR_BF16) return TR_EINVAL;
  if (V <= 0 || k <= 0 || k > V) return TR_EINVAL;
  if (!topk_static_fits(n_rows, V, k)) return TR_ECAPACITY;
  return launch_topk_static(d_logits, dtype, n_rows, V, k, d_topk, as_stream(stream)) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_op_matrix_update(tr_ctx *c, const int32_t *d_S, const int32_t *d_topk, void *stream) {
  if (c == nullptr || d_S == nullptr || d_topk == nullptr) return TR_EINVAL;
  return launch_matrix_update(c, d_S, d_topk, as_stream(stream)) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_op_tree_attention(tr_ctx *c, const tr_kv *kv, int32_t layer, int32_t n_heads, const void *d_q, void *d_out,
                               void *ws, size_t ws_bytes, void *stream) {
  if (c == nullptr || d_q == nullptr || d_out == nullptr) return TR_EINVAL;
  tr_status s = check_kv(kv);
  if (s != TR_OK) return s;
  if (layer < 0 || layer >= kv->n_layers || n_heads <= 0 || n_heads % kv->n_kv_heads != 0) return TR_EINVAL;
  if ((int64_t)kv->len_bound + c->tree.n_nodes > kv->capacity) return TR_ECAPACITY;
  const size_t need = ((size_t)ATTN_MAX_SPLITS * NP * n_heads * 2 * 4 + 255) / 256 * 256 +
                      (size_t)ATTN_MAX_SPLITS * NP * n_heads * kv->head_dim * 4;
  if (kv->dtype == TR_BF16 && (ws == nullptr || ws_bytes < need)) return TR_ECAPACITY;
  return run_tree_attention(*kv, layer, n_heads, c->tree, d_q, d_out, ws, as_stream(stream)) == hipSuccess ? TR_OK
                                                                                                            : TR_EHIP;
}

tr_status tr_op_linear(tr_ctx *c, const void *d_x, const void *d_w, int32_t dtype, int32_t layout, int32_t n_rows,
                       int32_t in_f, int32_t out_f, int32_t splits, float *d_y, void *ws, size_t ws_bytes,
                       void *stream) {
  if (c == nullptr || d_x == nullptr || d_w == nullptr || d_y == nullptr) return TR_EINVAL;
  if (dtype != TR_F32 && dtype != TR_BF16) return TR_EINVAL;
  if (layout != TR_ROW_MAJOR && layout != TR_PACKED) return TR_EINVAL;
  if (n_rows <= 0 || n_rows > (layout == TR_PACKED ? TR_PREFILL_ROWS : TR_MAX_NODES) || in_f <= 0 || out_f <= 0)
    return TR_EINVAL;
  if (layout == TR_PACKED) {
    if (dtype != TR_BF16) return TR_EINVAL;
    if (n_rows <= TR_MAX_NODES ? !gemm_mfma_supported(n_rows, in_f, out_f) : !gemm_wide_supported(n_rows, in_f, out_f))
      return TR_EINVAL;
    if (splits < 1 || splits > GEMM_MAX_SPLITS) return TR_EINVAL;
    if (ws == nullptr || ws_bytes < linear_workspace_bytes(n_rows, in_f, out_f, splits)) return TR_ECAPACITY;
  }
  return run_linear(d_x, d_w, dtype, layout, n_rows, in_f, out_f, splits, d_y, ws, as_stream(stream)) == hipSuccess
             ? TR_OK
             : TR_EHIP;
}

tr_status tr_pack_weight(const void *d_src, void *d_dst, int32_t out_f, int32_t in_f, void *stream) {
  if (d_src == nullptr || d_dst == nullptr || d_src == d_dst) return TR_EINVAL;
  if (out_f <= 0 || in_f <= 0 || out_f % 32 != 0 || in_f % 32 != 0) return TR_EINVAL;
  return launch_pack_weight((const bf16_t *)d_src, (bf16_t *)d_dst, out_f, in_f, 0, as_stream(stream)) == hipSuccess
             ? TR_OK
             : TR_EHIP;
}

tr_status tr_pack_weight_rope(const void *d_src, void *d_dst, int32_t out_f, int32_t in_f, int32_t head_dim,
                              void *stream) {
  if (d_src == nullptr || d_dst == nullptr || d_src == d_dst) return TR_EINVAL;
  if (out_f <= 0 || in_f <= 0 || out_f % 32 != 0 || in_f % 32 != 0) return TR_EINVAL;
  if (head_dim <= 0 || head_dim % 4 != 0 || out_f % head_dim != 0) return TR_EINVAL;
  return launch_pack_weight((const bf16_t *)d_src, (bf16_t *)d_dst, out_f, in_f, head_dim, as_stream(stream)) ==
                 hipSuccess
             ? TR_OK
             : TR_EHIP;
}

tr_status tr_op_stream(const void *d_src, void *d_dst, size_t bytes, void *stream) {
  if (d_src == nullptr || bytes == 0 || bytes % 16 != 0) return TR_EINVAL;
  return launch_stream(d_src, d_dst, bytes, as_stream(stream)) == hipSuccess ? TR_OK : TR_EHIP;
}

tr_status tr_profile_enable(tr_ctx *c, int32_t enable) {
  if (c == nullptr) return TR_EINVAL;
  Profiler &p = c->prof;
  if (enable && p.ev == nullptr) {
    p.ev = new (std::nothrow) hipEvent_t[2 * Profiler::MAX_PAIRS];
    p.cat = new (std::nothrow) int8_t[Profiler::MAX_PAIRS];
    if (p.ev == nullptr || p.cat == nullptr) return TR_ENOMEM;
    for (int i = 0; i < 2 * Profiler::MAX_PAIRS; ++i)
      if (hipEventCreate(&p.ev[i]) != hipSuccess) return TR_EHIP;
  }
  p.enabled = enable != 0;
  return TR_OK;
}

tr_status tr_profile_read(tr_ctx *c, tr_profile_entry *h, int32_t max_entries, int32_t *n_entries) {
  static const char *const names[PC_COUNT] = {"build_tree", "embed_rope_table", "residual_norm", "qkv_proj",
                                              "rope_kv_write", "tree_attention", "attention_merge", "o_proj",
                                              "gate_up_swiglu", "down_proj", "lm_head", "topk", "topk_merge",
                                              "accept_update", "compact_kv", "sample_tokens"};
  if (c == nullptr || h == nullptr || n_entries == nullptr || max_entries < 0) return TR_EINVAL;
  Profiler &p = c->prof;
  if (hipDeviceSynchronize() != hipSuccess) return TR_EHIP;
  double ms[PC_COUNT] = {0};
  int cnt[PC_COUNT] = {0};
  for (int i = 0; i < p.used; ++i) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, p.ev[2 * i], p.ev[2 * i + 1]) != hipSuccess) return TR_EHIP;
    ms[p.cat[i]] += t;
    cnt[p.cat[i]] += 1;
  }
  p.used = 0;
  int n = 0;
  for (int k = 0; k < PC_COUNT && n < max_entries; ++k) {
    if (cnt[k] == 0) continue;
    memset(&h[n], 0, sizeof(h[n]));
    strncpy(h[n].name, names[k], sizeof(h[n].name) - 1);
    h[n].launches = cnt[k];
    h[n].ms = ms[k];
    ++n;
  }
  *n_entries = n;
  return TR_OK;
}

} // extern "C"
