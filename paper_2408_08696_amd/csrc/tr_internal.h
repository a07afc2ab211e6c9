// Internal declarations shared by the translation units of libtr (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "tr.h"

namespace tr {

// ---------------------------------------------------------------------------------------------
// bf16 storage helpers (round-to-nearest-even; NaN inputs are not supported anywhere on the path)
// ---------------------------------------------------------------------------------------------
typedef uint16_t bf16_t;

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
  union { uint32_t u; float f; } c;
  c.u = ((uint32_t)b) << 16;
  return c.f;
}
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ inline float to_f32(T v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

inline size_t dtype_size(int32_t dt) { return dt == TR_BF16 ? 2 : 4; }

// Element offsets inside one (layer, kv head) block of the cache, head_dim 128, TR_KV_TILED.
// K: 16 positions x 32 d per KiB tile, tiles ordered (pos/16, d/32): the A operand of S^T = K Q^T.
// V: 16 d x 32 positions per KiB tile, tiles ordered (pos/32, d/16); inside a lane slot the 8 elements
//    are positions {4g..4g+3} of the first and of the second 16-position half (g = slot/16): the order in
//    which the S^T accumulators of two consecutive 16-key tiles sit in a lane.
__host__ __device__ inline size_t kv_k_index(int pos, int d) {
  return ((size_t)(pos >> 4) * 4 + (d >> 5)) * 512 + ((pos & 15) + 16 * ((d & 31) >> 3)) * 8 + (d & 7);
}
__host__ __device__ inline size_t kv_v_index(int pos, int d) {
  return ((size_t)(pos >> 5) * 8 + (d >> 4)) * 512 + ((d & 15) + 16 * ((pos & 15) >> 2)) * 8 + ((pos >> 4) & 1) * 4 +
         (pos & 3);
}

// ---------------------------------------------------------------------------------------------
// device copy of a tree: node i sits depth[i] below the root and may attend to the tree nodes
// whose bits are set in anc[i] (its ancestors and itself; 128 bits as two 64-bit words)
// ---------------------------------------------------------------------------------------------
struct TreeDev {
  int32_t n_nodes;
  int32_t n_layers;
  const int32_t *parent; // [n]
  const int32_t *rank;   // [n]
  const int32_t *depth;  // [n]
  const uint64_t *anc;   // [n][2]
};

// Workspace carve-up (byte offsets, all 256-aligned).  Buffers are sized for NP = TR_MAX_NODES rows; for models
// the packed path serves, the activation buffers (x, xn, q, attn, h, rope, ssq, and ypart as one complete sum)
// hold NPW rows, which is what one prompt-ingestion pass takes.
struct Workspace {
  size_t x;        // float  [NP, d]            residual stream
  size_t xn;       // T      [NP, d]            normalised activations
  size_t qkv;      // float  [NP, (H+2Hkv)*hd]  (generic path only)
  size_t q;        // T      [NP, H*hd]         rotated queries
  size_t attn;     // T      [NP, H*hd]         attention output
  size_t gu;       // float  [NP, 2F]           gate | up (generic path only)
  size_t h;        // T      [NP, F]            silu(gate)*up
  size_t rope;     // float  [NP, hd]           cos[hd/2] | sin[hd/2] per row
  size_t logits;   // float  [NP, V]            used when the caller passes no logits buffer
  size_t part_ml;  // float  [SPLITS, NP, H, 2] attention split partials: running max, sum
  size_t part_acc; // float  [SPLITS, NP, H, hd]
  size_t ypart;    // float  [GEMM_MAX_SPLITS, NP, d] K-split partial sums of o_proj / down_proj
  size_t ssq;      // float  [NP, ceil(d/1024)] per-row partial sums of squares of the residual stream
  size_t total;
};
constexpr int NP = TR_MAX_NODES;
constexpr int NPW = TR_PREFILL_ROWS;
constexpr int ATTN_MAX_SPLITS = 16;
constexpr int GEMM_MAX_SPLITS = 4;

Workspace plan_workspace(const tr_model &m);

// ---------------------------------------------------------------------------------------------
// optional per-kernel timing.  While enabled, every kernel of the step is launched with a start and a
// stop event attached to the dispatch itself (hipExtLaunchKernelGGL), so the elapsed time between the
// two is the kernel's own duration, without the launch latency an event pair recorded around a launch
// would include.
// ---------------------------------------------------------------------------------------------
enum ProfCat { PC_BUILD = 0, PC_EMBED, PC_NORM, PC_QKV, PC_ROPE, PC_ATTN, PC_ATTN_MERGE, PC_OPROJ, PC_GATEUP, PC_DOWN,
               PC_LMHEAD, PC_TOPK, PC_TOPK_MERGE, PC_ACCEPT, PC_COMPACT, PC_SAMPLE, PC_COUNT };
struct KernelTimer {
  hipEvent_t start = nullptr, stop = nullptr; // both null: launch untimed
};
struct Profiler {
  static constexpr int MAX_PAIRS = 8192;
  hipEvent_t *ev = nullptr; // 2 * MAX_PAIRS
  int8_t *cat = nullptr;    // MAX_PAIRS
  int used = 0;
  bool enabled = false;
  KernelTimer next(ProfCat c) {
    KernelTimer t;
    if (enabled && used < MAX_PAIRS) {
      cat[used] = (int8_t)c;
      t.start = ev[2 * used];
      t.stop = ev[2 * used + 1];
      ++used;
    }
    return t;
  }
};
inline KernelTimer prof_next(Profiler *p, ProfCat c) { return p != nullptr ? p->next(c) : KernelTimer{}; }

// One place through which every kernel of the library is launched.
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t smem, hipStream_t st, KernelTimer t,
                         Args... args) {
  if (t.start != nullptr)
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, st, t.start, t.stop, 0u, static_cast<KArgs>(args)...);
  else
    hipLaunchKernelGGL(kernel, grid, block, smem, st, static_cast<KArgs>(args)...);
  return hipGetLastError();
}

} // namespace tr

struct tr_ctx {
  int32_t V, k;
  int32_t device;
  int32_t *d_M;          // [V, k]
  tr::TreeDev tree;      // the static draft tree
  tr::TreeDev chain;     // chain of TR_MAX_NODES nodes (prefill chunks)
  void *d_tree_blob;     // backing store of both trees
  int32_t *d_step_L;     // committed length at the start of the current accept/update
  void *d_topk_cand;     // per-segment top-k candidates (two-stage top-k)
  int32_t update_mode;   // tr_update_mode bits
  tr::Profiler prof;
};

namespace tr {

// --- integer kernels (tr_int_kernels.hip) -------------------------------------------------------
hipError_t launch_build_tree(tr_ctx *c, const int32_t *d_root, int32_t *d_S, hipStream_t s);
// d_cand: scratch of topk_scratch_bytes() owned by the context (may be NULL: slower one-kernel path)
hipError_t launch_topk(const void *logits, int32_t dtype, int32_t rows, int32_t V, int32_t k,
                       int32_t *d_topk, void *d_cand, Profiler *prof, hipStream_t s);
size_t topk_scratch_bytes();
// the same two-stage kernels on the library's static device scratch (no allocation anywhere)
bool topk_static_fits(int32_t rows, int32_t V, int32_t k);
hipError_t launch_topk_static(const void *logits, int32_t dtype, int32_t rows, int32_t V, int32_t k,
                              int32_t *d_topk, hipStream_t s);
hipError_t launch_matrix_update(const tr_ctx *c, const int32_t *d_S, const int32_t *d_topk, hipStream_t s);
// d_tokens: the model's token per node, or NULL for the argmax (first top-k column)
hipError_t launch_accept_update(tr_ctx *c, const tr_kv *kv, const int32_t *d_S,
                                const int32_t *d_topk, const int32_t *d_tokens, tr_step_out *d_out, hipStream_t s);
hipError_t launch_sample_tokens(tr_ctx *c, const tr_kv *kv, const float *d_logits, const float *d_noise,
                                int32_t pos0, int32_t noise_rows, float inv_t, int32_t *d_tokens, hipStream_t s);
hipError_t launch_advance_len(int32_t *d_len, int32_t by, hipStream_t s);
hipError_t launch_stream(const void *src, void *dst, size_t bytes, hipStream_t s);

// --- forward pass (tr_forward.hip) -----------------------------------------------------------------
// Runs rows `tokens` through the model.  `write_logits` may be NULL (no LM head).
hipError_t run_forward(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n,
                       const int32_t *d_tokens, float *write_logits, void *ws, Profiler *prof, hipStream_t s);
// Prompt ingestion: rows one pass may take for this model and cache (NPW on the packed path with a tiled cache,
// else NP), and the pass itself: n consecutive prompt tokens, causal, keys / values appended at the committed
// length (which the caller advances afterwards), no logits.
int32_t prefill_rows(const tr_model &m, const tr_kv &kv);
hipError_t run_prefill_pass(const tr_model &m, const tr_kv &kv, const TreeDev &chain, int32_t n,
                            const int32_t *d_tokens, void *ws, hipStream_t s);
hipError_t run_tree_attention(const tr_kv &kv, int32_t layer, int32_t H, const TreeDev &tree,
                              const void *d_q, void *d_out, void *ws, hipStream_t s);
size_t linear_workspace_bytes(int32_t n, int32_t in_f, int32_t out_f, int32_t splits);
hipError_t run_linear(const void *x, const void *w, int32_t dtype, int32_t layout, int32_t n, int32_t in_f,
                      int32_t out_f, int32_t splits, float *y, void *ws, hipStream_t s);
bool model_layout_ok(const tr_model &m);

} // namespace tr
